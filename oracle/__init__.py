"""CPU oracle of the K-means hot path -- test infrastructure only (see cpu.py, abft.py)."""
