"""MI355X-native hot path of fault-tolerant K-means (assignment, update, Lloyd loop)."""
