"""How the matrix instructions round, held against exact arithmetic.  v_mfma_f32_32x32x16_bf16:  The error bounds of the
reduced-precision assignment (the counterpart of the paper's TF32 path, Section 3.1.5) budget 7 u
of an instruction's magnitude M = |accumulator| + sum |products| per instruction, u = 2^-24; no
document states how the instruction rounds, so this test is what the budget stands on: the 16
products of bf16 operands are exact, and the measured error of the sum stays below 6.25 u M on
random, wide-range, cancelling and one-sided operands."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2408_01391_amd import ablation

pytestmark = pytest.mark.gpu
U = 2.0 ** -24


def _to_bf16_bits(x):
    """float32 -> bf16 bit patterns, round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (b + 0x7FFF + ((b >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def _from_bf16_bits(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _run(A, B, C):
    """A [T,32,16], B [T,16,32] float32 (rounded to bf16 here), C [T,32,32] float32."""
    if not ablation._LIB_PATH.exists():
        pytest.skip("libftk_ablation.so not built (run python __graft_entry__.py)")
    dev = torch.device("cuda:0")
    Ab, Bb = _to_bf16_bits(A), _to_bf16_bits(B)
    Dd = ablation.mfma_bf16(torch.from_numpy(Ab.view(np.int16)).to(dev), torch.from_numpy(Bb.view(np.int16)).to(dev),
                            torch.from_numpy(np.ascontiguousarray(C, dtype=np.float32)).to(dev))
    torch.cuda.synchronize()
    a64 = _from_bf16_bits(Ab).astype(np.float64)
    b64 = _from_bf16_bits(Bb).astype(np.float64)
    c64 = C.astype(np.float64)
    exact = np.einsum("tik,tkj->tij", a64, b64) + c64           # products exact, 17 terms in double
    mag = np.einsum("tik,tkj->tij", np.abs(a64), np.abs(b64)) + np.abs(c64)
    err = np.abs(Dd.cpu().numpy().astype(np.float64) - exact)
    return err, mag, exact


def _ratio(err, mag):
    ok = mag > 0
    return float((err[ok] / (U * mag[ok])).max())


def test_layout_exact_on_small_integers():
    """Integer operands: every product and the sum are exact, so D must equal A B + C bit for bit
    (also pins the lane layout of the probe kernel)."""
    rng = np.random.default_rng(0)
    A = rng.integers(-8, 9, size=(64, 32, 16)).astype(np.float32)
    B = rng.integers(-8, 9, size=(64, 16, 32)).astype(np.float32)
    C = rng.integers(-100, 101, size=(64, 32, 32)).astype(np.float32)
    err, _, _ = _run(A, B, C)
    assert err.max() == 0.0


CASES = ["normal", "wide range", "accumulator dominant", "cancelling", "one-sided", "tiny accumulator"]


@pytest.mark.parametrize("case", CASES)
def test_error_of_one_instruction_is_below_the_budget(case):
    rng = np.random.default_rng(100 + CASES.index(case))
    T = 2048
    A = rng.normal(size=(T, 32, 16))
    B = rng.normal(size=(T, 16, 32))
    C = rng.normal(size=(T, 32, 32)) * 4.0
    if case == "wide range":
        A *= 2.0 ** rng.integers(-12, 13, size=A.shape)
        B *= 2.0 ** rng.integers(-12, 13, size=B.shape)
        C *= 2.0 ** rng.integers(-20, 21, size=C.shape)
    elif case == "accumulator dominant":
        C *= 2.0 ** 12
    elif case == "tiny accumulator":
        C *= 2.0 ** -20
    elif case == "one-sided":
        A, B, C = np.abs(A), np.abs(B), np.abs(C)
    A = A.astype(np.float32)
    B = B.astype(np.float32)
    C = C.astype(np.float32)
    if case == "cancelling":  # the accumulator nearly cancels the products: the result is tiny against M
        a64 = _from_bf16_bits(_to_bf16_bits(A)).astype(np.float64)
        b64 = _from_bf16_bits(_to_bf16_bits(B)).astype(np.float64)
        C = (-np.einsum("tik,tkj->tij", a64, b64) * (1.0 + rng.normal(size=C.shape) * 1e-3)).astype(np.float32)
    err, mag, _ = _run(A, B, C)
    worst = _ratio(err, mag)
    print("mfma bf16 rounding,", case, ": max error %.2f u M" % worst, flush=True)
    assert worst <= 6.25, "the instruction errs by %.2f u of its magnitude: the fast paths budget 7 u" % worst


def test_exponent_gaps_lose_at_most_three_guard_bits():
    """One large addend and sixteen small ones far below it: what is dropped of each small addend is
    below 2^-26 of the large one (three guard bits under the fp32 unit), so the sum of the losses
    stays inside the budget however the small addends are chosen."""
    rng = np.random.default_rng(4)
    T = 1024
    A = np.ones((T, 32, 16), dtype=np.float32)
    for shift in (20, 23, 24, 25, 26, 27, 30):
        B = (rng.uniform(1.0, 2.0, size=(T, 16, 32)) * 2.0 ** -shift).astype(np.float32)
        C = rng.uniform(1.0, 2.0, size=(T, 32, 32)).astype(np.float32)
        err, mag, _ = _run(A, B, C)
        worst = _ratio(err, mag)
        print("small addends at 2^-%d of the accumulator: max error %.2f u M" % (shift, worst), flush=True)
        assert worst <= 6.25


# ---- the fp32 and fp64 instructions of the main path -------------------------------------------
def _round_to(q, dtype):
    """Fraction -> nearest dtype value, ties to even, without double rounding."""
    d = float(q)  # correctly rounded double
    if dtype == np.float64:
        return d
    f = np.float32(d)
    cands = [np.nextafter(f, np.float32(-np.inf)), f, np.nextafter(f, np.float32(np.inf))]
    best = min(cands, key=lambda c: (abs(Fraction(float(c)) - q), int(np.float32(c).view(np.uint32)) & 1))
    return float(best)


def _fma_chain(a_row, b_col, c, dtype):
    """c, then one fused multiply-add per contraction step in index order, each rounded to dtype."""
    s = Fraction(float(c))
    for a, b in zip(a_row, b_col):
        s = Fraction(_round_to(Fraction(float(a)) * Fraction(float(b)) + s, dtype))
    return float(s)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_fp32_and_fp64_instructions_are_chains_of_fused_multiply_adds(dtype):
    """Every output equals, bit for bit, the accumulator followed by one fused multiply-add per
    contraction index in order (exact rational arithmetic rounded once per step): the chain the
    rounding band 2 (D + 4) u of the assignment assumes."""
    if not ablation._LIB_PATH.exists():
        pytest.skip("libftk_ablation.so not built (run python __graft_entry__.py)")
    rng = np.random.default_rng(11)
    m, k = (32, 2) if dtype == np.float32 else (16, 4)
    T = 6
    dev = torch.device("cuda:0")
    for scale in ("normal", "wide range", "cancelling"):
        A = rng.normal(size=(T, m, k))
        B = rng.normal(size=(T, k, m))
        C = rng.normal(size=(T, m, m))
        if scale == "wide range":
            A *= 2.0 ** rng.integers(-10, 11, size=A.shape)
            B *= 2.0 ** rng.integers(-10, 11, size=B.shape)
            C *= 2.0 ** rng.integers(-20, 21, size=C.shape)
        A, B = A.astype(dtype), B.astype(dtype)
        if scale == "cancelling":
            C = -np.einsum("tik,tkj->tij", A.astype(np.float64), B.astype(np.float64)) * (1 + 1e-4 * rng.normal(size=C.shape))
        C = C.astype(dtype)
        D = ablation.mfma_plain(torch.from_numpy(A).to(dev), torch.from_numpy(B).to(dev), torch.from_numpy(C).to(dev))
        torch.cuda.synchronize()
        D = D.cpu().numpy()
        mismatches = 0
        for t in range(T):
            for i in range(m):
                for j in range(m):
                    want = _fma_chain(A[t, i, :], B[t, :, j], C[t, i, j], dtype)
                    mismatches += int(dtype(want) != D[t, i, j])
        print("mfma", np.dtype(dtype).name, scale, ": outputs differing from the fma chain:", mismatches, "of", T * m * m, flush=True)
        assert mismatches == 0
