"""CPU checks of the closed forms the limb-decomposed GEMM relies on (Python integers / numpy, no GPU
code involved), of the workload generators and of bench.py's argument handling."""
import os
import subprocess
import sys

import numpy as np

from paper_2402_02320_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
M64 = (1 << 64) - 1
BIAS = 0x8080808080808080


def digits(a, limbs=8):
    """Balanced digits of a (mod 2^(8*limbs)) by the add-then-xor rule the pack kernels use."""
    mask = (1 << (8 * limbs)) - 1
    bias = int.from_bytes(b"\x80" * limbs, "little")
    t = ((a + bias) & mask) ^ bias
    out = []
    for i in range(limbs):
        byte = (t >> (8 * i)) & 0xFF
        out.append(byte - 256 if byte >= 128 else byte)
    return out


def test_balanced_digit_identity():
    rng = np.random.default_rng(1)
    vals = [0, 1, M64, 0x7F7F7F7F7F7F7F80, 0x8080808080808080, 0x7F, 0x80, 0xFF, 1 << 63] + \
        [int(v) for v in rng.integers(0, 1 << 64, size=2000, dtype=np.uint64)]
    for a in vals:
        s = digits(a)
        assert all(-128 <= d <= 127 for d in s)
        assert sum(d << (8 * i) for i, d in enumerate(s)) % (1 << 64) == a
    assert digits(0x7F7F7F7F7F7F7F80) == [-128] * 8        # the worst case the GPU test feeds


def test_two_limb_analogue_is_exhaustive():
    # 16-bit ring, 2 digits, 3 surviving pairs: every a against a spread of b
    bs = [0, 1, 0x7F80, 0x8080, 0xFFFF, 0x1234, 0xFEDC, 0x00FF, 0xFF00]
    for a in range(1 << 16):
        s = digits(a, 2)
        assert (s[0] + (s[1] << 8)) % (1 << 16) == a
        for b in bs:
            t = digits(b, 2)
            got = (s[0] * t[0] + ((s[0] * t[1] + s[1] * t[0]) << 8)) % (1 << 16)
            assert got == (a * b) % (1 << 16)


def test_36_pair_product_identity_and_dropped_pairs():
    rng = np.random.default_rng(2)
    for _ in range(2000):
        a, b = (int(v) for v in rng.integers(0, 1 << 64, size=2, dtype=np.uint64))
        s, t = digits(a), digits(b)
        kept = sum((s[i] * t[j]) << (8 * (i + j)) for i in range(8) for j in range(8) if i + j <= 7)
        dropped = sum((s[i] * t[j]) << (8 * (i + j)) for i in range(8) for j in range(8) if i + j > 7)
        assert kept % (1 << 64) == (a * b) % (1 << 64)
        assert dropped % (1 << 64) == 0
    assert sum(1 for i in range(8) for j in range(8) if i + j <= 7) == 36


def test_int32_accumulators_with_wraparound_recombine_exactly():
    # inner dimension at the per-launch maximum (2 * 511 k-tiles of 32), worst-case and random digits:
    # diagonals 0..3 must fit int32 exactly, diagonals 4..7 may wrap and still recombine to the right value
    ktot = 2 * 511 * 32
    assert 4 * ktot * (1 << 14) < (1 << 31)
    rng = np.random.default_rng(3)
    for worst in (True, False):
        if worst:
            a = np.full(ktot, 0x7F7F7F7F7F7F7F80, dtype=np.uint64)
            b = a.copy()
        else:
            a = rng.integers(0, 1 << 64, size=ktot, dtype=np.uint64)
            b = rng.integers(0, 1 << 64, size=ktot, dtype=np.uint64)
        sa = np.array([digits(int(v)) for v in a], dtype=np.int64)      # [ktot, 8]
        sb = np.array([digits(int(v)) for v in b], dtype=np.int64)
        want = sum(int(x) * int(y) for x, y in zip(a, b)) % (1 << 64)
        total = 0
        for d in range(8):
            exact = sum(int(np.dot(sa[:, i], sb[:, d - i])) for i in range(d + 1))
            if d <= 3:
                assert -(1 << 31) <= exact < (1 << 31)
            wrapped = (exact + (1 << 31)) % (1 << 32) - (1 << 31)       # what an int32 accumulator holds
            total += wrapped << (8 * d)
        assert total % (1 << 64) == want


def wrapped_diagonal_dot(a_vals, b_vals, limbs):
    """sum_k a_k b_k mod 2^(8 limbs) from int32 accumulators that wrap, one per diagonal."""
    sa = np.array([digits(int(v), limbs) for v in a_vals], dtype=object)
    sb = np.array([digits(int(v), limbs) for v in b_vals], dtype=object)
    total, exact_by_diag = 0, []
    for d in range(limbs):
        exact = sum(int(sum(int(x) * int(y) for x, y in zip(sa[:, i], sb[:, d - i]))) for i in range(d + 1))
        exact_by_diag.append(exact)
        total += ((exact + (1 << 31)) % (1 << 32) - (1 << 31)) << (8 * d)
    return total % (1 << (8 * limbs)), exact_by_diag


def test_four_digit_ring_never_needs_an_inner_dimension_split():
    # Z_2^32: 10 pairs, 4 diagonals, each needing at most 32 exact bits, so wrapped accumulators are
    # right at any length; the all-(-128) operands overflow int32 on diagonals 1..3 here
    assert sum(1 for i in range(4) for j in range(4) if i + j <= 3) == 10
    k = 70000
    a = [0x7F7F7F80] * k
    got, exact = wrapped_diagonal_dot(a, a, 4)
    assert all(abs(e) >= (1 << 31) for e in exact[1:])
    assert got == (k * 0x7F7F7F80 * 0x7F7F7F80) % (1 << 32)
    rng = np.random.default_rng(4)
    a, b = rng.integers(0, 1 << 32, size=(2, 3000), dtype=np.uint64)
    got, _ = wrapped_diagonal_dot(a, b, 4)
    assert got == sum(int(x) * int(y) for x, y in zip(a, b)) % (1 << 32)


def test_sixteen_digit_ring_chunk_limit():
    # Z_2^128: 136 pairs; diagonals 0..11 must be exact, which 2 * 170 k-tiles of 32 per launch guarantee
    assert sum(1 for i in range(16) for j in range(16) if i + j <= 15) == 136
    ktot = 2 * 170 * 32
    assert 12 * ktot * (1 << 14) < (1 << 31) <= 12 * (2 * 171 * 32) * (1 << 14)
    worst = int.from_bytes(b"\x80" + b"\x7f" * 15, "little")
    assert digits(worst, 16) == [-128] * 16
    a = [worst] * ktot
    got, exact = wrapped_diagonal_dot(a, a, 16)
    assert all(-(1 << 31) <= e < (1 << 31) for e in exact[:12])
    assert got == (ktot * worst * worst) % (1 << 128)


def test_missing_library_raises_instead_of_falling_back(monkeypatch, tmp_path):
    from paper_2402_02320_amd import spin
    monkeypatch.setattr(spin, "_lib", None)
    monkeypatch.setattr(spin, "LIB_PATH", str(tmp_path / "libspin.so"))
    try:
        spin.lib()
    except spin.SpinError as e:
        assert "not found" in str(e)
    else:
        raise AssertionError("a missing library must raise")


def test_product_code_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2402_02320_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, name)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, name
                assert "spin_oracle" not in text, name


def test_config_table_matches_the_benchmark_definition():
    c = workloads.CONFIGS
    assert (c[1].n, c[1].gemms[0].M, c[1].gemms[0].N, c[1].gemms[0].K) == (3, 64, 64, 64)
    assert (c[2].n, c[2].gemms[0].M, c[2].vec) == (2, 1024, 1 << 24)
    g3 = c[3].gemms[0]
    assert (c[3].n, g3.M, g3.K, g3.N) == (3, 128 * 32 * 32, 64 * 3 * 3, 64)
    assert (c[4].n, c[4].gemms[0].batch, c[4].gemms[0].K, c[4].gemms[1].K, c[4].vec) == (3, 64, 64, 128, 8 * 8 * 128 * 128)
    assert (c[5].n, c[5].gemms[0].M) == (5, 4096)
    assert all(v.f == 16 for v in c.values())


def test_im2col_reproduces_a_direct_convolution():
    rng = np.random.default_rng(4)
    fmap = rng.normal(size=(2, 3, 5, 6))
    w = rng.normal(size=(4, 3, 3, 3))                              # [out, in, 3, 3]
    cols = workloads.im2col_3x3(fmap)                              # [B*H*W, C*9]
    got = (cols @ w.reshape(4, -1).T).reshape(2, 5, 6, 4).transpose(0, 3, 1, 2)
    pad = np.pad(fmap, ((0, 0), (0, 0), (1, 1), (1, 1)))
    want = np.zeros((2, 4, 5, 6))
    for dy in range(3):
        for dx in range(3):
            want += np.einsum("bchw,oc->bohw", pad[:, :, dy:dy + 5, dx:dx + 6], w[:, :, dy, dx])
    assert np.allclose(got, want)


def test_plaintexts_are_seeded_and_shaped():
    X, Y = workloads.gemm_plaintexts(1)
    X2, _ = workloads.gemm_plaintexts(1)
    assert X.shape == (1, 64, 64) and Y.shape == (1, 64, 64) and (X == X2).all()
    assert np.abs(X).max() <= 1.0
    Xs, Ys = workloads.gemm_plaintexts(3, scale=2 / 128)
    assert Xs.shape == (1, 2048, 576) and Ys.shape == (1, 576, 64)
    Q, KT = workloads.gemm_plaintexts(4, 0, scale=1 / 8)
    assert Q.shape == (8, 128, 64) and KT.shape == (8, 64, 128)


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
