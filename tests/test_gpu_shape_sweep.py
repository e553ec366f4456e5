"""Seeded sweep over ragged Beaver-matmul shapes on every ring and GEMM path: sizes straddle the 32-wide MFMA
blocks, the 64/128-wide workgroup tiles and the 32-deep k-tiles, with party counts 1..8 and small batches.
Every output word is compared with the oracle."""
import numpy as np
import pytest
import torch

import oracle
from oracle import r128
from paper_2402_02320_amd import spin

pytestmark = pytest.mark.gpu
M32 = np.uint64(0xFFFFFFFF)


def shapes(seed, count, max_mn, max_k):
    rng = np.random.default_rng(seed)
    edges = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 255, 256, 257]
    out = []
    for _ in range(count):
        n = int(rng.integers(1, 9))
        batch = int(rng.integers(1, 4))
        pick = lambda hi: int(rng.choice([e for e in edges if e <= hi])) if rng.random() < 0.5 else int(rng.integers(1, hi + 1))
        out.append((n, batch, pick(max_mn), pick(max_mn), pick(max_k)))
    return out


def dev64(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def dev32(a):
    return torch.from_numpy(np.ascontiguousarray(a.astype(np.uint32)).view(np.int32)).cuda()


@pytest.mark.parametrize("path", [spin.LIMB_MFMA, spin.VALU])
def test_sweep_ring64(path):
    for idx, (n, batch, M, N, K) in enumerate(shapes(64, 40, 300, 200)):
        rng = np.random.default_rng(1000 + idx)
        X = rng.integers(0, 1 << 64, size=(n, batch, M, K), dtype=np.uint64)
        Y = rng.integers(0, 1 << 64, size=(n, batch, K, N), dtype=np.uint64)
        A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=idx)
        want = oracle.beaver_matmul(X, Y, A, B, C)
        got = spin.beaver_matmul(dev64(X), dev64(Y), dev64(A), dev64(B), dev64(C), path=path)
        assert (got.cpu().numpy().view(np.uint64) == want).all(), (n, batch, M, N, K)


@pytest.mark.parametrize("path", [spin.LIMB_MFMA, spin.VALU])
def test_sweep_ring32(path):
    for idx, (n, batch, M, N, K) in enumerate(shapes(32, 30, 300, 200)):
        rng = np.random.default_rng(2000 + idx)
        X = rng.integers(0, 1 << 32, size=(n, batch, M, K), dtype=np.uint64)
        Y = rng.integers(0, 1 << 32, size=(n, batch, K, N), dtype=np.uint64)
        A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=idx, l=32)
        want = oracle.beaver_matmul(X, Y, A, B, C, l=32)
        got = spin.ring32.beaver_matmul(dev32(X), dev32(Y), dev32(A), dev32(B), dev32(C), path=path)
        assert (got.cpu().numpy().view(np.uint32).astype(np.uint64) == want).all(), (n, batch, M, N, K)


@pytest.mark.parametrize("path", [spin.LIMB_MFMA, spin.VALU])
def test_sweep_ring128(path):
    for idx, (n, batch, M, N, K) in enumerate(shapes(128, 16, 150, 100)):
        rng = np.random.default_rng(3000 + idx)
        X = rng.integers(0, 1 << 64, size=(n, batch, M, K, 2), dtype=np.uint64)
        Y = rng.integers(0, 1 << 64, size=(n, batch, K, N, 2), dtype=np.uint64)
        A, B, C = r128.dealer_matmul(n, batch, M, N, K, seed=idx)
        want = r128.beaver_matmul(X, Y, A, B, C)
        got = spin.ring128.beaver_matmul(dev64(X), dev64(Y), dev64(A), dev64(B), dev64(C), path=path)
        assert (got.cpu().numpy().view(np.uint64) == want).all(), (n, batch, M, N, K)


def test_sweep_row_kernel_domain():
    # at most three parties, an even inner dimension, one to a few column tiles: the shapes the row-streaming limb
    # kernel takes (inner dimensions of 1 .. 40 k-tiles walk every phase of its three-slot ring), plain and with
    # the right operand stored transposed
    rng = np.random.default_rng(2024)
    for idx in range(120):
        n, batch = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        M = int(rng.choice([1, 31, 32, 33, 64, 95, 100, 257, 1000])) if rng.random() < 0.5 else int(rng.integers(1, 600))
        N = int(rng.choice([1, 31, 32, 33, 63, 64, 65, 96, 128, 130, 192])) if rng.random() < 0.6 else int(rng.integers(1, 200))
        K = 2 * int(rng.integers(1, 130)) if rng.random() < 0.8 else 2 * int(rng.integers(100, 640))
        r = np.random.default_rng(idx)
        X = r.integers(0, 1 << 64, size=(n, batch, M, K), dtype=np.uint64)
        Y = r.integers(0, 1 << 64, size=(n, batch, K, N), dtype=np.uint64)
        A, B, C = oracle.dealer_matmul(n, batch, M, N, K, seed=idx)
        want = oracle.beaver_matmul(X, Y, A, B, C)
        got = spin.beaver_matmul(dev64(X), dev64(Y), dev64(A), dev64(B), dev64(C), path=spin.LIMB_MFMA)
        assert (got.cpu().numpy().view(np.uint64) == want).all(), (n, batch, M, N, K)
        Yt, Bt = (dev64(np.ascontiguousarray(t.transpose(0, 1, 3, 2))) for t in (Y, B))
        got_t = spin.beaver_matmul(dev64(X), Yt, dev64(A), Bt, dev64(C), path=spin.LIMB_MFMA, y_transposed=True)
        assert torch.equal(got, got_t), (n, batch, M, N, K)
