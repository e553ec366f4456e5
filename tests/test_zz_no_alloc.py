"""spin_beaver_matmul_static, the entry point for callers that cannot allocate: called through the C ABI
on the library's built-in workspace and compared word for word with spin_beaver_matmul on a caller-provided
workspace (which the other tests compare with the oracle), on two calls in a row, the second with a smaller
input, so that whatever the first call left in the shared array must not matter."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2402_02320_amd import spin

pytestmark = pytest.mark.gpu

EWORKSPACE = 3


def operands(rng, n, batch, M, N, K):
    def u(shape):
        return torch.from_numpy(rng.integers(0, 1 << 64, size=shape, dtype=np.uint64).view(np.int64)).cuda()
    return u((n, batch, M, K)), u((n, batch, K, N)), u((n, batch, M, K)), u((n, batch, K, N)), u((n, batch, M, N))


@pytest.mark.parametrize("path", [pytest.param(spin.LIMB_MFMA, id="limb"), pytest.param(spin.VALU, id="valu")])
def test_static_workspace_call_matches_the_call_with_a_workspace(path):
    rng = np.random.default_rng(2024)
    # first a product that fills most of the array (3 parties, 64 attention-sized matrices: 32 MiB of fragments,
    # with a ragged 130 x 70 x 45 tail case after it), then smaller ones
    for n, batch, M, N, K in [(3, 64, 128, 128, 64), (3, 2, 130, 70, 45), (2, 1, 33, 31, 32), (5, 1, 1, 1, 1)]:
        X, Y, A, B, C = operands(rng, n, batch, M, N, K)
        assert spin.beaver_matmul_workspace_bytes(n, batch, M, N, K, path) <= spin.STATIC_WORKSPACE_BYTES
        want = spin.beaver_matmul(X, Y, A, B, C, path=path)
        got = torch.empty_like(C)
        spin.beaver_matmul_static(X, Y, A, B, C, got, path=path)
        assert torch.equal(got, want), (n, batch, M, N, K)
        # in place on C, as the other call allows
        Cc = C.clone()
        spin.beaver_matmul_static(X, Y, A, B, Cc, Cc, path=path)
        assert torch.equal(Cc, want), (n, batch, M, N, K)


def test_static_workspace_call_rejects_what_does_not_fit():
    L = spin.lib()
    n, M = 2, 2048                                        # 3 slots x 2 sides x 2048^2 x 8 bytes = 192 MiB of fragments
    assert spin.beaver_matmul_workspace_bytes(n, 1, M, M, M) > spin.STATIC_WORKSPACE_BYTES
    fake = ctypes.c_void_p(0x1000)                        # never dereferenced: the size check comes before any launch
    assert L.spin_beaver_matmul_static(n, 1, M, M, M, fake, fake, fake, fake, fake, fake, spin.LIMB_MFMA, None) == EWORKSPACE
    assert L.spin_beaver_matmul_static(n, 1, 0, M, M, fake, fake, fake, fake, fake, fake, spin.LIMB_MFMA, None) == 1
    assert L.spin_beaver_matmul_static(n, 1, 8, 8, 8, None, fake, fake, fake, fake, fake, spin.LIMB_MFMA, None) == 1
