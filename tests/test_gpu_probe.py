"""The MFMA-rate probe (a measurement aid of the library) computes what its header says: checked against
numpy integer matrix products built from the documented operand and accumulator layouts of
v_mfma_i32_32x32x32_i8 (lane l of an operand holds row l % 32, k = 16 (l / 32) .. + 15; accumulator
register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32)."""
import numpy as np
import pytest
import torch

from paper_2402_02320_amd import spin

pytestmark = pytest.mark.gpu


def fragment_matrix(frag_bytes):
    """1 KiB fragment -> 32 x 32 int8 matrix [row or column][k]."""
    lanes = frag_bytes.reshape(64, 16).view(np.int8)
    m = np.zeros((32, 32), dtype=np.int64)
    for l in range(64):
        m[l % 32, 16 * (l // 32):16 * (l // 32) + 16] = lanes[l]
    return m


@pytest.mark.parametrize("iters", [1, 3])
def test_probe_sums_match_numpy(iters):
    rng = np.random.default_rng(5)
    raw = rng.integers(0, 256, size=24 * 1024, dtype=np.uint8)
    ops = torch.from_numpy(raw.view(np.int64).copy()).cuda()
    sink = spin.probe_mfma(ops, blocks=2, iters=iters).cpu().numpy()
    frags = [fragment_matrix(raw[f * 1024:(f + 1) * 1024]) for f in range(24)]
    left = [frags[0:8], frags[8:16]]
    right = frags[16:24]
    total = np.zeros((32, 32), dtype=np.int64)
    for t in range(2):
        for da in range(8):
            for db in range(8 - da):
                total += left[t][da] @ right[db].T
    total *= iters
    want = np.zeros(64, dtype=np.int64)
    for l in range(64):
        rows = [8 * (r // 4) + 4 * (l // 32) + r % 4 for r in range(16)]
        want[l] = total[rows, l % 32].sum()
    want = ((want + 2 ** 31) % 2 ** 32) - 2 ** 31                  # the kernel's sum wraps as int32
    assert sink.shape == (512,)
    assert (sink.reshape(8, 64) == want[None, :]).all()            # every wave of every block the same


def test_probe_with_zero_operands_and_validation():
    ops = torch.zeros(24 * 128, dtype=torch.int64, device="cuda")
    assert int(spin.probe_mfma(ops, blocks=4, iters=10).abs().max()) == 0
    with pytest.raises(spin.SpinError):
        spin.probe_mfma(ops, blocks=0, iters=1, sink=torch.empty(256, dtype=torch.int64, device="cuda"))
