"""The calibration entry point that allocates nothing (hccs_calibrate_grid_static) against the
one that takes a caller's workspace (hccs_calibrate_grid): same sums in the same order, so the
objective tables and the arg-min must be equal bit for bit.  Two calls in a row, the second on a
smaller problem, so that anything the first call left in the library's static work buffer would
show; then the size limit."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_2604_02292_amd import binding, synth  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()


def _candidates(n, count, seed):
    g = np.random.default_rng(seed)
    bmax, f = 32767 // n, -(-256 // n)
    out = np.zeros((count, 4), np.int32)
    for i in range(count):
        D = int(g.integers(0, 128))
        B = int(g.integers(f, bmax + 1))
        out[i, :3] = (B, int(g.integers(0, min(127, (B - f) // max(D, 1)) + 1)), D)
    out[1, :3] = (bmax + 1, 0, 1)        # one inadmissible candidate: +infinity on both sides
    return out


def test_static_scratch_calibration_equals_workspace_calibration():
    lib = binding.lib()
    for shape, count in (((6, 4, 24, 128), 150), ((2, 3, 9, 64), 40)):   # the second call is the smaller one
        print(f"no-alloc calibration case shape={shape} candidates={count}", flush=True)
        H, n = shape[1], shape[3]
        x = torch.from_numpy(synth.make_workload("edge_encoder", shape=shape)["logits"]).cuda()
        alpha = np.linspace(0.04, 0.2, H)
        cand = _candidates(n, count, seed=n)
        want_obj, want_best = binding.calibrate_grid(x, alpha, cand[:, :3])
        cand_dev = torch.from_numpy(cand).cuda()
        obj = torch.full((H, count), -1.0, dtype=torch.float64, device="cuda")
        best = torch.full((H,), -7, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        binding.calibrate_grid_static(x, alpha, cand_dev, obj, best)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert np.array_equal(obj.cpu().numpy().view(np.uint64), want_obj.cpu().numpy().view(np.uint64))
        assert np.array_equal(best.cpu().numpy(), want_best.cpu().numpy())
        assert np.isinf(obj.cpu().numpy()[:, 1]).all() and np.isfinite(obj.cpu().numpy()[:, 0]).all()

    # a problem beyond the static buffer is refused before anything is launched
    B, H, Lq, Lk = 80, 8, 128, 128
    assert lib.hccs_calibrate_workspace_bytes(B, H, Lq, Lk) > 36 * 1024 * 1024
    obj = torch.full((H, 4), -1.0, dtype=torch.float64, device="cuda")
    best = torch.full((H,), -7, dtype=torch.int32, device="cuda")
    x = torch.zeros((B, H, Lq, Lk), dtype=torch.int8, device="cuda")
    with pytest.raises(binding.HccsError) as e:
        binding.calibrate_grid_static(x, [0.1] * H, torch.from_numpy(_candidates(Lk, 4, 1)).cuda(), obj, best)
    assert e.value.status == -10
    torch.cuda.synchronize()
    assert bool((obj == -1.0).all()) and bool((best == -7).all())
    # the largest calibration set it is sized for: 64 batches of [8, 128, 128]
    assert lib.hccs_calibrate_workspace_bytes(64, 8, 128, 128) <= 36 * 1024 * 1024
