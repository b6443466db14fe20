"""The entry points enqueue kernels only (no allocation, no memset, no synchronisation), so a
caller may capture them in a HIP graph.  Replays are interleaved with eager work and checked
against the eager result every time."""
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


def test_graph_replays_match_eager(oracle):
    w = synth.make_workload("edge_encoder", shape=(4, 8, 128, 128))
    a = synth.make_workload("fused_attention", shape=(2, 3, 256, 64))
    x = torch.from_numpy(w["logits"]).cuda()
    q, k, v = (torch.from_numpy(a[t]).cuda() for t in ("q", "k", "v"))
    p_eager = binding.calibrated_softmax_i8(x, w["table"], w["band"])
    p16_eager = binding.calibrated_softmax_i8_ex(x, w["table"], w["band"], out_scale_T=32767)
    o_eager = binding.attention_i8(q, k, v, a["table"], a["requant"], a["band"])
    torch.cuda.synchronize()
    want, rc = oracle.softmax(w["logits"], w["table"], w["band"])
    assert rc == 0 and np.array_equal(p_eager.cpu().numpy(), want)

    p = torch.zeros_like(p_eager)
    p16 = torch.zeros_like(p16_eager)
    o = torch.zeros_like(o_eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        binding.calibrated_softmax_i8(x, w["table"], w["band"], out=p)
        binding.calibrated_softmax_i8_ex(x, w["table"], w["band"], out_scale_T=32767, out=p16)
        binding.attention_i8(q, k, v, a["table"], a["requant"], a["band"], out=o)
    for rep in range(4):
        p.fill_(7)
        p16.fill_(7)
        o.fill_(7)
        scratch = torch.randn(1 << 20, device="cuda").sum()      # unrelated eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(p, p_eager) and torch.equal(p16, p16_eager) and torch.equal(o, o_eager), rep
        assert bool(torch.isfinite(scratch))
