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


def test_graph_replays_ragged_and_streaming(oracle):
    """The kernels with LDS exchange and barriers (ragged rows, both streaming fused forms, the resident fused form
    at a length that is no multiple of 64) under graph replay: every replay equals the eager result, which equals
    the oracle."""
    g0 = np.random.default_rng(5)
    xr = g0.integers(-128, 128, size=(3, 4, 61, 197), dtype=np.int8)
    tr = synth.head_params(4, 197, synth.BAND_STRICT, seed=9)
    shapes = [(1, 2, 70, 300, 64), (1, 1, 40, 2300, 64),      # two-pass and three-pass streaming forms
              (2, 3, 197, 197, 64)]                          # resident, partial last tiles
    att = []
    for Bt, H, Lq, Lk, d in shapes:
        q = g0.integers(-64, 64, size=(Bt, H, Lq, d), dtype=np.int8)
        k = g0.integers(-64, 64, size=(Bt, H, Lk, d), dtype=np.int8)
        v = g0.integers(-128, 128, size=(Bt, H, Lk, d), dtype=np.int8)
        att.append((q, k, v, synth.head_params(H, Lk, synth.BAND_U8, seed=Lk), synth.requant_params(H, seed=Lk)))
    x = torch.from_numpy(xr).cuda()
    dev = [tuple(torch.from_numpy(t).cuda() for t in a[:3]) for a in att]
    p_eager = binding.calibrated_softmax_i8(x, tr, synth.BAND_STRICT)
    o_eager = [binding.attention_i8(*dev[i], att[i][3], att[i][4], synth.BAND_U8) for i in range(len(att))]
    torch.cuda.synchronize()
    want, rc = oracle.softmax(xr, tr, synth.BAND_STRICT)
    assert rc == 0 and np.array_equal(p_eager.cpu().numpy(), want)
    for i, a in enumerate(att):
        want_o, rc = oracle.attention(a[0], a[1], a[2], a[3], a[4], synth.BAND_U8)
        assert rc == 0 and np.array_equal(o_eager[i].cpu().numpy(), want_o)

    p = torch.zeros_like(p_eager)
    o = [torch.zeros_like(t) for t in o_eager]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        binding.calibrated_softmax_i8(x, tr, synth.BAND_STRICT, out=p)
        for i in range(len(att)):
            binding.attention_i8(*dev[i], att[i][3], att[i][4], synth.BAND_U8, out=o[i])
    for rep in range(3):
        p.fill_(9)
        for t in o:
            t.fill_(9)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(p, p_eager), rep
        for i in range(len(att)):
            assert torch.equal(o[i], o_eager[i]), (rep, i)
