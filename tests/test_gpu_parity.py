"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element, bit-exact -- the method is a single-valued integer function."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_2604_02292_amd import binding, synth  # noqa: E402

THREADS = 16


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()   # raises if the library is not built: no fallback


def gpu_softmax(x, table, band, **kw):
    out = binding.calibrated_softmax_i8(torch.from_numpy(x).cuda(), table, band, **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check(x, table, band, oracle, label=""):
    print(f"case {label} shape={x.shape} band={band}", flush=True)
    want, rc = oracle.softmax(x, table, band, threads=THREADS)
    assert rc == 0
    got = gpu_softmax(x, table, band)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError(f"{label}: {bad.shape[0]} mismatches, first at {i}: got {got[i]} want {want[i]} "
                             f"row={x[i[:3]].tolist()[:32]} params={table[i[1]].tolist()}")


def mixed_logits(shape, seed):
    """Rows cycling through narrow, wide, saturating and constant distributions."""
    g = np.random.default_rng(seed)
    Bt, H, Lq, Lk = shape
    x = np.empty(shape, np.float64)
    sig = np.array([3.0, 24.0, 80.0, 0.0])[np.arange(Bt * H * Lq) % 4].reshape(Bt, H, Lq, 1)
    mu = g.uniform(-100, 100, size=(Bt, H, Lq, 1))
    x = mu + sig * g.standard_normal(shape)
    return np.clip(np.rint(x), -128, 127).astype(np.int8)


# every lane-group shape of the register kernel, full tiles and ragged tails
SHAPES = [
    ((1, 4, 64, 64), 1), ((3, 8, 37, 128), 1), ((2, 3, 50, 16), 1), ((2, 2, 33, 32), 1), ((2, 2, 20, 48), 1),
    ((1, 2, 21, 96), 1), ((1, 2, 19, 112), 1), ((1, 3, 9, 256), 1), ((1, 2, 7, 208), 1), ((2, 12, 40, 512), 1),
    ((1, 2, 130, 400), 1), ((1, 2, 5, 1024), 0), ((1, 2, 6, 880), 0), ((1, 2, 5, 2048), 0), ((1, 2, 9, 1536), 0),
    ((1, 2, 3, 4096), 0), ((1, 1, 5, 3216), 0), ((1, 1, 3, 8192), 0), ((1, 1, 2, 5008), 0), ((1, 1, 2, 16384), 0),
    ((1, 1, 2, 12304), 0), ((2, 1, 1, 64), 1), ((1, 1, 257, 64), 1), ((1, 1, 513, 128), 1),
    # lengths that are not multiples of 16, or beyond the register kernel
    ((1, 2, 5, 100), 1), ((1, 2, 3, 1), 1), ((1, 1, 4, 17), 1), ((1, 1, 3, 255), 0), ((1, 1, 2, 20000), 0),
    ((1, 1, 1, 65536), 0), ((1, 2, 2, 16400), 0),
    # one block per row: multiples of 16 beyond 16384
    ((1, 2, 3, 32768), 0), ((2, 1, 2, 40000), 0), ((1, 1, 5, 65520), 0),
    # either side of the lengths at which the row kernels change form
    ((1, 2, 5, 3952), 0), ((1, 2, 5, 3968), 0), ((1, 2, 3, 4112), 0), ((1, 1, 3, 8208), 0), ((1, 1, 2, 32784), 0),
]


@pytest.mark.parametrize("shape,band", SHAPES)
def test_softmax_u8_shapes(oracle, shape, band):
    H, n = shape[1], shape[3]
    table = synth.head_params(H, n, band, seed=n + 7 * H)
    check(mixed_logits(shape, seed=sum(shape)), table, band, oracle, "mixed")


@pytest.mark.parametrize("n,band", [(64, 1), (128, 1), (512, 1), (4096, 0), (100, 1), (197, 1), (300, 1), (1000, 0)])
def test_softmax_u8_degenerate_rows_and_params(oracle, n, band):
    shape = (1, 6, 16, n)   # 16 rows per head: lengths that are no multiple of 16 take the kernel that goes through LDS
    x = mixed_logits(shape, seed=n)
    x[0, :, 0] = -128
    x[0, :, 1] = 127
    x[0, :, 2] = -128
    x[0, :, 2, n // 2] = 127          # one-hot at full int8 range
    x[0, :, 3, ::2] = -128            # alternating extremes
    x[0, :, 3, 1::2] = 127
    x[0, :, 4] = np.arange(n) % 256 - 128
    bmax = 32767 // n if band == 1 else min(32767, (255 << 15) // n)
    f = -(-256 // n)
    table = np.array([[bmax, 0, 127], [bmax, (bmax - f) // 127, 127], [bmax, min(127, bmax - f), 1],
                      [f, 0, 0], [max(f, bmax // 2), 127 if bmax // 2 - f >= 127 else 0, 0],
                      [bmax, min(127, (bmax - f) // 64), 64]], np.int32)
    assert binding.validate_params(table, n, band) == (0, -1)
    check(x, table, band, oracle, "degenerate")


def test_softmax_in_place_and_unaligned(oracle):
    shape = (2, 4, 30, 128)
    x = mixed_logits(shape, 5)
    table = synth.head_params(4, 128, 1, seed=3)
    want, _ = oracle.softmax(x, table, 1)
    t = torch.from_numpy(x).cuda()
    out = binding.calibrated_softmax_i8(t, table, 1, out=t.view(torch.uint8))
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)
    # misaligned base pointers, input and output at different offsets inside a 16-byte line
    buf_in = torch.zeros(x.size + 16, dtype=torch.int8, device="cuda")
    buf_out = torch.zeros(x.size + 16, dtype=torch.uint8, device="cuda")
    buf_in[1:1 + x.size] = torch.from_numpy(x).cuda().view(-1)
    got = binding.calibrated_softmax_i8(buf_in[1:1 + x.size].view(shape), table, 1,
                                        out=buf_out[3:3 + x.size].view(shape))
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want)
    assert int(buf_out[:3].sum()) == 0 and int(buf_out[3 + x.size:].sum()) == 0


# ragged row lengths: every lane-group shape of the kernel, rows that start at every offset inside a
# 16-byte line, the longest register-resident length and the first one past it
RAGGED_SHAPES = [
    ((2, 3, 40, 1), 1), ((1, 2, 33, 7), 1), ((1, 2, 70, 33), 1), ((2, 2, 50, 49), 1), ((1, 3, 37, 50), 1),
    ((1, 2, 19, 100), 1), ((2, 2, 33, 113), 1), ((1, 2, 21, 127), 1), ((1, 2, 35, 129), 1), ((1, 2, 18, 225), 1),
    ((1, 2, 17, 241), 1), ((1, 1, 9, 500), 0), ((1, 2, 11, 1001), 0), ((1, 1, 7, 1009), 0), ((1, 2, 5, 2047), 0),
    ((1, 1, 5, 3000), 0), ((1, 1, 3, 4099), 0), ((1, 1, 3, 8100), 0), ((1, 1, 3, 16351), 0), ((1, 1, 2, 16353), 0),
    ((2, 3, 197, 197), 0), ((1, 5, 77, 77), 1), ((3, 2, 61, 250), 1), ((1, 2, 130, 999), 0), ((1, 64, 5, 21), 1),
    ((1, 2, 40, 500), 0), ((1, 2, 9, 1000), 0), ((1, 3, 33, 104), 1), ((1, 2, 21, 2040), 0), ((1, 2, 19, 252), 1),
    # rows through LDS (every lane layout): a head change inside every wave, every block, or rarely; one row in
    # the last block; the shortest and the longest length of each layout; lengths just outside
    ((2, 5, 16, 100), 1), ((3, 7, 17, 241), 1), ((1, 4, 23, 65), 1), ((5, 3, 65, 113), 1), ((1, 1, 129, 129), 1),
    ((1, 2, 64, 199), 1), ((4, 64, 16, 145), 1), ((2, 5, 16, 37), 1), ((1, 1, 129, 63), 1), ((2, 3, 15, 150), 1),
    ((2, 3, 33, 257), 1), ((1, 2, 50, 300), 1), ((3, 2, 16, 497), 1), ((1, 2, 21, 498), 1), ((2, 2, 19, 769), 0),
    ((1, 3, 35, 800), 0), ((2, 2, 16, 1009), 0), ((1, 2, 17, 1010), 0), ((1, 2, 40, 114), 1), ((1, 2, 40, 242), 1),
    # slabs shorter than a vector (the guard on the tensor's last vectors spans several rows and slabs)
    ((7, 3, 1, 5), 1), ((2, 2, 2, 3), 1), ((1, 1, 1, 1), 1), ((1, 1, 1, 15), 1), ((3, 1, 1, 17), 1), ((9, 1, 1, 2), 1),
    # ragged lengths beyond a wave's registers: one block per row
    ((1, 2, 2, 16401), 0), ((1, 1, 3, 40001), 0), ((1, 1, 2, 65535), 0), ((2, 1, 1, 32777), 0),
]


@pytest.mark.parametrize("shape,band", RAGGED_SHAPES)
def test_softmax_u8_ragged_lengths(oracle, shape, band):
    """The output tensor sits inside a larger buffer filled with a canary value: bytes before
    and after it stay untouched, also when the tensor's last byte is not at the end of a 16-byte line."""
    H, n = shape[1], shape[3]
    table = synth.head_params(H, n, band, seed=n + 7 * H)
    x = mixed_logits(shape, seed=sum(shape))
    print(f"case ragged shape={shape} band={band}", flush=True)
    want, rc = oracle.softmax(x, table, band, threads=THREADS)
    assert rc == 0
    buf = torch.full((x.size + 96,), 0xA5, dtype=torch.uint8, device="cuda")
    out = buf[32:32 + x.size].view(shape)
    binding.calibrated_softmax_i8(torch.from_numpy(x).cuda(), table, band, out=out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError(f"{bad.shape[0]} mismatches, first at {i}: got {got[i]} want {want[i]}")
    assert bool((buf[:32] == 0xA5).all()) and bool((buf[32 + x.size:] == 0xA5).all())
    # in place, and with the leading-bit reciprocal
    t = torch.from_numpy(x).cuda()
    binding.calibrated_softmax_i8(t, table, band, out=t.view(torch.uint8))
    torch.cuda.synchronize()
    assert np.array_equal(t.view(torch.uint8).cpu().numpy(), want)
    want_clb, _ = oracle.softmax(x, table, band, mode=2, threads=THREADS)
    got_clb = binding.calibrated_softmax_i8_ex(torch.from_numpy(x).cuda(), table, band, reciprocal=1)
    torch.cuda.synchronize()
    assert np.array_equal(got_clb.cpu().numpy(), want_clb)


@pytest.mark.parametrize("shape,off", [((2, 4, 30, 128), 5), ((1, 3, 33, 100), 9), ((2, 2, 17, 1000), 15),
                                       ((1, 2, 40, 64), 8), ((1, 2, 9, 4099), 3), ((3, 2, 50, 7), 1)])
def test_softmax_tensors_that_begin_inside_a_vector(oracle, shape, off):
    """Input and output begin the same number of elements behind a 16-byte boundary (a slice of
    a larger tensor): vectors are read and written where they lie; canaries around the output."""
    H, n = shape[1], shape[3]
    band = 1 if n * 8 <= 32767 else 0
    table = synth.head_params(H, n, band, seed=n + H)
    x = mixed_logits(shape, seed=sum(shape) + off)
    want, rc = oracle.softmax(x, table, band, threads=THREADS)
    assert rc == 0
    print(f"case offset shape={shape} off={off}", flush=True)
    buf_in = torch.zeros(x.size + 64, dtype=torch.int8, device="cuda")
    buf_in[off:off + x.size] = torch.from_numpy(x).cuda().view(-1)
    buf_out = torch.full((x.size + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    binding.calibrated_softmax_i8(buf_in[off:off + x.size].view(shape), table, band,
                                  out=buf_out[16 + off:16 + off + x.size].view(shape))
    torch.cuda.synchronize()
    assert np.array_equal(buf_out[16 + off:16 + off + x.size].view(shape).cpu().numpy(), want)
    assert bool((buf_out[:16 + off] == 0xA5).all()) and bool((buf_out[16 + off + x.size:] == 0xA5).all())
    if band == 1:   # 16-bit output: element offsets match when the output is `off` elements behind a boundary
        want16, _ = oracle.softmax(x, table, band, mode=1, threads=THREADS)
        buf16 = torch.full((x.size + 64,), 0x5A5A, dtype=torch.int16, device="cuda")
        o8 = off % 8
        b_in = torch.zeros(x.size + 64, dtype=torch.int8, device="cuda")
        b_in[o8:o8 + x.size] = torch.from_numpy(x).cuda().view(-1)
        binding.calibrated_softmax_i8_ex(b_in[o8:o8 + x.size].view(shape), table, band, out_scale_T=32767,
                                         out=buf16[8 + o8:8 + o8 + x.size].view(shape))
        torch.cuda.synchronize()
        got16 = buf16[8 + o8:8 + o8 + x.size].view(shape).cpu().numpy().view(np.uint16)
        assert np.array_equal(got16, want16)
        assert bool((buf16[:8 + o8] == 0x5A5A).all()) and bool((buf16[8 + o8 + x.size:] == 0x5A5A).all())


@pytest.mark.parametrize("shape,off_in,off_out", [((2, 4, 30, 128), 3, 11), ((1, 3, 33, 100), 7, 0),
                                                  ((1, 2, 9, 4099), 1, 14), ((1, 1, 2, 20001), 5, 9),
                                                  ((2, 2, 40, 64), 0, 13), ((1, 2, 3, 16384), 2, 2)])
def test_softmax_tensors_at_unrelated_offsets(oracle, shape, off_in, off_out):
    """Input and output begin at unrelated offsets inside a 16-byte line, in the 8-bit and (2-byte
    aligned) 16-bit output modes; canaries around the outputs."""
    H, n = shape[1], shape[3]
    band = 1 if n * 8 <= 32767 else 0
    table = synth.head_params(H, n, band, seed=n + H)
    x = mixed_logits(shape, seed=sum(shape) + off_in)
    print(f"case offsets shape={shape} in={off_in} out={off_out}", flush=True)
    buf_in = torch.zeros(x.size + 64, dtype=torch.int8, device="cuda")
    buf_in[off_in:off_in + x.size] = torch.from_numpy(x).cuda().view(-1)
    t_in = buf_in[off_in:off_in + x.size].view(shape)
    for mode, T, recip in ((0, 255, 0), (2, 255, 1)) + (((1, 32767, 0), (3, 32767, 1)) if band == 1 else ()):
        want, rc = oracle.softmax(x, table, band, mode=mode, threads=THREADS)
        assert rc == 0
        canary = 0x5A if T == 255 else 0x5A5A
        buf = torch.full((x.size + 64,), canary, dtype=torch.uint8 if T == 255 else torch.int16, device="cuda")
        t_out = buf[off_out:off_out + x.size].view(shape)
        binding.calibrated_softmax_i8_ex(t_in, table, band, out_scale_T=T, reciprocal=recip, out=t_out)
        torch.cuda.synchronize()
        got = t_out.cpu().numpy()
        got = got.view(np.uint16) if T == 32767 else got
        assert np.array_equal(got, want), f"mode {mode}"
        assert bool((buf[:off_out] == canary).all()) and bool((buf[off_out + x.size:] == canary).all())


def test_empty_tensors_and_size_limits(oracle):
    """Zero-sized tensors are a no-op; the largest head table (64) and a batch extent beyond 65535
    (no grid dimension is tied to it) go through."""
    for shape in [(0, 4, 8, 64), (3, 4, 0, 64)]:
        x = torch.empty(shape, dtype=torch.int8, device="cuda")
        out = binding.calibrated_softmax_i8(x, synth.head_params(4, 64, 1, seed=1), 1)
        torch.cuda.synchronize()
        assert out.shape == x.shape
    table = synth.head_params(64, 32, 1, seed=64)
    check(mixed_logits((2, 64, 3, 32), 64), table, 1, oracle, "64 heads")
    table = synth.head_params(1, 16, 1, seed=2)
    check(mixed_logits((70001, 1, 1, 16), 65535), table, 1, oracle, "70001 batches")
    table = synth.head_params(2, 100, 1, seed=3)
    check(mixed_logits((66000, 2, 1, 100), 66000), table, 1, oracle, "66000 batches, ragged rows")
    q, k, v = rect_qkv(66000, 33000, 2, 2, 16, 64)       # 66000 (batch, head) items through the streaming kernel
    check_attention(q, k, v, synth.head_params(2, 16, 1, seed=5), synth.requant_params(2, seed=5), 1, oracle,
                    "66000 items")
    q = torch.empty((0, 2, 64, 64), dtype=torch.int8, device="cuda")
    o = binding.attention_i8(q, q, q, synth.head_params(2, 64, 1, seed=1), synth.requant_params(2, seed=1), 1)
    torch.cuda.synchronize()
    assert o.shape == q.shape


def test_rejected_call_leaves_output_untouched():
    x = torch.zeros((1, 1, 4, 64), dtype=torch.int8, device="cuda")
    out = torch.full((1, 1, 4, 64), 77, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.HccsError) as e:
        binding.calibrated_softmax_i8(x, [[512, 0, 1]], 1, out=out)
    assert e.value.status == -7
    torch.cuda.synchronize()
    assert bool((out == 77).all())


def test_reciprocal_exhaustive(oracle):
    """Every row sum the 8-bit band admits goes through the kernels' reciprocal routine."""
    N = 255 << 15
    z = np.arange(256, N + 1, dtype=np.int64)
    want, rc = oracle.reciprocal_u8(z)
    assert rc == 0
    got = binding.reciprocal_u8(torch.from_numpy(z.astype(np.int32)).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().astype(np.int64), want)


def test_normalise_stage_sweep(oracle):
    """The exact-float normalise stage against integers, over constants and row sums that random rows
    rarely produce: Z = B (one element carries everything), Z at the ends of its range, reciprocals
    next to powers of two, and 300k random admissible combinations."""
    N = 255 << 15
    g = np.random.default_rng(42)
    count = 300_000
    B = g.integers(1, 32768, count)
    D = g.integers(0, 128, count)
    S = np.minimum(g.integers(0, 128, count), B // np.maximum(D, 1))
    Z = (np.maximum(B, 256) + (g.random(count) ** 3 * (N - np.maximum(B, 256)))).astype(np.int64)
    edge = []
    for b in (1, 2, 255, 256, 257, 4095, 16383, 32767):
        for s_, d_ in ((0, 0), (1, min(b, 127)), (min(127, b // 127), 127), (min(b, 127), 1)):
            for z in {max(b, 256), max(b, 256) + 1, 32767, 32768, 65535, 65536, N - 1, N, 8355, 261120, 522241}:
                if z >= max(b, 256) and s_ * d_ <= b:
                    edge.append((b, s_, d_, z))
    edge = np.array(edge, np.int64)
    B, S, D, Z = (np.concatenate([a, edge[:, i]]) for i, a in enumerate((B, S, D, Z)))
    assert np.all(S * D <= B) and np.all(B <= Z) and np.all(Z >= 256) and np.all(Z <= N)
    rho, rc = oracle.reciprocal_u8(Z)
    assert rc == 0
    delta = np.arange(256, dtype=np.int64)[None, :]
    want = ((B[:, None] - S[:, None] * np.minimum(delta, D[:, None])) * rho[:, None]) >> 15
    assert want.min() >= 0 and want.max() <= 255
    bsdz = torch.from_numpy(np.stack([B, S, D, Z], 1).astype(np.int32)).cuda()
    got = binding.normalise_table_u8(bsdz)
    torch.cuda.synchronize()
    got = got.cpu().numpy().astype(np.int64)
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"{bad.shape[0]} mismatches, first (B,S,D,Z)={B[bad[0,0]],S[bad[0,0]],D[bad[0,0]],Z[bad[0,0]]} delta={bad[0,1]}"


def test_other_stream(oracle):
    shape = (2, 8, 64, 128)
    x = mixed_logits(shape, 9)
    table = synth.head_params(8, 128, 1, seed=9)
    want, _ = oracle.softmax(x, table, 1)
    s = torch.cuda.Stream()
    t = torch.from_numpy(x).cuda()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        out = binding.calibrated_softmax_i8(t, table, 1)
    s.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)


# ---------------------------------------------------------------- 16-bit output and leading-bit reciprocal
MODES = {"i16": (32767, 0, 1), "clb_u8": (255, 1, 2), "clb_i16": (32767, 1, 3)}   # name -> (T, reciprocal, oracle mode)
MODE_SHAPES = [
    ((1, 4, 64, 64), 1), ((3, 8, 37, 128), 1), ((2, 3, 50, 16), 1), ((2, 2, 20, 48), 1), ((1, 3, 9, 256), 1),
    ((2, 12, 40, 512), 1), ((1, 2, 3, 4096), 1), ((1, 1, 2, 16384), 1), ((1, 2, 7, 208), 1), ((1, 2, 6, 880), 1),
    ((1, 2, 5, 100), 1), ((1, 1, 4, 17), 1), ((1, 2, 3, 1), 1), ((1, 1, 2, 20000), 1),
    ((1, 2, 5, 1024), 0), ((1, 2, 3, 4096), 0), ((1, 1, 3, 255), 0),
    ((1, 2, 2, 32752), 1), ((1, 1, 3, 16400), 1), ((1, 1, 2, 40000), 0),
    # ragged lengths in every mode (8-byte input vectors in the 16-bit modes)
    ((2, 3, 197, 197), 1), ((1, 2, 40, 500), 1), ((1, 2, 33, 24), 1), ((1, 2, 9, 1000), 1), ((1, 2, 7, 8200), 1),
    ((1, 3, 70, 7), 1), ((1, 2, 21, 127), 1), ((1, 2, 50, 9), 1), ((1, 1, 3, 16351), 1), ((1, 2, 5, 2047), 1),
    ((1, 2, 130, 129), 0), ((1, 2, 19, 72), 1), ((1, 1, 5, 16376), 1),
]


@pytest.mark.parametrize("mode", sorted(MODES))
@pytest.mark.parametrize("shape,band", MODE_SHAPES)
def test_softmax_other_modes(oracle, mode, shape, band):
    T, recip, omode = MODES[mode]
    if T == 32767 and band != 1:
        pytest.skip("the 16-bit path exists under the strict band only")
    H, n = shape[1], shape[3]
    table = synth.head_params(H, n, band, seed=n + 7 * H)
    x = mixed_logits(shape, seed=sum(shape) + omode)
    print(f"case mode={mode} shape={shape} band={band}", flush=True)
    want, rc = oracle.softmax(x, table, band, mode=omode, threads=THREADS)
    assert rc == 0
    got = binding.calibrated_softmax_i8_ex(torch.from_numpy(x).cuda(), table, band, out_scale_T=T, reciprocal=recip)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    if T == 32767:
        got = got.view(np.uint16)
    assert got.dtype == want.dtype
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError(f"{mode}: {bad.shape[0]} mismatches, first at {i}: got {got[i]} want {want[i]} "
                             f"params={table[i[1]].tolist()}")


@pytest.mark.parametrize("mode", sorted(MODES))
def test_other_modes_degenerate_and_saturating(oracle, mode):
    """Rows that make the leading-bit reciprocal overshoot (one dominant element, Z just below a
    power of two) and the extremes of the int8 range."""
    T, recip, omode = MODES[mode]
    n = 64
    shape = (1, 4, 16, n)
    x = mixed_logits(shape, seed=77)
    x[0, :, 0] = -128
    x[0, :, 0, 5] = 127
    x[0, :, 1] = 127
    x[0, :, 2, ::2] = -128
    table = np.array([[511, 3, 127], [500, 3, 127], [511, 0, 1], [260, 2, 127]], np.int32)
    assert binding.validate_params(table, n, 1) == (0, -1)
    want, rc = oracle.softmax(x, table, 1, mode=omode)
    assert rc == 0
    got = binding.calibrated_softmax_i8_ex(torch.from_numpy(x).cuda(), table, 1, out_scale_T=T, reciprocal=recip)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    got = got.view(np.uint16) if T == 32767 else got
    assert np.array_equal(got, want)
    # n = 16, one dominant element: s = [1100, 20, ...], Z = 1400, k = 10 -> 1100*rho overshoots T
    x16 = np.full((1, 1, 8, 16), -128, np.int8)
    x16[0, 0, :, 3] = 100
    x16[0, 0, 4:, 7] = 99
    t16 = np.array([[1100, 12, 90]], np.int32)
    assert binding.validate_params(t16, 16, 1) == (0, -1)
    want, rc = oracle.softmax(x16, t16, 1, mode=omode)
    assert rc == 0
    got = binding.calibrated_softmax_i8_ex(torch.from_numpy(x16).cuda(), t16, 1, out_scale_T=T, reciprocal=recip)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    got = got.view(np.uint16) if T == 32767 else got
    assert np.array_equal(got, want)
    if recip == 1:
        assert (want == T).any(), "the case was meant to reach saturation"


def test_edge_encoder_full_size_i16(oracle):
    w = synth.make_workload("edge_encoder", threads=THREADS)
    want, rc = oracle.softmax(w["logits"], w["table"], 1, mode=1, threads=THREADS)
    assert rc == 0
    got = binding.calibrated_softmax_i8_ex(torch.from_numpy(w["logits"]).cuda(), w["table"], 1, out_scale_T=32767)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint16), want)


# ---------------------------------------------------------------- grid-search calibration
def candidate_grid(n, count, seed):
    """Mostly admissible triples for row length n, plus a few that are not."""
    g = np.random.default_rng(seed)
    bmax = 32767 // n
    f = -(-256 // n)
    out = []
    while len(out) < count:
        D = int(g.integers(0, 128))
        B = int(g.integers(f, bmax + 1))
        S = int(g.integers(0, min(127, (B - f) // max(D, 1)) + 1))
        out.append((B, S, D))
    out[3] = (bmax + 1, 0, 1)          # ceiling violated
    out[7] = (f, 1, 127)               # negative floor
    out[11] = (bmax, 0, 128)           # Dmax out of range
    return np.array(out, np.int32)


@pytest.mark.parametrize("shape", [(6, 4, 24, 128), (3, 2, 5, 100), (2, 3, 9, 64), (1, 2, 7, 4096), (2, 1, 33, 16)])
def test_calibration_grid_search(oracle, shape):
    """Objective in double precision on both sides; sums are ordered differently, so values are
    compared to 1e-9 relative, and the arg-min is checked for validity against the oracle's table."""
    H, n = shape[1], shape[3]
    x = synth.make_workload("edge_encoder", shape=shape)["logits"] if n != 4096 else mixed_logits(shape, 4)
    alpha = np.linspace(0.04, 0.2, H)
    cand = candidate_grid(n, 150, seed=n)
    print(f"calibration case shape={shape}", flush=True)
    want, want_best, rc = oracle.calibrate(x, alpha, cand, threads=THREADS)
    assert rc == 0
    obj, best = binding.calibrate_grid(torch.from_numpy(x).cuda(), alpha, cand)
    torch.cuda.synchronize()
    obj, best = obj.cpu().numpy(), best.cpu().numpy()
    assert np.array_equal(np.isinf(obj), np.isinf(want))
    fin = np.isfinite(want)
    assert fin.any()
    assert np.allclose(obj[fin], want[fin], rtol=1e-9, atol=1e-12)
    for h in range(H):
        assert 0 <= best[h] < len(cand) and np.isfinite(want[h, best[h]])
        assert want[h, best[h]] <= want[h][fin[h]].min() * (1 + 1e-9) + 1e-12
    # reproducible to the bit
    obj2, best2 = binding.calibrate_grid(torch.from_numpy(x).cuda(), alpha, cand)
    torch.cuda.synchronize()
    assert np.array_equal(obj2.cpu().numpy(), obj) and np.array_equal(best2.cpu().numpy(), best)


def test_calibration_finds_the_exact_reproduction():
    import math
    x = np.tile(np.array([0, -1, 0, -1], np.int8), (2, 1, 3, 1))
    cand = [[200, 10, 12], [254, 100, 1], [254, 127, 1], [8192, 0, 0]]
    obj, best = binding.calibrate_grid(torch.from_numpy(x).cuda(), [math.log(2.0)], cand)
    torch.cuda.synchronize()
    assert best.cpu().tolist() == [2]
    assert abs(float(obj[0, 2])) < 1e-14 and float(obj[0, 0]) > 1e-4 and math.isinf(float(obj[0, 3]))


# ---------------------------------------------------------------- the named workloads
@pytest.mark.parametrize("name,shape", [
    ("pr1_ref", None), ("edge_encoder", (4, 8, 128, 128)), ("stress_rows", (2, 12, 512, 512)),
    ("long_row", (1, 16, 64, 4096)),
])
def test_workload_recipes_reduced(oracle, name, shape):
    w = synth.make_workload(name, shape=shape)
    check(w["logits"], w["table"], w["band"], oracle, name)


@pytest.mark.parametrize("name", ["edge_encoder", "stress_rows", "long_row"])
def test_workloads_full_size(oracle, name):
    """Full-size tensors, same launch configuration as the benchmark; the oracle runs
    over every element (OpenMP over rows)."""
    w = synth.make_workload(name, threads=THREADS)
    print(f"generated {name} {w['logits'].shape}", flush=True)
    x, table, band = w["logits"], w["table"], w["band"]
    got = gpu_softmax(x, table, band)
    print("gpu done", flush=True)
    want, rc = oracle.softmax(x, table, band, threads=THREADS)
    assert rc == 0
    assert np.array_equal(got, want)
    if name == "long_row":
        # the band of Eq. (11) at n = 4096 caps B at 7: the output is provably all zero
        strict = synth.head_params(x.shape[1], 4096, 1, seed=3)
        sub = np.ascontiguousarray(x[:1, :, :256])
        got0 = gpu_softmax(sub, strict, 1)
        want0, _ = oracle.softmax(sub, strict, 1, threads=THREADS)
        assert np.array_equal(got0, want0) and not got0.any()


# ---------------------------------------------------------------- fused block
def check_attention(q, k, v, table, rq, band, oracle, label=""):
    print(f"attention case {label} shape={q.shape}", flush=True)
    want, rc = oracle.attention(q, k, v, table, rq, band, threads=THREADS)
    assert rc == 0
    got = binding.attention_i8(torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(),
                               torch.from_numpy(v).cuda(), table, rq, band)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError(f"{label}: {bad.shape[0]} mismatches of {got.size}, first at {i}: "
                             f"got {got[i]} want {want[i]}")


@pytest.mark.parametrize("shape", [(1, 2, 64, 64), (2, 3, 128, 64), (1, 2, 256, 64), (1, 1, 192, 64),
                                   (1, 2, 320, 64), (1, 1, 384, 64), (1, 1, 448, 64), (1, 1, 512, 64),
                                   (5, 7, 64, 64)])
def test_attention_shapes(oracle, shape):
    w = synth.make_workload("fused_attention", shape=shape)
    check_attention(w["q"], w["k"], w["v"], w["table"], w["requant"], w["band"], oracle, "uniform")


def test_attention_full_range_inputs_and_large_multiplier(oracle):
    """int8 extremes in Q, K, V; multipliers that would leave 32 bits without the
    accumulator saturation; probabilities above 127 (8-bit band)."""
    g = np.random.default_rng(2)
    shape = (2, 4, 128, 64)
    q, k, v = (g.integers(-128, 128, size=shape, dtype=np.int8) for _ in range(3))
    q[0, 0, :4] = 127
    k[0, 0, :4] = 127
    q[0, 1, :4] = -128
    k[0, 1, :4] = -128
    v[0, :, :8] = -128
    table = np.array([[30000, 127, 127], [65280, 0, 0], [20000, 100, 127], [255, 1, 127]], np.int32)
    table[1] = [32767, 127, 100]
    assert binding.validate_params(table, 128, 0) == (0, -1)
    for rq in ([[4096, 23], [4096, 12], [1, 1], [2047, 16]],
               [[4096, 24], [1, 24], [4095, 24], [3000, 22]]):   # the top of the shift range
        check_attention(q, k, v, table, np.array(rq, np.int32), 0, oracle, f"extremes {rq}")


def rect_qkv(seed, Bt, H, Lq, Lk, d, lo=-64, hi=63):
    g = np.random.default_rng(seed)
    return (g.integers(lo, hi + 1, size=(Bt, H, Lq, d), dtype=np.int8),
            g.integers(lo, hi + 1, size=(Bt, H, Lk, d), dtype=np.int8),
            g.integers(lo, hi + 1, size=(Bt, H, Lk, d), dtype=np.int8))


# streaming kernel: rectangular blocks, key lengths beyond the resident kernel, ragged tails, d = 128
STREAM_SHAPES = [  # (Bt, H, Lq, Lk, d, band)
    (1, 2, 64, 128, 64, 1), (2, 3, 40, 256, 64, 1), (1, 2, 7, 48, 64, 1), (1, 1, 130, 80, 64, 1),
    (1, 2, 33, 1024, 64, 1), (1, 1, 20, 2064, 64, 0), (1, 2, 64, 64, 128, 1), (2, 2, 50, 272, 128, 1),
    (1, 1, 16, 4096, 128, 0), (1, 2, 100, 576, 64, 0), (3, 1, 1, 16, 64, 1), (1, 1, 70, 1040, 128, 0),
    # key lengths that are not a multiple of 16 (masked tail tile)
    (1, 2, 19, 100, 64, 1), (2, 1, 33, 1, 64, 1), (1, 2, 5, 17, 128, 1), (1, 1, 40, 255, 64, 1),
    (1, 2, 16, 1031, 64, 0), (1, 1, 9, 63, 128, 1), (1, 1, 3, 65, 64, 1), (1, 1, 5, 2049, 64, 0),
    (1, 1, 18, 2111, 128, 0), (1, 2, 17, 1999, 64, 0), (1, 1, 70, 2047, 128, 0),
    # block counts that are no multiple of the number of dies (block renumbering), whole and partial 128-key chunks
    (3, 3, 200, 96, 64, 1), (1, 5, 150, 130, 64, 1), (1, 11, 65, 128, 64, 1), (1, 3, 129, 384, 128, 1),
    (1, 1, 300, 2200, 64, 0),
    # 1024 < Lk <= 2048 in whole pairs of chunks: the keys of a row split over two waves
    (1, 2, 70, 1280, 64, 0), (1, 1, 40, 1536, 128, 0), (2, 1, 130, 1792, 64, 0), (1, 1, 17, 2048, 128, 0),
    # 2048 < Lk <= 4096 in whole sets of four chunks: four waves per row, two passes
    (1, 2, 70, 2560, 64, 0), (1, 1, 130, 3072, 64, 0), (2, 1, 33, 3584, 64, 0), (1, 1, 64, 4096, 64, 0),    # shares that end in a partial chunk: the largest rests that still split (254 and 508 keys beyond whole
    # chunk sets), a rest of one key (three of four shares get an empty partial chunk), and the lengths
    # just beyond, which fall back to one wave per row (1279) and to three passes (4095)
    (1, 1, 20, 2046, 64, 0), (1, 2, 18, 1279, 64, 0), (1, 1, 24, 4092, 64, 0), (1, 1, 17, 4095, 64, 0),
    (2, 1, 40, 3001, 64, 0), (1, 1, 33, 2561, 64, 0), (1, 2, 21, 1025, 64, 1),
]


@pytest.mark.parametrize("Bt,H,Lq,Lk,d,band", STREAM_SHAPES)
def test_attention_streaming_shapes(oracle, Bt, H, Lq, Lk, d, band):
    q, k, v = rect_qkv(Lq + Lk + d, Bt, H, Lq, Lk, d)
    table = synth.head_params(H, Lk, band, seed=Lk + d)
    rq = synth.requant_params(H, seed=Lk, shift=16, mult_lo=60, mult_hi=200)
    check_attention(q, k, v, table, rq, band, oracle, "streaming")


def test_attention_streaming_benchmark_shape_and_long_three_pass(oracle):
    """The streaming shape the benchmark times, [4,12,2048,2048,64] (two-pass kernel), at full size
    with the benchmark's own inputs, and three-pass cases beyond 4096 keys with several query tiles."""
    g = np.random.default_rng(7)
    Bs, Hs, Ls, ds = 4, 12, 2048, 64
    q, k, v = (g.integers(-64, 64, size=(Bs, Hs, Ls, ds), dtype=np.int8) for _ in range(3))
    check_attention(q, k, v, synth.head_params(Hs, Ls, synth.BAND_U8, seed=11), synth.requant_params(Hs, seed=11),
                    synth.BAND_U8, oracle, "benchmark streaming shape")
    for Bt, H, Lq, Lk, d in ((1, 2, 256, 4096, 64), (1, 2, 320, 4160, 128), (1, 1, 257, 5000, 64)):
        q, k, v = rect_qkv(Lq + Lk, Bt, H, Lq, Lk, d)
        check_attention(q, k, v, synth.head_params(H, Lk, 0, seed=Lk), synth.requant_params(H, seed=Lk), 0, oracle,
                        "three-pass")


def test_attention_streaming_rescale_kinds_and_extremes(oracle):
    """Every rescale form of the streaming kernel, full-range inputs, d = 128 (|acc| up to 2^21)."""
    g = np.random.default_rng(12)
    Bt, H, Lq, Lk, d = 1, 3, 24, 144, 128
    q = g.integers(-128, 128, size=(Bt, H, Lq, d), dtype=np.int8)
    k = g.integers(-128, 128, size=(Bt, H, Lk, d), dtype=np.int8)
    v = g.integers(-128, 128, size=(Bt, H, Lk, d), dtype=np.int8)
    q[0, 0, :3] = -128
    k[0, 0, :3] = -128
    table = np.array([[30000, 127, 127], [32767, 127, 100], [227, 1, 127]], np.int32)
    assert binding.validate_params(table, Lk, 0) == (0, -1)
    for rq in ([[100, 16], [7, 12], [255, 16]],          # high-half form
               [[100, 17], [900, 20], [3, 2]],           # shift form
               [[4096, 23], [4096, 12], [2047, 16]],     # accumulator saturation needed
               [[4096, 24], [1, 24], [2049, 24]]):       # the top of the shift range
        check_attention(q, k, v, table, np.array(rq, np.int32), 0, oracle, f"rescale {rq}")


@pytest.mark.parametrize("Lq,Lk,d", [(40, 2048, 64), (24, 1000, 128), (33, 2500, 64), (20, 2300, 128), (17, 300, 64)])
def test_attention_streaming_probabilities_above_127(oracle, Lq, Lk, d):
    """Tables that allow P > 127 (the kernels then feed P - 128 and add the offset back), with rows
    that reach it: one key far above all others, which sit at the window's edge."""
    g = np.random.default_rng(Lk + d)
    H = 2
    q = g.integers(40, 100, size=(1, H, Lq, d), dtype=np.int8)
    k = g.integers(-1, 2, size=(1, H, Lk, d), dtype=np.int8)
    v = g.integers(-128, 128, size=(1, H, Lk, d), dtype=np.int8)
    k[0, :, Lk // 3] = 127                                # the dominant key
    k[0, 1, Lk - 1] = 127                                 # a second one for head 1
    cap = (255 << 15) // Lk
    S, D = 32, 100
    table = np.array([[S * D + 1, S, D], [min(cap, 32767), S, D]], np.int32)   # floor 1, and the band's largest base
    assert binding.validate_params(table, Lk, 0) == (0, -1)
    rq = np.array([[40, 16], [3, 12]], np.int32)
    x, rc = oracle.requant_logits(q, k, rq)
    assert rc == 0
    p, rc = oracle.softmax(x, table, 0, threads=THREADS)
    assert rc == 0 and p[0, 0].max() > 127                # the case does reach beyond the signed range
    check_attention(q, k, v, table, rq, 0, oracle, f"P above 127, Lk={Lk} d={d}")


def test_attention_streaming_equals_resident_definition(oracle):
    """A square shape that the resident kernel takes, and its first 64 queries alone, which the streaming kernel
    takes (more than 448 keys, at most 64 queries): the same rows must come out."""
    w = synth.make_workload("fused_attention", shape=(1, 2, 512, 64))
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    o_res = binding.attention_i8(dev(w["q"]), dev(w["k"]), dev(w["v"]), w["table"], w["requant"], w["band"])
    o_str = binding.attention_i8(dev(w["q"][:, :, :64]), dev(w["k"]), dev(w["v"]), w["table"], w["requant"], w["band"])
    torch.cuda.synchronize()
    assert torch.equal(o_str, o_res[:, :, :64])


@pytest.mark.parametrize("Bt,H", [(257, 2), (65, 8)])
def test_attention_many_items_every_rescale_form(oracle, Bt, H):
    """Square blocks of 256 keys, more (batch, head) items than two per compute unit: probabilities
    below and above 127 and every rescale form, full-range inputs."""
    g = np.random.default_rng(Bt)
    shape = (Bt, H, 256, 64)
    q, k, v = (g.integers(-128, 128, size=shape, dtype=np.int8) for _ in range(3))
    strict = synth.head_params(H, 256, 1, seed=Bt)                       # B <= 127: P <= 127 for every row
    wide = synth.head_params(H, 256, 0, seed=Bt)
    wide[0] = (32640, 127, 127)                                          # one dominant key takes P to 255
    assert binding.validate_params(wide, 256, 0) == (0, -1)
    for table, band in ((strict, 1), (wide, 0)):
        for rq in ([[100 + h, 16] for h in range(H)], [[900 + h, 20] for h in range(H)],
                   [[4096 - h, 24 - (h % 3)] for h in range(H)]):
            check_attention(q, k, v, table, np.array(rq, np.int32), band, oracle,
                            f"items={Bt * H} band={band} rq={rq[0]}")


@pytest.mark.parametrize("L,params,p_top", [(256, (763, 38, 20), 127), (256, (261, 13, 20), 128), (256, (502, 25, 20), 126),
                                            (1280, (1281, 64, 20), 127), (1280, (1301, 65, 20), 128),
                                            (2304, (2301, 115, 20), 127), (2304, (2341, 117, 20), 128),
                                            (2560, (2551, 85, 30), 127), (2560, (2611, 87, 30), 128)])
def test_attention_largest_probability_at_the_signed_limit(oracle, L, params, p_top):
    """Tables whose largest possible probability is just below, at and just above 127 (the fused
    kernels feed P to the signed matrix unit as it is only when the table proves P <= 127), with
    rows that attain it: one key at the maximum, every other key beyond the window.  256 keys take
    the resident kernels, 1280 and 2560 the two-pass streaming kernel with the keys in two and four
    shares, 2304 the three-pass one."""
    g = np.random.default_rng(p_top + L)
    H, d = 2, 64
    Bt, Lq = (3, L) if L == 256 else (1, 48)
    q = g.integers(40, 100, size=(Bt, H, Lq, d), dtype=np.int8)
    k = g.integers(-1, 2, size=(Bt, H, L, d), dtype=np.int8)
    v = g.integers(-128, 128, size=(Bt, H, L, d), dtype=np.int8)
    k[:, :, 77] = 127                                     # the dominant key
    table = np.array([params, params], np.int32)
    assert binding.validate_params(table, L, 0) == (0, -1)
    rq = np.array([[40, 16], [40, 16]], np.int32)
    x, rc = oracle.requant_logits(q, k, rq)
    assert rc == 0
    p, rc = oracle.softmax(x, table, 0, threads=THREADS)
    assert rc == 0 and int(p.max()) == p_top              # the bound is attained
    check_attention(q, k, v, table, rq, 0, oracle, f"largest P = {p_top}, {L} keys")


SQUARE_LENGTHS = [1, 2, 15, 16, 17, 48, 63, 65, 100, 127, 129, 130, 191, 193, 197, 200, 208, 255, 257, 300, 319, 321,
                  383, 385, 400, 447, 449, 500, 511]


@pytest.mark.parametrize("L", SQUARE_LENGTHS)
def test_attention_square_blocks_of_any_length(oracle, L):
    """Square blocks whose length is no multiple of 64 (a vision encoder's 197 tokens among them): under the strict
    band (P <= 127 proven) the resident kernel takes them with its last key tiles partly or wholly absent, under
    a table that allows P > 127 the streaming kernel does.  Full-range inputs, every rescale form, and an output
    buffer with guard values before and behind it."""
    g = np.random.default_rng(1000 + L)
    Bt, H, d = 3, 3, 64
    q, k, v = (g.integers(-128, 128, size=(Bt, H, L, d), dtype=np.int8) for _ in range(3))
    k[0, 0, L - 1] = 127                                  # the last key matters: large logits on it
    q[0, 0, : min(L, 4)] = 127
    strict = synth.head_params(H, L, 1, seed=L)
    wide = _random_table(g, H, L, 0)
    wide[0] = (min((255 << 15) // L, 32640), 127, 127)
    assert binding.validate_params(wide, L, 0) == (0, -1)
    dev = lambda a: torch.from_numpy(a).cuda()
    for table, band in ((strict, 1), (wide, 0)):
        for rq in ([[100 + h, 16] for h in range(H)], [[900 + h, 20] for h in range(H)],
                   [[4096 - h, 24 - (h % 3)] for h in range(H)]):
            rq = np.array(rq, np.int32)
            print(f"square block L={L} band={band} rq={rq[0].tolist()}", flush=True)
            want, rc = oracle.attention(q, k, v, table, rq, band, threads=THREADS)
            assert rc == 0
            buf = torch.full((q.size + 512,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
            out = buf[256:256 + q.size].view(q.shape)
            binding.attention_i8(dev(q), dev(k), dev(v), table, rq, band, out=out)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), want), f"L={L} band={band} rq={rq[0].tolist()}"
            assert bool((buf[:256] == 0x5A5A5A5A).all()) and bool((buf[256 + q.size:] == 0x5A5A5A5A).all())


def test_attention_every_square_length_up_to_896(oracle):
    """Every length from 1 to 896 once, with tables that prove P <= 127 from three keys on (so all but the first two
    take the resident kernel), rows whose maximum is the last key, and inputs whose logits reach both saturations."""
    g = np.random.default_rng(512)
    H, d = 2, 64
    for L in range(1, 897):
        q, k, v = (g.integers(-128, 128, size=(1, H, L, d), dtype=np.int8) for _ in range(3))
        if L % 3 == 0:
            k[0, :, L - 1] = np.where(q[0, :, L // 2] >= 0, 127, -128)   # the last key is the largest for that query
        table = np.array([[300, 2, 20], [280, 1, 20]] if L < 7 else [[100, 2, 20], [60, 1, 20]] if L <= 327
                         else [[60, 1, 20], [50, 0, 9]] if L <= 546 else [[36, 1, 20], [30, 0, 9]], np.int32)
        assert binding.validate_params(table, L, 1) == (0, -1)
        rq = np.array([[3 + L % 50, 12], [900, 20]], np.int32)
        want, rc = oracle.attention(q, k, v, table, rq, 1, threads=THREADS)
        assert rc == 0
        got = binding.attention_i8(torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(),
                                   table, rq, 1)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want), f"L={L}"
    print("896 lengths equal", flush=True)


@pytest.mark.parametrize("L", [16, 64, 65, 100, 128, 197, 200, 256, 300, 320, 384, 390, 447, 448, 449, 511, 512, 513, 577, 640,
                               641, 700, 768, 769, 850, 896])
def test_attention_square_lengths_with_probabilities_above_127(oracle, L):
    """Resident lengths under tables that allow P > 127, with rows that reach it: one key far above the others,
    which sit at the window's edge; in head 1 that key is the last one, whose logit the partial-length kernel repeats
    in the slots behind it.  The matrix unit reads such a byte as P - 256 and the kernel makes up for it."""
    g = np.random.default_rng(2000 + L)
    Bt, H, d = 2, 2, 64
    q = g.integers(20, 100, size=(Bt, H, L, d), dtype=np.int8)
    k = g.integers(-1, 2, size=(Bt, H, L, d), dtype=np.int8)
    v = g.integers(-128, 128, size=(Bt, H, L, d), dtype=np.int8)
    k[:, 0, L // 3] = 127
    k[:, 1, L - 1] = 127
    q[0, 0, ::5] = g.integers(-3, 4, size=q[0, 0, ::5].shape, dtype=np.int8)   # rows without a dominant key in between
    floor = -(-256 // L) + 1
    S0 = 100 if L <= 640 else 70                          # n*B stays within the 8-bit band
    table = np.array([[S0 * 127 + floor, S0, 127], [32 * 100 + floor, 32, 100]], np.int32)
    assert binding.validate_params(table, L, 0) == (0, -1)
    for rq in ([[40, 16], [3, 12]], [[900, 20], [4096, 24]]):
        rq = np.array(rq, np.int32)
        x, rc = oracle.requant_logits(q, k, rq)
        assert rc == 0
        p, rc = oracle.softmax(x, table, 0, threads=THREADS)
        assert rc == 0 and p[:, 0].max() > 127 and p[:, 1, :, L - 1].max() > 127   # the case does reach beyond 127
        check_attention(q, k, v, table, rq, 0, oracle, f"P above 127, L={L} rq={rq[0].tolist()}")


RESIDENT_RECT = [(2, 3, 64, 256), (1, 2, 197, 256), (2, 2, 77, 197), (1, 3, 100, 400), (3, 2, 1, 256), (1, 2, 16, 384),
                 (1, 2, 250, 500), (1, 2, 128, 512), (1, 2, 65, 512), (1, 2, 64, 512), (2, 2, 192, 130), (1, 2, 193, 130),
                 (1, 2, 300, 448), (1, 2, 17, 1), (1, 2, 64, 63), (2, 1, 33, 447), (1, 1, 448, 385), (1, 2, 5, 449),
                 (2, 2, 197, 77), (1, 2, 128, 64), (1, 1, 1000, 64), (1, 2, 700, 300), (1, 1, 513, 512), (1, 2, 449, 385),
                 (1, 2, 100, 600), (1, 1, 700, 577), (2, 1, 65, 768), (1, 2, 64, 768), (1, 1, 300, 769), (1, 2, 1300, 641),
                 (1, 2, 900, 896), (1, 1, 65, 897), (2, 1, 200, 833)]


@pytest.mark.parametrize("Bt,H,Lq,Lk", RESIDENT_RECT)
def test_attention_resident_rectangular_blocks(oracle, Bt, H, Lq, Lk):
    """Head size 64, up to 896 keys, queries and keys of different counts: the resident kernel takes these (beyond 448
    keys only with more than 64 queries; the shapes just outside are here too and stream), in several blocks per
    item when there are more queries than key slots.  Full-range inputs, a table that proves P <= 127 and one that
    does not, two rescale forms, guard values around the output."""
    g = np.random.default_rng(Lq * 1000 + Lk)
    q, k, v = rect_qkv(Lq + Lk, Bt, H, Lq, Lk, 64, lo=-128, hi=127)
    k[:, 0, Lk - 1] = 127
    floor = -(-256 // Lk) + 1
    tables = [(synth.head_params(H, Lk, 1, seed=Lk), 1),
              (np.array([[(100 if Lk <= 640 else 70) * 127 + floor + h, 100 if Lk <= 640 else 70, 127] for h in range(H)],
                        np.int32), 0)]
    for table, band in tables:
        assert binding.validate_params(table, Lk, band) == (0, -1)
        for rq in ([[100 + h, 16] for h in range(H)], [[4096 - h, 24 - (h % 3)] for h in range(H)]):
            rq = np.array(rq, np.int32)
            want, rc = oracle.attention(q, k, v, table, rq, band, threads=THREADS)
            assert rc == 0
            buf = torch.full((q.size + 512,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
            out = buf[256:256 + q.size].view(q.shape)
            binding.attention_i8(torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(),
                                 table, rq, band, out=out)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), want), f"{(Bt, H, Lq, Lk)} band={band} rq={rq[0].tolist()}"
            assert bool((buf[:256] == 0x5A5A5A5A).all()) and bool((buf[256 + q.size:] == 0x5A5A5A5A).all())


def test_attention_vision_encoder_length_full_size(oracle):
    """[64, 12, 197, 197] with head size 64: as many items as the benchmark's fused shape, 197 tokens each."""
    g = np.random.default_rng(197)
    Bt, H, L, d = 64, 12, 197, 64
    q, k, v = (g.integers(-64, 64, size=(Bt, H, L, d), dtype=np.int8) for _ in range(3))
    check_attention(q, k, v, synth.head_params(H, L, 1, seed=197), synth.requant_params(H, seed=197), 1, oracle,
                    "197 tokens, full size")


def test_attention_full_size(oracle):
    w = synth.make_workload("fused_attention")
    check_attention(w["q"], w["k"], w["v"], w["table"], w["requant"], w["band"], oracle, "full")


# ---------------------------------------------------------------- seeded random sweeps
def _random_table(g, H, n, band):
    """Admissible per-head parameters: mostly the workload recipe, sometimes the corners of the band."""
    table = synth.head_params(H, n, band, seed=int(g.integers(1 << 30)))
    cap = (32767 if band == 1 else 255 << 15) // n
    for h in range(H):
        kind = int(g.integers(6))
        if kind == 0 and cap >= 1:                       # largest base the band allows, no slope
            table[h] = (min(cap, 32767), 0, int(g.integers(0, 128)))
        elif kind == 1:                                  # smallest admissible floor: n*(B - S*D) >= 256
            floor = -(-256 // n)
            S, D = int(g.integers(0, 4)), int(g.integers(0, 128))
            if floor + S * D <= min(cap, 32767):
                table[h] = (floor + S * D, S, D)
    assert binding.validate_params(table, n, band) == (0, -1)
    return table


def test_softmax_random_sweep(oracle):
    """500 seeded random cases over shapes, lengths, bands, output modes and value mixes."""
    g = np.random.default_rng(20260427)
    for case in range(500):
        Bt, H, Lq = int(g.integers(1, 4)), int(g.integers(1, 7)), int(g.integers(1, 70))
        pick = int(g.integers(5))
        if pick == 0:
            n = 16 * int(g.integers(1, 40))
        elif pick == 1:
            n = int(g.integers(1, 300))
        elif pick == 2:
            n = 8 * int(g.integers(1, 60))
        elif pick == 3:
            n = int(g.integers(300, 5000))
        else:
            n = int(g.integers(1, 40))
        band = int(g.integers(2))
        if band == 1 and n > 32767 // 2:
            band = 0
        mode = int(g.integers(4))
        if mode & 1 and band != 1:                       # 16-bit output exists under the strict band only
            mode &= 2
        table = _random_table(g, H, n, band)
        x = mixed_logits((Bt, H, Lq, n), seed=int(g.integers(1 << 30)))
        if g.integers(3) == 0:
            x = g.integers(-128, 128, size=x.shape, dtype=np.int8)
        print(f"sweep case {case}: shape={(Bt, H, Lq, n)} band={band} mode={mode}", flush=True)
        want, rc = oracle.softmax(x, table, band, mode=mode, threads=THREADS)
        assert rc == 0
        T, recip = (32767 if mode & 1 else 255), (1 if mode & 2 else 0)
        # a third of the cases run on tensors that begin `off` elements behind a 16-byte line (input
        # and output alike), a few of the 8-bit ones in place
        off = int(g.integers(1, 16)) if g.integers(3) == 0 else 0
        in_place = T == 255 and g.integers(8) == 0
        buf_in = torch.zeros(x.size + 32, dtype=torch.int8, device="cuda")
        buf_in[off:off + x.size] = torch.from_numpy(x).cuda().view(-1)
        t_in = buf_in[off:off + x.size].view(x.shape)
        if in_place:
            t_out = t_in.view(torch.uint8)
        else:
            buf_out = torch.full((x.size + 48,), 0x5A if T == 255 else 0x5A5A,
                                 dtype=torch.uint8 if T == 255 else torch.int16, device="cuda")
            lead = 16 + off if T == 255 else 8 + off      # elements: the same offset behind a 16-byte line
            t_out = buf_out[lead:lead + x.size].view(x.shape)
        binding.calibrated_softmax_i8_ex(t_in, table, band, out_scale_T=T, reciprocal=recip, out=t_out)
        torch.cuda.synchronize()
        got = t_out.cpu().numpy()
        if T == 32767:
            got = got.view(np.uint16)
        assert np.array_equal(got, want), f"case {case} shape={(Bt, H, Lq, n)} band={band} mode={mode} off={off}"
        if not in_place:
            canary = 0x5A if T == 255 else 0x5A5A
            assert bool((buf_out[:lead] == canary).all()) and bool((buf_out[lead + x.size:] == canary).all())


def test_attention_random_sweep(oracle):
    """200 seeded random fused blocks: resident and streaming shapes, both head sizes, every rescale form."""
    attention_sweep(oracle, 20260428, 200)


def test_attention_resident_random_sweep(oracle):
    """300 seeded random fused blocks with head size 64 and up to 896 keys: square, fewer and more queries than keys,
    tables with large and with small floors (probabilities above 127 possible), uniform keys and one dominant key
    (also as the last key), every rescale form."""
    g = np.random.default_rng(20260429)
    for case in range(300):
        Bt, H = int(g.integers(1, 4)), int(g.integers(1, 5))
        Lk = int(g.integers(1, 897)) if g.integers(4) else 64 * int(g.integers(1, 15))
        pick = int(g.integers(4))
        Lq = (Lk if pick == 0 else int(g.integers(1, 130)) if pick == 1 else int(g.integers(1, 1100)) if pick == 2
              else max(1, Lk + int(g.integers(-20, 21))))
        band = int(g.integers(2))
        table = _random_table(g, H, Lk, band)
        if g.integers(2):
            floor = -(-256 // Lk) + 1
            cap = min((32767 if band == 1 else 255 << 15) // Lk, 32767)
            for h in range(H):
                S, D = int(g.integers(1, 101)), int(g.integers(60, 128))
                if S * D + floor <= cap:
                    table[h] = (S * D + floor, S, D)
        assert binding.validate_params(table, Lk, band) == (0, -1)
        lo, hi = (-128, 128) if g.integers(2) else (-64, 64)
        q = g.integers(lo, hi, size=(Bt, H, Lq, 64), dtype=np.int8)
        k = g.integers(lo, hi, size=(Bt, H, Lk, 64), dtype=np.int8)
        v = g.integers(-128, 128, size=(Bt, H, Lk, 64), dtype=np.int8)
        peaky = g.integers(2) == 0
        if peaky:
            q = np.abs(q.astype(np.int16)).clip(0, 127).astype(np.int8)
            k = g.integers(-1, 2, size=k.shape, dtype=np.int8)
            k[:, :, int(g.integers(Lk))] = 127
            k[:, -1, Lk - 1] = 127
        kind = int(g.integers(3))
        if kind == 0:
            rq = np.stack([g.integers(1, 256, H), g.integers(10, 17, H)], 1)
        elif kind == 1:
            rq = np.stack([g.integers(1, 4097, H), g.integers(17, 25, H)], 1)
        else:
            rq = np.stack([g.integers(2048, 4097, H), g.integers(1, 25, H)], 1)
        check_attention(q, k, v, table, rq.astype(np.int32), band, oracle,
                        f"resident sweep {case} Lq={Lq} Lk={Lk} band={band} peaky={peaky} rq={kind}")


def attention_sweep(oracle, seed, cases):
    g = np.random.default_rng(seed)
    for case in range(cases):
        Bt, H = int(g.integers(1, 3)), int(g.integers(1, 5))
        d = 64 if g.integers(3) else 128
        pick = int(g.integers(6))
        if pick == 0:                                    # resident: square, multiple of 64, d = 64
            Lq = Lk = 64 * int(g.integers(1, 9))
            d = 64
        elif pick == 5:                                  # square, any length up to 512, d = 64
            Lq = Lk = int(g.integers(1, 513))
            d = 64
        elif pick == 1:
            Lq, Lk = int(g.integers(1, 200)), int(g.integers(1, 700))
        elif pick == 2:
            Lq, Lk = int(g.integers(1, 100)), int(g.integers(900, 2300))
        elif pick == 3:
            Lq, Lk = int(g.integers(1, 40)), 64 * int(g.integers(1, 40))
        else:                                            # keys in four shares, and just beyond
            Lq, Lk = int(g.integers(1, 70)), int(g.integers(2049, 4300))
        band = int(g.integers(2))
        if band == 1 and Lk > 4000:
            band = 0
        table = _random_table(g, H, Lk, band)
        full = g.integers(2) == 0
        lo, hi = (-128, 128) if full else (-64, 64)
        q = g.integers(lo, hi, size=(Bt, H, Lq, d), dtype=np.int8)
        k = g.integers(lo, hi, size=(Bt, H, Lk, d), dtype=np.int8)
        v = g.integers(-128, 128, size=(Bt, H, Lk, d), dtype=np.int8)
        kind = int(g.integers(3))
        if kind == 0:
            rq = np.stack([g.integers(1, 256, H), g.integers(10, 17, H)], 1)
        elif kind == 1:
            rq = np.stack([g.integers(1, 4097, H), g.integers(17, 25, H)], 1)
        else:
            rq = np.stack([g.integers(2048, 4097, H), g.integers(1, 25, H)], 1)
        check_attention(q, k, v, table, rq.astype(np.int32), band, oracle, f"sweep {case} Lq={Lq} Lk={Lk} d={d} rq={kind}")
