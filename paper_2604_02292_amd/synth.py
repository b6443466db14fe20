"""Seeded synthetic inputs: int8 attention logits, Q/K/V tensors and per-head
constants shaped like the workloads the method is measured on.

This module only *draws inputs*.  It holds none of the method's arithmetic
(no row maximum, distance, score, sum, reciprocal or normalisation); both the
GPU library's tests and the CPU oracle's tests feed on the bytes it returns.

Every tensor is produced block by block -- one (batch, head) slab per
counter-based Philox stream keyed by (seed, slab index) -- so the bytes do not
depend on how many threads generate them.

The real workloads these stand in for are int8 attention logits of small
encoder Transformers at sequence lengths 64 and 128 (Sec. V-A of the paper);
their data and weights are not available, so value distributions are chosen to
exercise the same paths: Gaussian rows with per-row offset and per-head spread,
heavy-tailed rows that hit both int8 clamps, rows with long runs of ties, and
long causally masked rows.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

N_U8 = 255 << 15          # numerator of the shifted reciprocal, Eq. (8)
BAND_U8, BAND_STRICT = 0, 1

# name -> (shape, band) of the five workloads
WORKLOADS = {
    "pr1_ref": ((1, 4, 64, 64), BAND_STRICT),
    "edge_encoder": ((256, 8, 128, 128), BAND_STRICT),
    "stress_rows": ((64, 12, 512, 512), BAND_STRICT),
    "long_row": ((4, 16, 4096, 4096), BAND_U8),
    "fused_attention": ((64, 12, 256, 64), BAND_STRICT),
}
WORKLOAD_SEED = {"pr1_ref": 0, "edge_encoder": 1, "stress_rows": 2, "long_row": 3,
                 "fused_attention": 4}


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def _to_int8(a):
    """Round to nearest (ties to even), then saturate to the int8 range."""
    return np.clip(np.rint(a), -128, 127).astype(np.int8)


def _map_slabs(fn, count, threads):
    if threads <= 1 or count <= 1:
        for i in range(count):
            fn(i)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fn, range(count)))


def head_params(H, n, band, seed):
    """H triples (B, S, Dmax), each inside the admissible band for row length n
    (Sec. IV-C; band 1 = Eq. (11), band 0 = the 8-bit path's constraints).
    Dmax ~ U{1..127}; S ~ U{0..min(127, (Bmax-f)//Dmax)}; B ~ U{S*Dmax+f..Bmax}
    with f = ceil(256/n) and Bmax the band's ceiling on B."""
    g = _rng(seed, 0xC0FFEE)
    bmax = 32767 // n if band == BAND_STRICT else min(32767, N_U8 // n)
    f = -(-256 // n)
    if bmax < f:
        raise ValueError(f"no admissible B for n={n} in band {band}")
    table = np.zeros((H, 3), dtype=np.int32)
    for h in range(H):
        D = int(g.integers(1, 128))
        S = int(g.integers(0, min(127, (bmax - f) // D) + 1))
        B = int(g.integers(S * D + f, bmax + 1))
        table[h] = (B, S, D)
    return table


def requant_params(H, seed, shift=16, mult_lo=96, mult_hi=256):
    """H pairs (mult, shift) for the fused block's int32 -> int8 rescale."""
    g = _rng(seed, 0xBEEF)
    out = np.zeros((H, 2), dtype=np.int32)
    out[:, 0] = g.integers(mult_lo, mult_hi + 1, size=H)
    out[:, 1] = shift
    return out


def gaussian_logits(shape, sigma, seed, threads=1):
    """round(N(0, sigma)) saturated to int8, any [B,H,Lq,Lk]."""
    Bt, H, Lq, Lk = shape
    out = np.empty(shape, dtype=np.int8)
    flat = out.reshape(Bt * H, Lq, Lk)

    def slab(i):
        g = _rng(seed, i)
        flat[i] = _to_int8(g.standard_normal((Lq, Lk), dtype=np.float32) * np.float32(sigma))

    _map_slabs(slab, Bt * H, threads)
    return out


def edge_encoder_logits(shape, seed, threads=1):
    """Per row an offset mu ~ U(-40,40); per head a spread sigma_h ~ U(8,40)."""
    Bt, H, Lq, Lk = shape
    sig = _rng(seed, 0x5161).uniform(8.0, 40.0, size=H).astype(np.float32)
    out = np.empty(shape, dtype=np.int8)
    flat = out.reshape(Bt * H, Lq, Lk)

    def slab(i):
        g = _rng(seed, i)
        mu = g.uniform(-40.0, 40.0, size=(Lq, 1)).astype(np.float32)
        z = g.standard_normal((Lq, Lk), dtype=np.float32)
        flat[i] = _to_int8(mu + sig[i % H] * z)

    _map_slabs(slab, Bt * H, threads)
    return out


def stress_logits(shape, seed, threads=1):
    """Row kind = global row index mod 3.
    0: Gaussian sigma 24.  1: Laplace(scale 20) around an offset cycling through
    -90, 0, +90 so both int8 clamps fire often.  2: runs of tied values, run length
    geometric with mean 32, run value round(N(0, 24))."""
    Bt, H, Lq, Lk = shape
    out = np.empty(shape, dtype=np.int8)
    flat = out.reshape(Bt * H, Lq, Lk)

    def slab(i):
        g = _rng(seed, i)
        rows = np.arange(Lq) + i * Lq
        kind = rows % 3
        block = np.empty((Lq, Lk), dtype=np.int8)
        k0 = np.nonzero(kind == 0)[0]
        block[k0] = _to_int8(g.standard_normal((k0.size, Lk), dtype=np.float32) * np.float32(24.0))
        k1 = np.nonzero(kind == 1)[0]
        offs = np.array([-90.0, 0.0, 90.0], dtype=np.float32)[(rows[k1] // 3) % 3][:, None]
        block[k1] = _to_int8(offs + g.laplace(0.0, 20.0, size=(k1.size, Lk)).astype(np.float32))
        k2 = np.nonzero(kind == 2)[0]
        total = k2.size * Lk
        if total:
            nruns = total // 8 + 64
            lens = g.geometric(1.0 / 32.0, size=nruns)
            while lens.sum() < total:
                lens = np.concatenate([lens, g.geometric(1.0 / 32.0, size=nruns)])
            vals = _to_int8(g.standard_normal(lens.size, dtype=np.float32) * np.float32(24.0))
            block[k2] = np.repeat(vals, lens)[:total].reshape(k2.size, Lk)
        flat[i] = block

    _map_slabs(slab, Bt * H, threads)
    return out


def causal_logits(shape, sigma, seed, threads=1):
    """round(N(0, sigma)); every key position after the query's is set to -128."""
    Bt, H, Lq, Lk = shape
    out = np.empty(shape, dtype=np.int8)
    flat = out.reshape(Bt * H, Lq, Lk)
    future = np.triu(np.ones((Lq, Lk), dtype=bool), k=1)

    def slab(i):
        g = _rng(seed, i)
        blk = _to_int8(g.standard_normal((Lq, Lk), dtype=np.float32) * np.float32(sigma))
        blk[future] = -128
        flat[i] = blk

    _map_slabs(slab, Bt * H, threads)
    return out


def uniform_qkv(shape, seed, lo=-64, hi=63):
    """Three int8 tensors [B,H,L,d] with integers uniform in [lo, hi]."""
    g = _rng(seed, 0x9137)
    return tuple(g.integers(lo, hi + 1, size=shape, dtype=np.int8) for _ in range(3))


def make_workload(name, threads=8, shape=None):
    """Inputs of one named workload.  `shape` overrides the size (same recipe,
    fewer batches/rows) for tests that need the oracle to finish quickly.
    Returns a dict: standalone workloads carry 'logits', 'table', 'band';
    the fused one carries 'q', 'k', 'v', 'table', 'requant', 'band'."""
    full_shape, band = WORKLOADS[name]
    shape = tuple(shape) if shape is not None else full_shape
    seed = WORKLOAD_SEED[name]
    H = shape[1]
    if name == "fused_attention":
        q, k, v = uniform_qkv(shape, seed)
        return {"name": name, "q": q, "k": k, "v": v, "band": band,
                "table": head_params(H, shape[2], band, seed),
                "requant": requant_params(H, seed)}
    n = shape[3]
    if name == "pr1_ref":
        x = gaussian_logits(shape, 24.0, seed, threads)
    elif name == "edge_encoder":
        x = edge_encoder_logits(shape, seed, threads)
    elif name == "stress_rows":
        x = stress_logits(shape, seed, threads)
    else:
        x = causal_logits(shape, 30.0, seed, threads)
    return {"name": name, "logits": x, "band": band, "table": head_params(H, n, band, seed)}
