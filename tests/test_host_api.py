"""Host-side behaviour of the C-ABI library that needs no GPU: the library loads,
exports every symbol the header declares, and its admissibility check agrees with
the oracle's on every boundary of Sec. IV-C.  Rejected calls launch nothing, so
the error paths of the compute entry points are exercised here with null device
pointers."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2604_02292_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_02292_amd.build import build
        build()
    return binding.lib()


def test_every_declared_symbol_is_exported(lib):
    header = "".join(open(os.path.join(ROOT, "include", f)).read()
                     for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    declared = set(re.findall(r"\b(hccs_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    assert binding.status_string(0) == "ok"
    for code in range(-10, 0):
        assert binding.status_string(code) != "unknown status"
    assert binding.status_string(-77) == "unknown status"


CASES = [
    (511, 0, 1, 64, 1), (512, 0, 1, 64, 1), (512, 0, 1, 64, 0), (130560, 0, 1, 64, 0),
    (32767, 0, 1, 255, 0), (32767, 0, 1, 256, 0), (100, 1, 96, 64, 1), (100, 1, 97, 64, 1),
    (100, 1, 101, 64, 1), (100, 1, 128, 64, 1), (100, 128, 0, 64, 1), (0, 0, 0, 64, 1),
    (7, 0, 127, 4096, 1), (8, 0, 127, 4096, 1), (2040, 15, 127, 4096, 0), (2041, 15, 127, 4096, 0),
    (100, -1, 5, 64, 1), (100, 1, -1, 64, 1), (32767, 127, 127, 65536, 0), (127, 1, 126, 256, 1),
]


@pytest.mark.parametrize("B,S,D,n,band", CASES)
def test_validator_agrees_with_oracle(lib, oracle, B, S, D, n, band):
    rc, bad = binding.validate_params([[B, S, D]], n, band)
    assert rc == oracle.check_params(B, S, D, n, band)
    assert bad == (-1 if rc == 0 else 0)


def test_validator_random_sweep_agrees_with_oracle(lib, oracle):
    g = np.random.default_rng(0)
    for _ in range(3000):
        n = int(g.choice([1, 2, 16, 32, 64, 100, 128, 256, 512, 4096, 65536]))
        B = int(g.integers(-2, 40000)) if g.random() < 0.5 else int(g.integers(1, max(2, 40000 // n)))
        S, D = int(g.integers(-1, 130)), int(g.integers(-1, 130))
        band = int(g.integers(0, 2))
        assert binding.validate_params([[B, S, D]], n, band)[0] == oracle.check_params(B, S, D, n, band)


def test_validator_reports_first_bad_head(lib):
    table = [[511, 0, 1], [511, 3, 100], [512, 0, 1], [0, 0, 0]]
    assert binding.validate_params(table, 64, 1) == (-7, 2)
    assert binding.validate_params(table[:2], 64, 1) == (0, -1)
    assert binding.validate_params(table, 64, 7)[0] == -4
    assert binding.validate_params(table, 0, 1)[0] == -2
    assert binding.validate_params(table, 65537, 1)[0] == -2


def test_synthetic_tables_are_admissible(lib):
    for name, (shape, band) in synth.WORKLOADS.items():
        n = shape[3] if name != "fused_attention" else shape[2]
        table = synth.head_params(shape[1], n, band, synth.WORKLOAD_SEED[name])
        assert binding.validate_params(table, n, band) == (0, -1)


def _softmax_rc(lib, ptr_in, ptr_out, B, H, Lq, Lk, table, T=255, band=1):
    arr, _ = binding.head_table(table)
    return lib.hccs_calibrated_softmax_i8(ctypes.c_void_p(ptr_in), ctypes.c_void_p(ptr_out), B, H, Lq, Lk, arr,
                                          T, band, None)


def test_softmax_rejections_launch_nothing(lib):
    ok = [[511, 0, 1]]
    assert _softmax_rc(lib, 0, 0, 1, 1, 4, 64, ok) == -1            # null device pointers
    assert _softmax_rc(lib, 4096, 8192, 1, 1, 4, 64, ok, T=32767) == -4
    assert _softmax_rc(lib, 4096, 8192, 1, 1, 4, 64, ok, band=3) == -4
    assert _softmax_rc(lib, 4096, 8192, 1, 1, 4, 64, [[512, 0, 1]]) == -7
    assert _softmax_rc(lib, 4096, 8192, 1, 1, 4, 64, [[100, 1, 97]]) == -6
    assert _softmax_rc(lib, 4096, 8192, 1, 1, 4, 64, [[100, 1, 101]]) == -5
    assert _softmax_rc(lib, 4096, 8192, -1, 1, 4, 64, ok) == -2
    assert _softmax_rc(lib, 4096, 8192, 1, 0, 4, 64, ok) == -2
    assert _softmax_rc(lib, 4096, 8192, 1, 65, 4, 64, ok * 65) == -2
    assert _softmax_rc(lib, 4096, 8192, 1, 1, 4, 0, ok) == -2
    assert _softmax_rc(lib, 4096, 8192, 1, 1, 4, 65537, ok) == -2
    assert _softmax_rc(lib, 4096, 8192, 1 << 20, 64, 32, 64, ok * 64) == -2   # 2^31 rows: one too many
    assert _softmax_rc(lib, 4096, 4096 + 64, 1, 1, 4, 64, ok) == -3  # partial overlap
    assert _softmax_rc(lib, 0, 0, 0, 1, 4, 64, ok) == 0             # empty tensor: no-op
    assert _softmax_rc(lib, 0, 0, 1, 1, 0, 64, ok) == 0


def test_ex_entry_point_rejections(lib):
    vp = ctypes.c_void_p
    ok, _ = binding.head_table([[511, 0, 1]])

    def call(a=4096, b=1 << 20, B=1, H=1, Lq=4, Lk=64, tab=ok, T=255, recip=0, band=1):
        return lib.hccs_calibrated_softmax_i8_ex(vp(a), vp(b), B, H, Lq, Lk, tab, T, recip, band, None)

    assert call(T=100) == -4 and call(recip=2) == -4 and call(band=5) == -4
    assert call(a=0) == -1
    assert call(T=32767, b=(1 << 20) + 1) == -3                   # odd address for 16-bit output
    assert call(T=32767, a=4096, b=4096) == -3                    # no in-place use in the 16-bit modes
    assert call(T=32767, a=4096, b=4096 + 128) == -3              # overlapping
    assert call(T=255, a=4096, b=4096 + 128) == -3
    # the 16-bit path enforces the strict band even if the caller names the wider one
    wide, _ = binding.head_table([[512, 0, 1]])
    assert call(tab=wide, band=0, T=255, a=0, b=0, B=0) == 0
    assert call(tab=wide, band=0, T=32767, a=0, b=0, B=0) == -7


def test_attention_rejections_launch_nothing(lib):
    arr, _ = binding.head_table([[127, 1, 126]])
    rq, _ = binding.requant_table([[128, 16]])
    vp = ctypes.c_void_p

    def call(q=4096, k=8192, v=12288, o=16384, B=1, H=1, L=256, d=64, rq_=rq, T=255, band=1, tab=arr):
        return lib.hccs_attention_i8(vp(q), vp(k), vp(v), vp(o), B, H, L, d, tab, rq_, T, band, None)

    assert call(q=0) == -1
    assert call(d=32) == -2 and call(L=0) == -2 and call(L=70000) == -2 and call(H=0) == -2
    assert call(L=1024) == -7                         # a valid shape now; this table is outside the band at n = 1024
    assert call(q=4100) == -3
    assert call(T=32767) == -4
    assert call(rq_=binding.requant_table([[4097, 16]])[0]) == -9
    assert call(rq_=binding.requant_table([[128, 25]])[0]) == -9
    assert call(rq_=binding.requant_table([[128, 0]])[0]) == -9
    assert call(tab=binding.head_table([[128, 1, 126]])[0]) == -7
    assert call(B=0, q=0, k=0, v=0, o=0) == 0

    def call_ex(q=4096, k=8192, v=12288, o=16384, B=1, H=1, Lq=40, Lk=256, d=64, band=1):
        return lib.hccs_attention_i8_ex(vp(q), vp(k), vp(v), vp(o), B, H, Lq, Lk, d, arr, rq, 255, band, None)

    assert call_ex(Lk=0) == -2 and call_ex(d=96) == -2 and call_ex(Lq=-1) == -2 and call_ex(B=1 << 26) == -2   # 2^31 rows and more
    assert call_ex(Lq=0, q=0, o=0) == 0               # no queries: nothing to do
    assert call_ex(k=0) == -1 and call_ex(o=16388) == -3
    assert call_ex(Lk=512) == -7                      # band is checked with n = Lk


def test_calibration_entry_point_rejections(lib):
    vp = ctypes.c_void_p
    assert lib.hccs_calibrate_workspace_bytes(2, 3, 4, 64) == (2 * 3 * 4 * (128 * 4 + 8) + 2 * 3 * 2048 + 3 * 2056
                                                              + 32768 * 8)   # + the table of logarithms
    assert lib.hccs_calibrate_workspace_bytes(0, 3, 4, 64) == -2
    assert lib.hccs_calibrate_workspace_bytes(2, 65, 4, 64) == -2
    assert lib.hccs_calibrate_workspace_bytes(1 << 20, 64, 32, 64) == -2
    al = (ctypes.c_double * 2)(0.1, 0.2)

    def call(x=4096, B=1, H=2, Lq=4, Lk=64, alpha=al, cand=8192, nc=5, obj=16384, best=32768, ws=65536, wsb=1 << 20):
        return lib.hccs_calibrate_grid(vp(x), B, H, Lq, Lk, alpha, vp(cand), nc, vp(obj), vp(best), vp(ws), wsb, None)

    assert call(x=0) == -1 and call(cand=0) == -1 and call(ws=0) == -1
    assert call(nc=0) == -2 and call(nc=70000) == -2 and call(B=0) == -2
    assert call(wsb=100) == -2                      # workspace too small
    assert call(ws=65540) == -3 and call(obj=16388) == -3
    assert call(alpha=(ctypes.c_double * 2)(0.1, 0.0)) == -4
    assert call(alpha=(ctypes.c_double * 2)(0.1, float("nan"))) == -4


def test_static_calibration_entry_point_rejections(lib):
    """The size limit and the shape checks come before anything touches a device."""
    vp = ctypes.c_void_p
    al = (ctypes.c_double * 8)(*([0.1] * 8))

    def call(B=1, H=8, Lq=4, Lk=64, nc=5):
        return lib.hccs_calibrate_grid_static(vp(4096), B, H, Lq, Lk, al, vp(8192), nc, vp(16384), vp(32768), None)

    assert lib.hccs_calibrate_workspace_bytes(64, 8, 128, 128) <= 36 << 20 < lib.hccs_calibrate_workspace_bytes(
        80, 8, 128, 128)
    assert call(B=80, Lq=128, Lk=128) == -10
    assert call(B=0) == -2 and call(H=65) == -2 and call(Lk=0) == -2
    assert binding.status_string(-10) != "unknown status"


def test_other_entry_points_reject_bad_arguments(lib):
    vp = ctypes.c_void_p
    assert lib.hccs_reciprocal_u8(vp(0), vp(0), 5, None) == -1
    assert lib.hccs_reciprocal_u8(vp(0), vp(0), -1, None) == -2
    assert lib.hccs_reciprocal_u8(vp(0), vp(0), 0, None) == 0
    assert lib.hccs_normalise_table_u8(vp(0), vp(0), 3, None) == -1
    assert lib.hccs_normalise_table_u8(vp(4100), vp(8192), 3, None) == -3
    assert lib.hccs_normalise_table_u8(vp(4096), vp(8192), -1, None) == -2
    assert lib.hccs_copy_bytes(vp(4096), vp(8192), 17, None) == -2
    assert lib.hccs_copy_bytes(vp(4097), vp(8192), 16, None) == -3
    sc = (ctypes.c_float * 1)(0.1)
    assert lib.hccs_exp_softmax_i8_f32(vp(4096), vp(8192), 1, 1, 4, 100, sc, None) == -2


def test_largest_probability_bound_is_attained_and_never_exceeded(lib, oracle):
    """The host-side bound that decides whether the fused kernels feed P to the signed matrix unit
    as it is: per head the probability of a row's maximum when every other key lies beyond the
    window.  Against the oracle: such a row attains the bound exactly, and no other row exceeds it."""
    g = np.random.default_rng(5)
    for n, band in ((256, 0), (256, 1), (64, 0), (1280, 0), (2304, 0), (17, 0)):
        tables = [synth.head_params(6, n, band, seed=n + band)]
        if band == 0:
            cap = (255 << 15) // n
            tables.append(np.array([[min(cap, 32767), 0, 0], [min(cap, 3000), 20, 100], [-(-256 // n) + 3 * 40, 3, 40]],
                                   np.int32))
        if n == 256 and band == 0:
            tables.append(np.array([[763, 38, 20], [261, 13, 20], [502, 25, 20]], np.int32))   # bounds 127, 128, 126
        for table in tables:
            assert binding.validate_params(table, n, band) == (0, -1)
            H = table.shape[0]
            bound = binding.largest_probability_u8(table, n)
            # one key at 127, the others 128 + Dmax and more below it (clamped whatever Dmax is)
            worst = np.full((1, H, 1, n), -128, np.int8)
            worst[..., n // 3] = 127
            p, rc = oracle.softmax(worst, table, band)
            assert rc == 0
            assert np.array_equal(p.reshape(H, n).max(axis=1), bound), (n, band, table.tolist(), bound)
            # random rows, narrow and wide spreads: never above the bound
            for spread in (3, 40, 128):
                x = g.integers(-spread, spread, size=(4, H, 64, n)).clip(-128, 127).astype(np.int8)
                p, rc = oracle.softmax(x, table, band)
                assert rc == 0
                assert (p.transpose(1, 0, 2, 3).reshape(H, -1).max(axis=1) <= bound).all()
    assert lib.hccs_largest_probability_u8(None, 1, 4, None) == -1
    one = np.zeros(3, np.int32)
    vp = ctypes.c_void_p
    assert lib.hccs_largest_probability_u8(one.ctypes.data_as(vp), 0, 4, one.ctypes.data_as(vp)) == -2
    assert lib.hccs_largest_probability_u8(one.ctypes.data_as(vp), 1, 0, one.ctypes.data_as(vp)) == -2


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(binding.HccsError):
        binding.lib()
