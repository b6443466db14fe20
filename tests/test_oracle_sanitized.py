"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer.

oracle/hccs_oracle.c is compiled together with oracle/sanitize_driver.c (a front end
that only moves arrays in and out) into an executable with
-fsanitize=address,undefined -fno-sanitize-recover=all, and the pinned cases run through
it: the hand-worked fixtures, every int8 row of length 2, the fused block's hand-worked
case and the top of its shift range, the reciprocal at the ends of its range, a small
calibration, and the error returns.  A sanitizer report aborts the executable, so each
case asserts exit status 0 and an empty stderr, and then the values against the fixtures,
the big-integer Python version, or exact integer arithmetic."""
import os
import struct
import subprocess

import numpy as np
import pytest

from conftest import ROOT, golden_files, read_golden
from oracle import hccs_ref

MODES = {"u8": 0, "i16": 1, "clb_u8": 2, "clb_i16": 3}
PY_ROW = {0: hccs_ref.row_u8, 1: hccs_ref.row_i16, 2: hccs_ref.row_clb_u8, 3: hccs_ref.row_clb_i16}


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "sanitize_driver")
    src = [os.path.join(ROOT, "oracle", f) for f in ("hccs_oracle.c", "sanitize_driver.c")]
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-Wall", "-Wextra",
                           "-o", exe] + src + ["-lm"])
    work = tmp_path_factory.mktemp("req")
    count = [0]

    def run(op, arrays, Bt=0, H=0, Lq=0, Lk=0, d=0, band=0, mode=0, threads=1, nc=0):
        count[0] += 1
        req, rep = str(work / f"q{count[0]}.bin"), str(work / f"r{count[0]}.bin")
        with open(req, "wb") as fh:
            fh.write(struct.pack("<12q", op, Bt, H, Lq, Lk, d, band, mode, threads, nc, 0, 0))
            for a in arrays:
                fh.write(np.ascontiguousarray(a).tobytes())
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
                   UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
        proc = subprocess.run([exe, req, rep], env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True,
                              timeout=300)
        assert proc.returncode == 0 and proc.stderr.strip() == "", f"sanitizer report:\n{proc.stderr[-4000:]}"
        with open(rep, "rb") as fh:
            blob = fh.read()
        os.remove(req), os.remove(rep)
        return struct.unpack("<q", blob[:8])[0], blob[8:]

    return run


@pytest.mark.parametrize("name", golden_files())
def test_golden_rows_sanitized(driver, name):
    g = read_golden(name)
    mode = MODES[g["mode"]]
    x = np.array(g["x"], np.int8)
    rc, blob = driver(6, [np.array(g["params"], np.int32), x], Lk=len(x), mode=mode)
    Z, rho = struct.unpack("<2q", blob[:16])
    p = np.frombuffer(blob[16:], np.uint16 if mode & 1 else np.uint8)
    assert rc == 0 and Z == g["Z"][0] and rho == g["rho"][0] and p.tolist() == g["p"]


@pytest.mark.parametrize("mode,params", [(0, (16383, 100, 127)), (1, (16383, 127, 127)), (2, (300, 2, 77)),
                                         (3, (16383, 127, 100))])
def test_all_rows_of_length_two_sanitized(driver, mode, params):
    """Every pair of int8 logits, all four output modes, against the big-integer version."""
    a = np.arange(-128, 128, dtype=np.int8)
    x = np.stack(np.meshgrid(a, a, indexing="ij"), -1).reshape(1, 1, 65536, 2)
    assert hccs_ref.admissible(*params, 2, 1)
    rc, blob = driver(1, [np.array([params], np.int32), x], Bt=1, H=1, Lq=65536, Lk=2, band=1, mode=mode, threads=2)
    got = np.frombuffer(blob, np.uint16 if mode & 1 else np.uint8).reshape(65536, 2)
    assert rc == 0
    rows = x.reshape(65536, 2).tolist()
    for i in range(0, 65536, 7):
        assert got[i].tolist() == PY_ROW[mode](rows[i], *params), rows[i]


def test_long_rows_and_wide_band_sanitized(driver):
    """Rows of 4096 and 65536 elements under the 8-bit band (the largest sums the oracle forms)."""
    g = np.random.default_rng(5)
    for n, params in ((4096, (2040, 15, 127)), (65536, (127, 0, 0)), (65536, (32767 // 300, 0, 3))):
        if not hccs_ref.admissible(*params, n, 0):
            params = (8355840 // n, 0, 0)
        x = g.integers(-128, 128, size=(1, 1, 2, n), dtype=np.int8)
        rc, blob = driver(1, [np.array([params], np.int32), x], Bt=1, H=1, Lq=2, Lk=n, band=0, mode=0)
        got = np.frombuffer(blob, np.uint8).reshape(2, n)
        assert rc == 0
        assert got[1].tolist() == hccs_ref.row_u8(x[0, 0, 1].tolist(), *params)


def test_fused_block_sanitized(driver):
    g = read_golden("a1_attention_tiny.txt")
    q, k, v = (np.array(g[t], np.int8).reshape(1, 1, 2, 1) for t in ("q", "k", "v"))
    table, rq = np.array([g["params"]], np.int32), np.array([g["requant"]], np.int32)
    rc, blob = driver(2, [table, rq, q, k, v], Bt=1, H=1, Lq=2, Lk=2, d=1, band=1)
    assert rc == 0 and np.frombuffer(blob, np.int32).tolist() == g["o"]
    rc, blob = driver(3, [rq, q, k], Bt=1, H=1, Lq=2, Lk=2, d=1)
    assert rc == 0 and np.frombuffer(blob, np.int8).tolist() == g["x"]
    # full-range operands at the ends of the rescale domain, rectangular, two threads
    rng = np.random.default_rng(9)
    Bt, H, Lq, Lk, d = 2, 3, 5, 24, 64
    q = rng.integers(-128, 128, size=(Bt, H, Lq, d), dtype=np.int8)
    k = rng.integers(-128, 128, size=(Bt, H, Lk, d), dtype=np.int8)
    v = rng.integers(-128, 128, size=(Bt, H, Lk, d), dtype=np.int8)
    q[0, 0, 0], k[0, 0, 0] = -128, -128                 # the largest accumulator, 64 * 2^14
    table = np.array([[1300, 10, 127], [1365, 0, 0], [700, 5, 100]], np.int32)
    rq = np.array([[4096, 24], [1, 1], [4096, 1]], np.int32)
    rc, blob = driver(2, [table, rq, q, k, v], Bt=Bt, H=H, Lq=Lq, Lk=Lk, d=d, band=1, threads=2)
    o = np.frombuffer(blob, np.int32).reshape(Bt, H, Lq, d)
    assert rc == 0
    for h in range(H):
        x = [[hccs_ref.requant(int(np.dot(q[1, h, i].astype(np.int64), k[1, h, j].astype(np.int64))),
                               int(rq[h, 0]), int(rq[h, 1])) for j in range(Lk)] for i in range(Lq)]
        for i in range(Lq):
            p = hccs_ref.row_u8(x[i], *table[h].tolist())
            assert o[1, h, i].tolist() == [sum(p[j] * int(v[1, h, j, t]) for j in range(Lk)) for t in range(d)]


def test_reciprocal_range_ends_sanitized(driver):
    N = 255 << 15
    Z = np.array([1, 2, 255, 256, 257, 32767, 32768, 65535, N - 1, N, N + 1, 2 ** 31 - 1], np.int64)
    rc, blob = driver(4, [Z], nc=len(Z))
    assert rc == 0 and np.frombuffer(blob, np.int64).tolist() == [N // int(z) for z in Z]


def test_calibration_sanitized(driver, oracle):
    """A small grid with inadmissible candidates among the admissible ones; the values are compared
    with the ordinary build of the same source (whose own pins are in test_oracle_calibration_pins)."""
    g = np.random.default_rng(3)
    Bt, H, Lq, Lk = 2, 2, 3, 32
    x = np.clip(np.rint(g.normal(0, 25, size=(Bt, H, Lq, Lk))), -128, 127).astype(np.int8)
    alpha = np.array([0.05, 0.2])
    cand = np.array([[1023, 7, 127], [1024, 0, 1], [500, 0, 0], [8, 0, 0], [7, 0, 0], [900, 90, 9], [100, 1, 128]],
                    np.int32)
    rc, blob = driver(5, [alpha, cand, x], Bt=Bt, H=H, Lq=Lq, Lk=Lk, nc=len(cand), threads=2)
    obj = np.frombuffer(blob[:H * len(cand) * 8], np.float64).reshape(H, len(cand))
    best = np.frombuffer(blob[H * len(cand) * 8:], np.int32)
    want, want_best, rc2 = oracle.calibrate(x, alpha, cand)
    assert rc == 0 and rc2 == 0
    assert np.array_equal(np.isinf(obj), np.isinf(want)) and np.isinf(obj[0]).tolist() == [False, True, False, False,
                                                                                            True, False, True]
    fin = np.isfinite(want)
    assert np.allclose(obj[fin], want[fin], rtol=1e-12) and best.tolist() == want_best.tolist()


def test_error_returns_sanitized(driver):
    """Rejected inputs return early: no write, no leak, the documented status."""
    x = np.zeros((1, 1, 2, 64), np.int8)
    for params, status in (((512, 0, 1), -7), ((100, 1, 97), -6), ((100, 1, 101), -5)):
        rc, blob = driver(1, [np.array([params], np.int32), x], Bt=1, H=1, Lq=2, Lk=64, band=1)
        assert rc == status and not np.frombuffer(blob, np.uint8).any()
    rc, _ = driver(1, [np.array([[511, 0, 1]], np.int32), x], Bt=1, H=1, Lq=2, Lk=64, band=0, mode=1)
    assert rc == -1                                      # the 16-bit modes exist under the strict band only
    q = np.zeros((1, 1, 2, 4), np.int8)
    for rq in ([4097, 16], [128, 25], [128, 0], [0, 4]):
        rc, _ = driver(2, [np.array([[511, 0, 1]], np.int32), np.array([rq], np.int32), q, q, q], Bt=1, H=1, Lq=2,
                       Lk=2, d=4, band=0)
        assert rc == -1, rq
        rc, _ = driver(3, [np.array([rq], np.int32), q, q], Bt=1, H=1, Lq=2, Lk=2, d=4)
        assert rc == -1, rq
    assert driver(7, [], Bt=511, H=0, Lq=1, Lk=64, band=1)[0] == 0
    assert driver(7, [], Bt=512, H=0, Lq=1, Lk=64, band=1)[0] == -7
    assert driver(7, [], Bt=32767, H=127, Lq=127, Lk=65536, band=0)[0] == -7
