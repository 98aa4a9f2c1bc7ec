"""The pure-host code -- the fp64 oracle's C loops and the library's argument validation -- under
AddressSanitizer and UndefinedBehaviorSanitizer (host only; nothing here touches a GPU).

tests/native/sanitize_driver.cpp is built with -fsanitize=address,undefined together with
oracle/linrec_oracle.c and csrc/linrec_validate.cpp, run on seeded cases whose buffers are exactly sized
heap arrays, and its results are compared with what the ordinary builds return for the same inputs.  Any
sanitizer report ends the driver with a non-zero status."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import paper_1709_04057_amd as lr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    d = tmp_path_factory.mktemp("sanitize")
    exe = str(d / "sanitize_driver")
    inc = "-I" + os.path.join(ROOT, "include")
    objs = []
    for cc, src, extra in (("gcc", os.path.join(ROOT, "oracle", "linrec_oracle.c"), ["-std=c99", "-ffp-contract=off"]),
                           ("g++", os.path.join(ROOT, "paper_1709_04057_amd", "csrc", "linrec_validate.cpp"), ["-std=c++17"]),
                           ("g++", os.path.join(ROOT, "tests", "native", "sanitize_driver.cpp"), ["-std=c++17"])):
        obj = str(d / (os.path.basename(src) + ".o"))
        subprocess.check_call([cc] + SAN + extra + ["-Wall", inc, "-c", src, "-o", obj])
        objs.append(obj)
    subprocess.check_call(["g++"] + SAN + objs + ["-o", exe, "-lm"])
    return exe, d


def _validation_records(rng, count):
    """Argument patterns for the validators: pointer VALUES (never dereferenced) that are null, equal,
    overlapping or apart, with small, empty, negative and overflowing shapes."""
    recs = []
    dims = [0, 1, 2, 3, 7, 64, 1 << 20, 1 << 39, 1 << 40, (1 << 40) + 1, (1 << 62), (1 << 63) - 1, -1, -(1 << 63)]
    for _ in range(count):
        kind = int(rng.integers(0, 10))
        T, B, n = (int(rng.choice(dims[:7])) if rng.random() < 0.7 else int(rng.choice(dims)) for _ in range(3))
        E = abs(T * B * n) % (1 << 44) if all(abs(v) < (1 << 21) for v in (T, B, n)) else 4096
        base = 1 << 32
        ptrs = []
        for _k in range(12):
            u = rng.random()
            if u < 0.15:
                ptrs.append(0)
            elif u < 0.3 and ptrs:
                ptrs.append(int(rng.choice(ptrs)))                       # exact alias of an earlier argument
            elif u < 0.4 and ptrs:
                ptrs.append(max(0, int(rng.choice(ptrs)) + 4 * int(rng.integers(-3, 4))))   # partial overlap
            else:
                ptrs.append(base + 16 * int(rng.integers(0, 64)) * max(E // 4, 1))
        recs.append([kind] + ptrs + [int(rng.integers(-1, 3)), T, B, n])
    return np.array(recs, dtype=np.int64)


def _library_status(rec):
    L = lr.lib()
    p = [ctypes.c_void_p(int(v)) if v else None for v in rec[1:13]]
    tau, T, B, n = (int(v) for v in rec[13:17])
    kind = int(rec[0])
    if kind == 0:
        return L.linrec_validate_forward(*p[:4], T, B, n)
    if kind == 1:
        return L.linrec_validate_backward(*p[:7], T, B, n)
    if kind == 2:
        return L.linrec_validate_forward_bf16(*p[:4], T, B, n)
    if kind == 3:
        return L.linrec_validate_backward_bf16(*p[:7], T, B, n)
    if kind == 4:
        return L.linrec_validate_gilr_forward(*p[:4], tau, T, B, n)
    if kind == 5:
        return L.linrec_validate_gilr_backward(*p[:8], tau, T, B, n)
    if kind == 6:
        return L.linrec_validate_lstm_cell_forward(*p[:7], T, B, n)
    if kind == 7:
        return L.linrec_validate_lstm_cell_backward(*p[:12], T, B, n)
    if kind == 8:
        return L.linrec_validate_gilr_forward_bf16(*p[:4], tau, T, B, n)
    return L.linrec_validate_lstm_cell_backward_bf16(*p[:12], T, B, n)


@pytest.mark.parametrize("T,C,tau,has_h0", [(1, 1, 1, 1), (2, 3, 0, 0), (17, 5, 1, 1), (64, 8, 0, 1), (3, 130, 1, 0),
                                              (0, 4, 1, 1), (5, 0, 1, 0)])
def test_oracle_and_validation_under_sanitizers(driver, oracle, T, C, tau, has_h0):
    exe, d = driver
    rng = np.random.default_rng(1000 * T + 10 * C + tau)
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    a = f32(rng.normal(0.5, 1.5, (T, C)))            # lambda (any sign, some beyond 1) / gate pre-activations
    b, z, o, e = (f32(rng.normal(size=(T, C))) for _ in range(4))
    h0 = f32(rng.normal(size=C))
    recs = _validation_records(rng, 200)
    case, res = str(d / f"case_{T}_{C}.bin"), str(d / f"res_{T}_{C}.bin")
    with open(case, "wb") as f:
        np.array([T, C, tau, has_h0, len(recs)], dtype=np.int64).tofile(f)
        for t in (a, b, z, o, e, h0):
            t.tofile(f)
        recs.tofile(f)
    p = subprocess.run([exe, case, res], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert p.returncode == 0, "sanitizer or driver failure:\n" + p.stdout[-4000:]

    # the same through the ordinary builds
    h0a = h0 if has_h0 else None
    want = []
    href = oracle.forward(a, b, h0a)
    want += [href]
    want += list(oracle.backward(a, f32(href), h0a, e))
    hg = oracle.gilr_forward(a, b, h0a, tau)
    want += [hg] + list(oracle.gilr_backward(a, b, f32(hg), h0a, e, tau))
    cref, hl = oracle.lstm_forward(a, b, z, o, h0a)
    want += [cref, hl] + list(oracle.lstm_backward(a, b, z, o, f32(cref), h0a, e))
    want = np.concatenate([np.asarray(w, dtype=np.float64).reshape(-1) for w in want])
    with open(res, "rb") as f:
        got = np.fromfile(f, dtype=np.float64, count=want.size)
        status = np.fromfile(f, dtype=np.int64)
    assert got.size == want.size and status.size == len(recs)
    # (same source, same -ffp-contract=off; only the optimisation level differs)
    np.testing.assert_allclose(got, want, rtol=1e-14, atol=1e-300)
    for rec, st in zip(recs, status):
        assert int(st) == _library_status(rec), rec.tolist()
