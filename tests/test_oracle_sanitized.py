"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the oracle is
compiled with gcc -fsanitize=address,undefined into a library of its own, and a child process
with the sanitizer runtime preloaded runs the oracle's entry points through ctypes on small
cases (brute-force comparison of the selection, merge, apply, delta) with inputs placed at the
very end of their buffers, so that any read or write past an array, a misaligned access or a
signed overflow aborts the child."""
import os
import shutil
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = textwrap.dedent(r"""
    import ctypes, itertools, sys
    import numpy as np
    lib = ctypes.CDLL(sys.argv[1])
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    lib.oracle_sparsify_layer.restype = ctypes.c_int
    lib.oracle_sparsify_layer.argtypes = [vp, vp, i64, f32, i64, vp, vp]
    def tight(a):
        # a copy that ends exactly at the end of its allocation (numpy allocates exactly nbytes)
        return np.array(a, copy=True)
    def ptr(a):
        return a.ctypes.data_as(vp)
    rng = np.random.default_rng(5)
    vals = np.array([0.0, -0.0, 1.0, -1.0, 2.5, 1e-42, -3.0, 2.5, np.inf, -np.inf], np.float32)
    checked = 0
    for d in (1, 2, 3, 5, 8):
        for trial in range(6):
            g = tight(rng.choice(vals, d).astype(np.float32))
            r0 = tight(rng.choice(vals[:8], d).astype(np.float32))
            for k in range(1, d + 1):
                r = tight(r0)
                oi, ov = np.empty(k, np.int32), np.empty(k, np.float32)
                assert lib.oracle_sparsify_layer(ptr(g), ptr(r), d, 0.5, k, ptr(oi), ptr(ov)) == 0
                acc = (r0 + np.float32(0.5) * g).astype(np.float32)
                key = acc.view(np.uint32) & 0x7FFFFFFF
                order = sorted(range(d), key=lambda i: (-int(key[i]), i))[:k]
                assert sorted(order) == list(oi), (d, k, oi, order)
                assert np.array_equal(ov.view(np.uint32), acc[oi].view(np.uint32))
                checked += 1
    # a two-layer model, three workers: model call, merge, apply and delta through the same build
    class Layer(ctypes.Structure):
        _fields_ = [("offset", i64), ("d", i64), ("rho", ctypes.c_double)]
    lib.oracle_topk_count.restype, lib.oracle_topk_count.argtypes = i64, [i64, ctypes.c_double]
    lib.oracle_sparsify_model.restype = ctypes.c_int
    lib.oracle_sparsify_model.argtypes = [vp, i32, vp, vp, f32, vp, vp]
    lib.oracle_merge_sparse.restype = ctypes.c_int
    lib.oracle_merge_sparse.argtypes = [vp, i32, vp, vp, i32, i64, vp]
    lib.oracle_apply_sparse.restype = ctypes.c_int
    lib.oracle_apply_sparse.argtypes = [vp, i32, vp, vp, i32, i64, vp]
    lib.oracle_delta_monitor.restype = ctypes.c_int
    lib.oracle_delta_monitor.argtypes = [vp, i32, vp, i64, vp, vp, i32, i64, vp]
    dims, rhos = (37, 5), (0.2, 0.5)
    layers = (Layer * 2)(Layer(0, dims[0], rhos[0]), Layer(dims[0], dims[1], rhos[1]))
    ks = [lib.oracle_topk_count(d, r) for d, r in zip(dims, rhos)]
    total, K, P = sum(dims), sum(ks), 3
    idx, val = np.empty(P * K, np.int32), np.empty(P * K, np.float32)
    res = np.zeros(P * total, np.float32)
    for p in range(P):
        g = tight(rng.standard_normal(total).astype(np.float32))
        r = tight(np.zeros(total, np.float32))
        oi, ov = np.empty(K, np.int32), np.empty(K, np.float32)
        assert lib.oracle_sparsify_model(ctypes.byref(layers), 2, ptr(g), ptr(r), 0.25, ptr(oi), ptr(ov)) == 0
        idx[p * K:(p + 1) * K], val[p * K:(p + 1) * K], res[p * total:(p + 1) * total] = oi, ov, r
    upd = tight(np.full(total, 7.0, np.float32))
    assert lib.oracle_merge_sparse(ctypes.byref(layers), 2, ptr(idx), ptr(val), P, K, ptr(upd)) == 0
    want = np.zeros(total, np.float32)
    for p in range(P):
        o = 0
        for (off, d), k in zip(((0, dims[0]), (dims[0], dims[1])), ks):
            for j in range(k):
                want[off + idx[p * K + o + j]] = np.float32(want[off + idx[p * K + o + j]] + val[p * K + o + j])
            o += k
    want = (want / np.float32(P)).astype(np.float32)
    assert np.array_equal(want.view(np.uint32), upd.view(np.uint32))
    param = tight(rng.standard_normal(total).astype(np.float32))
    expect = (param - want).astype(np.float32)
    assert lib.oracle_apply_sparse(ctypes.byref(layers), 2, ptr(idx), ptr(val), P, K, ptr(param)) == 0
    assert np.array_equal(param.view(np.uint32), expect.view(np.uint32))
    out3 = tight(np.empty(6, np.float64))
    assert lib.oracle_delta_monitor(ctypes.byref(layers), 2, ptr(res), total, ptr(idx), ptr(val), P, K, ptr(out3)) == 0
    assert np.all(np.isfinite(out3))
    print("sanitized oracle: %d selections checked" % checked)
    """)


def test_oracle_under_asan_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc is not installed")
    probe = subprocess.run([gcc, "-print-file-name=libasan.so"], capture_output=True, text=True)
    asan = probe.stdout.strip()
    if not asan or not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("the AddressSanitizer runtime is not installed")
    ubsan = subprocess.run([gcc, "-print-file-name=libubsan.so"], capture_output=True, text=True).stdout.strip()
    lib = str(tmp_path / "liblags_oracle_san.so")
    src = os.path.join(ROOT, "oracle", "lags_oracle.c")
    subprocess.check_call([gcc, "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-shared", "-fPIC", "-o", lib, src,
                           "-lm"])
    child = tmp_path / "child.py"
    child.write_text(CHILD)
    env = dict(os.environ)
    preload = asan + (":" + ubsan if os.path.isabs(ubsan) and os.path.exists(ubsan) else "")
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    out = subprocess.run([sys.executable, str(child), lib], env=env, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert "selections checked" in out.stdout
