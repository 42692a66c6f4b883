"""Exercises the host code of one sanitizer-instrumented library (run by tests/test_host_sanitizers.py in a process
whose LD_PRELOAD names the matching sanitizer runtime).  Loads the library with ctypes only: no torch, no GPU.

usage: host_sanitizer_driver.py znni <libznni_hostsan.so> | oracle <libznni_ref_san.so>
"""
import ctypes
import sys

import numpy as np


def i3(*v):
    return (ctypes.c_int * 3)(*v)


def drive_znni(path):
    L = ctypes.CDLL(path)
    sz = ctypes.c_size_t
    L.znni_status_string.restype = ctypes.c_char_p
    b = sz(0)
    p, ws, big = 0x1000, 0x100000, 1 << 40
    vp = ctypes.c_void_p
    n_ok = 0
    # transform sizes over the whole range, and the workspace / division / work / choice queries over many shapes
    for n in range(-2, 1100):
        L.znni_fft_size(n)
    rng = np.random.default_rng(5)
    for _ in range(400):
        S, f, fo = (int(v) for v in rng.integers(1, 70, 3))
        n = [int(v) for v in rng.integers(1, 400, 3)]
        k = [int(min(v, m)) for v, m in zip(rng.integers(1, 12, 3), n)]
        rc = L.znni_conv3d_fft_workspace_v(S, f, fo, i3(*n), i3(*k), ctypes.byref(b))
        if rc != 0:
            continue
        n_ok += 1
        full = b.value
        sub = i3(0, 0, 0)
        for frac in (1.0, 0.5, 0.2, 0.01):
            L.znni_conv3d_fft_sublayers_v(S, f, fo, i3(*n), i3(*k), sz(int(full * frac)), sub, ctypes.byref(b))
        nb, fl = (ctypes.c_double * 8)(), (ctypes.c_double * 8)()
        for flags in (0, 1, 4, 8, 16, 32, 64 | 1, 2):
            L.znni_conv3d_fft_stage_work_v(S, f, fo, i3(*n), i3(*k), flags, nb, fl)
        prim = ctypes.c_int(0)
        est = (ctypes.c_float * 2)()
        L.znni_conv3d_choose_v(S, f, fo, i3(*n), i3(*k), ctypes.byref(prim), est)
        L.znni_conv3d_workspace_v(S, f, fo, i3(*n), i3(*k), ctypes.byref(b))
        L.znni_conv3d_direct_workspace_v(S, f, fo, i3(*n), i3(*k), ctypes.byref(b))
        # calls that must stop in validation (too small a workspace, misaligned or missing pointers, bad flags)
        for args in ((vp(p), vp(p), None, vp(p), 0, vp(ws), sz(16)), (None, vp(p), None, vp(p), 0, vp(ws), sz(big)),
                     (vp(p + 4), vp(p), None, vp(p), 0, vp(ws), sz(big)), (vp(p), vp(p), None, vp(p), 1 << 20, vp(ws), sz(big))):
            assert L.znni_conv3d_fft_v(S, f, fo, i3(*n), i3(*k), *args, None) != 0
            assert L.znni_conv3d_fft_budget_v(S, f, fo, i3(*n), i3(*k), *args, None) != 0
            assert L.znni_conv3d_v(S, f, fo, i3(*n), i3(*k), *args, None) != 0
        assert L.znni_conv3d_fft_static_v(S, f, fo, i3(*n), i3(*k), None, vp(p), None, vp(p), 0, None) == -1
    for st in range(-9, 2):
        assert L.znni_status_string(st)
    for pw in ((2, 2, 2), (1, 3, 4), (5, 1, 1), (0, 1, 1)):
        L.znni_mpf(1, 1, i3(7, 7, 7), i3(*pw), vp(p), vp(p), None)
        L.znni_maxpool(1, 1, i3(8, 8, 8), i3(*pw), None, vp(p), None)
    assert n_ok > 100
    print(f"znni host code: {n_ok} shapes planned, no sanitizer report")


def drive_oracle(path):
    L = ctypes.CDLL(path)
    fp, dp, ip = (ctypes.POINTER(t) for t in (ctypes.c_float, ctypes.c_double, ctypes.c_int))
    rng = np.random.default_rng(6)
    for _ in range(40):
        S, f, fo = (int(v) for v in rng.integers(1, 4, 3))
        n = [int(v) for v in rng.integers(1, 9, 3)]
        k = [int(min(v, m)) for v, m in zip(rng.integers(1, 5, 3), n)]
        inp = rng.uniform(-1, 1, (S, f, *n)).astype(np.float32)
        w = rng.standard_normal((fo, f, *k)).astype(np.float32)
        bias = rng.standard_normal(fo).astype(np.float32)
        o = [a - c + 1 for a, c in zip(n, k)]
        out = np.empty((S, fo, *o), dtype=np.float64)
        for flags, bp in ((0, None), (1, bias.ctypes.data_as(fp))):
            rc = L.znni_ref_conv3d_f64_v(S, f, fo, *n, *k, inp.ctypes.data_as(fp), w.ctypes.data_as(fp), bp,
                                         out.ctypes.data_as(dp), flags, 2)
            assert rc == 0
            pts = np.stack([rng.integers(0, S, 50), rng.integers(0, fo, 50), rng.integers(0, o[0], 50),
                            rng.integers(0, o[1], 50), rng.integers(0, o[2], 50)], 1).astype(np.int32)
            got = np.empty(50, dtype=np.float64)
            rc = L.znni_ref_conv3d_points_f64(S, f, fo, *n, *k, inp.ctypes.data_as(fp), w.ctypes.data_as(fp), bp,
                                              pts.ctypes.data_as(ip), ctypes.c_long(50), got.ctypes.data_as(dp), flags, 2)
            assert rc == 0
            assert np.allclose(got, out[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3], pts[:, 4]], rtol=0, atol=1e-12)
        for p in ((1, 1, 1), (2, 2, 2), (1, 2, 3)):
            if all((a + 1) % q == 0 or q == 1 for a, q in zip(n, p)) and all(a >= q for a, q in zip(n, p)):
                m = [a // q for a, q in zip(n, p)]
                frag = np.empty((S * p[0] * p[1] * p[2], f, *m), dtype=np.float32)
                assert L.znni_ref_mpf(S, f, *n, *p, inp.ctypes.data_as(fp), frag.ctypes.data_as(fp)) == 0
            if all(a % q == 0 for a, q in zip(n, p)):
                m = [a // q for a, q in zip(n, p)]
                pool = np.empty((S, f, *m), dtype=np.float32)
                assert L.znni_ref_maxpool(S, f, *n, *p, inp.ctypes.data_as(fp), pool.ctypes.data_as(fp)) == 0
    print("oracle: no sanitizer report")


if __name__ == "__main__":
    {"znni": drive_znni, "oracle": drive_oracle}[sys.argv[1]](sys.argv[2])
