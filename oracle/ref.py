"""ctypes binding of the CPU oracle (oracle/znni_ref.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module; the product
package never does.  It holds no arithmetic of its own: every number comes from the C loops, which
write out the layer definition of Section IV (valid 3D convolution summed over input images, then bias
and transfer function) in fp64.
"""
import ctypes
import os

import numpy as np

from . import build as _build

RELU = 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        L.znni_ref_conv3d_f64_v.restype = ctypes.c_int
        L.znni_ref_conv3d_f64_v.argtypes = [ctypes.c_int] * 9 + [fp, fp, fp, dp, ctypes.c_uint, ctypes.c_int]
        L.znni_ref_conv3d_f64.restype = ctypes.c_int
        L.znni_ref_conv3d_f64.argtypes = [ctypes.c_int] * 5 + [fp, fp, fp, dp, ctypes.c_uint, ctypes.c_int]
        L.znni_ref_conv3d_points_f64.restype = ctypes.c_int
        L.znni_ref_conv3d_points_f64.argtypes = ([ctypes.c_int] * 9 + [fp, fp, fp, ip, ctypes.c_long, dp,
                                                                      ctypes.c_uint, ctypes.c_int])
        L.znni_ref_max_threads.restype = ctypes.c_int
        for fn in (L.znni_ref_maxpool, L.znni_ref_mpf):
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_int] * 8 + [fp, fp]
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _triple(v):
    if np.isscalar(v):
        return (int(v),) * 3
    v = tuple(int(t) for t in v)
    assert len(v) == 3
    return v


def max_threads() -> int:
    return int(lib().znni_ref_max_threads())


def conv3d(inp, w, bias=None, relu=False, nthreads=0):
    """Full layer.  inp [S,f,nx,ny,nz] fp32, w [fo,f,kx,ky,kz] fp32, bias [fo] or None -> fp64 [S,fo,n'...]."""
    inp, pin = _f32(inp)
    w, pw = _f32(w)
    S, f, nx, ny, nz = inp.shape
    fo, f2, kx, ky, kz = w.shape
    assert f2 == f, "w and inp disagree on the number of input images"
    pb = None
    if bias is not None:
        bias, pb = _f32(bias)
        assert bias.shape == (fo,)
    out = np.empty((S, fo, nx - kx + 1, ny - ky + 1, nz - kz + 1), dtype=np.float64)
    rc = lib().znni_ref_conv3d_f64_v(S, f, fo, nx, ny, nz, kx, ky, kz, pin, pw, pb,
                                     out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                     RELU if relu else 0, int(nthreads))
    if rc != 0:
        raise ValueError(f"znni_ref_conv3d_f64_v failed with status {rc}")
    return out


def conv3d_points(inp, w, bias, pts, relu=False, nthreads=0):
    """Layer output at the positions pts[:, (s, j, x, y, z)] only -> fp64 [npts]."""
    inp, pin = _f32(inp)
    w, pw = _f32(w)
    S, f, nx, ny, nz = inp.shape
    fo, f2, kx, ky, kz = w.shape
    assert f2 == f
    pb = None
    if bias is not None:
        bias, pb = _f32(bias)
    pts = np.ascontiguousarray(pts, dtype=np.int32)
    assert pts.ndim == 2 and pts.shape[1] == 5
    out = np.empty(pts.shape[0], dtype=np.float64)
    rc = lib().znni_ref_conv3d_points_f64(S, f, fo, nx, ny, nz, kx, ky, kz, pin, pw, pb,
                                          pts.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                          pts.shape[0],
                                          out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                          RELU if relu else 0, int(nthreads))
    if rc != 0:
        raise ValueError(f"znni_ref_conv3d_points_f64 failed with status {rc}")
    return out


def _pool(fn_name, inp, p, out_shape):
    inp, pin = _f32(inp)
    S, f, nx, ny, nz = inp.shape
    px, py, pz = _triple(p)
    if min(px, py, pz) < 1:
        raise ValueError("pooling window must be at least 1 on every axis")
    out = np.empty(out_shape(S, f, nx, ny, nz, px, py, pz), dtype=np.float32)
    rc = getattr(lib(), fn_name)(S, f, nx, ny, nz, px, py, pz, pin,
                                 out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc != 0:
        raise ValueError(f"{fn_name} failed with status {rc}")
    return out


def maxpool(inp, p):
    """Max pooling with window p (Section VI): inp [S,f,nx,ny,nz] fp32 -> fp32 [S,f,nx/px,ny/py,nz/pz]."""
    return _pool("znni_ref_maxpool", inp, p,
                 lambda S, f, nx, ny, nz, px, py, pz: (S, f, max(nx // px, 0), max(ny // py, 0), max(nz // pz, 0)))


def mpf(inp, p):
    """Max-pooling fragments with window p (Section VI): inp [S,f,nx,ny,nz] fp32 ->
    fp32 [S*px*py*pz, f, floor(nx/px), floor(ny/py), floor(nz/pz)], fragment (ox,oy,oz) of input s at batch
    index s*px*py*pz + (ox*py + oy)*pz + oz."""
    return _pool("znni_ref_mpf", inp, p,
                 lambda S, f, nx, ny, nz, px, py, pz: (S * px * py * pz, f, nx // px, ny // py, nz // pz))


def tolerance(inp, w, rel=1e-4):
    """Per-output-image error bound rel * max|x| * sum_{i,a,b,c} |w[j,i,a,b,c]| (one value per j)."""
    x = float(np.max(np.abs(np.asarray(inp, dtype=np.float64))))
    return rel * x * np.sum(np.abs(np.asarray(w, dtype=np.float64)), axis=(1, 2, 3, 4))
