"""Thin ctypes binding of libznni.so (declared in include/znni.h): argument marshalling only.

PyTorch is used for device memory and streams; every step of the layer runs in the library's HIP kernels.
There is no fallback: if the compiled library is missing, loading raises.
"""
import ctypes
import os

import torch  # imported before the library so both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libznni.so")

OK = 0
RELU = 1
MAC_REFERENCE = 2
MAC_SINGLE = 4
MAC_BATCH = 8
MAC_XDIRECT = 16
MAC_XBLOCK = 32
KEEP_KERNELS = 64
PASSES_REFERENCE = 128
STAGES = ("kernel_prep", "fwd_z", "fwd_y", "fwd_x", "mac", "inv_x", "inv_y", "inv_z")
EXPORTS = ("znni_version", "znni_status_string", "znni_fft_size", "znni_conv3d_fft_workspace",
           "znni_conv3d_fft", "znni_conv3d_fft_profile", "znni_conv3d_fft_workspace_v", "znni_conv3d_fft_v",
           "znni_conv3d_fft_profile_v", "znni_conv3d_fft_static_v", "znni_conv3d_fft_stage_work_v", "znni_conv3d_fft_sublayers_v", "znni_conv3d_fft_budget_v", "znni_conv3d_direct_workspace_v", "znni_conv3d_direct_v", "znni_conv3d_choose_v", "znni_conv3d_workspace_v", "znni_conv3d_v", "znni_mpf", "znni_maxpool",
           "znni_copy_probe")

_lib = None


class ZnniError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"znni status {status}: {message}")
        self.status = status


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_1606_05688_amd.build` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        i, u, vp, sz = ctypes.c_int, ctypes.c_uint, ctypes.c_void_p, ctypes.c_size_t
        L.znni_version.restype = i
        L.znni_status_string.restype = ctypes.c_char_p
        L.znni_status_string.argtypes = [i]
        L.znni_fft_size.restype = i
        L.znni_fft_size.argtypes = [i]
        L.znni_conv3d_fft_workspace.restype = i
        L.znni_conv3d_fft_workspace.argtypes = [i, i, i, i, i, ctypes.POINTER(sz)]
        L.znni_conv3d_fft.restype = i
        L.znni_conv3d_fft.argtypes = [i, i, i, i, i, vp, vp, vp, vp, u, vp, sz, vp]
        L.znni_conv3d_fft_profile.restype = i
        L.znni_conv3d_fft_profile.argtypes = [i, i, i, i, i, vp, vp, vp, vp, u, vp, sz, vp,
                                              ctypes.POINTER(ctypes.c_float)]
        i3 = ctypes.POINTER(ctypes.c_int)
        L.znni_conv3d_fft_workspace_v.restype = i
        L.znni_conv3d_fft_workspace_v.argtypes = [i, i, i, i3, i3, ctypes.POINTER(sz)]
        L.znni_conv3d_fft_v.restype = i
        L.znni_conv3d_fft_v.argtypes = [i, i, i, i3, i3, vp, vp, vp, vp, u, vp, sz, vp]
        L.znni_conv3d_fft_static_v.restype = i
        L.znni_conv3d_fft_static_v.argtypes = [i, i, i, i3, i3, vp, vp, vp, vp, u, vp]
        L.znni_conv3d_fft_stage_work_v.restype = i
        L.znni_conv3d_fft_stage_work_v.argtypes = [i, i, i, i3, i3, u, ctypes.POINTER(ctypes.c_double),
                                                   ctypes.POINTER(ctypes.c_double)]
        L.znni_conv3d_fft_profile_v.restype = i
        L.znni_conv3d_fft_profile_v.argtypes = [i, i, i, i3, i3, vp, vp, vp, vp, u, vp, sz, vp,
                                                ctypes.POINTER(ctypes.c_float)]
        L.znni_conv3d_fft_sublayers_v.restype = i
        L.znni_conv3d_fft_sublayers_v.argtypes = [i, i, i, i3, i3, sz, i3, ctypes.POINTER(sz)]
        L.znni_conv3d_fft_budget_v.restype = i
        L.znni_conv3d_fft_budget_v.argtypes = [i, i, i, i3, i3, vp, vp, vp, vp, u, vp, sz, vp]
        L.znni_conv3d_direct_workspace_v.restype = i
        L.znni_conv3d_direct_workspace_v.argtypes = [i, i, i, i3, i3, ctypes.POINTER(sz)]
        L.znni_conv3d_direct_v.restype = i
        L.znni_conv3d_direct_v.argtypes = [i, i, i, i3, i3, vp, vp, vp, vp, u, vp, sz, vp]
        L.znni_conv3d_choose_v.restype = i
        L.znni_conv3d_choose_v.argtypes = [i, i, i, i3, i3, i3, ctypes.POINTER(ctypes.c_float)]
        L.znni_conv3d_workspace_v.restype = i
        L.znni_conv3d_workspace_v.argtypes = [i, i, i, i3, i3, ctypes.POINTER(sz)]
        L.znni_conv3d_v.restype = i
        L.znni_conv3d_v.argtypes = [i, i, i, i3, i3, vp, vp, vp, vp, u, vp, sz, vp]
        for fn in (L.znni_mpf, L.znni_maxpool):
            fn.restype = i
            fn.argtypes = [i, i, i3, i3, vp, vp, vp]
        L.znni_copy_probe.restype = i
        L.znni_copy_probe.argtypes = [vp, vp, sz, vp]
        _lib = L
    return _lib


def _check(status):
    if status != OK:
        raise ZnniError(status, lib().znni_status_string(status).decode())


def znni_version():
    return int(lib().znni_version())


def znni_fft_size(n):
    return int(lib().znni_fft_size(int(n)))


def _triple(v):
    """An edge length or a sequence <x, y, z> -> ctypes int[3]."""
    t = (int(v),) * 3 if isinstance(v, int) else tuple(int(e) for e in v)
    assert len(t) == 3, "a size is one edge length or three (x, y, z)"
    return (ctypes.c_int * 3)(*t)


def znni_conv3d_fft_workspace(S, f, fo, n, k):
    """Workspace bytes for a layer; n and k are an edge length (cubic call) or (x, y, z) triples (general call)."""
    b = ctypes.c_size_t(0)
    if isinstance(n, int) and isinstance(k, int):
        _check(lib().znni_conv3d_fft_workspace(int(S), int(f), int(fo), n, k, ctypes.byref(b)))
    else:
        _check(lib().znni_conv3d_fft_workspace_v(int(S), int(f), int(fo), _triple(n), _triple(k), ctypes.byref(b)))
    return int(b.value)


def alloc_workspace(S, f, fo, n, k, device="cuda"):
    """A torch byte tensor large enough for the layer (torch allocations are at least 256-byte aligned)."""
    return torch.empty(znni_conv3d_fft_workspace(S, f, fo, n, k), dtype=torch.uint8, device=device)


def _flags(relu, mac_reference, keep_kernels=False):
    """mac_reference: False/True, or one of the strings 'single' / 'batch' / 'xdirect' / 'xblock' to force a
    multiply-accumulate form, or 'generic_passes' for the diagnostic that runs the generic transform passes."""
    m = {False: 0, None: 0, True: MAC_REFERENCE, "reference": MAC_REFERENCE, "single": MAC_SINGLE,
         "batch": MAC_BATCH, "xdirect": MAC_XDIRECT, "xblock": MAC_XBLOCK,
         "generic_passes": PASSES_REFERENCE}[mac_reference]
    return (RELU if relu else 0) | m | (KEEP_KERNELS if keep_kernels else 0)


def _marshal(inp, w, bias, out, workspace):
    assert inp.is_cuda and inp.dtype == torch.float32 and inp.is_contiguous() and inp.dim() == 5
    assert w.is_cuda and w.dtype == torch.float32 and w.is_contiguous() and w.dim() == 5
    S, f = inp.shape[0], inp.shape[1]
    n = tuple(int(e) for e in inp.shape[2:])
    fo = w.shape[0]
    k = tuple(int(e) for e in w.shape[2:])
    assert w.shape[1] == f, "kernel bank must be [f', f, kx, ky, kz]"
    oshape = (S, fo) + tuple(a - b + 1 for a, b in zip(n, k))
    if bias is not None:
        assert bias.is_cuda and bias.dtype == torch.float32 and bias.is_contiguous() and bias.shape == (fo,)
    if out is None:
        out = torch.empty([max(e, 0) for e in oshape], dtype=torch.float32, device=inp.device)
    else:
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        assert tuple(out.shape) == oshape
    if workspace is None:
        workspace = alloc_workspace(S, f, fo, n, k, inp.device)
    assert workspace.is_cuda and workspace.dtype == torch.uint8 and workspace.is_contiguous()
    return S, f, fo, n, k, out, workspace


def _cubic(n, k):
    return n[0] == n[1] == n[2] and k[0] == k[1] == k[2]


def znni_conv3d_fft(inp, w, bias=None, relu=False, out=None, workspace=None, stream=None,
                    mac_reference=False, keep_kernels=False):
    """out[S,f',n-k+1 per axis] = act(bias + valid 3D convolution of inp[S,f,nx,ny,nz] with w[f',f,kx,ky,kz]).

    Cubic shapes go through znni_conv3d_fft, all others through znni_conv3d_fft_v.
    Asynchronous on `stream` (a torch.cuda.Stream; default: torch's current stream).
    keep_kernels: the workspace (which must then be passed) still holds this w's stored transforms."""
    assert not keep_kernels or workspace is not None
    S, f, fo, n, k, out, workspace = _marshal(inp, w, bias, out, workspace)
    st = stream if stream is not None else torch.cuda.current_stream(inp.device)
    tail = (inp.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None, out.data_ptr(),
            _flags(relu, mac_reference, keep_kernels), workspace.data_ptr(), workspace.numel(), st.cuda_stream)
    if _cubic(n, k):
        _check(lib().znni_conv3d_fft(S, f, fo, n[0], k[0], *tail))
    else:
        _check(lib().znni_conv3d_fft_v(S, f, fo, _triple(n), _triple(k), *tail))
    return out


STATIC_SCRATCH_BYTES = 64 << 20


def znni_conv3d_fft_static(inp, w, bias=None, relu=False, out=None, stream=None, mac_reference=False):
    """znni_conv3d_fft on the library's own fixed scratch array instead of a caller's workspace (`out` should be
    passed by callers that must not allocate; without it torch allocates the result)."""
    S, f, fo, n, k, out, _ = _marshal(inp, w, bias, out, inp.new_empty(0, dtype=torch.uint8))
    st = stream if stream is not None else torch.cuda.current_stream(inp.device)
    _check(lib().znni_conv3d_fft_static_v(S, f, fo, _triple(n), _triple(k), inp.data_ptr(), w.data_ptr(),
                                          bias.data_ptr() if bias is not None else None, out.data_ptr(),
                                          _flags(relu, mac_reference), st.cuda_stream))
    return out


def znni_conv3d_fft_profile(inp, w, bias=None, relu=False, out=None, workspace=None, stream=None,
                            mac_reference=False, keep_kernels=False):
    """Same call with per-stage HIP-event timing; returns (out, {stage: milliseconds}).  Synchronises."""
    S, f, fo, n, k, out, workspace = _marshal(inp, w, bias, out, workspace)
    st = stream if stream is not None else torch.cuda.current_stream(inp.device)
    ms = (ctypes.c_float * len(STAGES))()
    tail = (inp.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None, out.data_ptr(),
            _flags(relu, mac_reference, keep_kernels), workspace.data_ptr(), workspace.numel(), st.cuda_stream, ms)
    if _cubic(n, k):
        _check(lib().znni_conv3d_fft_profile(S, f, fo, n[0], k[0], *tail))
    else:
        _check(lib().znni_conv3d_fft_profile_v(S, f, fo, _triple(n), _triple(k), *tail))
    return out, {name: float(ms[i]) for i, name in enumerate(STAGES)}


def znni_conv3d_fft_stage_work(S, f, fo, n, k, relu=False, mac_reference=False):
    """({stage: bytes the stage must move}, {stage: flops of its contraction}) for the kernels a call would run."""
    nb = (ctypes.c_double * len(STAGES))()
    fl = (ctypes.c_double * len(STAGES))()
    _check(lib().znni_conv3d_fft_stage_work_v(int(S), int(f), int(fo), _triple(n), _triple(k),
                                              _flags(relu, mac_reference), nb, fl))
    return ({name: float(nb[q]) for q, name in enumerate(STAGES)},
            {name: float(fl[q]) for q, name in enumerate(STAGES)})


def znni_conv3d_fft_sublayers(S, f, fo, n, k, budget_bytes):
    """Division of a layer for a workspace budget: ((S_i, f_i, f'_i), workspace bytes needed)."""
    sub = (ctypes.c_int * 3)()
    b = ctypes.c_size_t(0)
    _check(lib().znni_conv3d_fft_sublayers_v(int(S), int(f), int(fo), _triple(n), _triple(k), int(budget_bytes),
                                             sub, ctypes.byref(b)))
    return tuple(sub), int(b.value)


def znni_conv3d_fft_budget(inp, w, bias=None, relu=False, out=None, workspace=None, stream=None,
                           mac_reference=False):
    """The layer computed as sub-layers that fit `workspace` (a torch uint8 CUDA tensor, required)."""
    assert workspace is not None, "the workspace is the budget"
    S, f, fo, n, k, out, workspace = _marshal(inp, w, bias, out, workspace)
    st = stream if stream is not None else torch.cuda.current_stream(inp.device)
    _check(lib().znni_conv3d_fft_budget_v(S, f, fo, _triple(n), _triple(k), inp.data_ptr(), w.data_ptr(),
                                          bias.data_ptr() if bias is not None else None, out.data_ptr(),
                                          _flags(relu, mac_reference), workspace.data_ptr(), workspace.numel(),
                                          st.cuda_stream))
    return out


def znni_conv3d_direct_workspace(S, f, fo, n, k):
    b = ctypes.c_size_t(0)
    _check(lib().znni_conv3d_direct_workspace_v(int(S), int(f), int(fo), _triple(n), _triple(k), ctypes.byref(b)))
    return int(b.value)


def znni_conv3d_direct(inp, w, bias=None, relu=False, out=None, workspace=None, stream=None):
    """The layer by direct convolution on the matrix cores (same tensors and result as znni_conv3d_fft)."""
    assert inp.is_cuda and inp.dtype == torch.float32 and inp.is_contiguous() and inp.dim() == 5
    S, f = inp.shape[0], inp.shape[1]
    if workspace is None:
        workspace = torch.empty(znni_conv3d_direct_workspace(S, f, w.shape[0], tuple(inp.shape[2:]), tuple(w.shape[2:])),
                                dtype=torch.uint8, device=inp.device)
    S, f, fo, n, k, out, workspace = _marshal(inp, w, bias, out, workspace)
    st = stream if stream is not None else torch.cuda.current_stream(inp.device)
    _check(lib().znni_conv3d_direct_v(S, f, fo, _triple(n), _triple(k), inp.data_ptr(), w.data_ptr(),
                                      bias.data_ptr() if bias is not None else None, out.data_ptr(),
                                      RELU if relu else 0, workspace.data_ptr(), workspace.numel(), st.cuda_stream))
    return out


PRIMITIVES = ("fft", "direct")


def znni_conv3d_choose(S, f, fo, n, k):
    """(name of the primitive picked for this layer shape, {name: estimated milliseconds})."""
    prim = ctypes.c_int(0)
    est = (ctypes.c_float * 2)()
    _check(lib().znni_conv3d_choose_v(int(S), int(f), int(fo), _triple(n), _triple(k), ctypes.byref(prim), est))
    return PRIMITIVES[prim.value], {name: float(est[q]) for q, name in enumerate(PRIMITIVES)}


def znni_conv3d(inp, w, bias=None, relu=False, out=None, stream=None):
    """The layer by whichever primitive the library picks for its shape."""
    assert inp.is_cuda and inp.dtype == torch.float32 and inp.is_contiguous() and inp.dim() == 5
    assert w.is_cuda and w.dtype == torch.float32 and w.is_contiguous() and w.dim() == 5
    S, f, fo = inp.shape[0], inp.shape[1], w.shape[0]
    n, k = tuple(inp.shape[2:]), tuple(w.shape[2:])
    b = ctypes.c_size_t(0)
    _check(lib().znni_conv3d_workspace_v(S, f, fo, _triple(n), _triple(k), ctypes.byref(b)))
    ws = torch.empty(int(b.value), dtype=torch.uint8, device=inp.device)
    S, f, fo, n, k, out, ws = _marshal(inp, w, bias, out, ws)
    st = stream if stream is not None else torch.cuda.current_stream(inp.device)
    _check(lib().znni_conv3d_v(S, f, fo, _triple(n), _triple(k), inp.data_ptr(), w.data_ptr(),
                               bias.data_ptr() if bias is not None else None, out.data_ptr(),
                               RELU if relu else 0, ws.data_ptr(), ws.numel(), st.cuda_stream))
    return out


def _pool(fn, inp, p, oshape, out, stream):
    assert inp.is_cuda and inp.dtype == torch.float32 and inp.is_contiguous() and inp.dim() == 5
    S, f = inp.shape[0], inp.shape[1]
    n = tuple(int(e) for e in inp.shape[2:])
    p = tuple(int(e) for e in _triple(p))
    shape = oshape(S, f, n, p)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=inp.device)
    else:
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == shape
    st = stream if stream is not None else torch.cuda.current_stream(inp.device)
    _check(fn(S, f, _triple(n), _triple(p), inp.data_ptr(), out.data_ptr(), st.cuda_stream))
    return out


def znni_mpf(inp, p, out=None, stream=None):
    """Max-pooling fragments with window p (edge or (px,py,pz)): [S,f,nx,ny,nz] -> [S*px*py*pz, f, n//p ...]."""
    return _pool(lib().znni_mpf, inp, p,
                 lambda S, f, n, p: (S * p[0] * p[1] * p[2], f) + tuple(max(a // max(b, 1), 0) for a, b in zip(n, p)),
                 out, stream)


def znni_maxpool(inp, p, out=None, stream=None):
    """Max pooling with window p: [S,f,nx,ny,nz] -> [S, f, nx/px, ny/py, nz/pz]."""
    return _pool(lib().znni_maxpool, inp, p,
                 lambda S, f, n, p: (S, f) + tuple(max(a // max(b, 1), 0) for a, b in zip(n, p)), out, stream)


def znni_copy_probe(dst, src, stream=None):
    """Plain device copy src -> dst (same-size contiguous CUDA tensors); used to calibrate traffic counters."""
    assert dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    st = stream if stream is not None else torch.cuda.current_stream(src.device)
    _check(lib().znni_copy_probe(dst.data_ptr(), src.data_ptr(), nbytes, st.cuda_stream))
    return dst
