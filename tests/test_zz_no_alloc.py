"""The entry point that allocates nothing (znni_conv3d_fft_static_v: the library's own fixed scratch array instead
of a caller's workspace) against the ordinary entry point, through the C ABI."""
import ctypes
import sys

import numpy as np
import pytest
import torch

from paper_1606_05688_amd import binding as B

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _inputs(seed, S, f, fo, n, k, d):
    r = np.random.default_rng(seed)
    inp = r.uniform(-1, 1, (S, f) + tuple(n)).astype(np.float32)
    w = (r.standard_normal((fo, f) + tuple(k)) * (f * k[0] * k[1] * k[2]) ** -0.5).astype(np.float32)
    b = (r.standard_normal(fo) * np.sqrt(0.1)).astype(np.float32)
    return inp, w, b, tuple(torch.from_numpy(t).to(d) for t in (inp, w, b))


def test_static_scratch_entry_point_matches_workspace_entry_point(oracle):
    """Two calls in a row, the second on a smaller layer (the array still holds the first call's spectra), then a
    call on a side stream; each must equal the workspace entry point bit for bit (same kernels, same order) and meet
    the oracle bar."""
    d = torch.device("cuda:0")
    L = B.lib()
    i3 = lambda v: (ctypes.c_int * 3)(*v)
    cases = [(1, 8, 8, (64, 64, 64), (5, 5, 5)),        # the second benchmark layer: 27 MB of scratch
             (2, 3, 4, (20, 18, 33), (3, 2, 4)),        # smaller, anisotropic, padded transform sizes
             (3, 2, 2, (12, 12, 12), (3, 3, 3))]
    side = torch.cuda.Stream(device=d)
    for idx, (S, f, fo, n, k) in enumerate(cases):
        need = B.znni_conv3d_fft_workspace(S, f, fo, n, k)
        assert need <= B.STATIC_SCRATCH_BYTES
        inp, w, b, (ti, tw, tb) = _inputs(70 + idx, S, f, fo, n, k, d)
        oshape = (S, fo) + tuple(a - c + 1 for a, c in zip(n, k))
        ref_out = B.znni_conv3d_fft(ti, tw, tb, relu=True)
        got = torch.full(oshape, float("nan"), device=d)
        torch.cuda.synchronize()
        st = side if idx == 2 else torch.cuda.current_stream(d)
        _say(f"[no-alloc] call {idx}: {(S, f, fo, n, k)}, needs {need} of {B.STATIC_SCRATCH_BYTES} bytes")
        rc = L.znni_conv3d_fft_static_v(S, f, fo, i3(n), i3(k), ti.data_ptr(), tw.data_ptr(), tb.data_ptr(),
                                        got.data_ptr(), B.RELU, st.cuda_stream)
        assert rc == 0, B.lib().znni_status_string(rc)
        torch.cuda.synchronize()
        assert torch.equal(got, ref_out)
        exp = oracle.conv3d(inp, w, b, relu=True)
        tol = oracle.tolerance(inp, w)[None, :, None, None, None]
        assert np.all(np.abs(got.cpu().numpy() - exp) <= tol)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    d = torch.device("cuda:0")
    S, f, fo, n, k = 1, 40, 40, 128, 3
    assert B.znni_conv3d_fft_workspace(S, f, fo, n, k) > B.STATIC_SCRATCH_BYTES
    inp = torch.zeros((S, f, n, n, n), device=d)
    w = torch.zeros((fo, f, k, k, k), device=d)
    with pytest.raises(B.ZnniError) as e:
        B.znni_conv3d_fft_static(inp, w)
    assert e.value.status == -4
    # argument errors come before anything else, as for the workspace entry point
    L = B.lib()
    i3 = lambda v: (ctypes.c_int * 3)(*v)
    p = inp.data_ptr()
    assert L.znni_conv3d_fft_static_v(1, 1, 1, i3((8, 8, 8)), i3((3, 3, 3)), None, p, None, p, 0, None) == -1
    assert L.znni_conv3d_fft_static_v(1, 1, 1, i3((8, 8, 8)), i3((9, 3, 3)), p, p, None, p, 0, None) == -2
    assert L.znni_conv3d_fft_static_v(1, 1, 1, i3((8, 8, 8)), i3((3, 3, 3)), p, p, None, p, 256, None) == -5
    assert L.znni_conv3d_fft_static_v(1, 1, 1, i3((8, 8, 8)), i3((3, 3, 3)), p, p + 4, None, p, 0, None) == -7
