"""Host-side checks of the C-ABI library: it loads, exports what include/znni.h declares, sizes its workspace
sensibly, and turns every argument error into a status code before touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_1606_05688_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "znni.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(znni_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS)
    for name in names:
        assert hasattr(L, name), f"{name} is declared in include/znni.h but not exported"
    assert B.znni_version() >= 100


def test_status_strings():
    L = B.lib()
    seen = set()
    for st in range(0, -8, -1):
        s = L.znni_status_string(st)
        assert s and s not in seen
        seen.add(s)
    assert L.znni_status_string(-99) == b"unknown status"


def test_fft_size_is_the_nearest_in_register_length():
    def smooth(m):
        for p in (2, 3, 5, 7):
            while m % p == 0:
                m //= p
        return m == 1
    sizes = set()
    for n in range(1, 1025):
        m = B.znni_fft_size(n)
        assert smooth(m) and n <= m <= 1024 and 5 * m <= 6 * n + 5      # at most 20 % above n (rounded)
        assert B.znni_fft_size(m) == m                                   # a size maps to itself
        if n > 1:
            assert m >= B.znni_fft_size(n - 1)                           # monotone
        sizes.add(m)
    assert len([m for m in sizes if m >= 8]) == 46 and {1, 2, 3, 4, 5, 6} <= sizes and 7 not in sizes
    assert B.znni_fft_size(125) == 128 and B.znni_fft_size(126) == 128 and B.znni_fft_size(243) == 256
    assert B.znni_fft_size(17) == 20 and B.znni_fft_size(21) == 24 and B.znni_fft_size(7) == 8
    assert B.znni_fft_size(81) == 84 and B.znni_fft_size(162) == 168 and B.znni_fft_size(324) == 336
    assert B.znni_fft_size(540) == 576 and B.znni_fft_size(700) == 720 and B.znni_fft_size(1000) == 1024
    for n in (16, 64, 128, 320):
        assert B.znni_fft_size(n) == n          # the benchmark layers transform at their own size
    assert B.znni_fft_size(0) == 0 and B.znni_fft_size(-3) == 0 and B.znni_fft_size(1025) == 0


def test_workspace_holds_both_spectra_and_partial_kernel_transforms():
    for (S, f, fo, n, k) in [(1, 2, 3, 16, 3), (1, 8, 8, 64, 5), (8, 32, 32, 64, 7), (1, 48, 48, 320, 5)]:
        N = B.znni_fft_size(n)
        zc = N // 2 + 1
        fp, Mp = (f + 3) // 4 * 4, (fo + 15) // 16 * 16     # kernel transforms are stored padded to matrix-core tiles
        # ... with k values per kernel column along x, or 8 (and input images in groups of 8) where the route that
        # transforms x in blocks of eight exists: the workspace does not depend on the flags of a call
        blocks = k in (4, 5) and f >= 16
        need = 8 * zc * N * N * S * (f + fo) + 8 * zc * N * Mp * ((f + 7) // 8 * 8 * 8 if blocks else fp * k)
        got = B.znni_conv3d_fft_workspace(S, f, fo, n, k)
        assert need <= got <= 1.1 * need + (1 << 20)
    # the largest benchmark layer: far below the 304 GB a stored kernel-spectrum bank would take
    assert B.znni_conv3d_fft_workspace(1, 48, 48, 320, 5) < 21e9


@pytest.mark.parametrize("args,status", [
    ((0, 1, 1, 8, 3), -2), ((1, 0, 1, 8, 3), -2), ((1, 1, 0, 8, 3), -2), ((1, 1, 1, 8, 0), -2),
    ((1, 1, 1, 8, 9), -2), ((1, 1, 1, 0, 1), -2), ((70000, 1, 1, 8, 3), -2), ((1, 1, 1, 1025, 3), -3),
])
def test_workspace_query_rejects_bad_shapes(args, status):
    b = ctypes.c_size_t(0)
    assert B.lib().znni_conv3d_fft_workspace(*args, ctypes.byref(b)) == status
    assert B.lib().znni_conv3d_fft_workspace(1, 1, 1, 8, 3, None) == -1


def test_layer_call_validates_before_any_gpu_work():
    """Fake (never dereferenced) device addresses: each call must fail in validation."""
    L = B.lib()
    p, ws = 0x1000, 0x100000
    big = 1 << 40

    def call(S=1, f=1, fo=1, n=8, k=3, inp=p, w=p, bias=None, out=p, flags=0, wsp=ws, wsb=big):
        return L.znni_conv3d_fft(S, f, fo, n, k, inp, w, bias, out, flags, wsp, wsb, None)
    assert call(inp=None) == -1 and call(w=None) == -1 and call(out=None) == -1 and call(wsp=None) == -1
    assert call(k=9) == -2 and call(S=0) == -2
    assert call(n=1025, k=1) == -3
    assert call(flags=256) == -5 and call(flags=0x80000001) == -5
    assert call(flags=64 | 1, wsb=1024) == -4                 # keeping stored kernel transforms is a known flag
    # at most one of the three bits that pick a multiply-accumulate form
    assert call(flags=2 | 4) == -5 and call(flags=4 | 8) == -5 and call(flags=1 | 2 | 8) == -5 and call(flags=8 | 16) == -5 and call(flags=16 | 32) == -5
    assert call(flags=1 | 4, wsb=1024) == -4 and call(flags=8, wsb=1024) == -4     # one of them: validation goes on
    assert call(inp=p + 4) == -7 and call(out=p + 8) == -7 and call(wsp=ws + 128) == -7
    assert call(wsb=1024) == -4
    need = B.znni_conv3d_fft_workspace(1, 1, 1, 8, 3)
    assert call(wsb=need - 1) == -4
    ms = (ctypes.c_float * 8)()
    assert L.znni_conv3d_fft_profile(1, 1, 1, 8, 9, p, p, None, p, 0, ws, big, None, ms) == -2
    assert L.znni_conv3d_fft_profile(1, 1, 1, 8, 3, p, p, None, p, 0, ws, big, None, None) == -1
    assert L.znni_copy_probe(None, p, 64, None) == -1 and L.znni_copy_probe(p, p, 0, None) == -2
    assert L.znni_copy_probe(p, p, 24, None) == -2 and L.znni_copy_probe(p + 8, p, 64, None) == -7


def _i3(*v):
    return (ctypes.c_int * 3)(*v)


def test_general_shape_calls_validate_per_axis():
    L = B.lib()
    b = ctypes.c_size_t(0)
    q = lambda n, k: L.znni_conv3d_fft_workspace_v(1, 2, 2, _i3(*n), _i3(*k), ctypes.byref(b))
    assert q((8, 9, 10), (3, 2, 1)) == 0 and b.value > 0
    assert q((8, 9, 10), (9, 2, 1)) == -2 and q((8, 9, 10), (3, 10, 1)) == -2 and q((8, 9, 10), (3, 2, 11)) == -2
    assert q((8, 9, 0), (3, 2, 1)) == -2 and q((8, 9, 10), (3, 0, 1)) == -2
    assert q((8, 1025, 10), (3, 2, 1)) == -3
    assert L.znni_conv3d_fft_workspace_v(1, 2, 2, None, _i3(1, 1, 1), ctypes.byref(b)) == -1
    assert L.znni_conv3d_fft_workspace_v(1, 2, 2, _i3(8, 8, 8), None, ctypes.byref(b)) == -1
    p, ws, big = 0x1000, 0x100000, 1 << 40
    assert L.znni_conv3d_fft_v(1, 1, 1, _i3(8, 6, 4), _i3(3, 7, 1), p, p, None, p, 0, ws, big, None) == -2
    assert L.znni_conv3d_fft_v(1, 1, 1, None, _i3(3, 3, 1), p, p, None, p, 0, ws, big, None) == -1
    assert L.znni_conv3d_fft_v(1, 1, 1, _i3(8, 6, 4), _i3(3, 3, 1), p, p, None, p, 0, ws, 64, None) == -4
    ms = (ctypes.c_float * 8)()
    assert L.znni_conv3d_fft_profile_v(1, 1, 1, _i3(8, 6, 4), _i3(3, 3, 5), p, p, None, p, 0, ws, big, None, ms) == -2


def test_cubic_calls_are_the_general_calls_with_equal_axes():
    for (S, f, fo, n, k) in [(1, 2, 3, 16, 3), (2, 5, 7, 33, 4)]:
        assert B.znni_conv3d_fft_workspace(S, f, fo, n, k) == B.znni_conv3d_fft_workspace(S, f, fo, (n, n, n), (k, k, k))
    # the workspace follows the per-axis transform sizes: doubling one image axis grows it by 1.5x to 2x
    # (the stored kernel transforms do not grow with the x axis, the halved axis has Nz/2+1 bins)
    a = B.znni_conv3d_fft_workspace(1, 4, 4, (32, 32, 32), (3, 3, 3))
    for n in [(64, 32, 32), (32, 64, 32), (32, 32, 64)]:
        assert 1.5 * a < B.znni_conv3d_fft_workspace(1, 4, 4, n, (3, 3, 3)) < 2.1 * a


def test_pooling_calls_validate_before_any_gpu_work():
    L = B.lib()
    p = 0x1000
    for fn in (L.znni_mpf, L.znni_maxpool):
        assert fn(1, 1, None, _i3(2, 2, 2), p, p, None) == -1
        assert fn(1, 1, _i3(7, 7, 7), None, p, p, None) == -1
        assert fn(0, 1, _i3(8, 8, 8), _i3(1, 1, 1), p, p, None) == -2
        assert fn(1, 1, _i3(8, 8, 8), _i3(1, 0, 1), p, p, None) == -2
        assert fn(1, 1, _i3(8, 2, 8), _i3(1, 3, 1), p, p, None) == -2          # window larger than the image
        assert fn(1, 1, _i3(8, 8, 8), _i3(1, 1, 1), None, p, None) == -1
        assert fn(1, 1, _i3(8, 8, 8), _i3(1, 1, 1), p, p + 2, None) == -7
    # fragments need n + 1 divisible by p (where p > 1), plain pooling needs n divisible by p
    assert L.znni_mpf(1, 1, _i3(8, 7, 7), _i3(2, 2, 2), p, p, None) == -2
    assert L.znni_mpf(1, 1, _i3(9, 9, 9), _i3(5, 1, 1), p, p, None) == -3      # window above the supported 4
    assert L.znni_maxpool(1, 1, _i3(8, 7, 8), _i3(2, 2, 2), p, p, None) == -2


def test_sublayer_division_follows_the_stated_preference():
    S, f, fo, n, k = 8, 32, 32, (64, 64, 64), (7, 7, 7)
    full = B.znni_conv3d_fft_workspace(S, f, fo, n, k)
    assert B.znni_conv3d_fft_sublayers(S, f, fo, n, k, full) == ((S, f, fo), full)
    assert B.znni_conv3d_fft_sublayers(S, f, fo, n, k, 10 * full) == ((S, f, fo), full)
    prev = None
    one = B.znni_conv3d_fft_workspace(1, f, fo, n, k)
    for frac in (0.9, 0.6, 0.4, one / full):        # sub-batches while at least one whole input fits
        sub, need = B.znni_conv3d_fft_sublayers(S, f, fo, n, k, int(frac * full) + 1)
        assert sub[1:] == (f, fo) and 1 <= sub[0] < S and need <= frac * full + 1
        assert prev is None or sub[0] <= prev
        prev = sub[0]
        # one more input per sub-batch would not fit
        L = B.lib()
        sub3 = (ctypes.c_int * 3)()
        b = ctypes.c_size_t(0)
        assert B.znni_conv3d_fft_workspace(sub[0] + 1, f, fo, n, k) > frac * full + 1
    sub, need = B.znni_conv3d_fft_sublayers(S, f, fo, n, k, one - 1)
    assert sub[0] == 1 and (sub[1] < f or sub[2] < fo) and need <= one - 1
    # smallest division; below it the query fails and reports what that division needs
    L = B.lib()
    sub3 = (ctypes.c_int * 3)()
    b = ctypes.c_size_t(0)
    assert L.znni_conv3d_fft_sublayers_v(S, f, fo, _i3(*n), _i3(*k), 1024, sub3, ctypes.byref(b)) == -4
    floor = b.value
    assert 0 < floor < one
    assert B.znni_conv3d_fft_sublayers(S, f, fo, n, k, floor)[0] == (1, 1, 1)
    assert L.znni_conv3d_fft_sublayers_v(S, f, fo, _i3(*n), _i3(*k), floor - 1, sub3, ctypes.byref(b)) == -4
    assert L.znni_conv3d_fft_sublayers_v(S, f, fo, _i3(*n), _i3(*k), full, None, ctypes.byref(b)) == -1
    assert L.znni_conv3d_fft_sublayers_v(S, 0, fo, _i3(*n), _i3(*k), full, sub3, ctypes.byref(b)) == -2
    p = 0x1000
    assert L.znni_conv3d_fft_budget_v(S, f, fo, _i3(*n), _i3(*k), p, p, None, p, 0, 0x100000, 1024, None) == -4
    assert L.znni_conv3d_fft_budget_v(S, f, fo, _i3(*n), _i3(*k), None, p, None, p, 0, 0x100000, full, None) == -1
    assert L.znni_conv3d_fft_budget_v(S, f, fo, _i3(*n), _i3(*k), p, p, None, p, 64, 0x100000, full, None) == -5            # no kernels kept across sub-layers
    assert L.znni_conv3d_fft_budget_v(S, f, fo, _i3(*n), _i3(*k), p, p, None, p, 4 | 8, 0x100000, full, None) == -5


def test_primitive_choice_follows_kernel_size_and_image_count():
    # first layers (one or a few input images) and narrow layers with 2^3 kernels go direct; large kernels and wide
    # layers go through transforms
    assert B.znni_conv3d_choose(1, 1, 48, 128, 3)[0] == "direct"
    assert B.znni_conv3d_choose(1, 8, 80, 200, 2)[0] == "direct"
    assert B.znni_conv3d_choose(1, 16, 16, 128, 2)[0] == "direct"
    assert B.znni_conv3d_choose(1, 48, 48, 320, 5)[0] == "fft"
    assert B.znni_conv3d_choose(8, 32, 32, 64, 7)[0] == "fft"
    assert B.znni_conv3d_choose(1, 40, 40, 128, 3)[0] == "fft"
    # a kernel the direct primitive cannot stage leaves only the transform route, and the estimate says so
    prim, est = B.znni_conv3d_choose(1, 4, 4, 40, 9)
    assert prim == "fft" and est["direct"] < 0 < est["fft"]
    # estimates grow with the work
    assert B.znni_conv3d_choose(1, 8, 8, 64, 3)[1]["direct"] < B.znni_conv3d_choose(1, 8, 8, 64, 5)[1]["direct"]
    assert B.znni_conv3d_choose(1, 8, 8, 64, 3)[1]["fft"] < B.znni_conv3d_choose(1, 8, 8, 128, 3)[1]["fft"]
    L = B.lib()
    prim = ctypes.c_int(0)
    assert L.znni_conv3d_choose_v(1, 1, 1, _i3(8, 8, 8), _i3(3, 3, 3), None, None) == -1
    assert L.znni_conv3d_choose_v(1, 1, 1, _i3(8, 8, 8), _i3(9, 3, 3), ctypes.byref(prim), None) == -2
    b = ctypes.c_size_t(0)
    assert L.znni_conv3d_workspace_v(1, 1, 48, _i3(128, 128, 128), _i3(3, 3, 3), ctypes.byref(b)) == 0
    assert b.value == B.znni_conv3d_direct_workspace(1, 1, 48, 128, 3)
    assert L.znni_conv3d_workspace_v(1, 48, 48, _i3(64, 64, 64), _i3(5, 5, 5), ctypes.byref(b)) == 0
    assert b.value == B.znni_conv3d_fft_workspace(1, 48, 48, 64, 5)
    p = 0x1000
    assert L.znni_conv3d_v(1, 1, 48, _i3(128, 128, 128), _i3(3, 3, 3), p, p, None, p, 2, 0x100000, 1 << 40, None) == -5
    assert L.znni_conv3d_v(1, 1, 48, _i3(128, 128, 128), _i3(3, 3, 3), p, p, None, p, 0, 0x100000, 16, None) == -4
    # the form hints of the transform route do not change what a call does when the direct route is picked: they
    # pass validation (the call goes on to the workspace check) unless both are given
    for hint in (4, 8, 1 | 4, 16, 32, 64, 128, 64 | 128 | 8):
        assert L.znni_conv3d_v(1, 1, 48, _i3(128, 128, 128), _i3(3, 3, 3), p, p, None, p, hint, 0x100000, 16, None) == -4
    assert L.znni_conv3d_v(1, 1, 48, _i3(128, 128, 128), _i3(3, 3, 3), p, p, None, p, 4 | 8, 0x100000, 16, None) == -5
    assert L.znni_conv3d_v(1, 1, 48, _i3(128, 128, 128), _i3(3, 3, 3), p, p, None, p, 16 | 32, 0x100000, 16, None) == -5
    assert L.znni_conv3d_v(1, 1, 48, _i3(128, 128, 128), _i3(3, 3, 3), p, p, None, p, 256, 0x100000, 16, None) == -5
    assert L.znni_conv3d_direct_v(1, 1, 1, _i3(8, 8, 8), _i3(3, 3, 3), None, p, None, p, 0, 0x100000, 1 << 20, None) == -1
    assert L.znni_conv3d_direct_v(1, 1, 1, _i3(8, 8, 8), _i3(3, 3, 3), p, p, None, p, 2, 0x100000, 1 << 20, None) == -5
    assert L.znni_conv3d_direct_v(1, 1, 1, _i3(8, 8, 8), _i3(3, 3, 3), p, p, None, p + 1, 0, 0x100000, 1 << 20, None) == -7
    assert L.znni_conv3d_direct_v(1, 1, 1, _i3(8, 8, 8), _i3(3, 3, 3), p, p, None, p, 0, 0x100000, 8, None) == -4


def test_stage_work_follows_the_kernels_a_call_would_run():
    S, f, fo, n, k = 1, 48, 48, 320, 5
    zc, no = n // 2 + 1, n - k + 1
    img = 8 * zc * n * n                                     # one transformed image, bytes
    nb, fl = B.znni_conv3d_fft_stage_work(S, f, fo, n, k, mac_reference="single")
    assert nb["fwd_z"] == f * (4 * n ** 3 + img) and nb["fwd_y"] == f * 2 * img and nb["fwd_x"] == f * 2 * img
    assert nb["inv_x"] == fo * (img + 8 * zc * no * n) and nb["inv_z"] == fo * (8 * no * no * zc + 4 * no ** 3)
    assert nb["kernel_prep"] == 4 * f * fo * k ** 3 + 8 * zc * n * f * fo * k
    assert fl["mac"] == (8 * S + 8 * (k - 1)) * f * fo * zc * n * n and sum(fl.values()) == fl["mac"]
    # the same layer without transforming the x axis: no x stages, multiply-accumulate on n' of n columns
    nb, fl = B.znni_conv3d_fft_stage_work(S, f, fo, n, k, mac_reference="xdirect")
    assert nb["fwd_x"] == 0 and nb["inv_x"] == 0 and nb["fwd_y"] == f * 2 * img
    assert nb["inv_y"] == fo * (8 * zc * no * n + 8 * no * no * zc)
    assert fl["mac"] == 8 * k * S * f * fo * zc * n * no
    # ... or with the x axis transformed in blocks of eight, four outputs each: 8 stored values per kernel column and
    # 8 multiply-adds per block, image and kernel; kept kernel transforms cost nothing
    nb, fl = B.znni_conv3d_fft_stage_work(S, f, fo, n, k, mac_reference="xblock")
    assert nb["fwd_x"] == 0 and nb["kernel_prep"] == 4 * f * fo * k ** 3 + 8 * zc * n * f * fo * 8
    assert fl["mac"] == 8 * 8 * S * f * fo * zc * n * (no // 4)
    assert nb["mac"] == f * img + 8 * zc * n * f * fo * 8 + fo * 8 * zc * no * n
    assert B.lib().znni_conv3d_fft_stage_work_v is not None
    # small images: one kernel per side does the z and y transforms, and its stage carries the bytes of both
    nb, _ = B.znni_conv3d_fft_stage_work(8, 32, 32, 64, 7)
    assert nb["fwd_y"] == 0 and nb["inv_z"] == 0
    assert nb["fwd_z"] == 8 * 32 * (4 * 64 ** 3 + 8 * 33 * 64 * 64)
    assert nb["inv_y"] == 8 * 32 * (8 * 33 * 58 * 64 + 4 * 58 ** 3)
    L = B.lib()
    arr = (ctypes.c_double * 8)()
    assert L.znni_conv3d_fft_stage_work_v(1, 1, 1, _i3(8, 8, 8), _i3(3, 3, 3), 0, None, arr) == -1
    assert L.znni_conv3d_fft_stage_work_v(1, 1, 1, _i3(8, 8, 8), _i3(9, 3, 3), 0, arr, arr) == -2
    assert L.znni_conv3d_fft_stage_work_v(1, 1, 1, _i3(8, 8, 8), _i3(3, 3, 3), 256, arr, arr) == -5
