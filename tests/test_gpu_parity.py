"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle on the same seeded inputs.

Bar (per output voxel of output image j):  |gpu - oracle| <= 1e-4 * max|x| * sum_{i,a,b,c} |w[j,i,a,b,c]|.
Four of the five benchmark layers and every smaller layer are compared element by element; the largest benchmark
layer, too large for a full direct convolution on the host, is compared on a declared sample of voxels (all
corner blocks and face-centre patches of every output image, the mid-planes of one image, 2^20 uniformly random
positions), each computed by the oracle one voxel at a time.
"""
import sys

import numpy as np
import pytest
import torch

from paper_1606_05688_amd import binding as B
from paper_1606_05688_amd import workloads as W

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _run_gpu(inp, w, bias, relu, **kw):
    d = torch.device("cuda:0")
    ti = torch.from_numpy(inp).to(d)
    tw = torch.from_numpy(w).to(d)
    tb = torch.from_numpy(bias).to(d) if bias is not None else None
    out = B.znni_conv3d_fft(ti, tw, tb, relu=relu, **kw)
    torch.cuda.synchronize()
    return out


# The library's own pick of the multiply-accumulate form, then each route forced: x axis transformed (kernel
# spectrum folded into the contraction), x axis not transformed, x axis transformed in overlapping blocks of eight
# (up to 5 taps along x; the flag is ignored elsewhere).  Every layer shape below runs through all sets of kernels.
ROUTES = (False, "single", "xdirect", "xblock")


def _check_full(oracle, inp, w, bias, relu, label, routes=ROUTES):
    _say(f"[parity/full] {label} inp={inp.shape} w={w.shape} relu={relu} bias={'yes' if bias is not None else 'no'}")
    exp = oracle.conv3d(inp, w, bias, relu=relu)
    tol = oracle.tolerance(inp, w)
    for route in routes:
        got = _run_gpu(inp, w, bias, relu, mac_reference=route).cpu().numpy().astype(np.float64)
        assert got.shape == exp.shape
        err = np.abs(got - exp).max(axis=(0, 2, 3, 4))
        _say(f"    route {route or 'default'}: max err/tol per output image: {np.max(err / tol):.3e} "
             f"(worst abs {err.max():.3e})")
        assert np.all(np.isfinite(got))
        assert np.all(err <= tol), f"{label} route {route}: err {err} > tol {tol}"


def _rand(seed, S, f, fo, n, k):
    r = np.random.default_rng(seed)
    inp = r.uniform(-1, 1, (S, f, n, n, n)).astype(np.float32)
    w = (r.standard_normal((fo, f, k, k, k)) * (f * k ** 3) ** -0.5).astype(np.float32)
    b = (r.standard_normal(fo) * np.sqrt(0.1)).astype(np.float32)
    return inp, w, b


# (S, f, fo, n, k): transform sizes with every supported radix, tiles with ragged tails, n~ > n padding,
# odd sizes, k = 1 and k = n, single and many images.
SMALL = [
    (1, 1, 1, 8, 3),       # one radix-8 stage
    (2, 3, 2, 20, 3),      # 20 = 5*4, two tiles of lines with a ragged second one
    (1, 2, 2, 17, 4),      # 17 -> n~ = 18 = 3*3*2, padded lines
    (1, 1, 2, 33, 5),      # 33 -> 35 = 7*5
    (1, 3, 5, 24, 7),      # 24 = 3*8
    (2, 2, 2, 48, 2),      # even kernel
    (1, 4, 4, 40, 5),      # 40 = 5*8
    (1, 2, 3, 21, 1),      # k = 1: per-voxel matrix product, odd transform size 21 = 7*3
    (1, 2, 2, 6, 6),       # k = n: one output voxel per image
    (3, 1, 1, 1, 1),       # a single voxel
    (1, 5, 3, 50, 3),      # 50 = 5*5*2
    (1, 2, 2, 96, 3),      # 96 = 3*4*8, three stages
    (1, 1, 1, 125, 4),     # 125 -> 126 = 7*3*3*2
]


# Cubic images at every length that has a fused z+y kernel and is not in SMALL or the benchmark list, at the length
# itself (rows fill the transform length) or just below it (padded rows); 56, 72 and 120 also take the x passes
# whose tiles of lines are counted across rows.
FUSED_CUBIC = [(1, 2, 1, 10, 2), (1, 1, 2, 12, 3), (2, 1, 1, 14, 2), (1, 1, 1, 27, 3), (1, 2, 1, 32, 4),
               (1, 1, 1, 36, 2), (1, 1, 2, 55, 3), (1, 2, 1, 56, 4), (1, 1, 1, 72, 3), (1, 1, 1, 79, 5),
               (1, 1, 1, 100, 3), (1, 1, 1, 111, 2), (1, 1, 2, 118, 3), (1, 1, 1, 120, 2)]


@pytest.mark.parametrize("shape", FUSED_CUBIC, ids=lambda s: "S%d_f%dx%d_n%d_k%d" % s)
def test_fused_plane_kernel_lengths_full_compare(oracle, shape):
    S, f, fo, n, k = shape
    inp, w, b = _rand(500 + n + k, S, f, fo, n, k)
    _check_full(oracle, inp, w, b, True, f"fused {shape}")


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "S%d_f%dx%d_n%d_k%d" % s)
def test_small_layers_full_compare(oracle, shape):
    S, f, fo, n, k = shape
    inp, w, b = _rand(100 + n + k, S, f, fo, n, k)
    _check_full(oracle, inp, w, b, True, f"small {shape}")
    _check_full(oracle, inp, w, None, False, f"small {shape} linear", routes=(False,))


def _rand_v(seed, S, f, fo, n, k):
    r = np.random.default_rng(seed)
    inp = r.uniform(-1, 1, (S, f) + tuple(n)).astype(np.float32)
    w = (r.standard_normal((fo, f) + tuple(k)) * (f * k[0] * k[1] * k[2]) ** -0.5).astype(np.float32)
    b = (r.standard_normal(fo) * np.sqrt(0.1)).astype(np.float32)
    return inp, w, b


# (S, f, fo, <nx,ny,nz>, <kx,ky,kz>): image and kernel sizes that differ per axis (Section IV's general
# n = <nx,ny,nz>, k = <kx,ky,kz>), so that an axis mix-up anywhere in a pass, the kernel transform or a crop
# window changes the result.  Covers: all three transform sizes different; in-register and generic passes mixed
# in one layer; padded axes; tap counts with and without a specialised multiply-accumulate kernel; a kernel as
# long as the image on one axis; flat (one-voxel-thick) images and kernels.
ANISO = [
    (1, 2, 3, (12, 20, 16), (3, 2, 5)),
    (2, 3, 2, (16, 24, 40), (5, 3, 2)),       # z generic (40), x in-register (16)
    (1, 2, 2, (64, 18, 33), (7, 4, 3)),       # x in-register; y = 18, z 33 -> 35 padded
    (1, 4, 5, (21, 64, 17), (2, 7, 6)),       # y in-register, x 21 = 7*3, z 17 -> 18
    (1, 1, 2, (10, 15, 128), (4, 1, 9)),      # long contiguous axis, k = 1 on y
    (1, 2, 1, (128, 9, 14), (3, 9, 2)),       # kernel as long as the image on y: one output along y
    (2, 2, 2, (1, 30, 30), (1, 5, 5)),        # flat image: a batch of 2D convolutions
    (1, 3, 3, (30, 1, 25), (3, 1, 5)),
    (1, 2, 2, (28, 36, 1), (5, 3, 1)),
    (1, 48, 20, (16, 20, 24), (5, 3, 3)),     # many input images: several chunks / row blocks in the multiply-accumulate
    (2, 3, 2, (20, 62, 60), (3, 5, 3)),       # y and z share one transform length (64) with different extents and taps:
                                              # the fused z+y kernels, both sides
    (1, 2, 3, (81, 30, 31), (3, 2, 5)),       # ... with a generic x length (81): fused inverse, separate forward
    (3, 2, 2, (24, 111, 109), (2, 3, 4)),     # ... at the longest fused length (112), odd extents
]


@pytest.mark.parametrize("shape", ANISO, ids=lambda s: "S%d_f%dx%d_n%s_k%s" % (s[0], s[1], s[2], "x".join(map(str, s[3])), "x".join(map(str, s[4]))))
def test_anisotropic_layers_full_compare(oracle, shape):
    S, f, fo, n, k = shape
    inp, w, b = _rand_v(500 + sum(n) + sum(k), S, f, fo, n, k)
    _check_full(oracle, inp, w, b, True, f"aniso {shape}")
    _say(f"[parity/full] aniso {shape} plain multiply-accumulate")
    got = _run_gpu(inp, w, b, False, mac_reference=True).cpu().numpy().astype(np.float64)
    exp = oracle.conv3d(inp, w, b, relu=False)
    assert np.all(np.abs(got - exp) <= oracle.tolerance(inp, w)[None, :, None, None, None])


def test_anisotropic_delta_kernel_moves_each_axis_by_its_own_offset():
    """A one-tap kernel at (a0,b0,c0) of a <kx,ky,kz> kernel must return the image shifted by
    (kx-1-a0, ky-1-b0, kz-1-c0): exact in fp32 up to the transform's rounding, and wrong on any axis swap."""
    n, k, tap = (20, 16, 24), (4, 3, 5), (1, 2, 3)
    r = np.random.default_rng(77)
    inp = r.uniform(-1, 1, (1, 1) + n).astype(np.float32)
    w = np.zeros((1, 1) + k, dtype=np.float32)
    w[(0, 0) + tap] = 1.0
    got = _run_gpu(inp, w, None, False).cpu().numpy()
    o = [k[a] - 1 - tap[a] for a in range(3)]
    m = [n[a] - k[a] + 1 for a in range(3)]
    exp = inp[0, 0, o[0]:o[0] + m[0], o[1]:o[1] + m[1], o[2]:o[2] + m[2]]
    assert got.shape == (1, 1) + tuple(m)
    assert np.abs(got[0, 0] - exp).max() <= 1e-4


# Every transform length served by the in-register pass kernels, once along each axis (so every pass kind runs at
# every length), at the length itself and one below it (padded lines).
FAST_N = [8, 10, 12, 14, 16, 20, 24, 28, 32, 36, 40, 48, 56, 64, 72, 80, 84, 96, 100, 112, 120, 128, 144, 160, 168, 192, 200,
          224, 240, 256, 288, 320, 336, 384, 400, 448, 480, 512, 576, 640, 720, 768, 840, 896, 960, 1024]


@pytest.mark.parametrize("N", FAST_N)
def test_in_register_pass_lengths_along_each_axis(oracle, N):
    assert B.znni_fft_size(N) == N and B.znni_fft_size(N - 1) == N
    for axis in range(3):
        for n_ax in (N, N - 1):
            n = [12, 12, 12]
            n[axis] = n_ax
            k = [2, 3, 2]
            k[axis] = 3
            inp, w, b = _rand_v(1000 + N + axis, 1, 2, 2, n, k)
            _check_full(oracle, inp, w, b, True, f"in-register length {N} on axis {axis}, n = {n}")


# The generic pass kernels: the lengths they alone serve (below 7), and, forced by the diagnostic flag, lengths the
# in-register kernels would take: every radix (2, 3, 4, 5, 7, 8) occurs, long lines, padded lines.  Both sets of pass
# kernels must give the oracle's result, so they also check each other.
GENERIC = [(1, 2, 2, (2, 3, 5), (1, 2, 3)), (2, 1, 2, (6, 4, 5), (3, 3, 3)), (1, 2, 1, (3, 6, 4), (2, 5, 4)),
           (1, 1, 2, (576, 6, 10), (3, 2, 2)), (1, 2, 1, (6, 720, 5), (2, 3, 2)), (1, 1, 1, (10, 6, 1000), (2, 2, 5)),
           (1, 1, 1, (5, 336, 8), (1, 7, 1)), (1, 2, 3, (100, 84, 56), (3, 4, 5)), (2, 3, 2, (20, 64, 64), (5, 3, 3))]


@pytest.mark.parametrize("shape", GENERIC, ids=lambda s: "S%d_f%dx%d_n%s_k%s" % (s[0], s[1], s[2], "x".join(map(str, s[3])), "x".join(map(str, s[4]))))
def test_generic_pass_lengths_full_compare(oracle, shape):
    S, f, fo, n, k = shape
    inp, w, b = _rand_v(1100 + sum(n), S, f, fo, n, k)
    _check_full(oracle, inp, w, b, True, f"generic {shape}", routes=("generic_passes", False))


# Transform lengths served by the two-step in-register passes (16, 64, 128, 256, 320), at the length itself
# and just below it (zero-padded lines, ragged tiles of lines).
TWO_STEP = [(2, 2, 3, 16, 3), (1, 2, 2, 15, 2), (1, 3, 2, 64, 5), (2, 1, 2, 61, 4), (1, 2, 1, 128, 3),
            (1, 1, 2, 127, 6), (1, 1, 1, 256, 3), (1, 1, 1, 250, 2), (1, 1, 2, 320, 5), (1, 2, 1, 317, 3)]


@pytest.mark.parametrize("shape", TWO_STEP, ids=lambda s: "S%d_f%dx%d_n%d_k%d" % s)
def test_two_step_pass_lengths_full_compare(oracle, shape):
    S, f, fo, n, k = shape
    inp, w, b = _rand(300 + n + k, S, f, fo, n, k)
    _check_full(oracle, inp, w, b, True, f"two-step {shape}")


@pytest.mark.parametrize("idx", [0, 1])
def test_benchmark_layers_full_compare(oracle, idx):
    L = W.CONFIGS[idx]
    inp, w, b = W.make_inputs(L)
    _check_full(oracle, inp, w, b, L.relu, L.name)


@pytest.mark.parametrize("idx", [2, 3])
def test_benchmark_layers_every_voxel(oracle, idx):
    """The wide 3^3 layer (86 G multiply-adds on the host) and the batched 7^3 layer (548 G): every output voxel
    against the full direct convolution of the oracle, one input of the batch at a time."""
    L = W.CONFIGS[idx]
    _say(f"[parity/full] {L.name}: drawing inputs")
    inp, w, b = W.make_inputs(L)
    routes = (False, "single" if L.S == 1 else "batch", "xdirect", "xblock")
    outs = [_run_gpu(inp, w, b, L.relu, mac_reference=r) for r in routes]
    assert all(bool(torch.isfinite(o).all()) for o in outs)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    worst, checked = [0.0] * len(routes), 0
    for s in range(L.S):
        _say(f"    oracle: input {s + 1} of {L.S}")
        exp = oracle.conv3d(inp[s:s + 1], w, b, relu=L.relu)
        assert np.count_nonzero(exp) > 0.2 * exp.size
        checked += exp.size
        for q, (route, out) in enumerate(zip(routes, outs)):
            ratio = np.abs(out[s:s + 1].cpu().numpy() - exp) / tol
            worst[q] = max(worst[q], float(ratio.max()))
            assert np.all(ratio <= 1.0), f"{L.name}: route {route}: input {s}: err/tol {ratio.max():.3e}"
    _say(f"    {checked} output voxels checked (all {L.out_voxels}) on the routes {routes}: max err/tol {worst}")
    assert checked == L.out_voxels


def _gather(out, pts):
    tp = torch.from_numpy(pts.astype(np.int64)).to(out.device)
    return out[tp[:, 0], tp[:, 1], tp[:, 2], tp[:, 3], tp[:, 4]].cpu().numpy().astype(np.float64)


def test_largest_benchmark_layer_declared_sample(largest_layer_case):
    """48 -> 48 images of 320^3, 5^3 kernels: 9.1e12 multiply-adds, too many for a full direct convolution on the
    host.  Checked on every voxel of the 8 corner blocks (8^3) and 6 face-centre patches of every output image,
    the three mid-planes of one complete output image, and 2^20 uniformly random positions."""
    C = largest_layer_case
    L = C.layer
    assert len(C.pts) >= (1 << 20)
    for route in ROUTES[1:]:
        _say(f"[parity/sampled] {L.name}: {len(C.pts)} sampled output voxels; running the layer, route {route}")
        out = _run_gpu(C.inp, C.w, C.bias, L.relu, mac_reference=route)
        assert bool(torch.isfinite(out).all())
        got = _gather(out, C.pts)
        del out
        torch.cuda.empty_cache()
        ratio = np.abs(got - C.exp) / C.tol
        _say(f"    {len(C.pts)} output voxels checked; max err/tol {ratio.max():.3e}; "
             f"mean |out| {np.abs(C.exp).mean():.3e}")
        assert np.all(ratio <= 1.0)


def test_results_are_bitwise_reproducible_and_workspace_reusable():
    S, f, fo, n, k = 2, 3, 4, 40, 5
    inp, w, b = _rand(7, S, f, fo, n, k)
    d = torch.device("cuda:0")
    ws = B.alloc_workspace(S, f, fo, n, k, d)
    ws.fill_(0xFF)          # NaN bit patterns: the layer must not depend on workspace contents
    a = _run_gpu(inp, w, b, True, workspace=ws).clone()
    c = _run_gpu(inp, w, b, True, workspace=ws)
    assert torch.equal(a, c)
    e = _run_gpu(inp, w, b, True)
    assert torch.equal(a, e)


def test_runs_on_a_side_stream_and_profile_matches():
    S, f, fo, n, k = 1, 4, 4, 32, 3
    inp, w, b = _rand(9, S, f, fo, n, k)
    d = torch.device("cuda:0")
    ti, tw, tb = (torch.from_numpy(t).to(d) for t in (inp, w, b))
    ref_out = B.znni_conv3d_fft(ti, tw, tb, relu=True)
    torch.cuda.synchronize()
    st = torch.cuda.Stream(device=d)
    with torch.cuda.stream(st):
        o2 = B.znni_conv3d_fft(ti, tw, tb, relu=True, stream=st)
    st.synchronize()
    assert torch.equal(ref_out, o2)
    o3, ms = B.znni_conv3d_fft_profile(ti, tw, tb, relu=True)
    assert torch.equal(ref_out, o3)
    assert set(ms) == set(B.STAGES) and all(v >= 0 for v in ms.values())


@pytest.mark.parametrize("shape", [(1, 8, 8, 64, 5), (8, 4, 4, 22, 3), (1, 3, 2, 118, 3)],
                         ids=lambda s: "S%d_f%dx%d_n%d_k%d" % s)
def test_layer_call_can_be_captured_in_a_graph_and_replayed(shape):
    """The layer call only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset),
    so a launch-bound small layer can be captured once and replayed.  Every replay, with eager work and
    synchronisations in between and new input values each time, must equal the eager result bit for bit.
    (The last shape uses the fused kernels with more than 48 KB of LDS, whose launch sets a function attribute.)"""
    S, f, fo, n, k = shape
    d = torch.device("cuda:0")
    inp, w, b = (torch.from_numpy(t).to(d) for t in _rand(31 + n, S, f, fo, n, k))
    ws_g, ws_e = B.alloc_workspace(S, f, fo, n, k, d), B.alloc_workspace(S, f, fo, n, k, d)
    out_g = torch.empty((S, fo) + (n - k + 1,) * 3, device=d)
    out_e = torch.empty_like(out_g)
    _say(f"[graph] {shape}: warm-up")
    B.znni_conv3d_fft(inp, w, b, relu=True, out=out_g, workspace=ws_g)        # first-use set-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    _say(f"[graph] {shape}: capture")
    with torch.cuda.graph(g):
        B.znni_conv3d_fft(inp, w, b, relu=True, out=out_g, workspace=ws_g)
    for rep in range(4):
        inp.uniform_(-1, 1)                        # eager work between replays
        out_g.fill_(float("nan"))
        B.znni_conv3d_fft(inp, w, b, relu=True, out=out_e, workspace=ws_e)
        torch.cuda.synchronize()
        _say(f"[graph] {shape}: replay {rep}")
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), f"replay {rep} differs from the eager call"


@pytest.mark.parametrize("shape", [(1, 2, 3, 16, 3), (2, 5, 7, 24, 5), (1, 48, 48, 40, 5), (3, 6, 20, 20, 2),
                                   (1, 80, 100, 16, 3)],
                         ids=lambda s: "S%d_f%dx%d_n%d_k%d" % s)
def test_matrix_core_mac_agrees_with_plain_mac(oracle, shape):
    """The tiled matrix-core multiply-accumulate and the one-thread-per-bin kernel must agree to rounding,
    and both must meet the oracle bar (row/column padding, several row blocks, channel chunks)."""
    S, f, fo, n, k = shape
    inp, w, b = _rand(21 + f, S, f, fo, n, k)
    _say(f"[mac] {shape}")
    fast = _run_gpu(inp, w, b, False).cpu().numpy().astype(np.float64)
    plain = _run_gpu(inp, w, b, False, mac_reference=True).cpu().numpy().astype(np.float64)
    exp = oracle.conv3d(inp, w, b, relu=False)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    assert np.all(np.abs(fast - exp) <= tol)
    assert np.all(np.abs(plain - exp) <= tol)
    assert np.all(np.abs(fast - plain) <= 0.1 * tol)


# (S, f, fo, n, k): batch sizes below, at and above the 4-input groups, more than 16 inputs (two chunks), taps with
# and without compile-time kernels, transform sizes that are not multiples of the 16-bin tile, one and several
# rounds of output-image groups, image blocks that need two LDS fills; an odd transform length with at most 8
# inputs (no batch kernel there: the flag is ignored) and with more; a last bin tile of 8 and of 10 bins with a
# partial second chunk of input images.
BATCH = [(2, 3, 5, 16, 3), (4, 4, 4, 20, 5), (5, 2, 3, 24, 2), (8, 32, 32, 16, 7), (9, 6, 40, 18, 4), (20, 3, 7, 16, 3),
         (3, 70, 9, 16, 1), (8, 5, 70, 32, 6), (4, 3, 3, 5, 2), (12, 3, 3, 5, 2), (8, 9, 5, 22, 5), (7, 12, 4, 10, 3),
         (4, 3, 5, 14, 9), (10, 2, 3, 13, 11), (9, 5, 3, 12, 12),      # 9 to 12 taps: three steps of four
         # more than 16 inputs: workgroups of two tiles of 16 inputs; a second tile with one input, several workgroups
         # along the batch with a ragged last one, a partial chunk of input images
         (33, 9, 17, 16, 7), (40, 5, 20, 12, 5), (70, 12, 4, 10, 3)]


@pytest.mark.parametrize("shape", BATCH, ids=lambda s: "S%d_f%dx%d_n%d_k%d" % s)
def test_batch_mac_form_matches_oracle_and_single_form(oracle, shape):
    S, f, fo, n, k = shape
    inp, w, b = _rand(60 + S + fo, S, f, fo, n, k)
    _say(f"[mac/batch] {shape}")
    batch = _run_gpu(inp, w, b, False, mac_reference="batch").cpu().numpy().astype(np.float64)
    single = _run_gpu(inp, w, b, False, mac_reference="single").cpu().numpy().astype(np.float64)
    exp = oracle.conv3d(inp, w, b, relu=False)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    _say(f"    max err/tol: batch {np.max(np.abs(batch - exp) / tol):.3e}, single {np.max(np.abs(single - exp) / tol):.3e}")
    assert np.all(np.abs(batch - exp) <= tol)
    assert np.all(np.abs(single - exp) <= tol)
    assert np.all(np.abs(batch - single) <= 0.1 * tol)


# (S, f, fo, <nx,ny,nz>, <kx,ky,kz>) for the route that leaves the x axis untransformed: every tap count it has a
# kernel for (1 to 9 along x), row blocks of one to five tiles, 128-wide and 64-wide column blocks with ragged ends,
# several inputs per batch (columns run over (input, xo)), x extents that are no transform length at all (the axis is
# never padded), output rows shorter than a tile.
XDIRECT = [(1, 3, 2, (9, 16, 16), (1, 3, 3)), (1, 5, 17, (37, 12, 20), (2, 3, 2)), (2, 6, 33, (150, 8, 10), (3, 2, 3)),
           (1, 9, 49, (70, 10, 8), (4, 3, 2)), (3, 4, 65, (45, 8, 12), (5, 2, 2)), (1, 7, 80, (131, 8, 8), (6, 1, 3)),
           (1, 13, 48, (203, 10, 8), (7, 3, 1)), (2, 2, 20, (67, 12, 14), (8, 2, 2)), (1, 4, 40, (300, 8, 8), (9, 2, 2)),
           (1, 48, 48, (40, 16, 20), (5, 5, 5)), (4, 3, 3, (11, 20, 24), (11, 3, 3)), (1, 2, 2, (5, 14, 10), (3, 3, 3)),
           # blocks of eight along x: ragged last block, more than 32 blocks (wide and narrow column blocks), a number
           # of input images that is no multiple of 8 or 4, several inputs per batch, two row blocks, one block only
           (1, 19, 40, (141, 8, 10), (5, 2, 2)), (2, 20, 48, (70, 10, 8), (4, 3, 2)), (1, 16, 7, (203, 8, 8), (4, 2, 2)),
           (1, 33, 96, (77, 8, 12), (5, 2, 3)), (3, 24, 4, (8, 12, 10), (5, 3, 2)), (1, 17, 3, (300, 8, 8), (4, 2, 2)),
           # ... output images in row blocks of different heights (five tiles = 3 + 2, four = 2 + 2, seven = 3 + 2 + 2)
           (1, 16, 80, (50, 8, 10), (5, 2, 2)), (1, 24, 64, (37, 10, 8), (4, 3, 2)), (2, 17, 112, (30, 8, 8), (5, 2, 2)),
           (1, 16, 70, (170, 8, 8), (4, 2, 2)),
           # ... kernels of one and of more than five taps along y (the kernel transform of this route has a form for up
           # to five and a general one), more than 32 transform bins along y
           (1, 16, 16, (30, 12, 8), (4, 1, 3)), (1, 17, 20, (40, 16, 8), (5, 7, 2)), (1, 16, 5, (20, 45, 8), (5, 4, 3))]


@pytest.mark.parametrize("shape", XDIRECT, ids=lambda s: "S%d_f%dx%d_n%s_k%s" % (s[0], s[1], s[2], "x".join(map(str, s[3])), "x".join(map(str, s[4]))))
def test_untransformed_x_axis_route_matches_oracle_and_transformed_route(oracle, shape):
    S, f, fo, n, k = shape
    inp, w, b = _rand_v(900 + sum(n) + fo, S, f, fo, n, k)
    _say(f"[mac/xdirect] {shape}")
    xd = _run_gpu(inp, w, b, False, mac_reference="xdirect").cpu().numpy().astype(np.float64)
    xb = _run_gpu(inp, w, b, False, mac_reference="xblock").cpu().numpy().astype(np.float64)
    single = _run_gpu(inp, w, b, False, mac_reference="single").cpu().numpy().astype(np.float64)
    exp = oracle.conv3d(inp, w, b, relu=False)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    _say(f"    max err/tol: xdirect {np.max(np.abs(xd - exp) / tol):.3e}, xblock {np.max(np.abs(xb - exp) / tol):.3e}, "
         f"single {np.max(np.abs(single - exp) / tol):.3e}")
    assert np.all(np.abs(xd - exp) <= tol)
    assert np.all(np.abs(xb - exp) <= tol)
    assert np.all(np.abs(single - exp) <= tol)
    assert np.all(np.abs(xd - single) <= 0.1 * tol)
    assert np.all(np.abs(xb - single) <= 0.1 * tol)


ALL_FORMS = (False, "single", "batch", "xdirect", "xblock", "generic_passes")


@pytest.mark.parametrize("seed", range(36))
def test_random_shapes_match_oracle_in_every_form(oracle, seed):
    """Seeded random layers (batches of 1 to 40, 1 to 40 input and 1 to 100 output images, per-axis image sizes up to
    72 and kernels of 1 to 9 taps, drawn until the oracle's work stays below about a billion multiply-adds): every
    form of the multiply-accumulate and both sets of pass kernels against the oracle, on every voxel."""
    r = np.random.default_rng(7000 + seed)
    while True:
        S = int(r.choice([1, 1, 1, 2, 3, 5, 8, 9, 17, 24, 40]))
        f, fo = int(r.integers(1, 41)), int(r.integers(1, 101))
        k = tuple(int(v) for v in r.integers(1, 10, 3))
        n = tuple(int(k[a] + r.integers(0, 72 - k[a] + 1)) for a in range(3))
        macs = S * f * fo * k[0] * k[1] * k[2] * np.prod([n[a] - k[a] + 1 for a in range(3)], dtype=np.float64)
        vox = S * max(f, fo) * np.prod(n, dtype=np.float64)
        if macs <= 1.2e9 and vox <= 3e7:
            break
    inp, w, b = _rand_v(7100 + seed, S, f, fo, n, k)
    relu, bias = bool(seed & 1), (b if seed % 3 else None)
    _check_full(oracle, inp, w, bias, relu, f"random seed {seed}: S={S} f={f} fo={fo} n={n} k={k}", routes=ALL_FORMS)


@pytest.mark.parametrize("route", [False, "single", "batch", "xdirect", "xblock"], ids=lambda r: str(r or "default"))
def test_stored_kernel_transforms_can_be_kept_between_calls(oracle, route):
    """Inference applies one kernel bank to many inputs: a call that keeps the workspace's stored kernel transforms
    must equal a call that recomputes them, bit for bit, on new inputs; and it really does not read w."""
    S, f, fo, n, k = (4 if route == "batch" else 1), 16, 20, (36, 20, 24), (5, 3, 4)
    inp, w, b = _rand_v(321, S, f, fo, n, k)
    d = torch.device("cuda:0")
    ti, tw, tb = (torch.from_numpy(t).to(d) for t in (inp, w, b))
    ws = B.alloc_workspace(S, f, fo, n, k, d)
    first = B.znni_conv3d_fft(ti, tw, tb, relu=True, workspace=ws, mac_reference=route)
    exp = oracle.conv3d(inp, w, b, relu=True)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    assert np.all(np.abs(first.cpu().numpy() - exp) <= tol)
    inp2 = np.random.default_rng(322).uniform(-1, 1, inp.shape).astype(np.float32)
    ti2 = torch.from_numpy(inp2).to(d)
    fresh = B.znni_conv3d_fft(ti2, tw, tb, relu=True, mac_reference=route)
    junk = torch.full_like(tw, float("nan"))                    # would poison everything if it were read
    kept = B.znni_conv3d_fft(ti2, junk, tb, relu=True, workspace=ws, mac_reference=route, keep_kernels=True)
    torch.cuda.synchronize()
    assert torch.equal(kept, fresh)
    assert np.all(np.abs(kept.cpu().numpy() - oracle.conv3d(inp2, w, b, relu=True)) <= tol)


def test_calls_on_two_streams_with_two_workspaces_do_not_disturb_each_other():
    """The library keeps no device state of its own: calls on different streams with different workspaces may overlap
    in time.  Two layers of different shapes are enqueued alternately on two streams, several times, without any
    synchronisation in between; every result must equal the one computed alone, bit for bit."""
    d = torch.device("cuda:0")
    shapes = [(1, 16, 16, (72, 64, 64), (5, 5, 5)), (2, 12, 20, (40, 36, 48), (3, 3, 3))]
    layers = []
    for q, (S, f, fo, n, k) in enumerate(shapes):
        inp, w, b = (torch.from_numpy(t).to(d) for t in _rand_v(700 + q, S, f, fo, n, k))
        alone = B.znni_conv3d_fft(inp, w, b, relu=True)
        layers.append(dict(inp=inp, w=w, b=b, alone=alone, ws=B.alloc_workspace(S, f, fo, n, k, d),
                           outs=[torch.empty_like(alone) for _ in range(4)], st=torch.cuda.Stream(device=d)))
    torch.cuda.synchronize()
    for rep in range(4):
        for L in layers:
            with torch.cuda.stream(L["st"]):
                B.znni_conv3d_fft(L["inp"], L["w"], L["b"], relu=True, out=L["outs"][rep], workspace=L["ws"], stream=L["st"])
    torch.cuda.synchronize()
    for L in layers:
        for o in L["outs"]:
            assert torch.equal(o, L["alone"])


def test_relu_flag_and_null_bias(oracle):
    S, f, fo, n, k = 1, 2, 2, 16, 3
    inp, w, b = _rand(11, S, f, fo, n, k)
    lin = _run_gpu(inp, w, None, False)
    pre = _run_gpu(inp, w, b, False)
    act = _run_gpu(inp, w, b, True)
    assert torch.equal(act, torch.clamp_min(pre, 0))
    tb = torch.from_numpy(b).to(lin.device)
    assert torch.allclose(pre, lin + tb[None, :, None, None, None], atol=1e-6)


def test_copy_probe_copies():
    src = torch.arange(1 << 20, dtype=torch.float32, device="cuda:0")
    dst = torch.zeros_like(src)
    B.znni_copy_probe(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
