"""GPU parity of the direct-convolution primitive (through the C ABI) against the fp64 oracle, to the same
per-voxel bar as the transform route: |gpu - oracle| <= 1e-4 * max|x| * sum|w[j]|."""
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


def _rand(seed, S, f, fo, n, k):
    r = np.random.default_rng(seed)
    inp = r.uniform(-1, 1, (S, f) + tuple(n)).astype(np.float32)
    w = (r.standard_normal((fo, f) + tuple(k)) * (f * k[0] * k[1] * k[2]) ** -0.5).astype(np.float32)
    b = (r.standard_normal(fo) * np.sqrt(0.1)).astype(np.float32)
    return inp, w, b


def _gpu(inp, w, b, relu):
    d = torch.device("cuda:0")
    out = B.znni_conv3d_direct(torch.from_numpy(inp).to(d), torch.from_numpy(w).to(d),
                               torch.from_numpy(b).to(d) if b is not None else None, relu=relu)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


# (S, f, fo, n, k): tap counts that are and are not multiples of four, one to five row tiles and two row blocks,
# ragged tiles on every axis, several chunks of input images, a single input image (first layers), flat images,
# k = 1, k = n, anisotropic shapes.
CASES = [
    (1, 1, 1, (8, 8, 8), (3, 3, 3)),
    (2, 3, 5, (9, 10, 37), (2, 2, 2)),
    (1, 1, 48, (12, 13, 40), (3, 3, 3)),        # first layer: one input image, three row tiles
    (1, 20, 17, (11, 9, 35), (3, 3, 3)),        # three chunks of input images, two row tiles
    (1, 4, 64, (7, 9, 33), (2, 3, 4)),          # four row tiles
    (1, 3, 80, (6, 7, 20), (3, 2, 1)),          # five row tiles (narrow column blocks)
    (1, 2, 100, (5, 6, 18), (2, 2, 3)),         # two row blocks
    (2, 5, 7, (14, 6, 70), (5, 5, 5)),
    (1, 2, 3, (10, 12, 16), (7, 7, 7)),
    (1, 6, 6, (5, 1, 40), (1, 1, 1)),           # k = 1: per-voxel matrix product
    (1, 2, 2, (4, 5, 6), (4, 5, 6)),            # k = n: one output voxel
    (3, 2, 2, (1, 20, 33), (1, 3, 3)),          # flat images
    (1, 9, 4, (13, 21, 8), (4, 1, 6)),
    (1, 1, 20, (4, 5, 140), (2, 2, 3)),         # first layer, long tiles: two tiles along z, the second ragged
    (2, 2, 33, (3, 6, 260), (1, 2, 2)),         # long tiles: three tiles along z, a ragged third row tile
    (1, 1, 81, (5, 4, 131), (2, 2, 4)),         # long tiles in two row blocks, 128 outputs along z exactly
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "S%d_f%dx%d_n%s_k%s" % (c[0], c[1], c[2], "x".join(map(str, c[3])), "x".join(map(str, c[4]))))
def test_direct_matches_oracle(oracle, case):
    S, f, fo, n, k = case
    _say(f"[direct] {case}")
    inp, w, b = _rand(700 + sum(n) + sum(k) + fo, S, f, fo, n, k)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    for bias, relu in ((b, True), (None, False)):
        got = _gpu(inp, w, bias, relu)
        exp = oracle.conv3d(inp, w, bias, relu=relu)
        assert got.shape == exp.shape
        err = np.abs(got - exp)
        _say(f"    relu={relu}: max err/tol {np.max(err / tol):.3e}")
        assert np.all(err <= tol)


@pytest.mark.parametrize("idx", [0, 1])
def test_direct_on_benchmark_layers_full_compare(oracle, idx):
    L = W.CONFIGS[idx]
    inp, w, b = W.make_inputs(L)
    got = _gpu(inp, w, b, L.relu)
    exp = oracle.conv3d(inp, w, b, relu=L.relu)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    assert np.all(np.abs(got - exp) <= tol)


def test_direct_on_wide_layer_every_voxel(oracle):
    L = W.CONFIGS[2]                                  # 40 -> 40 images of 128^3, 3^3 kernels
    _say(f"[direct/full] {L.name}")
    inp, w, b = W.make_inputs(L)
    d = torch.device("cuda:0")
    ti, tw, tb = (torch.from_numpy(t).to(d) for t in (inp, w, b))
    out = B.znni_conv3d_direct(ti, tw, tb, relu=L.relu)
    exp = oracle.conv3d(inp, w, b, relu=L.relu)
    tol = oracle.tolerance(inp, w)
    ratio = np.abs(out.cpu().numpy() - exp) / tol[None, :, None, None, None]
    _say(f"    {exp.size} output voxels checked; max err/tol {ratio.max():.3e}")
    assert np.all(ratio <= 1.0)
    # and the two primitives agree with each other everywhere
    fft = B.znni_conv3d_fft(ti, tw, tb, relu=L.relu)
    tolj = torch.from_numpy(tol.astype(np.float32)).to(d)[None, :, None, None, None]
    assert bool(((out - fft).abs() <= 0.2 * tolj).all())


def test_direct_rejects_kernels_it_cannot_stage():
    with pytest.raises(B.ZnniError) as e:
        B.znni_conv3d_direct_workspace(1, 1, 1, (20, 20, 20), (9, 9, 9))
    assert e.value.status == -3


@pytest.mark.parametrize("case", [(1, 1, 20, (40, 40, 40), (3, 3, 3), "direct"), (1, 16, 16, (64, 64, 64), (5, 5, 5), "fft"),
                                  (2, 6, 6, (30, 30, 30), (2, 2, 2), "direct")],
                         ids=lambda c: "S%d_f%dx%d_n%d_k%d_%s" % (c[0], c[1], c[2], c[3][0], c[4][0], c[5]))
def test_auto_call_runs_the_picked_primitive_and_matches_oracle(oracle, case):
    S, f, fo, n, k, want = case
    assert B.znni_conv3d_choose(S, f, fo, n, k)[0] == want
    inp, w, b = _rand(800 + f + fo, S, f, fo, n, k)
    d = torch.device("cuda:0")
    ti, tw, tb = (torch.from_numpy(t).to(d) for t in (inp, w, b))
    got = B.znni_conv3d(ti, tw, tb, relu=True)
    same = (B.znni_conv3d_direct if want == "direct" else B.znni_conv3d_fft)(ti, tw, tb, relu=True)
    torch.cuda.synchronize()
    assert torch.equal(got, same)
    exp = oracle.conv3d(inp, w, b, relu=True)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - exp) <= tol)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_match_oracle_on_both_routes(oracle, seed):
    """Seeded random shapes (per-axis sizes and kernels, small batches, ragged everything): the direct primitive and
    the transform route against the oracle, and therefore against each other."""
    r = np.random.default_rng(9000 + seed)
    S, f, fo = int(r.integers(1, 4)), int(r.integers(1, 6)), int(r.integers(1, 40))
    k = tuple(int(v) for v in r.integers(1, 6, 3))
    n = tuple(int(k[a] + r.integers(0, 60 if a == 2 else 14)) for a in range(3))
    _say(f"[random] seed {seed}: S={S} f={f} fo={fo} n={n} k={k}")
    inp, w, b = _rand(9100 + seed, S, f, fo, n, k)
    exp = oracle.conv3d(inp, w, b, relu=True)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    got_d = _gpu(inp, w, b, True)
    d = torch.device("cuda:0")
    got_f = B.znni_conv3d_fft(torch.from_numpy(inp).to(d), torch.from_numpy(w).to(d), torch.from_numpy(b).to(d),
                              relu=True).cpu().numpy().astype(np.float64)
    assert got_d.shape == exp.shape and got_f.shape == exp.shape
    assert np.all(np.abs(got_d - exp) <= tol), "direct"
    assert np.all(np.abs(got_f - exp) <= tol), "transform"


@pytest.mark.parametrize("seed", range(12))
def test_random_cubic_shapes_match_oracle_on_both_routes(oracle, seed):
    """Seeded random cubic images (8^3 to 72^3: the transform route's fused plane kernels, at and below their
    lengths) on both routes against the oracle."""
    r = np.random.default_rng(9500 + seed)
    S, f, fo = int(r.integers(1, 3)), int(r.integers(1, 4)), int(r.integers(1, 4))
    kk = int(r.integers(1, 6))
    nn = int(r.integers(max(8, kk), 73))
    n, k = (nn, nn, nn), (kk, kk, kk)
    _say(f"[random cubic] seed {seed}: S={S} f={f} fo={fo} n={nn} k={kk}")
    inp, w, b = _rand(9600 + seed, S, f, fo, n, k)
    exp = oracle.conv3d(inp, w, b, relu=True)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    got_d = _gpu(inp, w, b, True)
    d = torch.device("cuda:0")
    got_f = B.znni_conv3d_fft(torch.from_numpy(inp).to(d), torch.from_numpy(w).to(d), torch.from_numpy(b).to(d),
                              relu=True).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got_d - exp) <= tol), "direct"
    assert np.all(np.abs(got_f - exp) <= tol), "transform"
