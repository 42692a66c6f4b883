"""GPU parity of the pooling kernels (through the C ABI) against the CPU oracle: selection of input values, so
the comparison is bit-exact."""
import sys

import numpy as np
import pytest
import torch

from paper_1606_05688_amd import binding as B

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _img(seed, S, f, n):
    return np.random.default_rng(seed).uniform(-1, 1, (S, f) + tuple(n)).astype(np.float32)


# (S, f, <nx,ny,nz>, <px,py,pz>): every window 1..4 on every axis, several tiles along y and z with ragged last
# tiles, several x chunks (more than 32 positions), images thinner than a tile, n = p (one voxel per fragment).
MPF_CASES = [
    (1, 1, (5, 5, 5), (2, 2, 2)),
    (2, 3, (7, 11, 9), (2, 3, 2)),
    (1, 2, (11, 7, 15), (4, 2, 4)),
    (1, 1, (3, 3, 3), (1, 1, 1)),
    (1, 2, (8, 5, 6), (3, 1, 1)),
    (1, 1, (5, 7, 4), (3, 4, 1)),
    (2, 2, (3, 5, 1), (2, 3, 1)),
    (1, 3, (71, 39, 35), (2, 2, 2)),          # three x chunks, ragged y tiles
    (1, 2, (20, 47, 299), (3, 4, 2)),         # three z tiles (64 fragment columns each), ragged
    (1, 1, (9, 33, 383), (1, 2, 3)),          # z tiles of 42 fragment columns
    (3, 2, (1, 63, 127), (1, 2, 2)),          # flat images: two-dimensional pooling
    (1, 2, (127, 1, 63), (4, 1, 4)),
    (1, 1, (5, 7, 7), (3, 4, 4)),
]


@pytest.mark.parametrize("case", MPF_CASES, ids=lambda c: "S%d_f%d_n%s_p%s" % (c[0], c[1], "x".join(map(str, c[2])), "x".join(map(str, c[3]))))
def test_mpf_matches_oracle_bit_exactly(oracle, case):
    S, f, n, p = case
    _say(f"[mpf] {case}")
    inp = _img(900 + sum(n) + sum(p), S, f, n)
    got = B.znni_mpf(torch.from_numpy(inp).cuda(), p)
    torch.cuda.synchronize()
    exp = oracle.mpf(inp, p)
    assert tuple(got.shape) == exp.shape
    assert np.array_equal(got.cpu().numpy(), exp)


def test_mpf_window_equal_to_image_gives_one_voxel_fragments(oracle):
    # the smallest image for a window p > 1 is n = 2p - 1: fragments of one voxel
    inp = _img(5, 1, 2, (7, 5, 3))
    got = B.znni_mpf(torch.from_numpy(inp).cuda(), (4, 3, 2)).cpu().numpy()
    assert got.shape == (24, 2, 1, 1, 1)
    assert np.array_equal(got, oracle.mpf(inp, (4, 3, 2)))


def test_mpf_benchmark_shape_sampled_fragments(oracle):
    """The benchmark's pooling workload (48 images of 255^3, window 2^3): whole fragments of a few images against
    the oracle, and every output voxel against the defining property checked on the GPU side with torch."""
    S, f, n, p = 1, 48, (255, 255, 255), (2, 2, 2)
    _say("[mpf] benchmark shape: drawing inputs")
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    inp = torch.rand((S, f) + n, device="cuda", generator=g) * 2 - 1
    out = B.znni_mpf(inp, p)
    torch.cuda.synchronize()
    assert tuple(out.shape) == (8, 48, 127, 127, 127)
    for i in (0, 17, 47):
        sub = inp[:, i:i + 1].cpu().numpy()
        exp = oracle.mpf(sub, p)
        assert np.array_equal(out[:, i:i + 1].cpu().numpy(), exp), f"image {i}"
    # fragment (ox,oy,oz) of every image is the strided max pooling of the shifted crop (library routine)
    for fr, (ox, oy, oz) in enumerate([(a, b, c) for a in range(2) for b in range(2) for c in range(2)]):
        ref = torch.nn.functional.max_pool3d(inp[:, :, ox:, oy:, oz:], 2, 2)
        assert torch.equal(out[fr:fr + 1], ref), f"fragment {fr}"


MAXPOOL_CASES = [(1, 1, (4, 4, 4), (2, 2, 2)), (2, 3, (6, 9, 8), (3, 3, 2)), (1, 2, (5, 70, 600), (5, 7, 2)),
                 (1, 1, (3, 3, 3), (1, 1, 1)), (1, 2, (8, 8, 8), (8, 8, 8)), (1, 2, (64, 64, 64), (2, 2, 2))]


@pytest.mark.parametrize("case", MAXPOOL_CASES, ids=lambda c: "S%d_f%d_n%s_p%s" % (c[0], c[1], "x".join(map(str, c[2])), "x".join(map(str, c[3]))))
def test_maxpool_matches_oracle_bit_exactly(oracle, case):
    S, f, n, p = case
    _say(f"[maxpool] {case}")
    inp = _img(950 + sum(n), S, f, n)
    got = B.znni_maxpool(torch.from_numpy(inp).cuda(), p)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.maxpool(inp, p))


def test_fragments_feed_the_convolutional_layer(oracle):
    """Pooling fragments followed by the FFT layer, as in the networks of Section VI's table: the fragment batch is
    an ordinary input batch of the next layer."""
    S, f, fo, n, p, k = 1, 3, 4, (23, 23, 23), (2, 2, 2), 3
    r = np.random.default_rng(31)
    inp = r.uniform(-1, 1, (S, f) + n).astype(np.float32)
    w = (r.standard_normal((fo, f, k, k, k)) * (f * k ** 3) ** -0.5).astype(np.float32)
    b = (r.standard_normal(fo) * 0.3).astype(np.float32)
    frag = B.znni_mpf(torch.from_numpy(inp).cuda(), p)
    out = B.znni_conv3d_fft(frag, torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda(), relu=True)
    torch.cuda.synchronize()
    fr = oracle.mpf(inp, p)
    exp = oracle.conv3d(fr, w, b, relu=True)
    tol = oracle.tolerance(fr, w)[None, :, None, None, None]
    assert tuple(out.shape) == exp.shape == (8, fo, 9, 9, 9)
    assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - exp) <= tol)
