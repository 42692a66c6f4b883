"""Pins for the CPU oracle: what the paper's layer definition and mathematics fix, none of it the oracle itself.

Each pin is a function `pin_*(conv)` taking a callable `conv(inp, w, bias, relu) -> fp64 array`, so the same
pins run (a) on the oracle, which must pass all of them, and (b) on deliberately wrong variants of a small
numpy reimplementation, each of which must be rejected by at least one pin -- evidence that a dropped term,
a wrong sign or index, or a transposed operand in the oracle would not go unnoticed.

Citations: layer equation and shapes -- Section IV; "valid" output size n-k+1 -- Sections II and IV; the
inverse transform of the point-wise product of equally padded transforms is the convolution -- Section III-A;
bias then transfer function when an output image is finished -- Section IV-A-3; rectified-linear -- Section V.
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers (no oracle code)
def _rng(seed):
    return np.random.default_rng(seed)


def _rand_layer(seed, S, f, fo, n, k, integer=False):
    r = _rng(seed)
    n3 = (n,) * 3 if np.isscalar(n) else tuple(n)
    k3 = (k,) * 3 if np.isscalar(k) else tuple(k)
    if integer:
        inp = r.integers(-4, 5, size=(S, f) + n3).astype(np.float32)
        w = r.integers(-3, 4, size=(fo, f) + k3).astype(np.float32)
        b = r.integers(-5, 6, size=fo).astype(np.float32)
    else:
        inp = r.uniform(-1, 1, size=(S, f) + n3).astype(np.float32)
        w = r.standard_normal((fo, f) + k3).astype(np.float32)
        b = r.standard_normal(fo).astype(np.float32)
    return inp, w, b


def _load_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([float(t) for t in line.split()])
    return np.array(rows)


# ----------------------------------------------------------------------------- the pins
def pin_golden_affine(conv):
    """Hand-derived worked example (tests/golden/affine_n3_k2.txt)."""
    x, y, z = np.meshgrid(np.arange(3), np.arange(3), np.arange(3), indexing="ij")
    inp = (1 + 9 * x + 3 * y + z).astype(np.float32)[None, None]
    w = np.arange(1, 9, dtype=np.float32).reshape(1, 1, 2, 2, 2)
    out = conv(inp, w, None, False)
    assert out.shape == (1, 1, 2, 2, 2)
    for xx, yy, zz, v in _load_rows("affine_n3_k2.txt"):
        assert out[0, 0, int(xx), int(yy), int(zz)] == v


def pin_golden_flip_1d(conv):
    """Hand-computed 1D example that separates convolution from cross-correlation."""
    inp = np.array([1, 2, 4, 8], dtype=np.float32).reshape(1, 1, 1, 1, 4)
    w = np.array([10, 1], dtype=np.float32).reshape(1, 1, 1, 1, 2)
    out = conv(inp, w, None, False)
    assert out.shape == (1, 1, 1, 1, 3)
    for zz, v in _load_rows("box_n4_k2_1d.txt"):
        assert out[0, 0, 0, 0, int(zz)] == v
    # the same line laid along x and along y
    for axis in (2, 3):
        shp_i = [1, 1, 1, 1, 1]
        shp_i[axis] = 4
        shp_w = [1, 1, 1, 1, 1]
        shp_w[axis] = 2
        o = conv(inp.reshape(shp_i), w.reshape(shp_w), None, False)
        assert o.ravel().tolist() == [21.0, 42.0, 84.0]


def pin_affine_moments(conv):
    """Affine image, arbitrary integer kernel: the sum collapses to kernel moments (closed form)."""
    n, k = (6, 5, 7), (3, 2, 4)
    r = _rng(11)
    w = r.integers(-3, 4, size=(2, 1) + k).astype(np.float32)
    gx, gy, gz = np.meshgrid(*[np.arange(t) for t in n], indexing="ij")
    c0, cx, cy, cz = 2.0, 5.0, -3.0, 7.0
    inp = (c0 + cx * gx + cy * gy + cz * gz).astype(np.float32)[None, None]
    out = conv(inp, w, None, False)
    a, b, c = np.meshgrid(*[np.arange(t) for t in k], indexing="ij")
    no = [n[d] - k[d] + 1 for d in range(3)]
    ox, oy, oz = np.meshgrid(*[np.arange(t) for t in no], indexing="ij")
    for j in range(2):
        wj = w[j, 0].astype(np.float64)
        m0, ma, mb, mc = wj.sum(), (a * wj).sum(), (b * wj).sum(), (c * wj).sum()
        exp = m0 * (c0 + cx * (ox + k[0] - 1) + cy * (oy + k[1] - 1) + cz * (oz + k[2] - 1)) \
            - cx * ma - cy * mb - cz * mc
        assert np.array_equal(out[0, j], exp)


def pin_delta_kernel(conv):
    """A kernel with a single unit tap at (a0,b0,c0) copies a shifted window of the matching input image."""
    S, f, n, k = 2, 3, (7, 6, 8), (3, 2, 4)
    inp, _, _ = _rand_layer(3, S, f, f, n, k)
    for tap in [(0, 1, 2), (2, 0, 3), (1, 1, 0)]:
        w = np.zeros((f, f) + k, dtype=np.float32)
        for j in range(f):
            w[j, (j + 1) % f, tap[0], tap[1], tap[2]] = 1.0     # output j reads input j+1: pins w[j][i] order
        out = conv(inp, w, None, False)
        no = [n[d] - k[d] + 1 for d in range(3)]
        for j in range(f):
            i = (j + 1) % f
            x0, y0, z0 = (k[0] - 1 - tap[0], k[1] - 1 - tap[1], k[2] - 1 - tap[2])
            exp = inp[:, i, x0:x0 + no[0], y0:y0 + no[1], z0:z0 + no[2]].astype(np.float64)
            assert np.array_equal(out[:, j], exp)


def pin_constant_input(conv):
    """Constant image c: every output voxel equals bias + c * (sum of the f kernels of that output image)."""
    S, f, fo, n, k = 1, 3, 2, 6, 3
    _, w, b = _rand_layer(5, S, f, fo, n, k, integer=True)
    inp = np.full((S, f, n, n, n), 3.0, dtype=np.float32)
    out = conv(inp, w, b, False)
    for j in range(fo):
        assert np.all(out[0, j] == b[j] + 3.0 * w[j].astype(np.float64).sum())


def pin_box_sums(conv):
    """All-ones kernel: outputs are box sums, obtained independently from a summed-volume table."""
    n, k = (7, 8, 6), (3, 4, 2)
    r = _rng(6)
    inp = r.integers(-9, 10, size=(1, 1) + n).astype(np.float32)
    w = np.ones((1, 1) + k, dtype=np.float32)
    out = conv(inp, w, None, False)[0, 0]
    sat = np.zeros(tuple(t + 1 for t in n))
    sat[1:, 1:, 1:] = inp[0, 0].astype(np.float64).cumsum(0).cumsum(1).cumsum(2)
    no = [n[d] - k[d] + 1 for d in range(3)]
    for x in range(no[0]):
        for y in range(no[1]):
            for z in range(no[2]):
                X, Y, Z = x + k[0], y + k[1], z + k[2]
                box = (sat[X, Y, Z] - sat[x, Y, Z] - sat[X, y, Z] - sat[X, Y, z]
                       + sat[x, y, Z] + sat[x, Y, z] + sat[X, y, z] - sat[x, y, z])
                assert out[x, y, z] == box


def pin_linearity_and_structure(conv):
    """Linear in the image and in the kernels; sum over input images; batch entries independent."""
    S, f, fo, n, k = 2, 3, 2, 6, 3
    inp1, w1, _ = _rand_layer(7, S, f, fo, n, k, integer=True)
    inp2, w2, _ = _rand_layer(8, S, f, fo, n, k, integer=True)
    o11 = conv(inp1, w1, None, False)
    assert np.array_equal(conv(inp1 + 2 * inp2, w1, None, False), o11 + 2 * conv(inp2, w1, None, False))
    assert np.array_equal(conv(inp1, w1 - 3 * w2, None, False), o11 - 3 * conv(inp1, w2, None, False))
    # O[s][j] = sum_i (single-image layer with kernel w[j][i])
    acc = np.zeros_like(o11)
    for i in range(f):
        acc += conv(inp1[:, i:i + 1], w1[:, i:i + 1], None, False)
    assert np.array_equal(acc, o11)
    # batch independence: entry s of a batched call equals the call on that entry alone
    for s in range(S):
        assert np.array_equal(conv(inp1[s:s + 1], w1, None, False)[0], o11[s])
    # output image j depends only on row j of the kernel bank
    for j in range(fo):
        assert np.array_equal(conv(inp1, w1[j:j + 1], None, False)[:, 0], o11[:, j])


def pin_translation(conv):
    """Shifting the image content by d shifts the output by d where both windows exist."""
    n, k, d = 9, 3, (2, 1, 3)
    inp, w, _ = _rand_layer(9, 1, 2, 2, n + 3, k, integer=True)
    big = conv(inp, w, None, False)
    sub = inp[:, :, d[0]:d[0] + n, d[1]:d[1] + n, d[2]:d[2] + n]
    small = conv(sub, w, None, False)
    m = n - k + 1
    assert np.array_equal(small, big[:, :, d[0]:d[0] + m, d[1]:d[1] + m, d[2]:d[2] + m])


def pin_separable(conv):
    """Kernel u (x) v (x) q: equals three successive 1D valid convolutions done with numpy.convolve."""
    n, k = (8, 7, 9), (3, 4, 2)
    r = _rng(10)
    inp = r.integers(-4, 5, size=n).astype(np.float32)
    u, v, q = [r.integers(-3, 4, size=t).astype(np.float64) for t in k]
    w = np.einsum("a,b,c->abc", u, v, q).astype(np.float32)
    out = conv(inp[None, None], w[None, None], None, False)[0, 0]
    t = np.apply_along_axis(lambda l: np.convolve(l, u, mode="valid"), 0, inp.astype(np.float64))
    t = np.apply_along_axis(lambda l: np.convolve(l, v, mode="valid"), 1, t)
    t = np.apply_along_axis(lambda l: np.convolve(l, q, mode="valid"), 2, t)
    assert np.array_equal(out, t)


def pin_degenerate_sizes(conv):
    """k = 1 is a per-voxel f' x f matrix product; k = n leaves one voxel, a flipped dot product."""
    S, f, fo, n = 2, 3, 4, 5
    inp, w, b = _rand_layer(12, S, f, fo, n, 1, integer=True)
    out = conv(inp, w, b, False)
    exp = np.einsum("ji,sixyz->sjxyz", w[:, :, 0, 0, 0].astype(np.float64), inp.astype(np.float64)) \
        + b.astype(np.float64)[None, :, None, None, None]
    assert np.array_equal(out, exp)
    inp, w, _ = _rand_layer(13, 1, 2, 2, 4, 4, integer=True)
    out = conv(inp, w, None, False)
    assert out.shape == (1, 2, 1, 1, 1)
    for j in range(2):
        assert out[0, j, 0, 0, 0] == np.sum(w[j].astype(np.float64)[:, ::-1, ::-1, ::-1] * inp[0])


def _dft_matrix(m, sign):
    idx = np.arange(m)
    return np.exp(sign * 2j * np.pi * np.outer(idx, idx) / m)


def pin_convolution_theorem(conv):
    """fp64 naive-DFT route: pad image and kernel to a common size m >= n, transform (explicit DFT matrices,
    no FFT library), multiply point-wise, inverse transform, crop [k-1, n-1].  Any common size works."""
    S, f, fo, n, k = 1, 2, 2, (6, 5, 7), (3, 2, 4)
    inp, w, _ = _rand_layer(14, S, f, fo, n, k)
    out = conv(inp, w, None, False)
    for extra in (0, 3):
        m = tuple(t + extra for t in n)
        F = [_dft_matrix(t, -1) for t in m]
        G = [_dft_matrix(t, +1) / t for t in m]

        def fwd(a):
            p = np.zeros(m, dtype=np.complex128)
            p[:a.shape[0], :a.shape[1], :a.shape[2]] = a
            return np.einsum("ax,by,cz,xyz->abc", F[0], F[1], F[2], p)

        for j in range(fo):
            acc = np.zeros(m, dtype=np.complex128)
            for i in range(f):
                acc += fwd(w[j, i]) * fwd(inp[0, i])
            full = np.einsum("xa,yb,zc,abc->xyz", G[0], G[1], G[2], acc)
            crop = full[k[0] - 1:n[0], k[1] - 1:n[1], k[2] - 1:n[2]]
            assert np.max(np.abs(crop.imag)) < 1e-12
            assert np.max(np.abs(crop.real - out[0, j])) < 1e-12


def pin_library_special_cases(conv):
    """scipy's direct valid convolution per (j, i) pair, and torch's fp64 conv3d with the kernel flipped."""
    from scipy.signal import convolve as sp_convolve
    import torch
    S, f, fo, n, k = 2, 3, 2, (7, 6, 8), (3, 3, 2)
    inp, w, b = _rand_layer(15, S, f, fo, n, k)
    out = conv(inp, w, b, False)
    for s in range(S):
        for j in range(fo):
            acc = np.zeros(out.shape[2:])
            for i in range(f):
                acc += sp_convolve(inp[s, i].astype(np.float64), w[j, i].astype(np.float64),
                                   mode="valid", method="direct")
            assert np.max(np.abs(acc + b[j] - out[s, j])) < 1e-12
    t = torch.nn.functional.conv3d(torch.from_numpy(inp).double(),
                                   torch.from_numpy(w).double().flip(2, 3, 4),
                                   torch.from_numpy(b).double())
    assert np.max(np.abs(t.numpy() - out)) < 1e-12


def pin_bias_and_transfer(conv):
    """Bias is per output image, added before the transfer function; ReLU = max(0, .)."""
    S, f, fo, n, k = 1, 2, 3, 6, 3
    inp, w, b = _rand_layer(16, S, f, fo, n, k, integer=True)
    lin = conv(inp, w, None, False)
    pre = conv(inp, w, b, False)
    assert np.array_equal(pre, lin + b.astype(np.float64)[None, :, None, None, None])
    act = conv(inp, w, b, True)
    assert np.array_equal(act, np.maximum(pre, 0.0))
    assert (pre < 0).any() and (pre > 0).any()
    # a bias large enough to lift everything above zero makes ReLU the identity ...
    big = np.full(fo, 1e4, dtype=np.float32)
    assert np.array_equal(conv(inp, w, big, True), lin + 1e4)
    # ... and one low enough zeroes the whole output
    assert not conv(inp, w, -big, True).any()


PINS = [pin_golden_affine, pin_golden_flip_1d, pin_affine_moments, pin_delta_kernel, pin_constant_input,
        pin_box_sums, pin_linearity_and_structure, pin_translation, pin_separable, pin_degenerate_sizes,
        pin_convolution_theorem, pin_library_special_cases, pin_bias_and_transfer]


# ----------------------------------------------------------------------------- the oracle passes every pin
@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_passes_pin(oracle, pin):
    pin(lambda inp, w, b, relu: oracle.conv3d(inp, w, b, relu=relu))


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_point_evaluator_passes_pin(oracle, pin):
    """The one-voxel-at-a-time evaluator, asked for every voxel, is held to the same pins."""
    def conv(inp, w, b, relu):
        S, fo = inp.shape[0], w.shape[0]
        no = [inp.shape[2 + d] - w.shape[2 + d] + 1 for d in range(3)]
        grid = np.stack(np.meshgrid(np.arange(S), np.arange(fo), *[np.arange(t) for t in no],
                                    indexing="ij"), -1).reshape(-1, 5)
        return oracle.conv3d_points(inp, w, b, grid, relu=relu).reshape(S, fo, *no)
    pin(conv)


def test_thread_count_does_not_change_result(oracle):
    inp, w, b = _rand_layer(17, 2, 3, 4, 9, 3)
    a = oracle.conv3d(inp, w, b, relu=True, nthreads=1)
    c = oracle.conv3d(inp, w, b, relu=True, nthreads=4)
    assert np.array_equal(a, c)


def test_oracle_rejects_bad_arguments(oracle):
    inp, w, b = _rand_layer(18, 1, 1, 1, 3, 4)      # kernel larger than image
    with pytest.raises(ValueError):
        oracle.conv3d(inp, w, b)
    inp, w, b = _rand_layer(18, 1, 1, 1, 4, 2)
    with pytest.raises(ValueError):
        oracle.conv3d_points(inp, w, b, np.array([[0, 0, 3, 0, 0]]))    # x = 3 is outside n' = 3


# ----------------------------------------------------------------------------- wrong variants are caught
def _variant(kind):
    """A small numpy layer with one planted mistake (kind) -- or none (kind == 'correct')."""
    def conv(inp, w, b, relu):
        inp = np.asarray(inp, dtype=np.float64)
        w = np.asarray(w, dtype=np.float64)
        S, f = inp.shape[:2]
        fo = w.shape[0]
        k = w.shape[2:]
        no = [inp.shape[2 + d] - k[d] + 1 for d in range(3)]
        out = np.zeros((S, fo, *no))
        ww = w
        if kind == "correlation":
            ww = w[:, :, ::-1, ::-1, ::-1]
        elif kind == "no_flip_z":
            ww = w[:, :, :, :, ::-1]
        elif kind == "no_flip_x":
            ww = w[:, :, ::-1]
        elif kind == "swap_kernel_xy" and k[0] == k[1]:
            ww = w.transpose(0, 1, 3, 2, 4)
        elif kind == "transpose_bank" and f == fo:
            ww = w.transpose(1, 0, 2, 3, 4)
        n_in = f - 1 if (kind == "drop_last_channel" and f > 1) else f
        for a in range(k[0]):
            for bb in range(k[1]):
                for c in range(k[2]):
                    x0, y0, z0 = k[0] - 1 - a, k[1] - 1 - bb, k[2] - 1 - c
                    if kind == "window_off_by_one" and a == k[0] - 1 and k[0] > 1:
                        x0 += 1
                    win = inp[:, :n_in, x0:x0 + no[0], y0:y0 + no[1], z0:z0 + no[2]]
                    if win.shape[2] != no[0]:
                        pad = np.zeros((S, n_in, no[0] - win.shape[2], no[1], no[2]))
                        win = np.concatenate([win, pad], 2)
                    out += np.einsum("ji,sixyz->sjxyz", ww[:, :n_in, a, bb, c], win)
        bv = np.zeros(fo) if b is None else np.asarray(b, dtype=np.float64)
        bv = bv[None, :, None, None, None]
        if kind == "bias_after_relu":
            return (np.maximum(out, 0) if relu else out) + bv
        if kind == "shared_bias":
            bv = np.full_like(bv, bv.ravel()[0])
        out = out + bv
        return np.maximum(out, 0) if relu else out
    return conv


def _rejected(conv):
    for pin in PINS:
        try:
            pin(conv)
        except AssertionError:
            return pin.__name__
    return None


def test_unmutated_variant_passes_all_pins():
    assert _rejected(_variant("correct")) is None


@pytest.mark.parametrize("kind", ["correlation", "no_flip_z", "no_flip_x", "swap_kernel_xy", "transpose_bank",
                                  "drop_last_channel", "window_off_by_one", "bias_after_relu", "shared_bias"])
def test_planted_mistake_is_rejected(kind):
    assert _rejected(_variant(kind)) is not None, f"no pin catches the mistake '{kind}'"
