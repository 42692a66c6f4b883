"""Pins for the pooling oracle (oracle/znni_ref_mpf.c): max pooling and max-pooling fragments of Section VI.

Nothing here re-types the oracle's loops: the expected values come from hand-worked fixtures, closed forms for
monotone images, single-spike images, library routines (torch max_pool3d on shifted crops, scipy's maximum
filter) and structural properties.  A small numpy variant with planted mistakes shows the pins reject them.
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    rows = []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([float(t) for t in line.split()])
    return rows


def _m(n, p):
    return tuple(a // b for a, b in zip(n, p))


def _frag(p, o):
    return (o[0] * p[1] + o[1]) * p[2] + o[2]


# Each pin takes mpf(inp[S,f,nx,ny,nz], p) -> [S*px*py*pz, f, mx, my, mz].

def pin_golden_1d(mpf):
    rows = _rows("mpf_1d_n5_p2.txt")
    img = np.array(rows[0], dtype=np.float32).reshape(1, 1, 1, 1, 5)
    out = mpf(img, (1, 1, 2))
    assert out.shape == (2, 1, 1, 1, 2)
    assert np.array_equal(out[:, 0, 0, 0, :], np.array(rows[1:3], dtype=np.float32))


def pin_golden_2d(mpf):
    rows = _rows("mpf_2d_n5x3_p2x2.txt")
    img = np.array(rows[:5], dtype=np.float32).reshape(1, 1, 1, 5, 3)
    out = mpf(img, (1, 2, 2))
    assert out.shape == (4, 1, 1, 2, 1)
    assert np.array_equal(out[:, 0, 0, :, 0], np.array(rows[5:9], dtype=np.float32))
    # the same image laid along (x, y) and (x, z) must give the same fragments: pins the axis roles
    out_xy = mpf(img.reshape(1, 1, 5, 3, 1), (2, 2, 1))
    assert np.array_equal(out_xy[:, 0, :, 0, 0], np.array(rows[5:9], dtype=np.float32))
    out_xz = mpf(img.reshape(1, 1, 5, 1, 3), (2, 1, 2))
    assert np.array_equal(out_xz[:, 0, :, 0, 0], np.array(rows[5:9], dtype=np.float32))


def pin_monotone_images(mpf):
    """Strictly increasing (decreasing) along every axis: the maximum of a block is its far (near) corner."""
    n, p = (11, 8, 9), (3, 1, 2)
    m = _m(n, p)
    g = np.meshgrid(*[np.arange(t) for t in n], indexing="ij")
    inc = (100 * g[0] + 10 * g[1] + g[2]).astype(np.float32)[None, None]
    dec = -inc
    oi, od = mpf(inc, p), mpf(dec, p)
    assert oi.shape == (6, 1) + m
    a = np.meshgrid(*[np.arange(t) for t in m], indexing="ij")
    for ox in range(p[0]):
        for oy in range(p[1]):
            for oz in range(p[2]):
                fr = _frag(p, (ox, oy, oz))
                far = 100 * (ox + p[0] * a[0] + p[0] - 1) + 10 * (oy + p[1] * a[1] + p[1] - 1) + (oz + p[2] * a[2] + p[2] - 1)
                near = 100 * (ox + p[0] * a[0]) + 10 * (oy + p[1] * a[1]) + (oz + p[2] * a[2])
                assert np.array_equal(oi[fr, 0], far.astype(np.float32))
                assert np.array_equal(od[fr, 0], -near.astype(np.float32))


def pin_single_spike(mpf):
    """One voxel at q is 1, the rest -1: fragment o shows the spike exactly at floor((q - o) / p) per axis,
    provided that block lies inside the fragment."""
    n, p = (7, 5, 11), (2, 3, 4)
    m = _m(n, p)
    for q in [(0, 0, 0), (6, 4, 10), (3, 2, 5), (1, 4, 6), (5, 1, 3)]:
        img = -np.ones((1, 1) + n, dtype=np.float32)
        img[(0, 0) + q] = 1.0
        out = mpf(img, p)
        for ox in range(p[0]):
            for oy in range(p[1]):
                for oz in range(p[2]):
                    o = (ox, oy, oz)
                    exp = -np.ones(m, dtype=np.float32)
                    pos = [(q[d] - o[d]) // p[d] if q[d] >= o[d] else -1 for d in range(3)]
                    if all(0 <= pos[d] < m[d] for d in range(3)):
                        exp[tuple(pos)] = 1.0
                    assert np.array_equal(out[_frag(p, o), 0], exp), (q, o)


def pin_window_one_is_identity(mpf):
    r = np.random.default_rng(3)
    inp = r.standard_normal((2, 3, 4, 5, 6)).astype(np.float32)
    assert np.array_equal(mpf(inp, (1, 1, 1)), inp)


def pin_batch_and_channel_layout(mpf):
    """Constant images tagged by (s, i): output tuple s*alpha + fragment holds image i's tag in channel i."""
    S, f, n, p = 3, 2, (5, 3, 7), (2, 2, 4)
    alpha = p[0] * p[1] * p[2]
    inp = np.empty((S, f) + n, dtype=np.float32)
    for s in range(S):
        for i in range(f):
            inp[s, i] = 10 * s + i
    out = mpf(inp, p)
    assert out.shape == (S * alpha, f) + _m(n, p)
    for s in range(S):
        for fr in range(alpha):
            for i in range(f):
                assert np.all(out[s * alpha + fr, i] == 10 * s + i)


def pin_library_max_pool_on_shifted_crops(mpf):
    """Fragment o is the ordinary strided max pooling (torch, floor mode) of the image cropped by o."""
    import torch
    S, f, n, p = 2, 2, (9, 11, 7), (2, 3, 2)
    r = np.random.default_rng(5)
    inp = r.standard_normal((S, f) + n).astype(np.float32)
    out = mpf(inp, p)
    alpha = p[0] * p[1] * p[2]
    t = torch.from_numpy(inp)
    for ox in range(p[0]):
        for oy in range(p[1]):
            for oz in range(p[2]):
                ref = torch.nn.functional.max_pool3d(t[:, :, ox:, oy:, oz:], kernel_size=p, stride=p).numpy()
                got = out[_frag(p, (ox, oy, oz))::alpha]
                assert np.array_equal(got, ref)


def pin_recombination_is_the_sliding_maximum(mpf):
    """Interleaving the fragments (voxel (a,b,c) of fragment o -> position o + p*(a,b,c)) gives the maximum over
    the window at every position of the image: the sliding-window result the fragments stand for."""
    from scipy.ndimage import maximum_filter
    n, p = (9, 8, 11), (2, 3, 4)
    r = np.random.default_rng(6)
    inp = r.standard_normal((1, 1) + n).astype(np.float32)
    out = mpf(inp, p)
    m = _m(n, p)
    dense = np.empty(tuple(p[d] * m[d] for d in range(3)), dtype=np.float32)
    for ox in range(p[0]):
        for oy in range(p[1]):
            for oz in range(p[2]):
                dense[ox::p[0], oy::p[1], oz::p[2]] = out[_frag(p, (ox, oy, oz)), 0]
    # scipy's maximum filter centres its window on each position; shifting the centre back by floor(p/2)
    # (origin) makes position x cover [x, x + p)
    full = maximum_filter(inp[0, 0], size=p, origin=tuple(-(t // 2) for t in p),
                          mode="constant", cval=-np.inf)
    assert np.array_equal(dense, full[:dense.shape[0], :dense.shape[1], :dense.shape[2]])
    # and without any library: maxima of shifted copies
    shifted = np.full(dense.shape, -np.inf, dtype=np.float32)
    for u in range(p[0]):
        for v in range(p[1]):
            for t in range(p[2]):
                shifted = np.maximum(shifted, inp[0, 0, u:u + dense.shape[0], v:v + dense.shape[1], t:t + dense.shape[2]])
    assert np.array_equal(dense, shifted)
    assert dense.shape == tuple(n[d] - p[d] + 1 for d in range(3))


MPF_PINS = [pin_golden_1d, pin_golden_2d, pin_monotone_images, pin_single_spike, pin_window_one_is_identity,
            pin_batch_and_channel_layout, pin_library_max_pool_on_shifted_crops,
            pin_recombination_is_the_sliding_maximum]


@pytest.mark.parametrize("pin", MPF_PINS, ids=lambda p: p.__name__)
def test_mpf_oracle_passes_pin(oracle, pin):
    pin(oracle.mpf)


def test_maxpool_oracle_against_hand_values_library_and_fragments(oracle):
    import torch
    # by hand: 1 x 2 x 4 image, window (1, 2, 2): blocks (1,5,2,0) -> 5 and (3,4,9,1) -> 9
    img = np.array([[1, 5, 3, 4], [2, 0, 9, 1]], dtype=np.float32).reshape(1, 1, 1, 2, 4)
    assert np.array_equal(oracle.maxpool(img, (1, 2, 2)).ravel(), [5, 9])
    r = np.random.default_rng(8)
    inp = r.standard_normal((2, 3, 6, 9, 8)).astype(np.float32)
    p = (2, 3, 4)
    out = oracle.maxpool(inp, p)
    assert np.array_equal(out, torch.nn.functional.max_pool3d(torch.from_numpy(inp), p, p).numpy())
    # the image with its last voxel per axis cut away satisfies the fragment size rule; its offset-0 fragment is
    # the max pooling without the last block per axis
    alpha = p[0] * p[1] * p[2]
    fr = oracle.mpf(inp[:, :, :-1, :-1, :-1], p)
    assert np.array_equal(fr[0::alpha], out[:, :, :-1, :-1, :-1])


def test_pooling_oracles_reject_bad_shapes(oracle):
    x = np.zeros((1, 1, 6, 6, 6), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.mpf(x, (2, 2, 2))           # 6 + 1 not divisible by 2
    with pytest.raises(ValueError):
        oracle.maxpool(x, (4, 2, 2))       # 6 not divisible by 4
    with pytest.raises(ValueError):
        oracle.mpf(x[:, :, :5, :5, :5], (2, 2, 0))
    assert oracle.mpf(x[:, :, :5, :5, :], (2, 3, 1)).shape == (6, 1, 2, 1, 6)


# ----------------------------------------------------------------------------- wrong variants are caught
def _variant(kind):
    def mpf(inp, p):
        inp = np.asarray(inp, dtype=np.float32)
        S, f = inp.shape[:2]
        n = inp.shape[2:]
        m = _m(n, p)
        alpha = p[0] * p[1] * p[2]
        out = np.empty((S * alpha, f) + m, dtype=np.float32)
        for ox in range(p[0]):
            for oy in range(p[1]):
                for oz in range(p[2]):
                    o = [ox, oy, oz]
                    if kind == "offset_from_far_end":
                        o = [p[d] - 1 - o[d] for d in range(3)]
                    w = list(p)
                    if kind == "window_too_short" and p[2] > 1:
                        w[2] -= 1
                    acc = None
                    for u in range(w[0]):
                        for v in range(w[1]):
                            for t in range(w[2]):
                                sl = inp[:, :, o[0] + u::p[0], o[1] + v::p[1], o[2] + t::p[2]][:, :, :m[0], :m[1], :m[2]]
                                if kind == "min_instead_of_max":
                                    acc = sl if acc is None else np.minimum(acc, sl)
                                else:
                                    acc = sl if acc is None else np.maximum(acc, sl)
                    fr = (ox * p[1] + oy) * p[2] + oz
                    if kind == "x_offset_fastest":
                        fr = (oz * p[1] + oy) * p[0] + ox
                    if kind == "fragment_major_batch":
                        out[fr * S:(fr + 1) * S] = acc
                    else:
                        out[fr::alpha] = acc
        return out
    return mpf


def _rejected(fn):
    for pin in MPF_PINS:
        try:
            pin(fn)
        except AssertionError:
            return pin.__name__
    return None


def test_unmutated_mpf_variant_passes_all_pins():
    assert _rejected(_variant("correct")) is None


@pytest.mark.parametrize("kind", ["offset_from_far_end", "window_too_short", "min_instead_of_max",
                                  "x_offset_fastest", "fragment_major_batch"])
def test_planted_mpf_mistake_is_rejected(kind):
    assert _rejected(_variant(kind)) is not None, f"no pin catches the mistake '{kind}'"
