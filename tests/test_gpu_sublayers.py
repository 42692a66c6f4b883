"""GPU parity of the layer computed as sub-layers under a workspace budget (Section VII-A) against the fp64 oracle,
to the same per-voxel bar as the whole-layer call, plus agreement with the whole-layer result."""
import sys

import numpy as np
import pytest
import torch

from paper_1606_05688_amd import binding as B

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


# (S, f, fo, n, k, fraction of the whole-layer workspace, expected kind of division)
CASES = [
    (5, 3, 4, (20, 20, 20), (3, 3, 3), 1.00, "whole"),
    (5, 3, 4, (20, 20, 20), (3, 3, 3), 0.55, "batches"),      # S_i = 2: chunks 2, 2, 1
    (5, 3, 4, (20, 20, 20), (3, 3, 3), 0.40, "batches"),      # S_i = 1
    (1, 24, 40, (24, 20, 16), (3, 5, 2), 0.60, "blocks"),     # blocks of input and output images, ragged last blocks
    (1, 24, 40, (24, 20, 16), (3, 5, 2), 0.25, "blocks"),
    (2, 10, 21, (16, 16, 16), (5, 5, 5), 0.30, "blocks"),     # S > 1 but not even one whole input fits
    (1, 7, 5, (33, 17, 21), (4, 2, 3), 0.70, "blocks"),       # padded transform sizes, blocks below the tile sizes
    (1, 48, 48, (16, 16, 16), (7, 7, 7), 0.30, "blocks"),     # specialised multiply-accumulate kernel (k = 7)
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "S%d_f%dx%d_n%s_k%s_%d%%" % (c[0], c[1], c[2], "x".join(map(str, c[3])), "x".join(map(str, c[4])), int(100 * c[5])))
def test_budgeted_layer_matches_oracle(oracle, case):
    S, f, fo, n, k, frac, kind = case
    full = B.znni_conv3d_fft_workspace(S, f, fo, n, k)
    budget = int(full * frac)
    sub, need = B.znni_conv3d_fft_sublayers(S, f, fo, n, k, budget)
    _say(f"[sublayers] {case}: division S_i={sub[0]} f_i={sub[1]} f'_i={sub[2]}, {need} of {budget} bytes")
    assert need <= budget
    if kind == "whole":
        assert sub == (S, f, fo)
    elif kind == "batches":
        assert sub[0] < S and sub[1:] == (f, fo)
    else:
        assert sub[0] == 1 and (sub[1] < f or sub[2] < fo)
    inp, w, b = _rand(40 + f + fo, S, f, fo, n, k)
    d = torch.device("cuda:0")
    ti, tw, tb = (torch.from_numpy(t).to(d) for t in (inp, w, b))
    ws = torch.empty(budget + 256, dtype=torch.uint8, device=d)
    ws.fill_(0xFF)                                   # NaN patterns: nothing may be read before it is written
    ws = ws[:budget]
    got = B.znni_conv3d_fft_budget(ti, tw, tb, relu=True, workspace=ws)
    whole = B.znni_conv3d_fft(ti, tw, tb, relu=True)
    torch.cuda.synchronize()
    exp = oracle.conv3d(inp, w, b, relu=True)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    err = np.abs(got.cpu().numpy().astype(np.float64) - exp)
    _say(f"    max err/tol {np.max(err / tol):.3e}")
    assert np.all(err <= tol)
    assert np.all(np.abs((got - whole).cpu().numpy()) <= 0.1 * tol)
    if kind != "blocks":
        assert torch.equal(got, whole)               # same arithmetic per input: bitwise equal


def test_largest_benchmark_layer_under_half_its_workspace(largest_layer_case):
    """The division the benchmark times: 48 -> 48 images of 320^3 with half of the whole-layer workspace, i.e.
    blocks of input and output images whose products are added into output spectra that live in a buffer of
    their own.  Compared with the whole-layer result on every voxel and with the oracle on the declared sample."""
    C = largest_layer_case
    L = C.layer
    n, k = (L.n,) * 3, (L.k,) * 3
    budget = B.znni_conv3d_fft_workspace(L.S, L.f, L.fo, n, k) // 2
    sub, need = B.znni_conv3d_fft_sublayers(L.S, L.f, L.fo, n, k, budget)
    _say(f"[sublayers] {L.name}: division S_i={sub[0]} f_i={sub[1]} f'_i={sub[2]}, {need} of {budget} bytes")
    assert sub[0] == 1 and sub[1] < L.f and sub[2] < L.fo
    d = torch.device("cuda:0")
    ti, tw, tb = (torch.from_numpy(t).to(d) for t in (C.inp, C.w, C.bias))
    ws = torch.empty(budget, dtype=torch.uint8, device=d)
    ws.fill_(0xFF)
    got = B.znni_conv3d_fft_budget(ti, tw, tb, relu=L.relu, workspace=ws)
    torch.cuda.synchronize()
    del ws
    whole = B.znni_conv3d_fft(ti, tw, tb, relu=L.relu)
    torch.cuda.synchronize()
    tj = torch.from_numpy(C.tol_j).to(d).float()[None, :, None, None, None]
    worst = float(((got - whole).abs() / tj).max())
    _say(f"    all {got.numel()} voxels: max |budget - whole| / tol = {worst:.3e}")
    assert worst <= 0.1
    tp = torch.from_numpy(C.pts.astype(np.int64)).to(d)
    g = got[tp[:, 0], tp[:, 1], tp[:, 2], tp[:, 3], tp[:, 4]].cpu().numpy().astype(np.float64)
    ratio = np.abs(g - C.exp) / C.tol
    _say(f"    {len(C.pts)} sampled voxels against the oracle: max err/tol {ratio.max():.3e}")
    assert np.all(ratio <= 1.0)


def test_blocks_accumulate_with_either_multiply_accumulate_form(oracle):
    S, f, fo, n, k = 1, 24, 40, (24, 20, 16), (3, 5, 2)
    budget = int(0.25 * B.znni_conv3d_fft_workspace(S, f, fo, n, k))
    inp, w, b = _rand(99, S, f, fo, n, k)
    d = torch.device("cuda:0")
    ti, tw, tb = (torch.from_numpy(t).to(d) for t in (inp, w, b))
    ws = torch.empty(budget, dtype=torch.uint8, device=d)
    exp = oracle.conv3d(inp, w, b, relu=True)
    tol = oracle.tolerance(inp, w)[None, :, None, None, None]
    for form in ("single", "batch", "reference", "xdirect", "xblock"):
        got = B.znni_conv3d_fft_budget(ti, tw, tb, relu=True, workspace=ws, mac_reference=form)
        torch.cuda.synchronize()
        assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - exp) <= tol), form


def test_budget_too_small_is_reported_not_run():
    S, f, fo, n, k = 1, 8, 8, (32, 32, 32), (3, 3, 3)
    with pytest.raises(B.ZnniError) as e:
        B.znni_conv3d_fft_sublayers(S, f, fo, n, k, 4096)
    assert e.value.status == -4
    d = torch.device("cuda:0")
    inp = torch.zeros((S, f) + n, device=d)
    w = torch.zeros((fo, f) + k, device=d)
    ws = torch.empty(4096, dtype=torch.uint8, device=d)
    with pytest.raises(B.ZnniError) as e:
        B.znni_conv3d_fft_budget(inp, w, None, workspace=ws)
    assert e.value.status == -4
