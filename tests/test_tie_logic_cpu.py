"""CPU checks of the tie handling the GPU parity tests use (tests/gpu_common.py): the tie set and
the admissible alternatives come from the oracle's pre-activations alone; another implementation's
ReLU / max-pool decisions are only compared against them.

A float32 PyTorch forward on the CPU stands in for "an implementation that accumulates in another
precision"; decisions are then planted by hand, inside and outside the band."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as O
import workloads
from tests import gpu_common as G


def _spec(pool=None, H=8, C=6, K=8, A=4):
    ls = workloads.LayerSpec("t", C, H, H, K, A=A)
    if pool:
        ls.pool_kind, ls.pool_k, ls.pool_stride, ls.pool_pad = 1, *pool
    return ls


def _inputs(ls, B=3, cls=5, seed=3):
    g = workloads.rng_for(seed, "tie-cpu", ls.C_in, ls.H_in, ls.pool_kind)
    x = g.standard_normal((B, ls.C_in, ls.H_in, ls.W_in)).astype(np.float32)
    labels = g.integers(0, cls, size=(B,)).astype(np.int32)
    p = workloads.gen_layer_params(seed, 0, ls, cls, bias_std=0.2)
    return x, labels, p


def _descs(ls, cls, head_pool=0):
    af = ls.aux_desc_fields(cls)
    af["head_pool"] = head_pool
    return O.layer_desc(**ls.layer_desc_fields()), O.aux_desc(**af)


def _f32_decisions(ls, oa, x, p):
    """Decisions of a float32 forward (torch, CPU) in the oracle's index convention."""
    t = {k: torch.from_numpy(v) for k, v in p.items() if v is not None}
    z = F.conv2d(torch.from_numpy(x), t["W"], t["b"], stride=ls.stride, padding=ls.pad)
    y = torch.relu(z)
    arg = None
    if ls.pool_kind:
        y, arg = F.max_pool2d(y, ls.pool_k, ls.pool_stride, ls.pool_pad, return_indices=True)
        arg = arg.numpy().astype(np.int32)
    u = torch.relu(F.conv2d(y, t["Wa"], t["ba"], padding=1))
    parg = None
    if oa.head_pool == 1:
        _, pi = F.adaptive_max_pool2d(u, (oa.pool_oh, oa.pool_ow), return_indices=True)
        parg = pi.numpy().reshape(x.shape[0], -1).astype(np.int32)
    return (u.numpy() > 0), y.numpy(), arg, parg


def _own_decisions(od, oa, x, p, labels):
    """The oracle's own decisions, laid out like another implementation's would be."""
    lf = O.layer_fwd(od, x, None, p["W"], p["b"], p["Wp"])
    af = O.aux_fwd_loss(oa, lf.Y, labels, p["Wa"], p["ba"], p["Wf"], p["bf"])
    return lf, af, [af.Upre > 0, lf.Y.copy(), None if lf.arg is None else lf.arg.copy(),
                    af.parg.copy() if oa.head_pool == 1 else None]


def _step(od, oa, ls, x, labels, p, dec):
    po = {k: (None if v is None else v.copy()) for k, v in p.items()}
    return G.oracle_step(od, oa, ls, x, None, labels, po, None, 0.0, 0.0, tuple(dec))


@pytest.mark.parametrize("pool", [None, (2, 2, 0), (3, 2, 1)])
@pytest.mark.parametrize("head_pool", [0, 1])
def test_float32_forward_is_accepted_and_matches(pool, head_pool):
    ls = _spec(pool)
    od, oa = _descs(ls, 5, head_pool)
    x, labels, p = _inputs(ls)
    _, _, g, ties = _step(od, oa, ls, x, labels, p, _f32_decisions(ls, oa, x, p))
    assert ties.differ == 0, str(ties)          # random data: no pre-activation that close to zero
    _, _, g_own = O.local_step(od, oa, x, None, labels, {k: (None if v is None else v.copy()) for k, v in p.items()},
                               None, 0.0, 0.0)
    for k in g_own:
        if g_own[k] is not None:
            assert np.array_equal(g[k], g_own[k]), k   # no alternative taken: the oracle's own gradients


def test_relu_flip_inside_the_band_is_an_admissible_outcome():
    ls = _spec()
    od, oa = _descs(ls, 5)
    x, labels, p = _inputs(ls)
    lf, _, _ = _own_decisions(od, oa, x, p, labels)
    e = (1, 2, 3, 4)
    others = np.abs(np.delete(lf.Z[:, e[1]].ravel(), np.ravel_multi_index((e[0], e[2], e[3]), lf.Z[:, 0].shape)))
    p["b"][e[1]] -= lf.Z[e]                      # that pre-activation is now zero to within rounding
    lf, af, dec = _own_decisions(od, oa, x, p, labels)
    band = G.tie_band(lf.Z, 9 * ls.C_in)
    assert abs(lf.Z[e]) <= band < others.min()
    on = lf.Z[e] > 0
    dec[1][e] = 0.0 if on else 1.0               # the other implementation took the other branch
    _, _, g, ties = _step(od, oa, ls, x, labels, p, dec)
    assert ties.differ == 1 and ties.in_band >= 1
    mz = lf.Z > 0
    mz[e] = not on
    ref = O.local_bwd(od, oa, x, None, lf, af, p["Wa"], p["Wf"], mask_u=af.Upre > 0, mask_z=mz)
    base = O.local_bwd(od, oa, x, None, lf, af, p["Wa"], p["Wf"])
    assert np.array_equal(g["W"], ref["W"]) and np.array_equal(g["b"], ref["b"])
    assert not np.array_equal(ref["b"], base["b"])


@pytest.mark.parametrize("which", ["layer", "aux"])
def test_relu_flip_outside_the_band_fails(which):
    ls = _spec()
    od, oa = _descs(ls, 5)
    x, labels, p = _inputs(ls)
    lf, af, dec = _own_decisions(od, oa, x, p, labels)
    if which == "layer":
        e = np.unravel_index(np.argmin(np.abs(lf.Z)), lf.Z.shape)   # the closest call of the whole tensor
        assert abs(lf.Z[e]) > G.tie_band(lf.Z, 9 * ls.C_in)
        dec[1][e] = 0.0 if lf.Z[e] > 0 else 1.0
    else:
        e = np.unravel_index(np.argmin(np.abs(af.Upre)), af.Upre.shape)
        assert abs(af.Upre[e]) > G.tie_band(af.Upre, 9 * ls.C_out)
        dec[0][e] = not dec[0][e]
    with pytest.raises(AssertionError, match="outside the tie band"):
        _step(od, oa, ls, x, labels, p, dec)


@pytest.mark.parametrize("pool", [(2, 2, 0), (3, 2, 1)])
def test_pool_routing_ties(pool):
    ls = _spec(pool, K=2)                        # two channels: the planted ties stay under the cap
    od, oa = _descs(ls, 5)
    x, labels, p = _inputs(ls)
    x[0, :, 0:5, 0:5] = 0.7                      # constant patch: conv outputs (1..3, 1..3) are exactly equal
    p["b"][:] = np.abs(p["b"]) + 4.0             # ... and positive in every channel
    lf, af, dec = _own_decisions(od, oa, x, p, labels)
    Wo = ls.Wo
    cell = (0, 1, 1, 1)                          # a window inside the constant patch
    t0 = int(lf.arg[cell])
    alt = t0 + 1 if pool[0] == 2 else t0 + Wo    # another cell of the same window, same value
    assert lf.Z[0, 1].ravel()[alt] == lf.Z[0, 1].ravel()[t0] > 0
    dec[2][cell] = alt
    _, _, g, ties = _step(od, oa, ls, x, labels, p, dec)
    assert ties.differ == 1 and ties.in_band >= 1
    arg2 = lf.arg.copy()
    arg2[cell] = alt
    ref = O.local_bwd(od, oa, x, None, O.LayerFwd(lf.Z, lf.Y, arg2), af, p["Wa"], p["Wf"])
    assert np.array_equal(g["W"], ref["W"])
    # routing to a cell of clearly lower value is no admissible alternative
    lf, af, dec = _own_decisions(od, oa, x, p, labels)
    cell = (1, 0, 2, 2)
    win = G._pool_windows(lf.Z, ls)[cell]
    hh = cell[2] * pool[1] - pool[2] + np.arange(pool[0])[:, None]
    ww = cell[3] * pool[1] - pool[2] + np.arange(pool[0])[None, :]
    flat = (hh * Wo + ww).ravel()
    worst = int(flat[np.argmin(np.where(np.isfinite(win), win, np.inf))])
    assert worst != lf.arg[cell]
    dec[2][cell] = worst
    dec[1][cell] = max(float(lf.Z[1, 0].ravel()[worst]), 1e-3)   # "on", through the wrong cell
    with pytest.raises(AssertionError, match="outside the tie band"):
        _step(od, oa, ls, x, labels, p, dec)


def test_caps_bound_the_tie_set_and_the_differing_decisions():
    s = G.TieStats()
    cap_t, cap_d = G.tie_caps(1_000_000)
    s.add("x", cap_t, cap_d, 1_000_000)
    with pytest.raises(AssertionError, match="inside the tie band"):
        s.add("x", cap_t + 1, 0, 1_000_000)
    with pytest.raises(AssertionError, match="differ"):
        s.add("x", 0, cap_d + 1, 1_000_000)


def test_band_is_about_1e_6_of_the_largest_value():
    g = np.random.default_rng(0)
    z = g.standard_normal(1_000_000)
    for K in (27, 576, 4608):
        b = G.tie_band(z, K)
        assert 1e-7 * np.abs(z).max() < b < 4e-6 * np.abs(z).max()
        assert (np.abs(z) <= b).sum() <= G.tie_caps(z.size)[0]
