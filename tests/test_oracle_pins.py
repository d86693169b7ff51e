"""Pins for the CPU oracle (no GPU): what the paper and the mathematics fix.

Each test is chosen so that a plausible slip in ``oracle/nfo.cpp`` (dropped term, wrong sign
or index, transposed operand, wrong window) fails at least one of them.
"""
import math
import os
from types import SimpleNamespace

import numpy as np
import pytest

import workloads
from tests import torch_ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _spec(C=2, H=5, W=5, K=3, A=2, R=3, S=3, stride=1, pad=1, pool=None, skip=0):
    ls = workloads.LayerSpec("t", C, H, W, K, R=R, S=S, stride=stride, pad=pad, A=A)
    if pool:
        ls.pool_kind, ls.pool_k, ls.pool_stride, ls.pool_pad = 1, *pool
    if skip == 1:
        ls.skip_kind, ls.skip_C, ls.skip_H, ls.skip_W, ls.skip_stride = 1, K, ls.Ho, ls.Wo, 1
    elif skip == 2:
        ls.skip_kind, ls.skip_C, ls.skip_stride = 2, 4, 2
        ls.skip_H, ls.skip_W = ls.Ho * 2, ls.Wo * 2 - 1  # odd width: last column never sampled
    return ls


def _setup(o, ls, B=2, Cls=3, seed=7, dtype=np.float64, relu=1, head_pool=0, loss_kind=0):
    d = o.layer_desc(**ls.layer_desc_fields())
    af = ls.aux_desc_fields(Cls)
    af["relu"] = relu
    af["head_pool"], af["loss_kind"] = head_pool, loss_kind
    a = o.aux_desc(**af)
    g = workloads.rng_for(seed, "pin", ls.C_in, ls.H_in, ls.C_out, ls.stride, ls.pool_kind, ls.skip_kind)
    x = g.standard_normal((B, ls.C_in, ls.H_in, ls.W_in)).astype(dtype)
    xs = None
    if ls.skip_kind:
        xs = g.standard_normal((B, ls.skip_C, ls.skip_H, ls.skip_W)).astype(dtype)
    labels = g.integers(0, Cls, size=(B,)).astype(np.int32)
    p = workloads.gen_layer_params(seed, 0, ls, Cls, dtype=dtype, bias_std=0.3)
    return d, a, x, xs, labels, p


def _loss(o, d, a, x, xs, labels, p):
    lf = o.layer_fwd(d, x, xs, p["W"], p["b"], p["Wp"])
    return o.aux_fwd_loss(a, lf.Y, labels, p["Wa"], p["ba"], p["Wf"], p["bf"]).loss


def _grads(o, d, a, x, xs, labels, p):
    lf = o.layer_fwd(d, x, xs, p["W"], p["b"], p["Wp"])
    af = o.aux_fwd_loss(a, lf.Y, labels, p["Wa"], p["ba"], p["Wf"], p["bf"])
    return lf, af, o.local_bwd(d, a, x, xs, lf, af, p["Wa"], p["Wf"])


SHAPES = {
    "plain5x5": dict(),
    "hp4": dict(H=4, W=4),
    "hp3_odd_overlap": dict(H=3, W=3),
    "hp2": dict(H=2, W=2),
    "hp1": dict(H=1, W=1),
    "rect": dict(H=6, W=3),
    "stride2": dict(H=7, W=6, stride=2),
    "pool2": dict(H=6, W=6, pool=(2, 2, 0)),
    "pool2_to1": dict(H=2, W=2, pool=(2, 2, 0)),
    "pool3s2p1": dict(H=7, W=7, pool=(3, 2, 1)),
    "stem7x7": dict(H=9, W=9, R=7, S=7, stride=2, pad=3, pool=(3, 2, 1)),
    "skip_identity": dict(C=3, K=3, skip=1),
    "skip_proj": dict(H=4, W=4, skip=2),
    "conv1x1": dict(R=1, S=1, pad=0),
}


# ---- P0: central finite differences of the loss, float64 -----------------------------------
@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("relu", [1, 0])
def test_finite_difference_gradients(oracle, name, relu):
    o = oracle
    if relu == 0 and name not in ("plain5x5", "pool2", "skip_proj"):
        pytest.skip("relu=0 variant checked on three shapes")
    ls = _spec(**SHAPES[name])
    d, a, x, xs, labels, p = _setup(o, ls, relu=relu)
    _, _, g = _grads(o, d, a, x, xs, labels, p)
    h = 1e-6
    for key in o.PARAM_NAMES:
        if p[key] is None:
            continue
        flat = p[key].reshape(-1)
        num = np.zeros_like(flat)
        for e in range(flat.size):
            keep = flat[e]
            flat[e] = keep + h
            lp = _loss(o, d, a, x, xs, labels, p)
            flat[e] = keep - h
            lm = _loss(o, d, a, x, xs, labels, p)
            flat[e] = keep
            num[e] = (lp - lm) / (2 * h)
        ana = g[key].reshape(-1)
        scale = max(np.abs(num).max(), 1e-3)
        assert np.abs(num - ana).max() <= 2e-6 * scale + 1e-8, (name, key, np.abs(num - ana).max(), scale)


# ---- library pin: the same step through PyTorch autograd (float64) --------------------------
@pytest.mark.parametrize("name", list(SHAPES))
def test_matches_torch_autograd(oracle, name):
    o = oracle
    ls = _spec(**SHAPES[name])
    d, a, x, xs, labels, p = _setup(o, ls, B=3, Cls=4, seed=11)
    lr, mu = 0.05, 0.9
    ref, final = torch_ref.local_step(SimpleNamespace(**ls.layer_desc_fields()),
                                      SimpleNamespace(**ls.aux_desc_fields(4)), x, xs, labels, p,
                                      lr, mu, steps=3)
    mom = {k: (None if v is None else np.zeros_like(v)) for k, v in p.items()}
    for step in range(3):
        Y, loss, g = o.local_step(d, a, x, xs, labels, p, mom, lr, mu)
        rl, rg, ry = ref[step]
        assert abs(loss - rl) <= 1e-12 * max(1, abs(rl))
        np.testing.assert_allclose(Y, ry, rtol=1e-12, atol=1e-13)
        for k in rg:
            np.testing.assert_allclose(g[k], rg[k], rtol=1e-9, atol=1e-12, err_msg=f"{name}:{k}:{step}")
    for k in final:
        np.testing.assert_allclose(p[k], final[k], rtol=1e-10, atol=1e-12, err_msg=f"{name}:{k}")


# ---- P1: the activation-size series printed in Fig. 13 (left) -------------------------------
def test_fig13_activation_sizes(oracle):
    series = {}
    for line in open(os.path.join(GOLDEN, "fig13_left_activation_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, *vals = line.split()
        series[name] = [int(v) for v in vals]
    vgg19 = workloads.vgg_layers([64, 64, 128, 128, 256, 256, 256, 256, 512, 512, 512, 512, 512, 512, 512, 512],
                                 {2, 4, 8, 12, 16})
    r18 = workloads.resnet_layers([2, 2, 2, 2])
    assert len(vgg19) == 16 and len(r18) == 17  # every convolution is its own local layer

    def sizes(layers):
        out = []
        for ls in layers:
            d = oracle.layer_desc(**ls.layer_desc_fields())
            Ho, Wo, Hp, Wp = oracle.layer_dims(d)
            assert (Ho, Wo, Hp, Wp) == (ls.Ho, ls.Wo, ls.Hp, ls.Wp)
            out.append(5 * ls.C_out * Hp * Wp)
        return out

    assert sizes(vgg19) == series["vgg19"]
    got = sizes(r18)
    assert got[:16] == series["resnet18"][:16]
    # The figure's last ResNet entry is after the backbone's global pooling (512*1*1*5); the
    # local layer itself emits 512x4x4 here (no global pool is attached to a local layer).
    assert got[16] == 5 * 512 * 4 * 4 and series["resnet18"][16] == 5 * 512


# ---- P2: zero linear weights => loss = ln(classes), and zeros propagate ---------------------
@pytest.mark.parametrize("Cls,expect", [(10, 2.302585), (100, 4.605170), (200, 5.298317)])
def test_ce_is_log_classes_at_zero_fc(oracle, Cls, expect):
    o = oracle
    ls = _spec(H=4, W=4)
    d, a, x, xs, labels, p = _setup(o, ls, B=4, Cls=Cls)
    p["Wf"][:] = 0
    p["bf"][:] = 0
    lf, af, g = _grads(o, d, a, x, xs, labels, p)
    assert abs(af.loss - math.log(Cls)) < 1e-12 and abs(af.loss - expect) < 1e-6
    want = np.full((4, Cls), 1.0 / Cls)
    want[np.arange(4), labels] -= 1.0
    np.testing.assert_allclose(af.dz, want / 4, rtol=0, atol=1e-15)
    assert np.all(g["Wa"] == 0) and np.all(g["W"] == 0) and np.all(g["b"] == 0) and np.all(g["ba"] == 0)
    np.testing.assert_allclose(g["bf"], af.dz.sum(0), atol=1e-15)


# ---- P3: locality ---------------------------------------------------------------------------
def test_locality_of_loss_and_gradients(oracle):
    o = oracle
    l1 = _spec(C=2, H=6, W=6, K=4)
    l2 = _spec(C=4, H=6, W=6, K=3)
    d1, a1, x, _, labels, p1 = _setup(o, l1, seed=1)
    d2, a2, _, _, _, p2 = _setup(o, l2, seed=2)
    x0 = x.copy()
    Y1, loss1, g1 = o.local_step(d1, a1, x, None, labels, {k: (None if v is None else v.copy()) for k, v in p1.items()}, None, 0.1, 0.0)
    assert np.array_equal(x, x0)  # the step writes nothing into its input
    # layer 2 trained from Y1 with two different sets of layer-2 parameters: layer 1 unaffected
    for scale in (1.0, -3.0):
        q2 = {k: (None if v is None else v * scale) for k, v in p2.items()}
        o.local_step(d2, a2, Y1, None, labels, q2, None, 0.1, 0.0)
        Y1b, loss1b, g1b = o.local_step(d1, a1, x, None, labels, {k: (None if v is None else v.copy()) for k, v in p1.items()}, None, 0.1, 0.0)
        assert loss1b == loss1 and np.array_equal(Y1, Y1b)
        for k in g1:
            if g1[k] is not None:
                assert np.array_equal(g1[k], g1b[k])


# ---- P4 / P5: cache equivalence and re-batching --------------------------------------------
def test_cache_equivalence_and_rebatching(oracle):
    o = oracle
    N, Cls = 10, 3
    l1 = _spec(C=2, H=6, W=6, K=4, pool=(2, 2, 0))
    l2 = _spec(C=4, H=3, W=3, K=3)
    d1, a1, _, _, _, p1 = _setup(o, l1, seed=1, dtype=np.float32)
    d2, a2, _, _, _, p2 = _setup(o, l2, seed=2, dtype=np.float32)
    g = workloads.rng_for(5, "cache")
    X = g.standard_normal((N, 2, 6, 6)).astype(np.float32)
    L = g.integers(0, Cls, size=(N,)).astype(np.int32)
    # train block 1 for a few steps at batch 4 (last batch partial), then freeze it
    for first in (0, 4, 8):
        o.local_step(d1, a1, X[first:first + 4], None, L[first:first + 4], p1, None, 0.05, 0.0)
    # fill the cache with the frozen weights, written in batches of 4,4,2
    cache = np.full((N, 4 * 3 * 3), np.nan, np.float32)
    clab = np.full((N,), -1, np.int32)
    for first in (0, 4, 8):
        y = o.layer_fwd(d1, X[first:first + 4], None, p1["W"], p1["b"]).Y
        o.cache_write(cache, clab, first, y, L[first:first + 4])
    full = o.layer_fwd(d1, X, None, p1["W"], p1["b"]).Y
    assert np.array_equal(cache, full.reshape(N, -1)) and np.array_equal(clab, L)
    # read at a different batch size (3: does not divide 10) and by a shuffled index list
    got = np.concatenate([o.cache_read(cache, clab, f, None, min(3, N - f), (4, 3, 3))[0] for f in range(0, N, 3)])
    assert np.array_equal(got, full)
    idx = np.array([7, 0, 9, 3, 3, 5], np.int64)
    xb, lb = o.cache_read(cache, clab, 0, idx, 6, (4, 3, 3))
    assert np.array_equal(xb, full[idx]) and np.array_equal(lb, L[idx])
    # one local step of block 2 from the cache == from recomputing block 1 forward on raw inputs
    pa = {k: (None if v is None else v.copy()) for k, v in p2.items()}
    pb = {k: (None if v is None else v.copy()) for k, v in p2.items()}
    Ya, la, ga = o.local_step(d2, a2, xb, None, lb, pa, None, 0.05, 0.0)
    recomputed = o.layer_fwd(d1, X[idx], None, p1["W"], p1["b"]).Y
    Yb, lbs, gb = o.local_step(d2, a2, recomputed, None, L[idx], pb, None, 0.05, 0.0)
    assert la == lbs and np.array_equal(Ya, Yb)
    for k in pa:
        if pa[k] is not None:
            assert np.array_equal(pa[k], pb[k]) and np.array_equal(ga[k], gb[k])


# ---- P6: ReLU and max-pool commute -----------------------------------------------------------
@pytest.mark.parametrize("pool", [(2, 2, 0), (3, 2, 1)])
def test_relu_maxpool_commute(oracle, pool):
    o = oracle
    ls = _spec(H=8, W=8, pool=pool)
    d, a, x, xs, labels, p = _setup(o, ls, B=3)
    lf = o.layer_fwd(d, x, xs, p["W"], p["b"])
    k, s, pd = pool
    Z = np.pad(lf.Z, ((0, 0), (0, 0), (pd, pd), (pd, pd)), constant_values=-np.inf)
    Hp, Wp = lf.Y.shape[2:]
    pooled = np.full(lf.Y.shape, -np.inf)
    for i in range(Hp):
        for j in range(Wp):
            pooled[:, :, i, j] = Z[:, :, i * s:i * s + k, j * s:j * s + k].max(axis=(2, 3))
    assert np.array_equal(np.maximum(pooled, 0), lf.Y)  # ReLU(pool(Z)) == pool(ReLU(Z))
    # the recorded arg-max points at an element equal to the emitted value (when positive)
    flatZ = lf.Z.reshape(*lf.Z.shape[:2], -1)
    picked = np.take_along_axis(flatZ, lf.arg.reshape(*lf.arg.shape[:2], -1).astype(np.int64), axis=2)
    assert np.array_equal(np.maximum(picked, 0).reshape(lf.Y.shape), lf.Y)


# ---- P7: convolution special cases -----------------------------------------------------------
def test_conv1x1_is_matmul_and_delta_kernels_shift(oracle):
    o = oracle
    g = workloads.rng_for(3, "p7")
    x = g.standard_normal((2, 3, 5, 4))
    W = g.standard_normal((4, 3, 1, 1))
    b = g.standard_normal((4,))
    d = o.layer_desc(3, 5, 4, 4, R=1, S=1, stride=1, pad=0)
    Z = o.layer_fwd(d, x, None, W, b).Z
    want = np.einsum("kc,nchw->nkhw", W[:, :, 0, 0], x) + b[None, :, None, None]
    np.testing.assert_allclose(Z, want, rtol=1e-13, atol=1e-13)
    # 3x3 delta kernels: centre = identity, off-centre = shift with zero fill
    d3 = o.layer_desc(3, 5, 4, 3, R=3, S=3, stride=1, pad=1)
    for (r, s) in [(1, 1), (0, 1), (2, 2), (1, 0)]:
        Wd = np.zeros((3, 3, 3, 3))
        for c in range(3):
            Wd[c, c, r, s] = 1.0
        Z = o.layer_fwd(d3, x, None, Wd, np.zeros(3)).Z
        want = np.zeros_like(x)
        dh, dw = r - 1, s - 1  # Z[i,j] = x[i+dh, j+dw]
        for i in range(5):
            for j in range(4):
                if 0 <= i + dh < 5 and 0 <= j + dw < 4:
                    want[:, :, i, j] = x[:, :, i + dh, j + dw]
        assert np.array_equal(Z, want)
    # stride 2: output cell (i,j) reads the window anchored at (2i-1, 2j-1)
    d2 = o.layer_desc(3, 5, 4, 3, R=3, S=3, stride=2, pad=1)
    Wd = np.zeros((3, 3, 3, 3))
    for c in range(3):
        Wd[c, c, 1, 1] = 1.0
    Z = o.layer_fwd(d2, x, None, Wd, np.zeros(3)).Z
    assert Z.shape == (2, 3, 3, 2) and np.array_equal(Z, x[:, :, ::2, ::2])


# ---- P8: head special cases ------------------------------------------------------------------
def test_aux_head_special_cases(oracle):
    o = oracle
    g = workloads.rng_for(4, "p8")
    # 1x1 input: only the centre tap of beta is used; adaptive pool 1 -> 2x2 replicates
    y = np.abs(g.standard_normal((2, 3, 1, 1)))
    Wa = g.standard_normal((2, 3, 3, 3))
    ba = g.standard_normal((2,))
    Wf = g.standard_normal((3, 8))
    bf = g.standard_normal((3,))
    a = o.aux_desc(3, 1, 1, 2, 3, relu=0)
    af = o.aux_fwd_loss(a, y, np.array([0, 2], np.int32), Wa, ba, Wf, bf)
    u = np.einsum("ak,nk->na", Wa[:, :, 1, 1], y[:, :, 0, 0]) + ba
    np.testing.assert_allclose(af.U[:, :, 0, 0], u, rtol=1e-13)
    np.testing.assert_allclose(af.Pq, np.repeat(u, 4, axis=1), rtol=1e-13)
    # 2x2 -> identity ; 4x4 -> 2x2 block means ; flatten order (a, i, j)
    for H in (2, 4, 6):
        y = g.standard_normal((2, 3, H, H))
        a = o.aux_desc(3, H, H, 2, 3, relu=1)
        af = o.aux_fwd_loss(a, y, np.array([1, 1], np.int32), Wa, ba, Wf, bf)
        h = H // 2
        want = af.U.reshape(2, 2, 2, h, 2, h).mean(axis=(3, 5)).reshape(2, 8)
        np.testing.assert_allclose(af.Pq, want, rtol=1e-13, atol=1e-15)
        assert af.U.min() >= 0
        np.testing.assert_allclose(af.z, af.Pq @ Wf.T + bf, rtol=1e-12, atol=1e-14)
    # odd input 3 -> windows [0,2) and [1,3) overlap
    y = g.standard_normal((1, 3, 3, 3))
    a = o.aux_desc(3, 3, 3, 2, 3, relu=0)
    af = o.aux_fwd_loss(a, y, np.array([0], np.int32), Wa, ba, Wf, bf)
    U = af.U[0]
    want = np.array([[U[q, i:i + 2, j:j + 2].mean() for i in (0, 1) for j in (0, 1)] for q in range(2)]).reshape(-1)
    np.testing.assert_allclose(af.Pq[0], want, rtol=1e-13)


# ---- P9: invariants ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["hp4", "pool2", "stride2"])
def test_invariants(oracle, name):
    o = oracle
    ls = _spec(**SHAPES[name])
    d, a, x, xs, labels, p = _setup(o, ls, B=4, Cls=5)
    lf, af, g = _grads(o, d, a, x, xs, labels, p)
    sm = np.exp(af.z - af.z.max(1, keepdims=True))
    sm /= sm.sum(1, keepdims=True)
    np.testing.assert_allclose(af.dz, (sm - np.eye(5)[labels]) / 4, atol=1e-15)
    np.testing.assert_allclose(af.dz.sum(1), 0, atol=1e-15)
    np.testing.assert_allclose(g["b"], g["dZ"].sum(axis=(0, 2, 3)), rtol=1e-12, atol=1e-15)
    # dZ vanishes wherever the pre-activation is not positive
    assert np.all(g["dZ"][lf.Z <= 0] == 0)
    if not d.pool_kind:
        assert np.array_equal(g["dZ"], np.where(lf.Z > 0, g["dY"], 0))
    else:
        # max-pool backward moves mass without changing it (where the max is positive)
        np.testing.assert_allclose(g["dZ"].sum(axis=(2, 3)), np.where(lf.Y > 0, g["dY"], 0).sum(axis=(2, 3)),
                                   rtol=1e-12, atol=1e-15)
    # average-pool backward conserves mass when windows partition the map (even sizes, relu off)
    a0 = o.aux_desc(**{**ls.aux_desc_fields(5), "relu": 0})
    af0 = o.aux_fwd_loss(a0, lf.Y, labels, p["Wa"], p["ba"], p["Wf"], p["bf"])
    g0 = o.local_bwd(d, a0, x, xs, lf, af0, p["Wa"], p["Wf"])
    if lf.Y.shape[2] % 2 == 0 and lf.Y.shape[3] % 2 == 0:
        dPq = af0.dz @ p["Wf"]
        np.testing.assert_allclose(g0["ba"], dPq.reshape(4, a.A, 4).sum(axis=(0, 2)), rtol=1e-12, atol=1e-15)


# ---- P10: batch-mean linearity and permutation invariance -----------------------------------
def test_batch_linearity_and_permutation(oracle):
    o = oracle
    ls = _spec(H=6, W=6, pool=(2, 2, 0))
    d, a, x, xs, labels, p = _setup(o, ls, B=6, Cls=4)
    _, af, g = _grads(o, d, a, x, xs, labels, p)
    _, af1, g1 = _grads(o, d, a, x[:3], None, labels[:3], p)
    _, af2, g2 = _grads(o, d, a, x[3:], None, labels[3:], p)
    assert abs(af.loss - 0.5 * (af1.loss + af2.loss)) < 1e-13
    perm = np.array([4, 2, 0, 5, 1, 3])
    _, afp, gp = _grads(o, d, a, np.ascontiguousarray(x[perm]), None, labels[perm], p)
    assert abs(af.loss - afp.loss) < 1e-13
    for k in ("W", "b", "Wa", "ba", "Wf", "bf"):
        np.testing.assert_allclose(g[k], 0.5 * (g1[k] + g2[k]), rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(g[k], gp[k], rtol=1e-11, atol=1e-14)


# ---- P11: SGD closed forms --------------------------------------------------------------------
def test_sgd_closed_forms(oracle):
    o = oracle
    g = workloads.rng_for(9, "sgd")
    w0 = g.standard_normal(100)
    gr = g.standard_normal(100)
    w = w0.copy()
    o.sgd_update(w, gr, None, 0.0, 0.0)
    assert np.array_equal(w, w0)
    o.sgd_update(w, gr, None, 0.1, 0.0)
    assert np.array_equal(w, w0 - 0.1 * gr)
    w, v = w0.copy(), np.zeros(100)
    o.sgd_update(w, gr, v, 0.1, 0.9)
    assert np.array_equal(v, gr)
    o.sgd_update(w, gr, v, 0.1, 0.9)
    np.testing.assert_allclose(w, w0 - 0.1 * gr * (2 + 0.9), rtol=1e-14)
    np.testing.assert_allclose(v, 1.9 * gr, rtol=1e-15)


# ---- P12: repeating a batch with a small learning rate lowers the loss ----------------------
def test_loss_decreases(oracle):
    o = oracle
    ls = _spec(C=3, H=8, W=8, K=8, A=4, pool=(2, 2, 0))
    d, a, x, xs, labels, p = _setup(o, ls, B=8, Cls=4)
    losses = [o.local_step(d, a, x, None, labels, p, None, 0.05, 0.0)[1] for _ in range(8)]
    assert all(b < a_ for a_, b in zip(losses, losses[1:]))


# ---- P13: shortcut special cases --------------------------------------------------------------
def test_skip_special_cases(oracle):
    o = oracle
    ls = _spec(C=3, K=3, skip=1)
    d, a, x, xs, labels, p = _setup(o, ls)
    lf = o.layer_fwd(d, x, xs, np.zeros_like(p["W"]), np.zeros_like(p["b"]))
    assert np.array_equal(lf.Y, np.maximum(xs, 0))
    ls = _spec(H=4, W=4, skip=2)
    d, a, x, xs, labels, p = _setup(o, ls)
    lf = o.layer_fwd(d, x, xs, np.zeros_like(p["W"]), np.zeros_like(p["b"]), p["Wp"])
    want = np.einsum("kc,nchw->nkhw", p["Wp"], xs[:, :, ::2, ::2])
    np.testing.assert_allclose(lf.Z, want, rtol=1e-13, atol=1e-15)


# ---- f32 entry points agree with f64 ones to float rounding ---------------------------------
def test_f32_matches_f64(oracle):
    o = oracle
    ls = _spec(C=3, H=8, W=8, K=8, A=4, pool=(2, 2, 0))
    d, a, x, xs, labels, p = _setup(o, ls, B=8, Cls=4)
    p32 = {k: (None if v is None else v.astype(np.float32)) for k, v in p.items()}
    p64 = {k: (None if v is None else v.astype(np.float32).astype(np.float64)) for k, v in p.items()}
    x32 = x.astype(np.float32)
    Y64, l64, g64 = o.local_step(d, a, x32.astype(np.float64), None, labels, p64, None, 0.05, 0.0)
    Y32, l32, g32 = o.local_step(d, a, x32, None, labels, p32, None, 0.05, 0.0)
    assert abs(l32 - l64) < 1e-6
    for k in g64:
        if g64[k] is not None:
            np.testing.assert_allclose(g32[k], g64[k], rtol=2e-5, atol=1e-6)


# ---- decision overrides: handing the oracle its own decisions changes nothing; flipping one
# ---- decision changes the gradient by exactly that element's contribution
def test_decision_overrides(oracle):
    o = oracle
    ls = _spec(H=6, W=6, pool=(2, 2, 0))
    d, a, x, xs, labels, p = _setup(o, ls, B=3, Cls=4)
    lf, af, g = _grads(o, d, a, x, xs, labels, p)
    g2 = o.local_bwd(d, a, x, xs, lf, af, p["Wa"], p["Wf"], mask_u=af.Upre > 0, mask_z=lf.Z > 0)
    for k in g:
        if g[k] is not None:
            assert np.array_equal(g[k], g2[k]), k
    assert np.array_equal(np.maximum(af.Upre, 0), af.U)
    mu = (af.Upre > 0).copy()
    on = np.argwhere(mu)[0]
    mu[tuple(on)] = False  # switch one active aux unit off
    g3 = o.local_bwd(d, a, x, xs, lf, af, p["Wa"], p["Wf"], mask_u=mu, mask_z=lf.Z > 0)
    assert not np.array_equal(g3["Wa"], g["Wa"]) and np.array_equal(g3["Wf"], g["Wf"])


# ---- a block of layers: Worker loop of Algorithm 2, cache sweep ------------------------------
def _block(o, kind, Cls=3, dtype=np.float64, seed=11):
    """Three local layers in a row.  'basic': plain conv with max-pool, then a basic block whose
    second conv adds the basic block's input; 'proj': a stride-2 basic block with a 1x1 projection
    shortcut from the block's input, then a plain conv."""
    if kind == "basic":
        specs = [workloads.LayerSpec("l0", 2, 8, 8, 4, A=2, pool_kind=1, pool_k=2, pool_stride=2),
                 workloads.LayerSpec("l1", 4, 4, 4, 4, A=3),
                 workloads.LayerSpec("l2", 4, 4, 4, 4, A=2, skip_kind=1, skip_C=4, skip_H=4, skip_W=4, skip_stride=1)]
        skip_src = [-1, -1, 1]
    else:
        specs = [workloads.LayerSpec("l0", 2, 6, 6, 4, A=2, stride=2),
                 workloads.LayerSpec("l1", 4, 3, 3, 4, A=2, skip_kind=2, skip_C=2, skip_H=6, skip_W=6, skip_stride=2),
                 workloads.LayerSpec("l2", 4, 3, 3, 3, A=2)]
        skip_src = [-1, 0, -1]
    layers = []
    for n, ls in enumerate(specs):
        d = o.layer_desc(**ls.layer_desc_fields())
        a = o.aux_desc(**ls.aux_desc_fields(Cls))
        p = workloads.gen_layer_params(seed, n, ls, Cls, dtype=dtype, bias_std=0.3)
        layers.append((d, a, p, skip_src[n]))
    return specs, layers


def _as_block_layers(o, layers, mu):
    out = []
    for d, a, p, s in layers:
        pc = {k: (None if v is None else v.copy()) for k, v in p.items()}
        mom = {k: (None if v is None else np.zeros_like(v)) for k, v in p.items()} if mu else None
        out.append(o.BlockLayer(d, a, pc, mom, s))
    return out


@pytest.mark.parametrize("kind", ["basic", "proj"])
@pytest.mark.parametrize("mu", [0.0, 0.9])
def test_block_epoch_matches_torch_autograd(oracle, kind, mu):
    """Three layers, shuffled order, partial last batch, two passes (so momentum and the updated
    weights matter): losses, final weights and momentum buffers against per-layer torch.optim.SGD."""
    o = oracle
    specs, layers = _block(o, kind)
    N, B, Cls = 7, 3, 3
    g = workloads.rng_for(3, "block-pin", kind)
    X = g.standard_normal((N, specs[0].C_in, specs[0].H_in, specs[0].W_in))
    lab = g.integers(0, Cls, size=(N,)).astype(np.int32)
    idx = g.permutation(N).astype(np.int64)
    bl = _as_block_layers(o, layers, mu)
    shape = X.shape[1:]
    cache = X.reshape(N, -1).copy()
    got = [o.block_train_epoch(bl, cache, lab, idx, N, B, shape, 0.05, mu) for _ in range(2)]
    batches = [idx[f:f + B] for f in range(0, N, B)]
    ref_losses, ref_final, ref_mom = torch_ref.block_epoch(layers, X, lab, batches * 2, 0.05, mu)
    np.testing.assert_allclose(np.concatenate(got), np.array(ref_losses), rtol=1e-10, atol=1e-12)
    for L, pf, mf in zip(bl, ref_final, ref_mom):
        for k, v in pf.items():
            np.testing.assert_allclose(L.params[k], v, rtol=1e-9, atol=1e-12, err_msg=k)
            if mu:
                np.testing.assert_allclose(L.mom[k], mf[k], rtol=1e-9, atol=1e-12, err_msg="v_" + k)


@pytest.mark.parametrize("kind", ["basic", "proj"])
def test_block_fill_cache_and_training_from_it(oracle, kind):
    """The sweep stores exactly the composed forward of the block (torch, float64); training the
    next block from that cache equals training it on activations recomputed from the raw inputs."""
    o = oracle
    specs, layers = _block(o, kind)
    N, Cls = 7, 3
    g = workloads.rng_for(4, "block-fill", kind)
    X = g.standard_normal((N, specs[0].C_in, specs[0].H_in, specs[0].W_in))
    lab = g.integers(0, Cls, size=(N,)).astype(np.int32)
    bl = _as_block_layers(o, layers, 0.0)
    last = specs[-1]
    out_shape = (last.C_out, last.Hp, last.Wp)
    cache_out = np.full((N, int(np.prod(out_shape))), np.nan)
    lab_out = np.full((N,), -1, np.int32)
    o.block_fill_cache(bl, X.reshape(N, -1).copy(), lab, N, 3, X.shape[1:], cache_out, lab_out)
    ref = torch_ref.block_forward(layers, X)
    np.testing.assert_allclose(cache_out.reshape(ref.shape), ref, rtol=1e-11, atol=1e-13)
    assert np.array_equal(lab_out, lab)
    # a one-layer second block, trained (a) from the cache, (b) from the recomputed activations
    nxt = workloads.LayerSpec("n", last.C_out, last.Hp, last.Wp, 3, A=2)
    d, a = o.layer_desc(**nxt.layer_desc_fields()), o.aux_desc(**nxt.aux_desc_fields(Cls))
    p = workloads.gen_layer_params(12, 0, nxt, Cls, dtype=np.float64, bias_std=0.3)
    idx = g.permutation(N).astype(np.int64)
    runs = []
    for src in (cache_out, ref.reshape(N, -1).copy()):
        blk = _as_block_layers(o, [(d, a, p, -1)], 0.9)
        losses = o.block_train_epoch(blk, src, lab_out, idx, N, 4, out_shape, 0.05, 0.9)
        runs.append((losses, blk[0].params))
    np.testing.assert_allclose(runs[0][0], runs[1][0], rtol=1e-9)
    for k, v in runs[0][1].items():
        if v is not None:
            np.testing.assert_allclose(v, runs[1][1][k], rtol=1e-8, atol=1e-12)


def test_block_epoch_is_the_sequence_of_local_steps(oracle):
    """Locality across layers: a layer's update inside the block pass depends only on its own
    input batch — perturbing layer 2's parameters leaves layer 0's and 1's results untouched,
    and the tensor handed on is the one computed with the pre-update weights."""
    o = oracle
    specs, layers = _block(o, "basic")
    N, Cls = 4, 3
    g = workloads.rng_for(5, "block-local")
    X = g.standard_normal((N, 2, 8, 8))
    lab = g.integers(0, Cls, size=(N,)).astype(np.int32)
    a_run = _as_block_layers(o, layers, 0.0)
    b_run = _as_block_layers(o, layers, 0.0)
    b_run[2].params["W"] += 0.5
    la = o.block_train_epoch(a_run, X.reshape(N, -1).copy(), lab, None, N, 4, X.shape[1:], 0.1, 0.0)
    lb = o.block_train_epoch(b_run, X.reshape(N, -1).copy(), lab, None, N, 4, X.shape[1:], 0.1, 0.0)
    assert np.array_equal(la[:, :2], lb[:, :2]) and la[0, 2] != lb[0, 2]
    for n in (0, 1):
        for k, v in a_run[n].params.items():
            assert v is None or np.array_equal(v, b_run[n].params[k])
    # pre-update hand-over: layer 1's first loss equals the head loss on layer 0's output under
    # layer 0's ORIGINAL weights
    d0, a0, p0, _ = layers[0]
    d1, a1, p1, _ = layers[1]
    y0 = o.layer_fwd(d0, X, None, p0["W"], p0["b"]).Y
    y1 = o.layer_fwd(d1, y0, None, p1["W"], p1["b"]).Y
    want = o.aux_fwd_loss(a1, y1, lab, p1["Wa"], p1["ba"], p1["Wf"], p1["bf"]).loss
    assert abs(la[0, 1] - want) < 1e-12


# ---- head variants the paper names: max pooling as F_n, mean squared error as the loss --------
VARIANTS = {"max_ce": (1, 0), "avg_mse": (0, 1), "max_mse": (1, 1)}
VARIANT_SHAPES = ["plain5x5", "hp4", "hp3_odd_overlap", "hp2", "hp1", "rect", "pool2", "skip_proj"]


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("name", VARIANT_SHAPES)
def test_variant_finite_difference_gradients(oracle, name, variant):
    o = oracle
    hp, lk = VARIANTS[variant]
    ls = _spec(**SHAPES[name])
    d, a, x, xs, labels, p = _setup(o, ls, head_pool=hp, loss_kind=lk)
    _, _, g = _grads(o, d, a, x, xs, labels, p)
    h = 1e-6
    for key in o.PARAM_NAMES:
        if p[key] is None:
            continue
        flat = p[key].reshape(-1)
        num = np.zeros_like(flat)
        for e in range(flat.size):
            keep = flat[e]
            flat[e] = keep + h
            lp = _loss(o, d, a, x, xs, labels, p)
            flat[e] = keep - h
            lm = _loss(o, d, a, x, xs, labels, p)
            flat[e] = keep
            num[e] = (lp - lm) / (2 * h)
        ana = g[key].reshape(-1)
        scale = max(np.abs(num).max(), 1e-3)
        assert np.abs(num - ana).max() <= 2e-6 * scale + 1e-8, (name, variant, key, np.abs(num - ana).max(), scale)


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("name", VARIANT_SHAPES)
def test_variant_matches_torch_autograd(oracle, name, variant):
    o = oracle
    hp, lk = VARIANTS[variant]
    ls = _spec(**SHAPES[name])
    d, a, x, xs, labels, p = _setup(o, ls, B=3, Cls=4, seed=11, head_pool=hp, loss_kind=lk)
    lr, mu = 0.05, 0.9
    ta = SimpleNamespace(**ls.aux_desc_fields(4), head_pool=hp, loss_kind=lk)
    ref, final = torch_ref.local_step(SimpleNamespace(**ls.layer_desc_fields()), ta, x, xs, labels, p, lr, mu, steps=3)
    mom = {k: (None if v is None else np.zeros_like(v)) for k, v in p.items()}
    for step in range(3):
        Y, loss, g = o.local_step(d, a, x, xs, labels, p, mom, lr, mu)
        rl, rg, ry = ref[step]
        assert abs(loss - rl) <= 1e-12 * max(1, abs(rl))
        for k in rg:
            np.testing.assert_allclose(g[k], rg[k], rtol=1e-9, atol=1e-12, err_msg=f"{name}:{variant}:{k}:{step}")
    for k in final:
        np.testing.assert_allclose(p[k], final[k], rtol=1e-10, atol=1e-12, err_msg=f"{name}:{variant}:{k}")


def test_variant_closed_forms(oracle):
    o = oracle
    g = workloads.rng_for(6, "variants")
    B, Cls = 5, 4
    y = np.abs(g.standard_normal((B, 3, 6, 6)))
    Wa, ba = g.standard_normal((2, 3, 3, 3)), g.standard_normal((2,))
    labels = g.integers(0, Cls, size=(B,)).astype(np.int32)
    # MSE at zero linear weights: every logit is 0, the one-hot target has one 1 -> loss = 1/Cls,
    # dL/dz = 2 (0 - t) / (B Cls)
    a = o.aux_desc(3, 6, 6, 2, Cls, loss_kind=1)
    af = o.aux_fwd_loss(a, y, labels, Wa, ba, np.zeros((Cls, 8)), np.zeros((Cls,)))
    assert abs(af.loss - 1.0 / Cls) < 1e-15
    t = np.eye(Cls)[labels]
    np.testing.assert_allclose(af.dz, -2.0 * t / (B * Cls), rtol=1e-14)
    # MSE with logits forced to the target by the bias of a one-class-per-sample batch is 0
    Wf, bf = g.standard_normal((Cls, 8)), g.standard_normal((Cls,))
    af = o.aux_fwd_loss(a, y, labels, Wa, ba, Wf, bf)
    want = np.mean((af.Pq @ Wf.T + bf - t) ** 2)
    assert abs(af.loss - want) < 1e-13
    # max pooling: windows of a 6x6 map are its 3x3 quadrants; parg points at the maximum; 2x2 map:
    # max == avg == identity
    am = o.aux_desc(3, 6, 6, 2, Cls, head_pool=1)
    afm = o.aux_fwd_loss(am, y, labels, Wa, ba, Wf, bf)
    want = afm.U.reshape(B, 2, 2, 3, 2, 3).max(axis=(3, 5)).reshape(B, 8)
    assert np.array_equal(afm.Pq, want)
    flatU = afm.U.reshape(B, 2, 36)
    pa = afm.parg.reshape(B, 2, 4)
    assert np.array_equal(np.take_along_axis(flatU, pa.astype(np.int64), axis=2).reshape(B, 8), afm.Pq)
    hh, ww = pa // 6, pa % 6
    cells = np.arange(4).reshape(1, 1, 4)
    assert np.all(hh // 3 == cells // 2) and np.all(ww // 3 == cells % 2)
    y2 = np.abs(g.standard_normal((B, 3, 2, 2)))
    a2m, a2a = o.aux_desc(3, 2, 2, 2, Cls, head_pool=1), o.aux_desc(3, 2, 2, 2, Cls)
    assert np.array_equal(o.aux_fwd_loss(a2m, y2, labels, Wa, ba, Wf, bf).Pq,
                          o.aux_fwd_loss(a2a, y2, labels, Wa, ba, Wf, bf).Pq)
    # an all-zero window (everything cut by the head's ReLU): first element selected, no gradient
    y0 = np.zeros((1, 3, 4, 4))
    a0 = o.aux_desc(3, 4, 4, 2, Cls, head_pool=1)
    af0 = o.aux_fwd_loss(a0, y0, labels[:1], Wa, -np.abs(ba), Wf, bf)
    assert np.array_equal(af0.parg.reshape(2, 2, 2), np.broadcast_to(np.array([[0, 2], [8, 10]]), (2, 2, 2)))
    ls = workloads.LayerSpec("t", 3, 4, 4, 3, A=2)
    d0 = o.layer_desc(**ls.layer_desc_fields())
    x0 = g.standard_normal((1, 3, 4, 4))
    W0, b0 = g.standard_normal((3, 3, 3, 3)), g.standard_normal((3,))
    lf = o.layer_fwd(d0, x0, None, W0, b0)
    af0 = o.aux_fwd_loss(a0, lf.Y, labels[:1], Wa * 0, -np.abs(ba) - 1, Wf, bf)
    gr = o.local_bwd(d0, a0, x0, None, lf, af0, Wa * 0, Wf)
    assert not gr["Wa"].any() and not gr["W"].any() and gr["Wf"].shape == (Cls, 8)


# ---- early-exit evaluation: prediction and accuracy ---------------------------------------------
def test_prediction_closed_forms_and_torch(oracle):
    import torch
    import torch.nn.functional as F
    o = oracle
    g = workloads.rng_for(8, "predict")
    B, Cls = 9, 5
    y = np.abs(g.standard_normal((B, 3, 6, 6)))
    Wa, ba = g.standard_normal((2, 3, 3, 3)), g.standard_normal((2,))
    Wf, bf = g.standard_normal((Cls, 8)), g.standard_normal((Cls,))
    a = o.aux_desc(3, 6, 6, 2, Cls)
    z, pred = o.aux_predict(a, y, Wa, ba, Wf, bf)
    # library pin: the head through torch
    u = torch.relu(F.conv2d(torch.tensor(y), torch.tensor(Wa), torch.tensor(ba), padding=1))
    zt = F.linear(F.adaptive_avg_pool2d(u, (2, 2)).flatten(1), torch.tensor(Wf), torch.tensor(bf))
    np.testing.assert_allclose(z, zt.numpy(), rtol=1e-12, atol=1e-13)
    assert np.array_equal(pred, zt.argmax(1).numpy())
    # zero linear weights: the bias alone decides -> every sample gets argmax(bf)
    _, p0 = o.aux_predict(a, y, Wa, ba, Wf * 0, bf)
    assert np.all(p0 == int(np.argmax(bf)))
    # all logits equal: the lowest class index
    _, p1 = o.aux_predict(a, y, Wa, ba, Wf * 0, bf * 0 + 0.25)
    assert np.all(p1 == 0)
    # two equal maxima: the lower index of the two
    b2 = np.array([0.0, 3.0, -1.0, 3.0, 1.0])
    _, p2 = o.aux_predict(a, y, Wa, ba, Wf * 0, b2)
    assert np.all(p2 == 1)
    # relabelling the classes relabels the predictions
    perm = np.array([3, 0, 4, 1, 2])
    _, pp = o.aux_predict(a, y, Wa, ba, Wf[perm], bf[perm])
    assert np.array_equal(perm[pp], pred)


def test_block_evaluate_and_exit_selection(oracle):
    import torch
    import torch.nn.functional as F
    o = oracle
    specs, layers = _block(o, "basic")
    N, Cls = 11, 3
    g = workloads.rng_for(9, "block-eval")
    X = g.standard_normal((N, 2, 8, 8))
    lab = g.integers(0, Cls, size=(N,)).astype(np.int32)
    bl = _as_block_layers(o, layers, 0.0)
    counts = []
    for e in range(3):
        preds, correct = o.block_evaluate(bl, e, X.reshape(N, -1).copy(), lab, N, 4, X.shape[1:])
        feats = torch.tensor(torch_ref.block_forward(layers[:e + 1], X))
        d, a, p, _ = layers[e]
        u = torch.relu(F.conv2d(feats, torch.tensor(p["Wa"]), torch.tensor(p["ba"]), padding=1))
        zt = F.linear(F.adaptive_avg_pool2d(u, (2, 2)).flatten(1), torch.tensor(p["Wf"]), torch.tensor(p["bf"]))
        assert np.array_equal(preds, zt.argmax(1).numpy().astype(np.int32))
        assert correct == int((preds == lab).sum())
        counts.append(correct)
    # a head that always answers class c is right exactly on the samples labelled c
    for L in bl:
        L.params["Wf"][:] = 0
        L.params["bf"][:] = np.array([0.0, 1.0, 0.5])
    preds, correct = o.block_evaluate(bl, 1, X.reshape(N, -1).copy(), lab, N, 5, X.shape[1:])
    assert np.all(preds == 1) and correct == int((lab == 1).sum())
    # exit selection: highest accuracy; ties -> fewest parameters; then the earliest
    assert o.select_exit([5, 9, 9, 7], [10, 20, 30, 40]) == 1
    assert o.select_exit([5, 9, 9, 7], [10, 30, 20, 40]) == 2
    assert o.select_exit([9, 9, 9], [10, 10, 10]) == 0
    assert o.select_exit([1, 2, 3], [10, 20, 30]) == 2
    assert 0 <= o.select_exit(counts, [1, 2, 3]) < 3
