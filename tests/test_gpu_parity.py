"""GPU parity: every C-ABI call of include/nf.h against the CPU oracle, element by element,
on the same seeded inputs.  Tolerance: 1e-4 relative (norm-wise and max-wise per tensor,
relative on the scalar loss); bit-exact for copies and indices.
"""
import numpy as np
import pytest
import torch

import oracle as O
import workloads
from paper_2402_14139_amd import binding as nf
from paper_2402_14139_amd import layout
from tests import gpu_common as G

pytestmark = pytest.mark.gpu


def S(C, H, W, K, A, R=3, S_=None, stride=1, pad=None, pool=None, skip=0, skip_C=0):
    S_ = R if S_ is None else S_
    pad = R // 2 if pad is None else pad
    ls = workloads.LayerSpec("t", C, H, W, K, R=R, S=S_, stride=stride, pad=pad, A=A)
    if pool:
        ls.pool_kind, ls.pool_k, ls.pool_stride, ls.pool_pad = 1, *pool
    if skip == 1:
        ls.skip_kind, ls.skip_C, ls.skip_H, ls.skip_W, ls.skip_stride = 1, K, ls.Ho, ls.Wo, 1
    elif skip == 2:
        ls.skip_kind, ls.skip_C, ls.skip_stride = 2, skip_C, 2
        ls.skip_H, ls.skip_W = ls.Ho * 2, ls.Wo * 2 - 1
    return ls


# name -> (spec, B, classes); sizes span several tiles and ragged tails in M, N and K
CASES = {
    "ragged_small": (S(8, 9, 7, 40, 12), 3, 10),
    "scalar_paths_c3_k6_a5": (S(3, 10, 10, 6, 5), 5, 7),
    "stride2": (S(16, 14, 14, 32, 8, stride=2), 4, 10),
    "pool2": (S(8, 12, 12, 24, 8, pool=(2, 2, 0)), 6, 10),
    "stem7x7_pool3s2p1": (S(3, 20, 20, 16, 8, R=7, stride=2, pad=3, pool=(3, 2, 1)), 4, 20),
    "skip_identity": (S(16, 8, 8, 16, 4, skip=1), 5, 10),
    "skip_projection": (S(32, 4, 4, 32, 4, skip=2, skip_C=16), 7, 10),
    "emits_1x1": (S(32, 2, 2, 32, 16, pool=(2, 2, 0)), 9, 10),
    "odd_3x3_overlapping_avg_windows": (S(8, 3, 3, 8, 4), 4, 5),
    "head_a32_n64": (S(16, 8, 8, 64, 32), 8, 100),
    "n160_two_tiles_a80": (S(32, 8, 8, 160, 80), 6, 200),
    "many_m_tiles": (S(16, 16, 16, 64, 16), 40, 10),
    "conv1x1": (S(16, 6, 6, 24, 8, R=1, pad=0), 4, 10),
    "rect_5x3_filter": (S(8, 9, 8, 16, 8, R=5, S_=3, pad=1), 3, 10),
    # skinny heads: split reduction of the aux conv forward (long reduction, few row tiles) and
    # the 4x4x1-MFMA weight gradient in each of its (groups, channels-per-lane) shapes
    "skinny_a4_c256_split": (S(16, 6, 6, 256, 4), 5, 10),
    "skinny_a8_c128_split": (S(8, 8, 8, 128, 8), 6, 10),
    "skinny_a12_c136_ragged": (S(8, 5, 7, 136, 12), 3, 10),
    "skinny_a16_c64_pool": (S(8, 12, 12, 64, 16, pool=(2, 2, 0)), 4, 10),
    "skinny_a4_c64_one_row_images": (S(8, 1, 9, 64, 4), 7, 10),
}


@pytest.mark.parametrize("name", list(CASES))
def test_local_step_matches_oracle(name):
    spec, B, cls = CASES[name]
    print(f"case {name}: B={B}", flush=True)
    out, final = G.run_step_both(spec, cls, B, seed=100, lr=0.05, mu=0.9, steps=2)
    G.check_step_results(name, out, final)


VARIANTS = {"maxpool_ce": (1, 0), "avgpool_mse": (0, 1), "maxpool_mse": (1, 1)}


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("name", ["ragged_small", "scalar_paths_c3_k6_a5", "pool2", "odd_3x3_overlapping_avg_windows",
                                  "emits_1x1", "head_a32_n64", "n160_two_tiles_a80", "skinny_a4_c256_split",
                                  "skinny_a12_c136_ragged"])
def test_head_variants_match_oracle(name, variant):
    """Max pooling as the head's down-sampling F_n and mean squared error as the loss (the
    alternatives the paper names next to average pooling and cross-entropy)."""
    spec, B, cls = CASES[name]
    hp, lk = VARIANTS[variant]
    print(f"case {name} {variant}: B={B}", flush=True)
    out, final = G.run_step_both(spec, cls, B, seed=102, lr=0.05, mu=0.9, steps=2, head_pool=hp, loss_kind=lk)
    G.check_step_results(f"{name}/{variant}", out, final)


def test_local_step_no_relu_head_no_momentum():
    spec, B, cls = CASES["pool2"]
    out, final = G.run_step_both(spec, cls, B, seed=101, lr=0.01, mu=0.0, steps=2, relu=0)
    G.check_step_results("relu0", out, final)


def test_cfg1_as_written():
    """Single local layer, batch 8, 3x32x32 -> 16, head 16->8, FC 32->10, lr 0.01, no momentum,
    zero biases, seed 0; outputs: loss, all weight grads, updated weights, emitted 16x32x32
    activation (pre-update weights) and the cached activation (forward with updated weights)."""
    cfg = workloads.config("cfg1")
    spec, B, cls = cfg.layers[0], cfg.blocks[0].batch, cfg.n_classes
    x, labels = workloads.gen_batch(cfg.seed, 0, B, cfg.in_shape, cls)
    p = workloads.gen_layer_params(cfg.seed, 0, spec, cls)
    (d, a), (od, oa) = G.descs(spec, cls)
    L = G.gpu_layer(spec, cls, p, B, False)
    xd, ld = G.to_dev(layout.act_to_lib(x)), G.to_dev(labels)
    y = L.step(xd, None, ld, cfg.lr, cfg.momentum)
    torch.cuda.synchronize()
    po = {k: (None if v is None else v.copy()) for k, v in p.items()}
    oY, oloss, og = O.local_step(od, oa, x, None, labels, po, None, cfg.lr, cfg.momentum)
    assert abs(float(L.loss.item()) - oloss) <= G.REL * abs(oloss)
    G.assert_close("y_step", layout.act_from_lib(y.cpu().numpy()), oY)
    gg, gp = L.params_numpy("g"), L.params_numpy("p")
    for k in ("W", "b", "Wa", "ba", "Wf", "bf"):
        G.assert_close("grad " + k, gg[k], og[k])
        G.assert_close("updated " + k, gp[k], po[k])
    # cached activation: forward with the updated weights -> cache write -> cache read
    se = spec.C_out * spec.Hp * spec.Wp
    cache = torch.full((B, se), float("nan"), device="cuda")
    clab = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    y2 = L.forward(xd)
    nf.nf_cache_write(cache, clab, B, se, 0, B, y2, ld)
    xo = torch.empty_like(y2)
    lo = torch.empty_like(clab)
    nf.nf_cache_read(cache, clab, B, se, 0, None, B, xo, lo)
    torch.cuda.synchronize()
    ref = O.layer_fwd(od, x, None, po["W"], po["b"]).Y
    G.assert_close("cache", layout.act_from_lib(xo.cpu().numpy()), ref)
    assert torch.equal(xo, y2) and torch.equal(lo, ld)


# ---- the separate entry points give the same results as the oracle's separate functions ----
@pytest.mark.parametrize("name", ["pool2", "skip_projection", "head_a32_n64"])
def test_separate_calls(name):
    spec, B, cls = CASES[name]
    x, xs, labels, p = G.make_inputs(spec, B, cls, seed=7)
    (d, a), (od, oa) = G.descs(spec, cls)
    L = G.gpu_layer(spec, cls, p, B, True)
    xd = G.to_dev(layout.act_to_lib(x))
    xsd = G.to_dev(None if xs is None else layout.act_to_lib(xs))
    ld = G.to_dev(labels)
    y = L.forward(xd, xsd)
    L.aux_loss(y, ld)
    L.backward(xd, xsd, y)
    torch.cuda.synchronize()
    lf = O.layer_fwd(od, x, xs, p["W"], p["b"], p["Wp"])
    af = O.aux_fwd_loss(oa, lf.Y, labels, p["Wa"], p["ba"], p["Wf"], p["bf"])
    og = O.local_bwd(od, oa, x, xs, lf, af, p["Wa"], p["Wf"])
    G.assert_close("y", layout.act_from_lib(y.cpu().numpy()), lf.Y)
    assert abs(float(L.loss.item()) - af.loss) <= G.REL * abs(af.loss)
    gg = L.params_numpy("g")
    for k in G.PARAM_NAMES:
        if og[k] is not None:
            G.assert_close("grad " + k, gg[k], og[k])
    # parameters untouched by forward/backward
    before = layout.params_to_lib(p, spec.A)
    for k, v in L.p.items():
        if v is not None:
            assert np.array_equal(v.cpu().numpy(), before[k])
    # update line
    L.sgd(0.05, 0.9)
    L.sgd(0.05, 0.9)
    torch.cuda.synchronize()
    gp, gv = L.params_numpy("p"), L.params_numpy("v")
    for k in G.PARAM_NAMES:
        if p[k] is None:
            continue
        w, v = p[k].copy(), np.zeros_like(p[k])
        O.sgd_update(w, og[k], v, 0.05, 0.9)
        O.sgd_update(w, og[k], v, 0.05, 0.9)
        G.assert_close("sgd w " + k, gp[k], w)
        G.assert_close("sgd v " + k, gv[k], v)


def test_sgd_odd_sizes_and_no_momentum():
    g = workloads.rng_for(3, "sgd-gpu")
    sizes = [1, 3, 4, 5, 1023, 4096 + 2]
    w = [g.standard_normal(n).astype(np.float32) for n in sizes]
    gr = [g.standard_normal(n).astype(np.float32) for n in sizes]
    wd, gd = [G.to_dev(t) for t in w], [G.to_dev(t) for t in gr]
    nf.nf_sgd_update(0.1, 0.0, wd, gd, None)
    torch.cuda.synchronize()
    for a, b, c in zip(wd, w, gr):
        ref = b.copy()
        O.sgd_update(ref, c, None, 0.1, 0.0)
        G.assert_close("sgd", a.cpu().numpy(), ref, rel=1e-6)


def test_cache_write_read_rebatching_bit_exact():
    N, se = 37, 4 * 3 * 5  # rows of 60 floats; also an odd row length below
    for se in (60, 7):
        g = workloads.rng_for(4, "cache-gpu", se)
        data = g.standard_normal((N, se)).astype(np.float32)
        labs = g.integers(0, 10, size=(N,)).astype(np.int32)
        # rows start 16-byte aligned only when se % 4 == 0; the odd case goes through a padded row
        row = se if se % 4 == 0 else 8
        cache = torch.full((N, row), float("nan"), device="cuda")
        clab = torch.full((N,), -1, dtype=torch.int32, device="cuda")
        src = np.zeros((N, row), np.float32)
        src[:, :se] = data
        for first in range(0, N, 8):  # write at batch 8 (last one partial)
            b = min(8, N - first)
            nf.nf_cache_write(cache, clab, N, row, first, b, G.to_dev(src[first:first + b]), G.to_dev(labs[first:first + b]))
        torch.cuda.synchronize()
        assert np.array_equal(cache.cpu().numpy(), src) and np.array_equal(clab.cpu().numpy(), labs)
        got = []
        for first in range(0, N, 5):  # read at batch 5: does not divide 37 nor 8
            b = min(5, N - first)
            xo = torch.empty((b, row), device="cuda")
            lo = torch.empty((b,), dtype=torch.int32, device="cuda")
            nf.nf_cache_read(cache, clab, N, row, first, None, b, xo, lo)
            got.append(xo.cpu().numpy())
        assert np.array_equal(np.concatenate(got), src)
        idx = g.permutation(N)[:11].astype(np.int64)
        xo = torch.empty((11, row), device="cuda")
        lo = torch.empty((11,), dtype=torch.int32, device="cuda")
        nf.nf_cache_read(cache, clab, N, row, 0, G.to_dev(idx), 11, xo, lo)
        ref_x, ref_l = O.cache_read(src, labs, 0, idx, 11, (row,))
        assert np.array_equal(xo.cpu().numpy(), ref_x) and np.array_equal(lo.cpu().numpy(), ref_l)


def test_block_from_cache_equals_recompute():
    """Training block k+1 from the cache equals recomputing block k forward on the raw inputs."""
    cls, N = 10, 24
    l1 = S(3, 12, 12, 16, 8, pool=(2, 2, 0))
    l2 = S(16, 6, 6, 24, 8)
    g = workloads.rng_for(8, "cache-equiv")
    X = g.standard_normal((N, 3, 12, 12)).astype(np.float32)
    Lb = g.integers(0, cls, size=(N,)).astype(np.int32)
    p1 = workloads.gen_layer_params(8, 0, l1, cls, bias_std=0.1)
    p2 = workloads.gen_layer_params(8, 1, l2, cls, bias_std=0.1)
    L1 = G.gpu_layer(l1, cls, p1, 8, True)
    Xd, Ld = G.to_dev(layout.act_to_lib(X)), G.to_dev(Lb)
    for first in range(0, N, 8):  # train block 1 at batch 8
        L1.step(Xd[first:first + 8], None, Ld[first:first + 8], 0.05, 0.9)
    se = 16 * 6 * 6
    cache = torch.empty((N, se), device="cuda")
    clab = torch.empty((N,), dtype=torch.int32, device="cuda")
    for first in range(0, N, 8):  # frozen sweep fills the cache
        y = L1.forward(Xd[first:first + 8])
        nf.nf_cache_write(cache, clab, N, se, first, 8, y, Ld[first:first + 8])
    idx = G.to_dev(np.array([5, 23, 0, 11, 17, 2, 8, 19, 3, 14, 21, 6], np.int64))  # block 2 at batch 12
    xin = torch.empty((12, 6, 6, 16), device="cuda")
    lin = torch.empty((12,), dtype=torch.int32, device="cuda")
    nf.nf_cache_read(cache, clab, N, se, 0, idx, 12, xin, lin)
    La = G.gpu_layer(l2, cls, p2, 12, True)
    Lr = G.gpu_layer(l2, cls, p2, 12, True)
    ya = La.step(xin, None, lin, 0.05, 0.9)
    xre = L1.forward(Xd[idx])
    yr = Lr.step(xre, None, Ld[idx], 0.05, 0.9)
    torch.cuda.synchronize()
    assert torch.equal(xin, xre) and torch.equal(ya, yr) and float(La.loss.item()) == float(Lr.loss.item())
    for k in G.PARAM_NAMES:
        if La.p[k] is not None:
            assert torch.equal(La.p[k], Lr.p[k]) and torch.equal(La.g[k], Lr.g[k])
    # and the cached rows match the oracle's forward with the trained weights
    tp = L1.params_numpy("p")
    (_, _), (od, _) = G.descs(l1, cls)
    ref = O.layer_fwd(od, X, None, tp["W"], tp["b"]).Y
    G.assert_close("cache rows", layout.act_from_lib(cache.view(N, 6, 6, 16).cpu().numpy()), ref)


@pytest.mark.parametrize("name", ["many_m_tiles", "skinny_a8_c128_split", "skinny_a4_c256_split", "skip_projection",
                                  "n160_two_tiles_a80"])
def test_run_to_run_determinism(name):
    """Split reductions are summed in a fixed order: gradients, updated weights and the loss are
    bitwise equal from run to run (tiled and 4x4x1 weight gradients, split aux forward)."""
    spec, B, cls = CASES[name]
    x, xs, labels, p = G.make_inputs(spec, B, cls, seed=5)
    res = []
    for _ in range(2):
        L = G.gpu_layer(spec, cls, p, B, True)
        L.step(G.to_dev(layout.act_to_lib(x)), G.to_dev(None if xs is None else layout.act_to_lib(xs)), G.to_dev(labels),
               0.05, 0.9)
        torch.cuda.synchronize()
        out = {"g_" + k: v.clone() for k, v in L.g.items() if v is not None}
        out.update({"p_" + k: v.clone() for k, v in L.p.items() if v is not None})
        out["loss"] = L.loss.clone()
        res.append(out)
    for k in res[0]:
        assert torch.equal(res[0][k], res[1][k]), k


def _random_case(seed):
    """A seeded random local layer: channel counts with and without the multiples of 4 the vector
    paths need, odd map sizes, every filter size / stride / pooling / shortcut the library accepts."""
    g = np.random.default_rng(1000 + seed)
    C = int(g.choice([3, 4, 6, 8, 12, 16, 20, 32]))
    K = int(g.choice([4, 6, 8, 12, 16, 24, 40, 64, 72]))
    A = int(g.choice([1, 3, 4, 8, 12, 16, 20, 32]))
    R = int(g.choice([1, 3, 3, 3, 5]))
    stride = int(g.choice([1, 1, 2]))
    H, W = int(g.integers(max(R, 2), 15)), int(g.integers(max(R, 2), 15))
    pool = None
    kind = int(g.integers(0, 4))
    spec = S(C, H, W, K, A, R=R, stride=stride)
    if kind == 1 and spec.Ho >= 2 and spec.Wo >= 2:
        pool = (2, 2, 0)
    elif kind == 2 and spec.Ho >= 3 and spec.Wo >= 3:
        pool = (3, 2, 1)
    skip = 0
    if pool is None and stride == 1 and kind == 3 and R == 3 and C == K:
        skip = 1
    elif pool is None and stride == 1 and kind == 3:
        skip = 2
    spec = S(C, H, W, K, A, R=R, stride=stride, pool=pool, skip=skip, skip_C=int(g.choice([4, 8, 6])))
    return spec, int(g.integers(2, 9)), int(g.choice([2, 10, 37]))


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_match_oracle(seed):
    spec, B, cls = _random_case(seed)
    print(f"random case {seed}: C={spec.C_in} {spec.H_in}x{spec.W_in} K={spec.C_out} A={spec.A} R={spec.R} "
          f"stride={spec.stride} pool={spec.pool_kind, spec.pool_k} skip={spec.skip_kind} B={B} cls={cls}", flush=True)
    # a small learning rate: with a handful of samples a larger one fits the batch in one step, and
    # the second step's gradient (softmax - onehot ~ 1e-12) is then rounding noise on both sides
    out, final = G.run_step_both(spec, cls, B, seed=200 + seed, lr=0.002, mu=0.9, steps=2,
                                 head_pool=seed % 2, loss_kind=(seed // 2) % 2)
    G.check_step_results(f"random{seed}", out, final)


@pytest.mark.parametrize("name", ["stride2", "skip_projection", "skinny_a8_c128_split"])
def test_eight_steps_stay_within_tolerance(name):
    """Eight consecutive local steps (momentum 0.9) on one batch: the fp32 library and the oracle
    stay within the tolerance step after step — rounding differences do not accumulate beyond it."""
    spec, B, cls = CASES[name]
    out, final = G.run_step_both(spec, cls, B, seed=103, lr=0.005, mu=0.9, steps=8)
    G.check_step_results(name + "/8steps", out, final)
    losses = [o[1][0] for o in out]
    assert losses[-1] < losses[0], losses
