"""Profiler linear models and the Partitioner (Algorithm 1): pins for the oracle
(oracle/partition.py) and, further down, the library's host functions against it.  No GPU."""
import os

import numpy as np
import pytest

from oracle import partition as OP

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        out[k] = v
    return out


def _closed_form(b, rho):
    """Independent statement of the grouping: cut between consecutive layers i, i+1 exactly when
    |b[i+1] - b[i]| > rho * b[i]; a block's batch size is the minimum over its layers."""
    cuts = [0] + [i + 1 for i in range(len(b) - 1) if abs(b[i + 1] - b[i]) > rho * b[i]] + [len(b)]
    return [(list(range(s, e)), min(b[s:e])) for s, e in zip(cuts[:-1], cuts[1:])]


def test_paper_max_batches_and_hand_evaluated_blocks():
    r = _rows("fig6_max_batch_vgg19.txt")
    t = [int(v) for v in r["max_batch"]]
    b = [min(v, 512) for v in t]
    blocks = OP.group(b, 0.4)
    want = [tuple(int(x) for x in item.split(":")) for item in r["blocks_limit512_rho0.4"]]
    assert [(ls[0] + 1, bs) for ls, bs in blocks] == want
    assert blocks == _closed_form(b, 0.4)
    assert sum(len(ls) for ls, _ in blocks) == 16


@pytest.mark.parametrize("seed", range(20))
def test_grouping_equals_closed_form_and_invariants(seed):
    g = np.random.default_rng(seed)
    n = int(g.integers(1, 40))
    b = [int(v) for v in g.integers(1, 600, size=n)]
    if seed % 3 == 0:                      # runs of equal and slowly varying values
        b = sorted(b)
    rho = float(g.choice([0.0, 0.1, 0.4, 0.7, 1.5]))
    blocks = OP.group(b, rho)
    assert blocks == _closed_form(b, rho)
    flat = [i for ls, _ in blocks for i in ls]
    assert flat == list(range(n))                                  # contiguous cover, in order
    for ls, bs in blocks:
        assert bs == min(b[i] for i in ls)
        for i, j in zip(ls[:-1], ls[1:]):
            assert abs(b[j] - b[i]) <= rho * b[i]
    for (la, _), (lb, _) in zip(blocks[:-1], blocks[1:]):
        assert abs(b[lb[0]] - b[la[-1]]) > rho * b[la[-1]]
    if rho == 0.0 and len(set(b)) == n:
        assert len(blocks) == n                                    # all different: singletons


def test_linear_models_on_the_papers_series():
    r = _rows("fig5_memory_vs_batch_vgg11.txt")
    x = [float(v) for v in r["batch"]]
    for k in ("L1", "L2", "L3", "L4", "L5", "L6", "L7", "L8"):
        y = [float(v) for v in r[k]]
        slope, icpt = OP.fit_linear(x, y)
        ps, pi = np.polyfit(x, y, 1)
        assert abs(slope - ps) <= 1e-9 * abs(ps) and abs(icpt - pi) <= 1e-7 * max(1.0, abs(pi))
        # the series are close to lines ("linearly correlates with the batch size")
        pred = np.array(x) * slope + icpt
        assert np.abs(pred - np.array(y)).max() <= 0.04 * max(y)
    # L1 is an exact line through the origin up to the plot's rounding: 17.2 MB per image
    s1, i1 = OP.fit_linear(x, [float(v) for v in r["L1"]])
    assert abs(s1 - 17.19) < 0.01 and abs(i1) < 0.3
    # two points: the line through them
    assert OP.fit_linear([10, 30], [7.0, 15.0]) == pytest.approx((0.4, 3.0))


def test_max_batch_and_partition_end_to_end():
    # mem = 100 + 20 b, budget 630 -> 26 ; exact fit 530/20 = 26.5 -> 26 ; boundary 120+... -> exact
    assert OP.max_batch((20.0, 100.0), 630.0) == 26
    assert OP.max_batch((20.0, 110.0), 630.0) == 26
    assert OP.max_batch((20.0, 10.0), 630.0) == 31
    assert OP.max_batch((20.0, 700.0), 630.0) == 0
    # brute force over integer batch sizes
    g = np.random.default_rng(7)
    for _ in range(200):
        s, c, M = float(g.uniform(0.1, 50)), float(g.uniform(0, 300)), float(g.uniform(50, 2000))
        t = OP.max_batch((s, c), M)
        assert c + s * t <= M + 1e-9 or t == 0
        assert c + s * (t + 1) > M - 1e-9
    # the VGG-11 models of the paper under the 630 MB budget it quotes for VGG-19, limit 512
    r = _rows("fig5_memory_vs_batch_vgg11.txt")
    x = [float(v) for v in r["batch"]]
    models = [OP.fit_linear(x, [float(v) for v in r[f"L{i}"]]) for i in range(1, 9)]
    b, blocks = OP.partition(models, 630.0, 512, 0.4)
    assert b[0] == 36 and b == sorted(b) and b[-1] == 512          # 630 / 17.19 = 36.6
    assert blocks == _closed_form(b, 0.4)
    assert blocks[0][1] == 36 and blocks[-1][1] == 512


# ---- the library's host functions (C ABI, no device work) against the oracle --------------------
@pytest.fixture(scope="module")
def nf():
    from paper_2402_14139_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2402_14139_amd import build
        build.build()
    binding.lib()
    return binding


def test_library_fit_and_partition_match_oracle(nf):
    r = _rows("fig5_memory_vs_batch_vgg11.txt")
    x = [float(v) for v in r["batch"]]
    models = []
    for i in range(1, 9):
        y = [float(v) for v in r[f"L{i}"]]
        s, c = nf.nf_fit_linear(x, y)
        os_, oc = OP.fit_linear(x, y)
        assert abs(s - os_) <= 1e-12 * abs(os_) and abs(c - oc) <= 1e-9 * max(1.0, abs(oc))
        models.append((s, c))
    for M in (100.0, 630.0, 4000.0):
        for rho in (0.0, 0.4, 0.7):
            b, blocks = nf.nf_partition(models, M, 512, rho)
            ob, oblocks = OP.partition(models, M, 512, rho)
            assert b == ob and blocks == [(ls[0], bs) for ls, bs in oblocks], (M, rho)
    # the paper's printed per-layer maximum batch sizes: models with slope 1, intercept 0 and a
    # budget of t reproduce t
    t = [int(v) for v in _rows("fig6_max_batch_vgg19.txt")["max_batch"]]
    got = []
    for ti in t:
        b, _ = nf.nf_partition([(1.0, 0.0)], float(ti), 512, 0.4)
        got.append(b[0])
    assert got == [min(v, 512) for v in t]
    lm = [(630.0 / (v + 0.5), 0.0) for v in t]            # each layer fits exactly t[v] samples in 630
    b, blocks = nf.nf_partition(lm, 630.0, 512, 0.4)
    assert b == [min(v, 512) for v in t]
    assert [(f + 1, bs) for f, bs in blocks] == [(1, 30), (4, 60), (5, 90), (9, 195), (13, 512)]


@pytest.mark.parametrize("seed", range(10))
def test_library_partition_random(nf, seed):
    g = np.random.default_rng(100 + seed)
    n = int(g.integers(1, 50))
    models = [(float(g.uniform(0.05, 40)), float(g.uniform(0, 200))) for _ in range(n)]
    M, B, rho = float(g.uniform(100, 5000)), int(g.integers(1, 1024)), float(g.choice([0.0, 0.2, 0.4, 1.0]))
    b, blocks = nf.nf_partition(models, M, B, rho)
    ob, oblocks = OP.partition(models, M, B, rho)
    assert b == ob and blocks == [(ls[0], bs) for ls, bs in oblocks]


def test_library_byte_model_and_profile(nf):
    """The byte count is what a caller really allocates for one local step: checked against a
    plain sum over the tensors of the step; it is affine in B apart from the alignment and split
    choices of the workspace (split-reduction partials), so the fitted line predicts it only to within 25 %; Algorithm 1
    on the ResNet-18-style network under 256 MiB yields non-decreasing block batch sizes."""
    import workloads
    cfg = workloads.config("cfg3")
    models = []
    for ls in cfg.layers:
        d, a = nf.LayerDesc(**ls.layer_desc_fields()), nf.AuxDesc(**ls.aux_desc_fields(cfg.n_classes))
        for B in (8, 64):
            got = nf.nf_layer_step_bytes(d, a, B, True)
            params = ls.C_out * ls.C_in * ls.R * ls.S + ls.C_out + (ls.C_out * ls.skip_C if ls.skip_kind == 2 else 0)
            params += ls.A * 9 * ls.C_out + ls.A + cfg.n_classes * 4 * ls.A + cfg.n_classes
            act = B * (ls.C_in * ls.H_in * ls.W_in + ls.C_out * ls.Hp * ls.Wp
                       + (ls.skip_C * ls.skip_H * ls.skip_W if ls.skip_kind else 0))
            want = 4 * (3 * params + act) + 4 * B + 4 + nf.nf_workspace_bytes(d, a, B)
            assert got == want
            assert nf.nf_layer_step_bytes(d, a, B, False) == want - 4 * params
        batches = [16, 32, 64, 128, 256]
        s, c = nf.nf_profile_layer(d, a, True, batches)
        os_, oc = OP.fit_linear(batches, [nf.nf_layer_step_bytes(d, a, B, True) for B in batches])
        assert abs(s - os_) <= 1e-9 * os_ and abs(c - oc) <= 1e-6 * max(1.0, abs(oc))
        for B in (48, 200):
            exact = nf.nf_layer_step_bytes(d, a, B, True)
            assert abs(s * B + c - exact) <= 0.25 * exact, (ls.name, B, s * B + c, exact)
        models.append((s, c))
    b, blocks = nf.nf_partition(models, float(256 << 20), 512, 0.4)
    ob, oblocks = OP.partition(models, float(256 << 20), 512, 0.4)
    assert b == ob and blocks == [(ls[0], bs) for ls, bs in oblocks]
    sizes = [bs for _, bs in blocks]
    assert sizes == sorted(sizes) and 0 < sizes[0] < sizes[-1] <= 512 and len(blocks) >= 2
    print("cfg3 under 256 MiB:", b, blocks)


def test_library_partition_rejects_bad_arguments(nf):
    import ctypes as C
    L = nf.lib()
    R = (nf.LinearModel * 2)(nf.LinearModel(1.0, 0.0), nf.LinearModel(2.0, 0.0))
    o = (C.c_int32 * 2)()
    nb = C.c_int32()
    assert L.nf_partition(2, None, 10.0, 8, 0.4, None, o, o, C.byref(nb)) == nf.NF_ERR_NULL
    assert L.nf_partition(0, R, 10.0, 8, 0.4, None, o, o, C.byref(nb)) == nf.NF_ERR_BAD_DESC
    assert L.nf_partition(2, R, 10.0, 0, 0.4, None, o, o, C.byref(nb)) == nf.NF_ERR_BAD_DESC
    assert L.nf_partition(2, R, 10.0, 8, -0.1, None, o, o, C.byref(nb)) == nf.NF_ERR_BAD_DESC
    assert L.nf_partition(2, R, 10.0, 8, 0.4, None, o, o, C.byref(nb)) == nf.NF_OK and nb.value >= 1
    m = nf.LinearModel()
    x = (C.c_double * 2)(4.0, 4.0)
    assert L.nf_fit_linear(2, x, x, C.byref(m)) == nf.NF_ERR_BAD_DESC      # equal batch sizes: no line
    assert L.nf_fit_linear(1, x, x, C.byref(m)) == nf.NF_ERR_BAD_DESC
