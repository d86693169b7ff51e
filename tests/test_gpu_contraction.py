"""GPU parity of the optional contraction modes NF_CONTRACT_BF16X6 / NF_CONTRACT_BF16X9: the wide
convolutions and weight gradients on the bf16 matrix cores, each fp32 operand cut into three bfloat16
pieces, six or all nine piece products per multiply-add.

Same oracle, same seeded inputs, same tolerances (1e-4 relative; ReLU / arg-max decisions compared
inside the oracle's own tie band) as the default mode: the mode is a different way to carry out an
fp32 contraction, not a lower precision.  The whole GPU suite can also be run in this mode with
NF_CONTRACTION=bf16x6 (or bf16x9) in the environment.
"""
import numpy as np
import pytest

import workloads
from paper_2402_14139_amd import binding as B
from tests import gpu_common as G

pytestmark = pytest.mark.gpu


MODES = {"bf16x6": B.NF_CONTRACT_BF16X6, "bf16x9": B.NF_CONTRACT_BF16X9}


@pytest.fixture(params=list(MODES))
def split_mode(request):
    prev = B.nf_contraction(MODES[request.param])
    yield request.param
    B.nf_contraction(prev)


def _run(cfg_name, li, batch, steps=1):
    cfg = workloads.config(cfg_name)
    spec = cfg.layers[li]
    mode = {v: k for k, v in MODES.items()}[B.nf_contraction()]
    print(f"{cfg_name} layer {li} ({spec.name}) B={batch} {mode}", flush=True)
    out, final = G.run_step_both(spec, cfg.n_classes, batch, seed=cfg.seed * 100 + li, lr=cfg.lr, mu=cfg.momentum,
                                 steps=steps, bias_std=0.05)
    G.check_step_results(f"{cfg_name}[{li}] {mode}", out, final)
    return out, final


# cfg3: 128 / 256 / 512 filters, stride-2 layers with the 1x1 projection appended to the reduction
# (6, 10, 14), identity shortcuts (8, 12, 16), plain ones; full block batch = the shapes bench.py times
@pytest.mark.parametrize("li", [5, 6, 7, 8, 9, 10, 12, 13, 14, 15, 16])
def test_cfg3_wide_layers_full_batch(split_mode, li):
    cfg = workloads.config("cfg3")
    _run("cfg3", li, cfg.blocks[cfg.layers[li].block].batch)


# cfg2: pooled layers, 2x2 .. 4x4 maps (the forward reduction is split over workgroups there)
@pytest.mark.parametrize("li", [1, 2, 3, 4, 5, 7])
def test_cfg2_wide_layers_full_batch(split_mode, li):
    _run("cfg2", li, 128)


# ragged sizes: a batch that leaves the last 128-row tile and the last reduction step partly filled,
# two steps with momentum
@pytest.mark.parametrize("cfg_name,li,batch", [("cfg3", 10, 37), ("cfg3", 14, 75), ("cfg2", 3, 13), ("cfg4", 9, 5)])
def test_ragged_batches_two_steps(split_mode, cfg_name, li, batch):
    _run(cfg_name, li, batch, steps=2)


def test_mode_changes_the_kernels_and_keeps_the_accuracy():
    """One 512-filter layer in all modes against the fp64 oracle: the forward output's error in the
    split modes stays within twice the error of the fp32 matrix-core instructions (measured: equal),
    and the modes do differ in the last bits (i.e. the switch reaches the kernels)."""
    cfg = workloads.config("cfg3")
    li = 15
    spec = cfg.layers[li]
    batch = 64
    errs, ys = {}, {}
    for mode in (B.NF_CONTRACT_F32, B.NF_CONTRACT_BF16X6, B.NF_CONTRACT_BF16X9):
        prev = B.nf_contraction(mode)
        try:
            out, _ = G.run_step_both(spec, cfg.n_classes, batch, seed=777, lr=cfg.lr, mu=cfg.momentum, steps=1,
                                     bias_std=0.05)
        finally:
            B.nf_contraction(prev)
        (_, _, gy), (_, _, oy), _ = out[0]
        errs[mode] = float(np.sqrt(np.mean((np.asarray(gy, dtype=np.float64) - np.asarray(oy, dtype=np.float64)) ** 2)))
        ys[mode] = np.asarray(gy)
    print(f"rms error of y against the oracle: fp32 MFMA {errs[0]:.3e}, bf16x6 {errs[1]:.3e}, "
          f"bf16x9 {errs[2]:.3e}", flush=True)
    assert errs[B.NF_CONTRACT_BF16X6] <= 2.0 * errs[B.NF_CONTRACT_F32] + 1e-9
    assert errs[B.NF_CONTRACT_BF16X9] <= 2.0 * errs[B.NF_CONTRACT_F32] + 1e-9
    assert not np.array_equal(ys[0], ys[1])
    assert not np.array_equal(ys[0], ys[2])


def test_split_mode_is_deterministic(split_mode):
    cfg = workloads.config("cfg3")
    spec = cfg.layers[11]
    runs = []
    for _ in range(2):
        out, final = G.run_step_both(spec, cfg.n_classes, 32, seed=4242, lr=cfg.lr, mu=cfg.momentum, steps=2,
                                     bias_std=0.05)
        runs.append((out, final))
    for ((la, ga, ya), _, _), ((lb, gb, yb), _, _) in zip(runs[0][0], runs[1][0]):
        assert la == lb
        assert np.array_equal(ya, yb)
        for k in G.PARAM_NAMES:
            if ga[k] is not None:
                assert np.array_equal(ga[k], gb[k]), k
    (pa, va), (pb, vb) = runs[0][1][0], runs[1][1][0]
    for k in G.PARAM_NAMES:
        if pa[k] is not None:
            assert np.array_equal(pa[k], pb[k]), k
            if va is not None:
                assert np.array_equal(va[k], vb[k]), k


def test_narrow_layers_are_untouched_by_the_mode():
    """A 64-filter layer has no wide contraction: both modes run the same kernels, bit for bit."""
    cfg = workloads.config("cfg3")
    spec = cfg.layers[1]
    res = {}
    for mode in (B.NF_CONTRACT_F32, B.NF_CONTRACT_BF16X6, B.NF_CONTRACT_BF16X9):
        prev = B.nf_contraction(mode)
        try:
            out, final = G.run_step_both(spec, cfg.n_classes, 16, seed=99, lr=cfg.lr, mu=cfg.momentum, steps=1,
                                         bias_std=0.05)
        finally:
            B.nf_contraction(prev)
        res[mode] = (out[0][0], final[0][0])
    (la, ga, ya), pa = res[B.NF_CONTRACT_F32]
    for other in (B.NF_CONTRACT_BF16X6, B.NF_CONTRACT_BF16X9):
        (lb, gb, yb), pb = res[other]
        assert la == lb and np.array_equal(ya, yb)
        for k in G.PARAM_NAMES:
            if ga[k] is not None:
                assert np.array_equal(ga[k], gb[k]), k
                assert np.array_equal(pa[k], pb[k]), k
