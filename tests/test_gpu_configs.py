"""GPU parity on the benchmark configurations' own layer shapes.

* the ResNet-18-style configuration at FULL block batch sizes (64/128/256/512), i.e. in the
  launch configuration bench.py times: every one of its 17 layers, whole local step against
  the oracle;
* every layer of the VGG-11-style configuration and sampled layers of the VGG-16- and
  ResNet-34-style ones at a reduced batch (the oracle is a plain loop nest).
"""
import pytest

import workloads
from tests import gpu_common as G

pytestmark = pytest.mark.gpu


def _run(cfg_name, li, B, steps=1):
    cfg = workloads.config(cfg_name)
    spec = cfg.layers[li]
    print(f"{cfg_name} layer {li} ({spec.name}) B={B}", flush=True)
    out, final = G.run_step_both(spec, cfg.n_classes, B, seed=cfg.seed * 100 + li, lr=cfg.lr, mu=cfg.momentum,
                                 steps=steps, bias_std=0.05)
    G.check_step_results(f"{cfg_name}[{li}]", out, final)


@pytest.mark.parametrize("li", list(range(17)))
def test_cfg3_full_batch(li):
    cfg = workloads.config("cfg3")
    _run("cfg3", li, cfg.blocks[cfg.layers[li].block].batch)


@pytest.mark.parametrize("li", list(range(8)))
def test_cfg2_all_layers_small_batch(li):
    _run("cfg2", li, 8, steps=2)


@pytest.mark.parametrize("li", list(range(8)))
def test_cfg2_all_layers_full_batch(li):
    """The VGG-11-style configuration at its own batch size 128.  Its late layers have 2x2 .. 4x4
    maps: few output tiles, so the forward, the head's convolution and the data gradient all run
    with a split reduction."""
    _run("cfg2", li, 128)


@pytest.mark.parametrize("li", [0, 1, 3, 6, 9, 12])
def test_cfg4_sampled_layers_small_batch(li):
    _run("cfg4", li, 2)


@pytest.mark.parametrize("li", [0, 1, 8, 16, 32])
def test_cfg5_sampled_layers_small_batch(li):
    _run("cfg5", li, 2)


@pytest.mark.parametrize("cfg_name,li", [("cfg3_aan", 5), ("cfg3_aan", 6), ("cfg3_aan", 10), ("cfg3_aan", 16),
                                         ("cfg3_ll256", 0), ("cfg3_ll256", 2)])
def test_wide_heads_full_batch(cfg_name, li):
    """The paper's own head widths (32 before the first down-sampling, 256 after; 256 everywhere
    for classic local learning) on the ResNet-18-style network at full block batch: the head's
    convolution, its weight gradient and its data gradient are then full-width MFMA GEMMs."""
    cfg = workloads.config(cfg_name)
    _run(cfg_name, li, cfg.blocks[cfg.layers[li].block].batch)


@pytest.mark.parametrize("cfg_name,li", [("cfg4", 0), ("cfg4", 1), ("cfg4", 3), ("cfg4", 6), ("cfg4", 8), ("cfg4", 12),
                                         ("cfg5", 0), ("cfg5", 1), ("cfg5", 7), ("cfg5", 8), ("cfg5", 15),
                                         ("cfg5", 16), ("cfg5", 21), ("cfg5", 27), ("cfg5", 28)])
def test_cfg4_cfg5_sampled_layers_full_batch(cfg_name, li):
    """The VGG-16- and ResNet-34-style configurations at their own block batch sizes (32 ... 512):
    64x64 and 128x128 inputs, the 7x7 stride-2 stem with its 3x3/s2/p1 max-pool, pooled VGG layers,
    stride-2 and projection-shortcut layers, the 512-sample stage-3 layers."""
    cfg = workloads.config(cfg_name)
    _run(cfg_name, li, cfg.blocks[cfg.layers[li].block].batch)
