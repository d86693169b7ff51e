"""GPU parity on the benchmark configurations' own layer shapes.

* the ResNet-18-style configuration at FULL block batch sizes (64/128/256/512), i.e. in the
  launch configuration bench.py times: every one of its 17 layers, whole local step against
  the oracle;
* every layer of the VGG-11-style configuration at a reduced batch (two steps) and at its own;
* every distinct layer of the VGG-16- and ResNet-34-style configurations at its block's own batch
  size, plus sampled ones at a reduced batch.
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


def distinct_layers(cfg_name):
    """Index of the first layer of every distinct (layer descriptor, head width, block batch size)
    of a configuration, and for every layer the representative it equals."""
    cfg = workloads.config(cfg_name)
    first, rep = {}, []
    for i, ls in enumerate(cfg.layers):
        key = (tuple(sorted(ls.layer_desc_fields().items())), ls.A, cfg.blocks[ls.block].batch)
        rep.append(first.setdefault(key, i))
    return sorted(set(rep)), rep


@pytest.mark.parametrize("cfg_name,li", [(c, i) for c in ("cfg4", "cfg5") for i in distinct_layers(c)[0]])
def test_cfg4_cfg5_every_layer_full_batch(cfg_name, li):
    """The VGG-16- and ResNet-34-style configurations at their own block batch sizes (32 ... 512):
    every layer, one whole local step against the oracle.  Layers that repeat an earlier one exactly
    (same descriptor, head width and batch size: 1 of 13 and 16 of 33) are represented by it.
    Covers 64x64 and 128x128 inputs, the 7x7 stride-2 stem with its 3x3/s2/p1 max-pool, pooled VGG
    layers, stride-2 and projection-shortcut layers, identity shortcuts, the 512-sample stage-3 layers."""
    cfg = workloads.config(cfg_name)
    _run(cfg_name, li, cfg.blocks[cfg.layers[li].block].batch)
