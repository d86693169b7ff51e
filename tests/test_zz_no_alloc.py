"""nf_local_step_static (the entry point for callers that cannot allocate: its scratch is a static
device array inside the library) against nf_local_step with a caller workspace: same kernels, so
every output must be bit-for-bit equal.  Two calls in a row, the second on a smaller input, so the
second runs over whatever the first left in the shared array."""
import numpy as np
import pytest
import torch

import workloads
from paper_2402_14139_amd import binding as nf
from paper_2402_14139_amd import layout
from paper_2402_14139_amd.layer import PARAM_NAMES, LocalLayer
from tests import gpu_common as G

pytestmark = pytest.mark.gpu


def _case(spec, cls, B, seed, lr=0.01, mu=0.9, steps=2):
    """Runs `steps` local steps from the same start through both entry points; returns the two
    result lists (y, loss, gradients, parameters, momentum as device tensors)."""
    x, xs, labels, p = G.make_inputs(spec, B, cls, seed)
    xd, xsd, ld = G.to_dev(layout.act_to_lib(x)), G.to_dev(None if xs is None else layout.act_to_lib(xs)), G.to_dev(labels)
    res = []
    for static in (False, True):
        L = G.gpu_layer(spec, cls, p, B, True)
        assert L.ws_bytes <= nf.NF_STATIC_SCRATCH_BYTES
        out = []
        for _ in range(steps):
            y = L.new_output(B)
            if static:
                nf.nf_local_step_static(L.d, L.a, lr, mu, B, xd, xsd, ld, L.sp, L.sa, L.sgp, L.sga, L.svp, L.sva,
                                        y, L.loss)
            else:
                nf.nf_local_step(L.d, L.a, lr, mu, B, xd, xsd, ld, L.sp, L.sa, L.sgp, L.sga, L.svp, L.sva, y,
                                 L.loss, L.ws)
            torch.cuda.synchronize()
            out.append([y, L.loss.clone()] + [getattr(L, w)[k].clone() for w in ("g", "p", "v") for k in PARAM_NAMES
                                              if L.p[k] is not None])
        res.append(out)
    return res


def _assert_same(tag, res):
    ws_res, static_res = res
    for si, (a, b) in enumerate(zip(ws_res, static_res)):
        for ti, (u, v) in enumerate(zip(a, b)):
            assert torch.isfinite(v).all(), f"{tag} step {si} tensor {ti}: non-finite"
            assert torch.equal(u, v), f"{tag} step {si} tensor {ti}: static-scratch call differs from nf_local_step"
            G.assert_close(f"{tag} step {si} tensor {ti}", v.cpu().numpy(), u.cpu().numpy())


def test_static_scratch_step_equals_workspace_step_twice_in_a_row():
    L = workloads.LayerSpec
    big = L("big", 64, 16, 16, 64, A=16, skip_kind=1, skip_C=64, skip_H=16, skip_W=16, skip_stride=1)
    small = L("small", 8, 12, 12, 24, A=8, pool_kind=1, pool_k=2, pool_stride=2)
    print("nf_local_step_static: big  64->64 16x16 identity shortcut B=48", flush=True)
    _assert_same("big", _case(big, 100, 48, seed=301))
    print("nf_local_step_static: small 8->24 12x12 pooled B=5", flush=True)
    _assert_same("small", _case(small, 10, 5, seed=302))


def test_static_scratch_full_size_layer():
    """A ResNet-18-style stage-4 layer at its block batch size 512 (89 MiB of scratch)."""
    cfg = workloads.config("cfg3")
    spec = cfg.layers[15]
    print("nf_local_step_static: cfg3 layer 15 B=512", flush=True)
    _assert_same("cfg3[15]", _case(spec, cfg.n_classes, 512, seed=303, lr=1e-3, steps=1))
