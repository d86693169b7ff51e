"""Helpers shared by the GPU parity tests: run the library on numpy inputs given in the
paper's notation and hand back numpy results in the same notation."""
import numpy as np
import torch

import oracle as O
import workloads
from paper_2402_14139_amd import binding as nf
from paper_2402_14139_amd import layout
from paper_2402_14139_amd.layer import PARAM_NAMES, LocalLayer

REL = 1e-4  # tolerance of the build target: 1e-4 relative on losses, gradients, updated weights


def assert_close(name, got, ref, rel=REL):
    """norm-wise and max-wise relative error against the oracle (element-wise relative error
    is meaningless for gradients, which have entries arbitrarily close to zero)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    nr, mr = np.linalg.norm(ref), np.abs(ref).max() if ref.size else 0.0
    diff = got - ref
    if nr == 0.0:
        assert np.abs(got).max() <= 1e-30, f"{name}: oracle is all-zero, library is not"
        return
    e2, em = np.linalg.norm(diff) / nr, np.abs(diff).max() / mr
    assert e2 <= rel and em <= rel, f"{name}: l2 rel {e2:.3e}, max rel {em:.3e} (limit {rel:g})"


def to_dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def descs(spec, n_classes, relu=1):
    lf = spec.layer_desc_fields()
    af = spec.aux_desc_fields(n_classes)
    af["relu"] = relu
    return (nf.LayerDesc(**lf), nf.AuxDesc(**af)), (O.layer_desc(**lf), O.aux_desc(**af))


def make_inputs(spec, B, n_classes, seed, bias_std=0.1, post_relu_input=False):
    g = workloads.rng_for(seed, "gpu-parity", spec.C_in, spec.H_in, spec.C_out, spec.stride, B)
    x = g.standard_normal((B, spec.C_in, spec.H_in, spec.W_in)).astype(np.float32)
    if post_relu_input:
        x = np.maximum(x, 0)
    xs = None
    if spec.skip_kind:
        xs = np.maximum(g.standard_normal((B, spec.skip_C, spec.skip_H, spec.skip_W)), 0).astype(np.float32)
    labels = g.integers(0, n_classes, size=(B,)).astype(np.int32)
    p = workloads.gen_layer_params(seed, 0, spec, n_classes, bias_std=bias_std)
    return x, xs, labels, p


def gpu_layer(spec, n_classes, p, B, momentum, relu=1):
    (d, a), _ = descs(spec, n_classes, relu)
    return LocalLayer(d, a, layout.params_to_lib(p, spec.A), B, momentum)


def run_step_both(spec, n_classes, B, seed, lr, mu, steps=1, relu=1, bias_std=0.1):
    """Runs `steps` local steps on the same batch through the library and the oracle; returns
    per-step (loss, grads, y) for both and the final params/momentum for both."""
    x, xs, labels, p = make_inputs(spec, B, n_classes, seed, bias_std)
    (_, _), (od, oa) = descs(spec, n_classes, relu)
    L = gpu_layer(spec, n_classes, p, B, mu != 0, relu)
    xd, xsd, ld = to_dev(layout.act_to_lib(x)), to_dev(None if xs is None else layout.act_to_lib(xs)), to_dev(labels)
    po = {k: (None if v is None else v.copy()) for k, v in p.items()}
    mo = {k: (None if v is None else np.zeros_like(v)) for k, v in p.items()} if mu != 0 else None
    out = []
    for _ in range(steps):
        y = L.step(xd, xsd, ld, lr, mu)
        torch.cuda.synchronize()
        g_loss = float(L.loss.item())
        g_grads = L.params_numpy("g")
        g_y = layout.act_from_lib(y.cpu().numpy())
        oY, oloss, ograds = O.local_step(od, oa, x, xs, labels, po, mo, lr, mu)
        out.append(((g_loss, g_grads, g_y), (oloss, ograds, oY)))
    final = (L.params_numpy("p"), L.params_numpy("v") if mu != 0 else None), (po, mo)
    return out, final


def check_step_results(tag, out, final):
    for si, ((gl, gg, gy), (ol, og, oy)) in enumerate(out):
        assert abs(gl - ol) <= REL * abs(ol), f"{tag} step {si}: loss {gl} vs {ol}"
        assert_close(f"{tag} step {si} y", gy, oy)
        for k in PARAM_NAMES:
            if og[k] is not None:
                assert_close(f"{tag} step {si} grad {k}", gg[k], og[k])
    (gp, gv), (op, ov) = final
    for k in PARAM_NAMES:
        if op[k] is not None:
            assert_close(f"{tag} updated {k}", gp[k], op[k])
            if ov is not None:
                assert_close(f"{tag} momentum {k}", gv[k], ov[k])
