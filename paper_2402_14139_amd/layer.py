"""Device-side state of one local layer (parameters, gradients, momentum, workspace) and the
calls of include/nf.h on it.  Host bookkeeping only — all arithmetic is in libnf's kernels.

Paper: one local layer = theta_n with its auxiliary head (beta_n, gamma_n), trained by the
body of Algorithm 2.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as nf
from . import layout

PARAM_NAMES = ("W", "b", "Wp", "Wa", "ba", "Wf", "bf")


def make_descs(spec, n_classes):
    """(LayerDesc, AuxDesc) from a workloads.LayerSpec-like object."""
    d = nf.LayerDesc(**spec.layer_desc_fields())
    a = nf.AuxDesc(**spec.aux_desc_fields(n_classes))
    return d, a


class LocalLayer:
    def __init__(self, d: nf.LayerDesc, a: nf.AuxDesc, params_lib: dict, max_batch: int, momentum: bool,
                 device="cuda", own_workspace: bool = True):
        if not torch.cuda.is_available():
            raise RuntimeError("LocalLayer needs a GPU: the library has no CPU path")
        nf.lib()
        self.d, self.a, self.device = d, a, device
        self.max_batch = max_batch
        self.Ho, self.Wo, self.Hp, self.Wp = nf.nf_layer_out_dims(d)
        self.p = {k: (None if params_lib.get(k) is None else torch.from_numpy(np.ascontiguousarray(params_lib[k])).to(device))
                  for k in PARAM_NAMES}
        self.g = {k: (None if v is None else torch.zeros_like(v)) for k, v in self.p.items()}
        self.v = {k: (None if v is None else torch.zeros_like(v)) for k, v in self.p.items()} if momentum else None
        # layers driven through the block-level calls share the block's workspace instead
        self.ws_bytes = nf.nf_workspace_bytes(d, a, max_batch) if own_workspace else 0
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device) if own_workspace else None
        self.loss = torch.zeros(1, dtype=torch.float32, device=device)
        self._structs()

    def _structs(self):
        lp = lambda t: nf.layer_params(t["W"], t["b"], t["Wp"])          # noqa: E731
        ap = lambda t: nf.aux_params(t["Wa"], t["ba"], t["Wf"], t["bf"])  # noqa: E731
        self.sp, self.sa = lp(self.p), ap(self.p)
        self.sgp, self.sga = lp(self.g), ap(self.g)
        self.svp, self.sva = (lp(self.v), ap(self.v)) if self.v is not None else (None, None)

    def new_output(self, B):
        return torch.empty((B, self.Hp, self.Wp, self.d.C_out), dtype=torch.float32, device=self.device)

    def forward(self, x, x_skip=None, y=None):
        B = x.shape[0]
        y = self.new_output(B) if y is None else y
        nf.nf_layer_fwd(self.d, B, x, x_skip, self.sp, y, self.ws)
        return y

    def aux_loss(self, y, labels):
        nf.nf_aux_fwd_loss(self.d, self.a, y.shape[0], y, labels, self.sa, self.loss, self.ws)
        return self.loss

    def backward(self, x, x_skip, y):
        nf.nf_local_bwd_wgrad(self.d, self.a, x.shape[0], x, x_skip, y, self.sp, self.sa, self.sgp, self.sga,
                              self.ws)

    def sgd(self, lr, momentum):
        names = [k for k in PARAM_NAMES if self.p[k] is not None]
        nf.nf_sgd_update(lr, momentum, [self.p[k] for k in names], [self.g[k] for k in names],
                         [self.v[k] for k in names] if (self.v is not None and momentum != 0) else None)

    def step(self, x, x_skip, labels, lr, momentum, y=None):
        """One pass of the Algorithm 2 body; returns y (emitted with the pre-update weights)."""
        B = x.shape[0]
        y = self.new_output(B) if y is None else y
        nf.nf_local_step(self.d, self.a, lr, momentum, B, x, x_skip, labels, self.sp, self.sa, self.sgp, self.sga,
                         self.svp, self.sva, y, self.loss, self.ws)
        return y

    def params_numpy(self, which="p"):
        src = getattr(self, which)
        lib_np = {k: (None if v is None else v.detach().cpu().numpy()) for k, v in src.items()}
        return layout.params_from_lib(lib_np, self.a.A, self.a.pool_oh, self.a.pool_ow)
