"""Controller of NeuroFlux (arXiv 2402.14139, "Modules" and "Trained Output CNN") on top of the
library's block-level calls: partition the network into blocks (Profiler models + Algorithm 1),
train the blocks one after the other (each from the cache the previous one left), fill the next
cache once a block is trained, evaluate every early exit on a validation set and pick the output
model.  Host bookkeeping only — every arithmetic step is a call of include/nf.h.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import binding as nf

PROBE_BATCHES = (16, 32, 64, 128, 256)


@dataclass
class BlockPlan:
    first: int      # index of the block's first layer
    last: int       # index of its last layer (inclusive)
    batch: int


def plan_blocks(specs, n_classes, momentum: bool, memory_budget_bytes: float, batch_limit: int, rho: float = 0.4,
                probe_batches=PROBE_BATCHES):
    """Profiler + Partitioner.  ``specs``: layer tables (``layer_desc_fields()``,
    ``aux_desc_fields(n_classes)``, ``skip_kind``, ``skip_src`` = index of the layer whose input
    is the shortcut).  Returns (per-layer batch sizes, list of BlockPlan).

    The paper does not say what happens when Algorithm 1 cuts between the two convolutions of a
    residual basic block; here such a cut is removed (the two blocks are merged, the merged
    block taking the smaller batch size), because the second convolution needs the basic
    block's input, which only exists inside the block that computes the first."""
    models = []
    for ls in specs:
        d, a = nf.LayerDesc(**ls.layer_desc_fields()), nf.AuxDesc(**ls.aux_desc_fields(n_classes))
        models.append(nf.nf_profile_layer(d, a, momentum, list(probe_batches)))
    b, blocks = nf.nf_partition(models, float(memory_budget_bytes), int(batch_limit), float(rho))
    if min(b) <= 0:
        raise ValueError(f"a layer does not fit the memory budget even at batch size 1: {b}")
    firsts = [f for f, _ in blocks] + [len(specs)]
    plans = [BlockPlan(firsts[k], firsts[k + 1] - 1, bs) for k, (_, bs) in enumerate(blocks)]
    return b, respect_shortcuts(plans, specs)


def respect_shortcuts(plans, specs):
    """Merges a block into its predecessor(s) until every shortcut source lies inside the block."""
    def needs_earlier(p):
        return any(specs[l].skip_kind and specs[l].skip_src < p.first for l in range(p.first, p.last + 1))

    out = []
    for p in plans:
        while needs_earlier(p) and out:
            q = out.pop()
            p = BlockPlan(q.first, p.last, min(q.batch, p.batch))
        out.append(p)
    return out


class Trainer:
    """Device state of a whole network and the Controller's loop over its blocks."""

    def __init__(self, specs, n_classes, params, plans, momentum: bool, device="cuda", head_pool=0, loss_kind=0):
        import torch
        from . import layout
        from .layer import LocalLayer
        if not torch.cuda.is_available():
            raise RuntimeError("Trainer needs a GPU: the library has no CPU path")
        self.torch, self.specs, self.n_classes, self.plans, self.device = torch, specs, n_classes, plans, device
        self.momentum = momentum
        self.layers, self.blocks, self.ws = [], [], []
        for plan in plans:
            Ls = []
            for li in range(plan.first, plan.last + 1):
                ls = specs[li]
                d, a = nf.LayerDesc(**ls.layer_desc_fields()), nf.AuxDesc(**ls.aux_desc_fields(n_classes))
                a.head_pool, a.loss_kind = head_pool, loss_kind
                Ls.append(LocalLayer(d, a, layout.params_to_lib(params[li], ls.A), plan.batch, momentum, device,
                                     own_workspace=False))
            skip = [(-1 if not specs[li].skip_kind else specs[li].skip_src - plan.first)
                    for li in range(plan.first, plan.last + 1)]
            blk = nf.make_block([l.d for l in Ls], [l.a for l in Ls], skip, [l.sp for l in Ls], [l.sa for l in Ls],
                                [l.sgp for l in Ls], [l.sga for l in Ls], [l.svp for l in Ls] if momentum else None,
                                [l.sva for l in Ls] if momentum else None)
            self.layers += Ls
            self.blocks.append(blk)
            self.ws.append(torch.empty(nf.nf_block_workspace_bytes(blk, plan.batch), dtype=torch.uint8, device=device))

    def _sample_elems(self, k):
        """Row length of the cache that feeds block k (k == len(plans): the network's output)."""
        if k == 0:
            f = self.specs[0]
            return f.C_in * f.H_in * f.W_in
        last = self.specs[self.plans[k - 1].last]
        return last.C_out * last.Hp * last.Wp

    def _sweep(self, k, cache, labels, n):
        """Forward-only sweep of block k with its current weights: the cache of block k+1."""
        torch = self.torch
        out = torch.empty((n, self._sample_elems(k + 1)), dtype=torch.float32, device=self.device)
        olab = torch.empty((n,), dtype=torch.int32, device=self.device)
        nf.nf_block_fill_cache(self.blocks[k], self.plans[k].batch, n, cache, labels, n, out, olab, n, self.ws[k])
        return out, olab

    def train(self, data, labels, epochs: int, lr: float, mu: float, seed: int = 0, prefetch_stream=None):
        """Blocks are trained one after the other; block k reads the cache block k-1 left.
        ``data`` [N, C*H*W] rows in the library's layout (H, W, C), ``labels`` int32 [N], both on
        the device.  Returns the per-block loss tensors [epochs, n_batches, n_layers] (device)."""
        torch = self.torch
        N = data.shape[0]
        cache, clab, losses = data, labels, []
        for k, plan in enumerate(self.plans):
            nb = (N + plan.batch - 1) // plan.batch
            lk = torch.zeros((epochs, nb, plan.last - plan.first + 1), dtype=torch.float32, device=self.device)
            for e in range(epochs):
                perm = np.random.Generator(np.random.Philox(key=[seed, k * 1000003 + e])).permutation(N)
                idx = torch.from_numpy(perm.astype(np.int64)).to(self.device)
                nf.nf_block_train_epoch(self.blocks[k], lr, mu, plan.batch, N, cache, clab, N, idx, lk[e], self.ws[k],
                                        prefetch_stream=prefetch_stream)
            losses.append(lk)
            if k + 1 < len(self.plans):
                cache, clab = self._sweep(k, cache, clab, N)
        return losses

    def evaluate_exits(self, data, labels):
        """Number of correct predictions of every early exit (one per layer) on a validation set,
        and the parameter count of the model that ends at that exit."""
        torch = self.torch
        N = data.shape[0]
        cache, clab = data, labels
        correct, n_params, body = [], [], 0
        pred = torch.empty((N,), dtype=torch.int32, device=self.device)
        cnt = torch.zeros((1,), dtype=torch.int32, device=self.device)
        li = 0
        for k, plan in enumerate(self.plans):
            for e in range(plan.last - plan.first + 1):
                nf.nf_block_evaluate(self.blocks[k], e, plan.batch, N, cache, clab, N, pred, cnt, self.ws[k])
                correct.append(int(cnt.item()))
                L = self.layers[li]
                body += sum(L.p[n].numel() for n in ("W", "b", "Wp") if L.p[n] is not None)
                n_params.append(body + sum(L.p[n].numel() for n in ("Wa", "ba", "Wf", "bf")))
                li += 1
            if k + 1 < len(self.plans):
                cache, clab = self._sweep(k, cache, clab, N)
        return correct, n_params

    def select_exit(self, correct, n_params) -> int:
        return nf.nf_select_exit(correct, n_params)

    def predict(self, data, exit_layer: int):
        """Classes predicted by the early-exit model that ends after layer ``exit_layer`` (global
        index) for ``data`` [N, C*H*W] (library layout, on the device).  Returns int32 [N]."""
        torch = self.torch
        N = data.shape[0]
        pred = torch.empty((N,), dtype=torch.int32, device=self.device)
        cache = data
        for k, plan in enumerate(self.plans):
            if exit_layer <= plan.last:
                nf.nf_block_evaluate(self.blocks[k], exit_layer - plan.first, plan.batch, N, cache, None, N, pred,
                                     None, self.ws[k])
                return pred
            dummy = torch.zeros((N,), dtype=torch.int32, device=self.device)
            cache, _ = self._sweep(k, cache, dummy, N)
        raise ValueError("exit_layer beyond the network")

    # The Controller keeps idle blocks on a storage device; here that is a plain .npz of all
    # parameters (and momentum buffers) in the library's layout, keyed by layer index.
    def save(self, path):
        out = {}
        for li, L in enumerate(self.layers):
            for which in ("p", "v"):
                src = getattr(L, which)
                if src is None:
                    continue
                for name, tns in src.items():
                    if tns is not None:
                        out[f"{which}.{li}.{name}"] = tns.detach().cpu().numpy()
        np.savez(path, **out)

    def load(self, path):
        with np.load(path, allow_pickle=False) as z:
            for li, L in enumerate(self.layers):
                for which in ("p", "v"):
                    src = getattr(L, which)
                    if src is None:
                        continue
                    for name, tns in src.items():
                        key = f"{which}.{li}.{name}"
                        if tns is not None and key in z:
                            tns.copy_(self.torch.from_numpy(z[key]).to(self.device))
