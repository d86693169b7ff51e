"""A PyTorch (CPU, float64, autograd) evaluation of one local step, used ONLY to pin the
CPU oracle to a library routine.  It is not part of the oracle and not part of the product.

Paper: Eq. 1 (conv, down-sampling, ReLU), Eq. 2 (aux conv, pooling, linear), Eq. 3
(cross-entropy, batch mean), Algorithm 2 (gradients of theta_n, beta_n, gamma_n only).
"""
import torch
import torch.nn.functional as F


def local_loss(d, a, x, x_skip, labels, p):
    """d, a: descriptor structs (attribute access); p: dict of float64 torch tensors."""
    z = F.conv2d(x, p["W"], p["b"], stride=d.stride, padding=d.pad)
    if d.skip_kind == 1:
        z = z + x_skip
    elif d.skip_kind == 2:
        z = z + F.conv2d(x_skip, p["Wp"][:, :, None, None], None, stride=d.skip_stride)
    y = torch.relu(z)
    if d.pool_kind:
        y = F.max_pool2d(y, d.pool_k, d.pool_stride, d.pool_pad)
    u = F.conv2d(y, p["Wa"], p["ba"], stride=1, padding=a.pad)
    if a.relu:
        u = torch.relu(u)
    pool = F.adaptive_max_pool2d if getattr(a, "head_pool", 0) == 1 else F.adaptive_avg_pool2d
    q = pool(u, (a.pool_oh, a.pool_ow)).flatten(1)
    logits = F.linear(q, p["Wf"], p["bf"])
    if getattr(a, "loss_kind", 0) == 1:
        loss = F.mse_loss(logits, F.one_hot(labels.long(), logits.shape[1]).to(logits.dtype), reduction="mean")
    else:
        loss = F.cross_entropy(logits, labels.long(), reduction="mean")
    return loss, y


def local_step(d, a, x, x_skip, labels, params, lr, mu, steps=1):
    """Runs ``steps`` local steps on the same batch with torch.optim.SGD; returns the list of
    (loss, grads, Y) per step and the final params / momentum buffers."""
    p = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()
         if v is not None}
    opt = torch.optim.SGD(list(p.values()), lr=lr, momentum=mu)
    xt = torch.tensor(x, dtype=torch.float64)
    xs = None if x_skip is None else torch.tensor(x_skip, dtype=torch.float64)
    lt = torch.tensor(labels)
    out = []
    for _ in range(steps):
        opt.zero_grad()
        loss, y = local_loss(d, a, xt, xs, lt, p)
        loss.backward()
        out.append((float(loss.detach()), {k: v.grad.detach().numpy().copy() for k, v in p.items()},
                    y.detach().numpy().copy()))
        opt.step()
    final = {k: v.detach().numpy().copy() for k, v in p.items()}
    return out, final


def block_epoch(layers, X, labels, batches, lr, mu):
    """Independent (autograd, float64) statement of a block's training pass.

    layers: list of (d, a, params dict of numpy arrays, skip_src); batches: list of index
    arrays.  Every layer has its own torch.optim.SGD; the tensor handed to the next layer is
    the one computed before the update, detached.  Returns (losses [n_batches][n_layers],
    final params per layer, momentum buffers per layer)."""
    ps, opts = [], []
    for _, _, params, _ in layers:
        p = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()
             if v is not None}
        ps.append(p)
        opts.append(torch.optim.SGD(list(p.values()), lr=lr, momentum=mu))
    Xt, Lt = torch.tensor(X, dtype=torch.float64), torch.tensor(labels)
    losses = []
    for sel in batches:
        sel = torch.as_tensor(sel, dtype=torch.long)
        inputs, lab, row = [Xt[sel]], Lt[sel], []
        for n, (d, a, _, skip_src) in enumerate(layers):
            xs = None if skip_src < 0 else inputs[skip_src]
            opts[n].zero_grad()
            loss, y = local_loss(d, a, inputs[n], xs, lab, ps[n])
            loss.backward()
            opts[n].step()
            row.append(float(loss.detach()))
            inputs.append(y.detach())
        losses.append(row)
    final = [{k: v.detach().numpy().copy() for k, v in p.items()} for p in ps]
    mom = [{k: (opts[n].state[v]["momentum_buffer"].numpy().copy() if mu else None) for k, v in p.items()}
           for n, p in enumerate(ps)]
    return losses, final, mom


def block_forward(layers, X):
    """Forward-only composition of a block's layers (float64)."""
    inputs = [torch.tensor(X, dtype=torch.float64)]
    with torch.no_grad():
        for n, (d, a, params, skip_src) in enumerate(layers):
            p = {k: torch.tensor(v, dtype=torch.float64) for k, v in params.items() if v is not None}
            xs = None if skip_src < 0 else inputs[skip_src]
            z = F.conv2d(inputs[n], p["W"], p["b"], stride=d.stride, padding=d.pad)
            if d.skip_kind == 1:
                z = z + xs
            elif d.skip_kind == 2:
                z = z + F.conv2d(xs, p["Wp"][:, :, None, None], None, stride=d.skip_stride)
            y = torch.relu(z)
            if d.pool_kind:
                y = F.max_pool2d(y, d.pool_k, d.pool_stride, d.pool_pad)
            inputs.append(y)
    return inputs[-1].numpy()
