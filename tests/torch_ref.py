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
    q = F.adaptive_avg_pool2d(u, (a.pool_oh, a.pool_ow)).flatten(1)
    logits = F.linear(q, p["Wf"], p["bf"])
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
