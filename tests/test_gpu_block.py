"""GPU parity of the block-level calls (nf_block_train_epoch, nf_block_fill_cache): against the
oracle's block pass (1e-4 relative on every loss, updated weight and momentum buffer; bit-exact
cache contents for the copies), and bit-for-bit against the same pass issued call by call through
the single-layer entry points, with and without the prefetch stream."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads
from paper_2402_14139_amd import binding as nf
from paper_2402_14139_amd import layout
from paper_2402_14139_amd.layer import PARAM_NAMES, LocalLayer
from tests import gpu_common as G

pytestmark = pytest.mark.gpu


def _small_block(kind):
    L = workloads.LayerSpec
    if kind == "pool_basic":   # pooled plain layer, then a basic block with identity shortcut
        specs = [L("l0", 8, 12, 12, 24, A=8, pool_kind=1, pool_k=2, pool_stride=2),
                 L("l1", 24, 6, 6, 24, A=12),
                 L("l2", 24, 6, 6, 24, A=4, skip_kind=1, skip_C=24, skip_H=6, skip_W=6, skip_stride=1)]
        skip = [-1, -1, 1]
    else:                      # stride-2 basic block with projection shortcut from the block input, then plain
        specs = [L("l0", 16, 10, 10, 40, A=8, stride=2),
                 L("l1", 40, 5, 5, 40, A=16, skip_kind=2, skip_C=16, skip_H=10, skip_W=10, skip_stride=2),
                 L("l2", 40, 5, 5, 32, A=4)]
        skip = [-1, 0, -1]
    return specs, skip


class GpuBlock:
    """Device state of a block + the nf_block struct over it."""

    def __init__(self, specs, skip, cls, params, B, momentum):
        self.specs, self.skip = specs, skip
        self.layers = []
        for ls, p in zip(specs, params):
            d, a = nf.LayerDesc(**ls.layer_desc_fields()), nf.AuxDesc(**ls.aux_desc_fields(cls))
            self.layers.append(LocalLayer(d, a, layout.params_to_lib(p, ls.A), B, momentum))
        Ls = self.layers
        self.blk = nf.make_block([l.d for l in Ls], [l.a for l in Ls], skip, [l.sp for l in Ls], [l.sa for l in Ls],
                                 [l.sgp for l in Ls], [l.sga for l in Ls],
                                 [l.svp for l in Ls] if momentum else None, [l.sva for l in Ls] if momentum else None)
        self.ws = torch.empty(nf.nf_block_workspace_bytes(self.blk, B), dtype=torch.uint8, device="cuda")

    def state(self):
        out = []
        for l in self.layers:
            for which in ("p", "v"):
                src = getattr(l, which)
                if src is not None:
                    out += [src[k].clone() for k in PARAM_NAMES if src[k] is not None]
        return out


def _gen(specs, cls, N, seed):
    g = workloads.rng_for(seed, "gpu-block", specs[0].C_in, specs[0].H_in, len(specs))
    f = specs[0]
    X = g.standard_normal((N, f.C_in, f.H_in, f.W_in)).astype(np.float32)
    lab = g.integers(0, cls, size=(N,)).astype(np.int32)
    idx = g.permutation(N).astype(np.int64)
    params = [workloads.gen_layer_params(seed, n, ls, cls, bias_std=0.1) for n, ls in enumerate(specs)]
    return X, lab, idx, params


@pytest.mark.parametrize("kind", ["pool_basic", "proj"])
@pytest.mark.parametrize("mu", [0.0, 0.9])
@pytest.mark.parametrize("prefetch", [False, True])
def test_block_epoch_matches_oracle(kind, mu, prefetch):
    specs, skip = _small_block(kind)
    cls, N, B, lr = 10, 20, 6, 0.02           # batches of 6, 6, 6, 2; two passes
    X, lab, idx, params = _gen(specs, cls, N, seed=21)
    gb = GpuBlock(specs, skip, cls, params, B, mu != 0)
    cache = G.to_dev(layout.act_to_lib(X).reshape(N, -1))
    clab, didx = G.to_dev(lab), G.to_dev(idx)
    nb = (N + B - 1) // B
    losses = torch.full((2, nb, len(specs)), float("nan"), device="cuda")
    main = torch.cuda.Stream()
    side = torch.cuda.Stream() if prefetch else None
    main.wait_stream(torch.cuda.current_stream())
    for e in range(2):
        nf.nf_block_train_epoch(gb.blk, lr, mu, B, N, cache, clab, N, didx, losses[e], gb.ws, stream=main,
                                prefetch_stream=side)
    main.synchronize()

    # The oracle's block pass, in lock-step with the same pass issued call by call on the GPU.  Where
    # the oracle's own pre-activation is a tie within fp32 rounding, its step takes the admissible
    # alternative the kernels took (see gpu_common.oracle_step: the kernels' decisions are only
    # compared, never handed to the oracle), so both follow the same trajectory.
    manual = GpuBlock(specs, skip, cls, params, B, mu != 0)
    obl = []
    for ls, p, s in zip(specs, params, skip):
        od, oa = O.layer_desc(**ls.layer_desc_fields()), O.aux_desc(**ls.aux_desc_fields(cls))
        pc = {k: (None if v is None else v.copy()) for k, v in p.items()}
        mom = {k: (None if v is None else np.zeros_like(v)) for k, v in p.items()} if mu else None
        obl.append(O.BlockLayer(od, oa, pc, mom, s))
    f = specs[0]
    xbuf = torch.empty((B, f.H_in, f.W_in, f.C_in), device="cuda")
    lbuf = torch.empty((B,), dtype=torch.int32, device="cuda")
    acts, man_losses, ties = [], [], G.TieStats()

    def step(j, n, L, x, xs, lb):
        nbj = x.shape[0]
        if n == 0:
            nf.nf_cache_read(cache, clab, N, cache.shape[1], 0, didx[j * B:j * B + nbj], nbj, xbuf, lbuf)
            acts.clear()
            acts.append(xbuf[:nbj])
        gl = manual.layers[n]
        y = gl.step(acts[n], None if skip[n] < 0 else acts[skip[n]], lbuf, lr, mu)
        torch.cuda.synchronize()
        acts.append(y)
        man_losses.append(float(gl.loss.item()))
        dec = G.gpu_decisions(gl, specs[n], nbj, y.cpu().numpy())
        oy, oloss, _, _ = G.oracle_step(L.d, L.a, specs[n], x, xs, lb, L.params, L.mom, lr, mu, dec, stats=ties)
        return oy, oloss

    ref = np.stack([O.block_train_epoch(obl, X.reshape(N, -1), lab, idx, N, B, X.shape[1:], lr, mu, step=step)
                    for _ in range(2)])
    print(f"  {ties}", flush=True)
    got = losses.cpu().numpy()
    assert np.array_equal(got.reshape(-1), np.array(man_losses, np.float32)), "block call != call-by-call sequence"
    assert all(torch.equal(a, b) for a, b in zip(gb.state(), manual.state())), "block call != call-by-call sequence"
    assert np.all(np.abs(got - ref) <= G.REL * np.abs(ref)), (got, ref)
    for n, (l, ob) in enumerate(zip(gb.layers, obl)):
        gp = l.params_numpy("p")
        gv = l.params_numpy("v") if mu else None
        for k in PARAM_NAMES:
            if ob.params[k] is not None:
                G.assert_close(f"layer {n} updated {k}", gp[k], ob.params[k])
                if mu:
                    G.assert_close(f"layer {n} momentum {k}", gv[k], ob.mom[k])


@pytest.mark.parametrize("kind", ["pool_basic", "proj"])
def test_block_fill_cache_matches_oracle(kind):
    specs, skip = _small_block(kind)
    cls, N, B = 10, 20, 6
    X, lab, _, params = _gen(specs, cls, N, seed=22)
    gb = GpuBlock(specs, skip, cls, params, B, False)
    last = specs[-1]
    se_out = last.C_out * last.Hp * last.Wp
    cache = G.to_dev(layout.act_to_lib(X).reshape(N, -1))
    clab = G.to_dev(lab)
    out = torch.full((N + 3, se_out), float("nan"), device="cuda")
    olab = torch.full((N + 3,), -1, dtype=torch.int32, device="cuda")
    nf.nf_block_fill_cache(gb.blk, B, N, cache, clab, N, out, olab, N + 3, gb.ws)
    torch.cuda.synchronize()
    obl = [O.BlockLayer(O.layer_desc(**ls.layer_desc_fields()), O.aux_desc(**ls.aux_desc_fields(cls)), p, None, s)
           for ls, p, s in zip(specs, params, skip)]
    ref = np.full((N, se_out), np.nan, np.float32)
    rlab = np.full((N,), -1, np.int32)
    O.block_fill_cache(obl, X.reshape(N, -1), lab, N, B, X.shape[1:], ref, rlab)
    got = out.cpu().numpy()
    assert np.all(np.isnan(got[N:])) and np.all(olab.cpu().numpy()[N:] == -1), "rows beyond n_items were touched"
    assert np.array_equal(olab.cpu().numpy()[:N], rlab)
    got_nchw = layout.act_from_lib(got[:N].reshape(N, last.Hp, last.Wp, last.C_out))
    G.assert_close("cache rows", got_nchw, ref.reshape(got_nchw.shape))
    # the sweep is the single-layer forward calls in a row: bit-exact against issuing them by hand
    x = torch.empty((B, specs[0].H_in, specs[0].W_in, specs[0].C_in), device="cuda")
    lb = torch.empty((B,), dtype=torch.int32, device="cuda")
    manual = torch.empty((N, se_out), device="cuda")
    mlab = torch.empty((N,), dtype=torch.int32, device="cuda")
    for first in range(0, N, B):
        n = min(B, N - first)
        nf.nf_cache_read(cache, clab, N, cache.shape[1], first, None, n, x, lb)
        acts = [x]
        for li, l in enumerate(gb.layers):
            acts.append(l.forward(acts[li][:n], None if skip[li] < 0 else acts[skip[li]][:n]))
        nf.nf_cache_write(manual, mlab, N, se_out, first, n, acts[-1], lb)
    torch.cuda.synchronize()
    assert torch.equal(manual, out[:N]) and torch.equal(mlab, olab[:N])


def _cfg_block(cfg_name, k, B, momentum, seed=5):
    cfg = workloads.config(cfg_name)
    b = cfg.blocks[k]
    specs = [cfg.layers[i] for i in b.layers]
    skip = [(-1 if not ls.skip_kind else ls.skip_src - b.layers[0]) for ls in specs]
    params = [workloads.gen_layer_params(seed, i, ls, cfg.n_classes) for i, ls in zip(b.layers, specs)]
    return cfg, specs, skip, params


@pytest.mark.parametrize("cfg_name,k", [("cfg3", 1), ("cfg3", 3), ("cfg2", 0)])
def test_block_epoch_is_the_sequence_of_local_steps_full_size(cfg_name, k):
    """At the benchmark's own shapes and batch sizes: the block pass, with and without the
    prefetch stream, leaves bit-for-bit the weights, momentum buffers and losses that the same
    nf_cache_read / nf_local_step calls leave when issued one by one."""
    cfg0 = workloads.config(cfg_name)
    B = cfg0.blocks[k].batch
    cfg, specs, skip, params = _cfg_block(cfg_name, k, B, True)
    N = 2 * B + B // 2                       # two full batches and a partial one
    f = specs[0]
    g = torch.Generator(device="cuda").manual_seed(3)
    cache = torch.randn((N, f.H_in * f.W_in * f.C_in), device="cuda", generator=g).abs_()
    clab = torch.randint(0, cfg.n_classes, (N,), device="cuda", generator=g, dtype=torch.int32)
    idx = torch.randperm(N, device="cuda", generator=g)
    lr, mu = 1e-3, 0.9
    nb = (N + B - 1) // B
    results = []
    for mode in ("manual", "block", "block_prefetch"):
        gb = GpuBlock(specs, skip, cfg.n_classes, params, B, True)
        losses = torch.zeros((nb, len(specs)), device="cuda")
        if mode == "manual":
            x = torch.empty((B, f.H_in, f.W_in, f.C_in), device="cuda")
            lb = torch.empty((B,), dtype=torch.int32, device="cuda")
            for j in range(nb):
                n = min(B, N - j * B)
                nf.nf_cache_read(cache, clab, N, cache.shape[1], 0, idx[j * B:j * B + n], n, x, lb)
                acts = [x[:n]]
                for li, l in enumerate(gb.layers):
                    acts.append(l.step(acts[li], None if skip[li] < 0 else acts[skip[li]], lb, lr, mu))
                    losses[j, li] = l.loss[0]
        else:
            main = torch.cuda.Stream()
            side = torch.cuda.Stream() if mode == "block_prefetch" else None
            main.wait_stream(torch.cuda.current_stream())
            nf.nf_block_train_epoch(gb.blk, lr, mu, B, N, cache, clab, N, idx, losses, gb.ws, stream=main,
                                    prefetch_stream=side)
            main.synchronize()
        torch.cuda.synchronize()
        results.append((losses.clone(), gb.state()))
        del gb
    base_l, base_s = results[0]
    assert torch.isfinite(base_l).all()
    for mode, (l, s) in zip(("block", "block_prefetch"), results[1:]):
        assert torch.equal(l, base_l), mode
        assert len(s) == len(base_s) and all(torch.equal(a, b) for a, b in zip(s, base_s)), mode


# ---- early-exit evaluation -----------------------------------------------------------------------
def _check_predictions(tag, pred_gpu, logits_ref, pred_ref):
    """Predictions are integers decided by fp32 logits: they must equal the oracle's wherever the
    oracle's best logit leads the runner-up by more than rounding, and otherwise be one of the
    classes within rounding of the best."""
    z = np.asarray(logits_ref, np.float64)
    top = z.max(axis=1)
    tol = 2e-5 * np.abs(z).max()
    near = z >= (top - tol)[:, None]
    clear = near.sum(axis=1) == 1
    assert np.array_equal(pred_gpu[clear], pred_ref[clear]), f"{tag}: prediction differs away from a tie"
    assert np.all(near[np.arange(len(pred_gpu)), pred_gpu]), f"{tag}: predicted class is not a maximum"
    return int((~clear).sum())


@pytest.mark.parametrize("case", ["a8", "a5_scalar", "a80_wide", "a4_split"])
def test_aux_predict_matches_oracle(case):
    L = workloads.LayerSpec
    spec, B, cls = {"a8": (L("t", 8, 12, 12, 24, A=8), 37, 10),
                    "a5_scalar": (L("t", 3, 10, 10, 6, A=5), 5, 7),
                    "a80_wide": (L("t", 32, 8, 8, 160, A=80), 6, 200),
                    "a4_split": (L("t", 16, 6, 6, 256, A=4), 5, 10)}[case]
    x, _, labels, p = G.make_inputs(spec, B, cls, seed=31)
    (d, a), (od, oa) = G.descs(spec, cls)
    gl = G.gpu_layer(spec, cls, p, B, False)
    y = gl.forward(G.to_dev(layout.act_to_lib(x)))
    pred = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    cnt = torch.full((1,), 1000, dtype=torch.int32, device="cuda")
    logits = torch.empty((B, cls), device="cuda")
    nf.nf_aux_predict(gl.d, gl.a, B, y, G.to_dev(labels), gl.sa, pred, cnt, False, logits, gl.ws)
    nf.nf_aux_predict(gl.d, gl.a, B, y, G.to_dev(labels), gl.sa, pred, cnt, True, None, gl.ws)   # accumulates
    torch.cuda.synchronize()
    oy = O.layer_fwd(od, x, None, p["W"], p["b"]).Y
    z, opred = O.aux_predict(oa, oy, p["Wa"], p["ba"], p["Wf"], p["bf"])
    G.assert_close("logits", logits.cpu().numpy(), z)
    pg = pred.cpu().numpy()
    _check_predictions(case, pg, z, opred)
    assert int(cnt.item()) == 2 * int((pg == labels).sum())
    # without labels nothing is counted
    nf.nf_aux_predict(gl.d, gl.a, B, y, None, gl.sa, pred, None, False, None, gl.ws)
    torch.cuda.synchronize()
    assert np.array_equal(pred.cpu().numpy(), pg)


def test_aux_predict_ties_go_to_the_lowest_class():
    spec, B, cls = workloads.LayerSpec("t", 8, 6, 6, 16, A=8), 4, 300
    x, _, labels, p = G.make_inputs(spec, B, cls, seed=32)
    p["Wf"][:] = 0
    p["bf"][:] = -1.0
    p["bf"][[257, 40, 299]] = 2.5                 # three equal maxima, the lowest in another thread's stride
    gl = G.gpu_layer(spec, cls, p, B, False)
    y = gl.forward(G.to_dev(layout.act_to_lib(x)))
    pred = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    cnt = torch.zeros((1,), dtype=torch.int32, device="cuda")
    lab = np.array([40, 257, 40, 0], np.int32)
    nf.nf_aux_predict(gl.d, gl.a, B, y, G.to_dev(lab), gl.sa, pred, cnt, False, None, gl.ws)
    torch.cuda.synchronize()
    assert pred.cpu().tolist() == [40] * B and int(cnt.item()) == 2


@pytest.mark.parametrize("kind", ["pool_basic", "proj"])
def test_block_evaluate_matches_oracle(kind):
    specs, skip = _small_block(kind)
    cls, N, B = 10, 23, 6
    X, lab, _, params = _gen(specs, cls, N, seed=23)
    gb = GpuBlock(specs, skip, cls, params, B, False)
    cache = G.to_dev(layout.act_to_lib(X).reshape(N, -1))
    clab = G.to_dev(lab)
    obl = [O.BlockLayer(O.layer_desc(**ls.layer_desc_fields()), O.aux_desc(**ls.aux_desc_fields(cls)), p, None, s)
           for ls, p, s in zip(specs, params, skip)]
    counts, ocounts = [], []
    for e in range(len(specs)):
        pred = torch.full((N + 2,), -7, dtype=torch.int32, device="cuda")
        cnt = torch.full((1,), 999, dtype=torch.int32, device="cuda")
        nf.nf_block_evaluate(gb.blk, e, B, N, cache, clab, N, pred, cnt, gb.ws)
        torch.cuda.synchronize()
        pg = pred.cpu().numpy()
        assert np.all(pg[N:] == -7)
        opred, ocorrect = O.block_evaluate(obl, e, X.reshape(N, -1), lab, N, B, X.shape[1:])
        # the oracle's logits for the margin test
        inputs = [X]
        for n in range(e + 1):
            xs = None if skip[n] < 0 else inputs[skip[n]]
            inputs.append(O.layer_fwd(obl[n].d, inputs[n], xs, params[n]["W"], params[n]["b"], params[n].get("Wp")).Y)
        z, _ = O.aux_predict(obl[e].a, inputs[-1], params[e]["Wa"], params[e]["ba"], params[e]["Wf"], params[e]["bf"])
        ties = _check_predictions(f"{kind} exit {e}", pg[:N], z, opred)
        assert int(cnt.item()) == int((pg[:N] == lab).sum())
        if ties == 0:
            assert int(cnt.item()) == ocorrect
        counts.append(int(cnt.item()))
        ocounts.append(ocorrect)
    n_params = np.cumsum([sum(v.size for k, v in p.items() if v is not None and k in ("W", "b", "Wp")) for p in params])
    assert nf.nf_select_exit(counts, [int(v) for v in n_params]) == O.select_exit(counts, [int(v) for v in n_params])


def test_block_epoch_under_graph_capture():
    """The block pass allocates nothing and records no memset, so a caller can capture it in a HIP
    graph: three replays (with eager work and synchronisations in between) leave bit-for-bit the
    state that three eager calls leave, checked after every replay."""
    specs, skip = _small_block("proj")
    cls, N, B, lr, mu = 10, 12, 6, 0.02, 0.9
    X, lab, idx, params = _gen(specs, cls, N, seed=24)
    cache = G.to_dev(layout.act_to_lib(X).reshape(N, -1))
    clab, didx = G.to_dev(lab), G.to_dev(idx)
    nb = N // B
    eager = GpuBlock(specs, skip, cls, params, B, True)
    el = torch.zeros((nb, len(specs)), device="cuda")
    eager_states = []
    for _ in range(3):
        nf.nf_block_train_epoch(eager.blk, lr, mu, B, N, cache, clab, N, didx, el, eager.ws)
        torch.cuda.synchronize()
        eager_states.append(([s.clone() for s in eager.state()], el.clone()))
    cap = GpuBlock(specs, skip, cls, params, B, True)
    gl = torch.zeros((nb, len(specs)), device="cuda")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        nf.nf_block_train_epoch(cap.blk, lr, mu, B, N, cache, clab, N, didx, gl, cap.ws)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 16, device="cuda")
    for r in range(3):
        graph.replay()
        scratch.add_(1.0).sum().item()          # eager work and a synchronisation between replays
        torch.cuda.synchronize()
        want_state, want_loss = eager_states[r]
        assert torch.equal(gl, want_loss), f"losses differ after replay {r}"
        assert all(torch.equal(a, b) for a, b in zip(cap.state(), want_state)), f"state differs after replay {r}"


def test_block_graph_captured_by_the_library():
    """nf_block_graph_create / launch / destroy: the library captures the block pass itself.  Three
    launches (with eager work and synchronisations in between, on a stream of the caller) leave
    bit-for-bit the state that three eager calls leave, checked after every launch; a new shuffle
    written into the same index buffer is picked up by the next launch; argument errors come back
    as from nf_block_train_epoch and leave no handle."""
    specs, skip = _small_block("proj")
    cls, N, B, lr, mu = 10, 12, 6, 0.02, 0.9
    X, lab, idx, params = _gen(specs, cls, N, seed=25)
    cache = G.to_dev(layout.act_to_lib(X).reshape(N, -1))
    clab = G.to_dev(lab)
    idx2 = np.ascontiguousarray(idx[::-1])
    nb = N // B
    eager = GpuBlock(specs, skip, cls, params, B, True)
    el = torch.zeros((nb, len(specs)), device="cuda")
    eidx = G.to_dev(idx)
    eager_states = []
    for r in range(3):
        if r == 2:
            eidx.copy_(torch.from_numpy(idx2))
        nf.nf_block_train_epoch(eager.blk, lr, mu, B, N, cache, clab, N, eidx, el, eager.ws)
        torch.cuda.synchronize()
        eager_states.append(([s.clone() for s in eager.state()], el.clone()))
    cap = GpuBlock(specs, skip, cls, params, B, True)
    gl = torch.zeros((nb, len(specs)), device="cuda")
    gidx = G.to_dev(idx)
    torch.cuda.synchronize()
    # a workspace that is too small: the error of nf_block_train_epoch, and no handle
    with pytest.raises(nf.NfError) as e:
        nf.nf_block_graph_create(cap.blk, lr, mu, B, N, cache, clab, N, gidx, gl, cap.ws[:256])
    assert e.value.status == nf.NF_ERR_WORKSPACE
    # refused while the per-launch event timing is on
    nf.nf_prof_begin()
    try:
        with pytest.raises(nf.NfError) as e:
            nf.nf_block_graph_create(cap.blk, lr, mu, B, N, cache, clab, N, gidx, gl, cap.ws)
        assert e.value.status == nf.NF_ERR_UNSUPPORTED
    finally:
        nf.nf_prof_end()
    print("create", flush=True)
    g = nf.nf_block_graph_create(cap.blk, lr, mu, B, N, cache, clab, N, gidx, gl, cap.ws)
    torch.cuda.synchronize()
    # creating the graph ran nothing
    assert all(torch.equal(a, b) for a, b in zip(cap.state(), GpuBlock(specs, skip, cls, params, B, True).state()))
    stream = torch.cuda.Stream()
    scratch = torch.zeros(1 << 16, device="cuda")
    try:
        for r in range(3):
            if r == 2:
                gidx.copy_(torch.from_numpy(idx2))
                torch.cuda.synchronize()
            print(f"launch {r}", flush=True)
            nf.nf_block_graph_launch(g, stream=stream)
            stream.synchronize()
            scratch.add_(1.0).sum().item()      # eager work and a synchronisation between launches
            torch.cuda.synchronize()
            want_state, want_loss = eager_states[r]
            assert torch.equal(gl, want_loss), f"losses differ after launch {r}"
            assert all(torch.equal(a, b) for a, b in zip(cap.state(), want_state)), f"state differs after launch {r}"
    finally:
        nf.nf_block_graph_destroy(g)


def test_block_graph_keeps_the_contraction_mode_of_its_creation():
    """A graph created in the split-operand mode runs the split kernels whatever the mode is when it
    is launched, and the other way round (cfg3's 256-filter block at full size): each graph
    reproduces, bit for bit, the eager pass made in the mode of its creation, and the two modes
    differ from each other."""
    cfg0 = workloads.config("cfg3")
    k = 2
    B = cfg0.blocks[k].batch
    cfg, specs, skip, params = _cfg_block("cfg3", k, B, True)
    N = B + B // 2
    f = specs[0]
    g = torch.Generator(device="cuda").manual_seed(7)
    cache = torch.randn((N, f.H_in * f.W_in * f.C_in), device="cuda", generator=g).abs_()
    clab = torch.randint(0, cfg.n_classes, (N,), device="cuda", generator=g, dtype=torch.int32)
    idx = torch.randperm(N, device="cuda", generator=g)
    lr, mu = 1e-3, 0.9
    nb = (N + B - 1) // B
    modes = (nf.NF_CONTRACT_F32, nf.NF_CONTRACT_BF16X6)
    start = nf.nf_contraction()
    eager, graphs = {}, {}
    try:
        for m in modes:
            nf.nf_contraction(m)
            gb = GpuBlock(specs, skip, cfg.n_classes, params, B, True)
            losses = torch.zeros((nb, len(specs)), device="cuda")
            nf.nf_block_train_epoch(gb.blk, lr, mu, B, N, cache, clab, N, idx, losses, gb.ws)
            torch.cuda.synchronize()
            eager[m] = (losses.clone(), [t.clone() for t in gb.state()])
            del gb
            cap = GpuBlock(specs, skip, cfg.n_classes, params, B, True)
            gl = torch.zeros((nb, len(specs)), device="cuda")
            graphs[m] = (nf.nf_block_graph_create(cap.blk, lr, mu, B, N, cache, clab, N, idx, gl, cap.ws), cap, gl)
        # launch each graph with the OTHER mode in force
        for m, other in zip(modes, modes[::-1]):
            nf.nf_contraction(other)
            h, cap, gl = graphs[m]
            print(f"launch graph created in mode {m} under mode {other}", flush=True)
            nf.nf_block_graph_launch(h)
            torch.cuda.synchronize()
            want_l, want_s = eager[m]
            assert torch.equal(gl, want_l), m
            assert all(torch.equal(a, b) for a, b in zip(cap.state(), want_s)), m
        assert not all(torch.equal(a, b) for a, b in zip(eager[modes[0]][1], eager[modes[1]][1]))
    finally:
        nf.nf_contraction(start)
        for h, _, _ in graphs.values():
            nf.nf_block_graph_destroy(h)
