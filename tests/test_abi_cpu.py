"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2402_14139_amd import binding as nf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(nf.LIB_PATH):
        from paper_2402_14139_amd import build
        build.build()
    return nf.lib()


def test_exports_every_declared_symbol(L):
    text = open(os.path.join(ROOT, "include", "nf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(nf_[a-z_]+)\s*\(", text))
    assert declared == set(nf.EXPORTS), declared ^ set(nf.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def _layer(**kw):
    base = dict(C_in=8, H_in=8, W_in=8, C_out=16, R=3, S=3, stride=1, pad=1, pool_kind=0, pool_k=0, pool_stride=0,
                pool_pad=0, skip_kind=0, skip_C=0, skip_H=0, skip_W=0, skip_stride=0)
    base.update(kw)
    return nf.LayerDesc(**base)


def _aux(**kw):
    base = dict(C_in=16, H_in=8, W_in=8, A=8, R=3, S=3, pad=1, relu=1, pool_oh=2, pool_ow=2, n_classes=10)
    base.update(kw)
    return nf.AuxDesc(**base)


def test_out_dims_and_workspace(L):
    assert nf.nf_layer_out_dims(_layer()) == (8, 8, 8, 8)
    assert nf.nf_layer_out_dims(_layer(stride=2)) == (4, 4, 4, 4)
    assert nf.nf_layer_out_dims(_layer(pool_kind=1, pool_k=2, pool_stride=2)) == (8, 8, 4, 4)
    assert nf.nf_layer_out_dims(_layer(H_in=128, W_in=128, R=7, S=7, stride=2, pad=3, pool_kind=1, pool_k=3,
                                       pool_stride=2, pool_pad=1)) == (64, 64, 32, 32)
    fwd_only = nf.nf_workspace_bytes(_layer(), None, 4)
    full = nf.nf_workspace_bytes(_layer(), _aux(), 4)
    assert 0 < fwd_only <= full and full % 256 == 0
    assert nf.nf_workspace_bytes(_layer(), _aux(), 8) > full


@pytest.mark.parametrize("cfg_name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_workspace_of_every_benchmark_layer(L, cfg_name):
    """Host-side sizing only: the workspace of every layer of every configuration holds at least
    the tensors the step keeps there (dL/dZ, U, dU), its named regions lie inside it, and it
    stays far below the 288 GB of the device."""
    import workloads
    cfg = workloads.config(cfg_name)
    for ls in cfg.layers:
        B = cfg.blocks[ls.block].batch
        d, a = nf.LayerDesc(**ls.layer_desc_fields()), nf.AuxDesc(**ls.aux_desc_fields(cfg.n_classes))
        total = nf.nf_workspace_bytes(d, a, B)
        conv_out = 4 * B * ls.Ho * ls.Wo * ls.C_out
        u = 4 * B * ls.Hp * ls.Wp * ls.A
        assert conv_out + 2 * u <= total < (8 << 30), (cfg_name, ls.name, total)
        for which in (nf.NF_WS_AUX_ACT, nf.NF_WS_POOL_ARG):
            off, nbytes = nf.nf_workspace_region(d, a, B, which)
            assert off % 256 == 0 and off + nbytes <= total
        off, nbytes = nf.nf_workspace_region(d, a, B, nf.NF_WS_AUX_ACT)
        assert nbytes == u
        assert nf.nf_workspace_bytes(d, None, B) <= total


@pytest.mark.parametrize("desc,status", [
    (dict(C_in=0), nf.NF_ERR_BAD_DESC),
    (dict(H_in=1, W_in=1, pad=0), nf.NF_ERR_BAD_DESC),          # filter larger than padded input
    (dict(pool_kind=2, pool_k=2, pool_stride=2), nf.NF_ERR_UNSUPPORTED),
    (dict(pool_kind=1, pool_k=2, pool_stride=2, pool_pad=2), nf.NF_ERR_BAD_DESC),
    (dict(skip_kind=1, skip_C=16, skip_H=4, skip_W=8), nf.NF_ERR_BAD_DESC),
    (dict(skip_kind=2, skip_C=8, skip_H=8, skip_W=8, skip_stride=2), nf.NF_ERR_BAD_DESC),  # reads past x_skip
    (dict(skip_kind=3), nf.NF_ERR_BAD_DESC),
    (dict(stride=9), nf.NF_ERR_UNSUPPORTED),
])
def test_bad_layer_descriptors(L, desc, status):
    out = C.c_size_t()
    assert L.nf_workspace_bytes(C.byref(_layer(**desc)), None, 4, C.byref(out)) == status


def test_bad_aux_and_pairing(L):
    out = C.c_size_t()
    d = _layer()
    assert L.nf_workspace_bytes(C.byref(d), C.byref(_aux(C_in=8)), 4, C.byref(out)) == nf.NF_ERR_BAD_DESC
    assert L.nf_workspace_bytes(C.byref(d), C.byref(_aux(A=0)), 4, C.byref(out)) == nf.NF_ERR_BAD_DESC
    assert L.nf_workspace_bytes(C.byref(d), C.byref(_aux(R=3, S=5)), 4, C.byref(out)) == nf.NF_ERR_UNSUPPORTED
    assert L.nf_workspace_bytes(C.byref(d), C.byref(_aux()), 0, C.byref(out)) == nf.NF_ERR_BAD_DESC
    assert L.nf_workspace_bytes(C.byref(d), C.byref(_aux()), 4, None) == nf.NF_ERR_NULL
    assert L.nf_workspace_bytes(None, None, 4, C.byref(out)) == nf.NF_ERR_NULL


def test_calls_validate_before_enqueue(L):
    """Fake (never dereferenced) device addresses: every call must fail in validation."""
    d, a = _layer(), _aux()
    good, odd = 0x10000, 0x10004
    p = nf.LayerParams(good, good, None)
    ap = nf.AuxParams(good, good, good, good)
    ws_bytes = nf.nf_workspace_bytes(d, a, 4)
    # NULL pointers
    assert L.nf_layer_fwd(C.byref(d), 4, None, None, C.byref(p), good, good, ws_bytes, None) == nf.NF_ERR_NULL
    assert L.nf_layer_fwd(C.byref(d), 4, good, None, None, good, good, ws_bytes, None) == nf.NF_ERR_NULL
    assert L.nf_layer_fwd(C.byref(d), 4, good, None, C.byref(nf.LayerParams(good, None, None)), good, good,
                          ws_bytes, None) == nf.NF_ERR_NULL
    dsk = _layer(skip_kind=1, skip_C=16, skip_H=8, skip_W=8)
    assert L.nf_layer_fwd(C.byref(dsk), 4, good, None, C.byref(p), good, good, ws_bytes, None) == nf.NF_ERR_NULL
    # misaligned pointer
    assert L.nf_layer_fwd(C.byref(d), 4, odd, None, C.byref(p), good, good, ws_bytes, None) == nf.NF_ERR_BAD_DESC
    # workspace: missing, misaligned, too small
    dp = _layer(pool_kind=1, pool_k=2, pool_stride=2)
    need = nf.nf_workspace_bytes(dp, None, 4)
    assert L.nf_layer_fwd(C.byref(dp), 4, good, None, C.byref(p), good, None, need, None) == nf.NF_ERR_WORKSPACE
    assert L.nf_layer_fwd(C.byref(dp), 4, good, None, C.byref(p), good, 0x10010, need, None) == nf.NF_ERR_WORKSPACE
    assert L.nf_layer_fwd(C.byref(dp), 4, good, None, C.byref(p), good, good, need - 1, None) == nf.NF_ERR_WORKSPACE
    assert L.nf_aux_fwd_loss(C.byref(d), C.byref(a), 4, good, good, C.byref(ap), good, good, ws_bytes - 1,
                             None) == nf.NF_ERR_WORKSPACE
    assert L.nf_aux_fwd_loss(C.byref(d), C.byref(a), 4, good, None, C.byref(ap), good, good, ws_bytes,
                             None) == nf.NF_ERR_NULL
    assert L.nf_local_bwd_wgrad(C.byref(d), C.byref(a), 4, good, None, good, C.byref(p), C.byref(ap), C.byref(p),
                                None, good, ws_bytes, None) == nf.NF_ERR_NULL
    s = nf.SgdDesc(0.1, 0.9)
    assert L.nf_local_step(C.byref(d), C.byref(a), C.byref(s), 4, good, None, good, C.byref(p), C.byref(ap),
                           C.byref(p), C.byref(ap), None, None, good, good, good, ws_bytes,
                           None) == nf.NF_ERR_NULL  # momentum without momentum buffers
    # cache ranges
    assert L.nf_cache_write(good, good, 10, 64, 8, 4, good, good, None) == nf.NF_ERR_CACHE_RANGE
    assert L.nf_cache_write(good, good, 10, 64, -1, 4, good, good, None) == nf.NF_ERR_CACHE_RANGE
    assert L.nf_cache_write(good, None, 10, 64, 0, 4, good, good, None) == nf.NF_ERR_NULL
    assert L.nf_cache_read(good, good, 10, 64, 7, None, 4, good, good, None) == nf.NF_ERR_CACHE_RANGE
    assert L.nf_cache_read(good, good, 10, 0, 0, None, 4, good, good, None) == nf.NF_ERR_BAD_DESC
    # sgd
    arr = (C.c_void_p * 1)(good)
    n1 = (C.c_int64 * 1)(16)
    assert L.nf_sgd_update(C.byref(s), 1, arr, arr, None, n1, None) == nf.NF_ERR_NULL
    assert L.nf_sgd_update(C.byref(s), 17, arr, arr, arr, n1, None) == nf.NF_ERR_BAD_DESC
    assert L.nf_sgd_update(C.byref(s), 1, arr, arr, arr, (C.c_int64 * 1)(0), None) == nf.NF_ERR_BAD_DESC


def test_strerror(L):
    assert nf.strerror(0) == "ok"
    for code in range(-7, 0):
        assert nf.strerror(code) and nf.strerror(code) != "unknown status"
    assert nf.strerror(-99) == "unknown status"


def test_static_scratch_entry_point_validates_and_rejects_oversize(L):
    """nf_local_step_static validates like nf_local_step and rejects a step whose workspace
    exceeds the static array, all before any device work (so it is checkable without a GPU)."""
    good = 0x10000
    p, ap = nf.LayerParams(good, good, None), nf.AuxParams(good, good, good, good)
    s = nf.SgdDesc(0.01, 0.0)

    def call(d, a, B, x=good, labels=good, y=good, loss=good):
        return L.nf_local_step_static(C.byref(d), C.byref(a), C.byref(s), B, x, None, labels, C.byref(p), C.byref(ap),
                                      C.byref(p), C.byref(ap), None, None, y, loss, None)

    d = _layer(C_in=64, H_in=64, W_in=64, C_out=64)
    a = _aux(C_in=64, H_in=64, W_in=64, A=64, n_classes=200)
    need = nf.nf_workspace_bytes(d, a, 64)
    assert need > nf.NF_STATIC_SCRATCH_BYTES
    assert call(d, a, 64) == nf.NF_ERR_SCRATCH_LIMIT
    assert "static" in nf.strerror(nf.NF_ERR_SCRATCH_LIMIT)
    small_d, small_a = _layer(), _aux()
    assert nf.nf_workspace_bytes(small_d, small_a, 4) <= nf.NF_STATIC_SCRATCH_BYTES
    assert call(small_d, small_a, 4, x=None) == nf.NF_ERR_NULL
    assert call(small_d, small_a, 4, y=good + 4) == nf.NF_ERR_BAD_DESC
    assert call(small_d, small_a, 0) == nf.NF_ERR_BAD_DESC
    text = open(os.path.join(ROOT, "include", "nf.h")).read()
    m = re.search(r"#define NF_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", text)
    assert m and int(m.group(1)) << int(m.group(2)) == nf.NF_STATIC_SCRATCH_BYTES


# ---- block-level calls: everything below fails (or only sizes things) before any enqueue ----------
def _cfg_block(cfg_name, k, good=0x10000, with_mom=True):
    import workloads
    cfg = workloads.config(cfg_name)
    b = cfg.blocks[k]
    specs = [cfg.layers[i] for i in b.layers]
    descs = [nf.LayerDesc(**ls.layer_desc_fields()) for ls in specs]
    auxs = [nf.AuxDesc(**ls.aux_desc_fields(cfg.n_classes)) for ls in specs]
    skip = [(-1 if not ls.skip_kind else ls.skip_src - b.layers[0]) for ls in specs]
    lp = [nf.LayerParams(good, good, good if ls.skip_kind == 2 else None) for ls in specs]
    apar = [nf.AuxParams(good, good, good, good) for _ in specs]
    blk = nf.make_block(descs, auxs, skip, lp, apar, lp, apar, lp if with_mom else None, apar if with_mom else None)
    return cfg, b, specs, blk


@pytest.mark.parametrize("cfg_name,k", [("cfg3", 0), ("cfg3", 3), ("cfg2", 0), ("cfg5", 0), ("cfg5", 2)])
def test_block_workspace(L, cfg_name, k):
    cfg, b, specs, blk = _cfg_block(cfg_name, k)
    B = b.batch
    total = nf.nf_block_workspace_bytes(blk, B)
    up = lambda v: (v + 255) // 256 * 256  # noqa: E731
    f = specs[0]
    want = 2 * (up(4 * B * f.C_in * f.H_in * f.W_in) + up(4 * B))
    want += sum(up(4 * B * ls.C_out * ls.Hp * ls.Wp) for ls in specs)
    want += up(max(nf.nf_workspace_bytes(blk._keep["layers"][i], blk._keep["aux"][i], B) for i in range(len(specs))))
    assert total == want and total < (16 << 30)


@pytest.mark.parametrize("cfg_name", ["cfg4", "cfg5"])
def test_every_layer_has_a_full_batch_parity_case(cfg_name):
    """The GPU parity suite runs one representative per distinct (descriptor, head width, batch
    size); every layer of the configuration must equal its representative field by field."""
    import workloads
    from tests.test_gpu_configs import distinct_layers
    cfg = workloads.config(cfg_name)
    tested, rep = distinct_layers(cfg_name)
    assert len(rep) == len(cfg.layers)
    for i, ls in enumerate(cfg.layers):
        r = cfg.layers[rep[i]]
        assert rep[i] in tested and rep[i] <= i
        assert ls.layer_desc_fields() == r.layer_desc_fields() and ls.A == r.A
        assert cfg.blocks[ls.block].batch == cfg.blocks[r.block].batch


def test_cfg5_blocks_fit_the_memory_budget(L):
    """The ResNet-34-style configuration sizes its blocks under a fixed 16 GiB budget for
    activations + weights (the budget M that Algorithm 1 consumes).  Batch sizes are given, so the
    budget is an assertion: while block k is trained, device memory holds its input cache and the
    cache it fills for block k+1 (all 16 384 samples, labels included), the block's workspace
    (double-buffered input batch, every layer's emitted batch, the largest single-layer workspace)
    and parameters + gradients + momentum buffers of its layers and heads."""
    import workloads
    cfg = workloads.config("cfg5")
    budget, N = cfg.extra["memory_budget_bytes"], cfg.n_samples
    assert budget == 16 << 30 and N == 16384
    peak = 0
    for k, b in enumerate(cfg.blocks):
        _, _, specs, blk = _cfg_block("cfg5", k)
        f, last = specs[0], specs[-1]
        cache_in = N * (4 * f.C_in * f.H_in * f.W_in + 4)
        cache_out = N * (4 * last.C_out * last.Hp * last.Wp + 4)
        ws = nf.nf_block_workspace_bytes(blk, b.batch)
        params = 0
        for ls in specs:
            F = 4 * ls.A
            n = ls.C_out * ls.C_in * ls.R * ls.S + ls.C_out + (ls.C_out * ls.skip_C if ls.skip_kind == 2 else 0)
            n += ls.A * ls.C_out * 9 + ls.A + cfg.n_classes * F + cfg.n_classes
            params += 3 * 4 * n                              # weights, gradients, momentum
        total = cache_in + cache_out + ws + params
        print(f"cfg5 block {k} (B={b.batch}, {len(specs)} layers): caches {(cache_in + cache_out) / 2**30:.2f} GiB, "
              f"workspace {ws / 2**30:.3f} GiB, parameters x3 {params / 2**30:.3f} GiB, total {total / 2**30:.2f} GiB")
        assert total <= budget, (k, total)
        peak = max(peak, total)
    assert peak > budget // 4    # the budget is not vacuous: the early blocks use a good part of it


def test_block_calls_validate_before_enqueue(L):
    good = 0x10000
    cfg, b, specs, blk = _cfg_block("cfg3", 1)
    B, n = b.batch, len(specs)
    need = nf.nf_block_workspace_bytes(blk, B)
    s = nf.SgdDesc(0.01, 0.9)
    out = C.c_size_t()

    def train(blk_, sgd=s, n_items=4 * B, cap=8 * B, idx=None, ws=good << 8, ws_bytes=need, cache=good, lab=good,
              losses=good, B_=B):
        return L.nf_block_train_epoch(C.byref(blk_), C.byref(sgd), B_, n_items, cache, lab, cap, idx, losses, ws,
                                      ws_bytes, None, None)

    def fill(blk_, n_items=4 * B, cap_in=8 * B, cap_out=8 * B, ws_bytes=need, cin=good, cout=good):
        return L.nf_block_fill_cache(C.byref(blk_), B, n_items, cin, good, cap_in, cout, good, cap_out, good << 8,
                                     ws_bytes, None)

    assert L.nf_block_workspace_bytes(None, B, C.byref(out)) == nf.NF_ERR_NULL
    assert L.nf_block_workspace_bytes(C.byref(blk), B, None) == nf.NF_ERR_NULL
    assert L.nf_block_workspace_bytes(C.byref(blk), 0, C.byref(out)) == nf.NF_ERR_BAD_DESC
    # argument errors
    assert train(blk, cache=None) == nf.NF_ERR_NULL
    assert train(blk, losses=None) == nf.NF_ERR_NULL
    assert train(blk, n_items=0) == nf.NF_ERR_BAD_DESC
    assert train(blk, n_items=9 * B) == nf.NF_ERR_CACHE_RANGE          # contiguous rows beyond the cache
    assert train(blk, ws_bytes=need - 1) == nf.NF_ERR_WORKSPACE
    assert train(blk, ws=(good << 8) + 16) == nf.NF_ERR_WORKSPACE
    assert train(blk, cache=good + 4) == nf.NF_ERR_BAD_DESC
    assert fill(blk, n_items=9 * B) == nf.NF_ERR_CACHE_RANGE
    assert fill(blk, cap_out=B) == nf.NF_ERR_CACHE_RANGE
    assert fill(blk, ws_bytes=16) == nf.NF_ERR_WORKSPACE
    assert fill(blk, cout=None) == nf.NF_ERR_NULL
    # momentum without momentum buffers
    _, _, _, nomom = _cfg_block("cfg3", 1, with_mom=False)
    assert train(nomom) == nf.NF_ERR_NULL
    # structure errors: broken chain, missing / wrong shortcut wiring, empty block, missing parameters
    descs = [nf.LayerDesc(**ls.layer_desc_fields()) for ls in specs]
    auxs = [nf.AuxDesc(**ls.aux_desc_fields(cfg.n_classes)) for ls in specs]
    skip = [(-1 if not ls.skip_kind else ls.skip_src - b.layers[0]) for ls in specs]
    lp = [nf.LayerParams(good, good, good) for _ in specs]
    apar = [nf.AuxParams(good, good, good, good) for _ in specs]
    chain = nf.make_block(descs[:1] + descs[2:], auxs[:1] + auxs[2:], None, lp[:-1], apar[:-1], lp[:-1], apar[:-1],
                          lp[:-1], apar[:-1])
    assert L.nf_block_workspace_bytes(C.byref(chain), B, C.byref(out)) == nf.NF_ERR_BAD_DESC
    assert any(ls.skip_kind for ls in specs)
    noskip = nf.make_block(descs, auxs, None, lp, apar, lp, apar, lp, apar)
    assert train(noskip) == nf.NF_ERR_BAD_DESC
    late = nf.make_block(descs, auxs, [n + 3 if v >= 0 else -1 for v in skip], lp, apar, lp, apar, lp, apar)
    assert train(late) == nf.NF_ERR_BAD_DESC
    wrong = nf.make_block(descs, auxs, [(v + 1 if v >= 0 and v + 1 <= i and specs[i].skip_kind == 2 else v)
                                        for i, v in enumerate(skip)], lp, apar, lp, apar, lp, apar)
    if [v for v in skip] != [wrong._keep["skip_src"][i] for i in range(n)]:
        assert train(wrong) == nf.NF_ERR_BAD_DESC                         # projection source of another shape
    empty = nf.make_block(descs, auxs, skip, lp, apar, lp, apar, lp, apar)
    empty.n_layers = 0
    assert train(empty) == nf.NF_ERR_BAD_DESC
    nop = nf.make_block(descs, auxs, skip, [nf.LayerParams(good, None, good)] * n, apar, lp, apar, lp, apar)
    assert train(nop) == nf.NF_ERR_NULL
    assert fill(nop) == nf.NF_ERR_NULL
    nohead = nf.make_block(descs, None, skip, lp, None)
    assert train(nohead) == nf.NF_ERR_NULL
    # a misaligned pointer in ANY per-layer struct is an argument error of the block call itself
    # (nothing is enqueued), not an error of the per-layer call it would reach mid-pass
    odd = good + 4
    last = n - 1
    for which in ("p", "ap", "gp", "ga", "vp", "va"):
        lp2, ap2 = list(lp), list(apar)
        if which in ("p", "gp", "vp"):
            lp2[last] = nf.LayerParams(good, odd, good)
        else:
            ap2[last] = nf.AuxParams(good, good, odd, good)
        args = dict(p=lp, ap=apar, gp=lp, ga=apar, vp=lp, va=apar)
        args[which] = lp2 if which in ("p", "gp", "vp") else ap2
        bad = nf.make_block(descs, auxs, skip, args["p"], args["ap"], args["gp"], args["ga"], args["vp"], args["va"])
        assert train(bad) == nf.NF_ERR_BAD_DESC, which
    assert L.nf_block_workspace_bytes(C.byref(nohead), B, C.byref(out)) == nf.NF_OK and out.value < need


def test_evaluation_calls_validate_before_enqueue(L):
    good = 0x10000
    d, a = _layer(), _aux()
    ap = nf.AuxParams(good, good, good, good)
    need = nf.nf_workspace_bytes(d, a, 4)

    def pred(y=good, lab=good, cnt=good, out=good, ws_bytes=need, a_=a):
        return L.nf_aux_predict(C.byref(d), C.byref(a_), 4, y, lab, C.byref(ap), out, cnt, 0, None, good << 8, ws_bytes,
                                None)

    assert pred(y=None) == nf.NF_ERR_NULL
    assert pred(out=None) == nf.NF_ERR_NULL
    assert pred(lab=None) == nf.NF_ERR_NULL            # a counter without labels
    assert pred(cnt=None) == nf.NF_ERR_NULL            # labels without a counter
    assert pred(ws_bytes=need - 1) == nf.NF_ERR_WORKSPACE
    assert pred(a_=_aux(head_pool=2)) == nf.NF_ERR_UNSUPPORTED
    assert pred(a_=_aux(loss_kind=5)) == nf.NF_ERR_UNSUPPORTED
    cfg, b, specs, blk = _cfg_block("cfg3", 1)
    B = b.batch
    bneed = nf.nf_block_workspace_bytes(blk, B)

    def ev(e=0, n_items=2 * B, cap=4 * B, ws_bytes=bneed, pred_out=good, blk_=blk):
        return L.nf_block_evaluate(C.byref(blk_), e, B, n_items, good, good, cap, pred_out, good, good << 8, ws_bytes,
                                   None)

    assert ev(e=-1) == nf.NF_ERR_BAD_DESC
    assert ev(e=len(specs)) == nf.NF_ERR_BAD_DESC
    assert ev(n_items=5 * B) == nf.NF_ERR_CACHE_RANGE
    assert ev(pred_out=None) == nf.NF_ERR_NULL
    assert L.nf_block_evaluate(C.byref(blk), 0, B, 2 * B, good, None, 4 * B, good, good, good << 8, bneed,
                               None) == nf.NF_ERR_NULL      # a counter without labels
    assert ev(ws_bytes=bneed // 2) == nf.NF_ERR_WORKSPACE
    out = C.c_int32()
    one = (C.c_int64 * 1)(3)
    assert L.nf_select_exit(0, one, one, C.byref(out)) == nf.NF_ERR_BAD_DESC
    assert L.nf_select_exit(1, None, one, C.byref(out)) == nf.NF_ERR_NULL
    assert nf.nf_select_exit([5, 9, 9, 7], [10, 30, 20, 40]) == 2
    assert nf.nf_select_exit([5, 9, 9, 7], [10, 20, 30, 40]) == 1
    assert nf.nf_select_exit([4, 4], [7, 7]) == 0


def test_contraction_mode_switch():
    """nf_contraction: returns the previous mode, -1 only queries, unknown modes are refused and
    leave the mode as it was."""
    prev = nf.nf_contraction()
    assert prev in (nf.NF_CONTRACT_F32, nf.NF_CONTRACT_BF16X6, nf.NF_CONTRACT_BF16X9)
    try:
        assert nf.nf_contraction(nf.NF_CONTRACT_BF16X9) == prev
        assert nf.nf_contraction(prev) == nf.NF_CONTRACT_BF16X9
        assert nf.nf_contraction(nf.NF_CONTRACT_BF16X6) == prev
        assert nf.nf_contraction() == nf.NF_CONTRACT_BF16X6
        assert nf.nf_contraction(nf.NF_CONTRACT_F32) == nf.NF_CONTRACT_BF16X6
        with pytest.raises(nf.NfError) as e:
            nf.nf_contraction(7)
        assert e.value.status == nf.NF_ERR_BAD_DESC
        assert nf.nf_contraction() == nf.NF_CONTRACT_F32
    finally:
        nf.nf_contraction(prev)


def test_block_graph_handles_without_a_device():
    """The graph entry points' argument checks that need no GPU."""
    L = nf.lib()
    assert L.nf_block_graph_create(None, None, 1, 1, None, None, 1, None, None, None, 0, None) == nf.NF_ERR_NULL
    assert L.nf_block_graph_launch(None, None) == nf.NF_ERR_NULL
    assert L.nf_block_graph_destroy(None) == nf.NF_OK
