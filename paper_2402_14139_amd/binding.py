"""Thin ctypes binding over libnf.so (include/nf.h): argument marshalling only.

Every step of the local training step runs in the library's HIP kernels; PyTorch is used
for device memory (``torch.empty(..., device='cuda')``, ``data_ptr()``) and the current
stream.  There is no CPU fallback: without the built library, or without a GPU, the compute
calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnf.so")

NF_OK = 0
NF_ERR_NULL, NF_ERR_BAD_DESC, NF_ERR_UNSUPPORTED, NF_ERR_WORKSPACE, NF_ERR_CACHE_RANGE, NF_ERR_DEVICE = (
    -1, -2, -3, -4, -5, -6)
NF_ERR_SCRATCH_LIMIT = -7
NF_STATIC_SCRATCH_BYTES = 128 << 20
NF_CONTRACT_F32, NF_CONTRACT_BF16X6, NF_CONTRACT_BF16X9 = 0, 1, 2

EXPORTS = ("nf_strerror", "nf_layer_out_dims", "nf_workspace_bytes", "nf_layer_fwd", "nf_aux_fwd_loss",
           "nf_local_bwd_wgrad", "nf_sgd_update", "nf_cache_write", "nf_cache_read", "nf_local_step",
           "nf_prof_begin", "nf_prof_end", "nf_workspace_region", "nf_block_workspace_bytes",
           "nf_block_train_epoch", "nf_block_fill_cache", "nf_layer_step_bytes", "nf_fit_linear",
           "nf_profile_layer", "nf_partition", "nf_aux_predict", "nf_block_evaluate", "nf_select_exit",
           "nf_device_info", "nf_local_step_static", "nf_contraction", "nf_block_graph_create",
           "nf_block_graph_launch", "nf_block_graph_destroy")

NF_WS_AUX_ACT, NF_WS_POOL_ARG, NF_WS_HEAD_ARG = 0, 1, 2
NF_HEAD_POOL_AVG, NF_HEAD_POOL_MAX = 0, 1
NF_LOSS_CE, NF_LOSS_MSE = 0, 1


class NfError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


class LayerDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "C_in", "H_in", "W_in", "C_out", "R", "S", "stride", "pad",
        "pool_kind", "pool_k", "pool_stride", "pool_pad",
        "skip_kind", "skip_C", "skip_H", "skip_W", "skip_stride")]


class AuxDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "C_in", "H_in", "W_in", "A", "R", "S", "pad", "relu", "pool_oh", "pool_ow", "n_classes",
        "head_pool", "loss_kind")]


class SgdDesc(C.Structure):
    _fields_ = [("lr", C.c_float), ("momentum", C.c_float)]


class LayerParams(C.Structure):
    _fields_ = [("W", C.c_void_p), ("b", C.c_void_p), ("Wp", C.c_void_p)]


class ProfRecord(C.Structure):
    _fields_ = [("kernel", C.c_char * 48), ("launches", C.c_int64), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


class AuxParams(C.Structure):
    _fields_ = [("Wa", C.c_void_p), ("ba", C.c_void_p), ("Wf", C.c_void_p), ("bf", C.c_void_p)]


class LinearModel(C.Structure):
    _fields_ = [("slope", C.c_double), ("intercept", C.c_double)]


class Block(C.Structure):
    """nf_block: host arrays of n_layers descriptors / parameter structs."""
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(LayerDesc)), ("aux", C.POINTER(AuxDesc)),
                ("skip_src", C.POINTER(C.c_int32)), ("p", C.POINTER(LayerParams)), ("ap", C.POINTER(AuxParams)),
                ("gp", C.POINTER(LayerParams)), ("ga", C.POINTER(AuxParams)), ("vp", C.POINTER(LayerParams)),
                ("va", C.POINTER(AuxParams))]


_lib = None


def lib():
    """Loads libnf.so; raises if it has not been built (no fallback of any kind)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2402_14139_amd.build` "
                               "(or __graft_entry__.build()); there is no fallback path")
        # PyTorch ships its own copy of the HIP runtime; it must be in the process before libnf.so
        # is loaded, so that both use the same runtime (with two runtimes the second one finds no
        # device and every launch of libnf fails)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.nf_strerror.restype = C.c_char_p
        L.nf_strerror.argtypes = [C.c_int32]
        for name in EXPORTS[1:]:
            getattr(L, name).restype = C.c_int32
        L.nf_layer_out_dims.argtypes = [C.POINTER(LayerDesc)] + [C.POINTER(C.c_int32)] * 4
        L.nf_workspace_bytes.argtypes = [C.POINTER(LayerDesc), C.POINTER(AuxDesc), C.c_int32, C.POINTER(C.c_size_t)]
        L.nf_layer_fwd.argtypes = [C.POINTER(LayerDesc), C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(LayerParams),
                                   C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.nf_aux_fwd_loss.argtypes = [C.POINTER(LayerDesc), C.POINTER(AuxDesc), C.c_int32, C.c_void_p, C.c_void_p,
                                      C.POINTER(AuxParams), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.nf_local_bwd_wgrad.argtypes = [C.POINTER(LayerDesc), C.POINTER(AuxDesc), C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.POINTER(LayerParams), C.POINTER(AuxParams),
                                         C.POINTER(LayerParams), C.POINTER(AuxParams), C.c_void_p, C.c_size_t,
                                         C.c_void_p]
        L.nf_sgd_update.argtypes = [C.POINTER(SgdDesc), C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                    C.POINTER(C.c_void_p), C.POINTER(C.c_int64), C.c_void_p]
        L.nf_cache_write.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_void_p,
                                     C.c_void_p, C.c_void_p]
        L.nf_cache_read.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_void_p]
        L.nf_local_step.argtypes = [C.POINTER(LayerDesc), C.POINTER(AuxDesc), C.POINTER(SgdDesc), C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.POINTER(LayerParams), C.POINTER(AuxParams), C.POINTER(LayerParams),
                                    C.POINTER(AuxParams), C.POINTER(LayerParams), C.POINTER(AuxParams),
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.nf_local_step_static.argtypes = L.nf_local_step.argtypes[:15] + [C.c_void_p]
        L.nf_prof_end.argtypes = [C.POINTER(ProfRecord), C.c_int32, C.POINTER(C.c_int32)]
        L.nf_workspace_region.argtypes = [C.POINTER(LayerDesc), C.POINTER(AuxDesc), C.c_int32, C.c_int32,
                                          C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.nf_block_workspace_bytes.argtypes = [C.POINTER(Block), C.c_int32, C.POINTER(C.c_size_t)]
        L.nf_block_train_epoch.argtypes = [C.POINTER(Block), C.POINTER(SgdDesc), C.c_int32, C.c_int64, C.c_void_p,
                                           C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                           C.c_void_p, C.c_void_p]
        L.nf_block_graph_create.argtypes = [C.POINTER(Block), C.POINTER(SgdDesc), C.c_int32, C.c_int64, C.c_void_p,
                                            C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                            C.POINTER(C.c_void_p)]
        L.nf_block_graph_launch.argtypes = [C.c_void_p, C.c_void_p]
        L.nf_block_graph_destroy.argtypes = [C.c_void_p]
        L.nf_block_fill_cache.argtypes = [C.POINTER(Block), C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64,
                                          C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
        L.nf_aux_predict.argtypes = [C.POINTER(LayerDesc), C.POINTER(AuxDesc), C.c_int32, C.c_void_p, C.c_void_p,
                                     C.POINTER(AuxParams), C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                     C.c_size_t, C.c_void_p]
        L.nf_block_evaluate.argtypes = [C.POINTER(Block), C.c_int32, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p,
                                        C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.nf_select_exit.argtypes = [C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        L.nf_device_info.argtypes = [C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.nf_contraction.argtypes = [C.c_int32]
        L.nf_layer_step_bytes.argtypes = [C.POINTER(LayerDesc), C.POINTER(AuxDesc), C.c_int32, C.c_int32,
                                          C.POINTER(C.c_size_t)]
        L.nf_fit_linear.argtypes = [C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(LinearModel)]
        L.nf_profile_layer.argtypes = [C.POINTER(LayerDesc), C.POINTER(AuxDesc), C.c_int32, C.c_int32,
                                       C.POINTER(C.c_int32), C.POINTER(LinearModel)]
        L.nf_partition.argtypes = [C.c_int32, C.POINTER(LinearModel), C.c_double, C.c_int32, C.c_double,
                                   C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                   C.POINTER(C.c_int32)]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().nf_strerror(int(status)).decode()


def _check(rc, where):
    if rc != NF_OK:
        raise NfError(rc, where)


def _ptr(t):
    """Device pointer of a torch tensor (or None / raw int passthrough)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def layer_params(W=None, b=None, Wp=None) -> LayerParams:
    return LayerParams(_ptr(W), _ptr(b), _ptr(Wp))


def aux_params(Wa=None, ba=None, Wf=None, bf=None) -> AuxParams:
    return AuxParams(_ptr(Wa), _ptr(ba), _ptr(Wf), _ptr(bf))


def nf_layer_out_dims(d: LayerDesc):
    o = [C.c_int32() for _ in range(4)]
    _check(lib().nf_layer_out_dims(C.byref(d), *[C.byref(v) for v in o]), "nf_layer_out_dims")
    return tuple(int(v.value) for v in o)


def nf_workspace_bytes(d: LayerDesc, a: AuxDesc | None, B: int) -> int:
    out = C.c_size_t()
    _check(lib().nf_workspace_bytes(C.byref(d), C.byref(a) if a is not None else None, B, C.byref(out)),
           "nf_workspace_bytes")
    return int(out.value)


def nf_workspace_region(d: LayerDesc, a: AuxDesc | None, B: int, which: int):
    """(byte offset, byte size) of an intermediate inside the workspace."""
    off, nb = C.c_size_t(), C.c_size_t()
    _check(lib().nf_workspace_region(C.byref(d), C.byref(a) if a is not None else None, B, which, C.byref(off),
                                     C.byref(nb)), "nf_workspace_region")
    return int(off.value), int(nb.value)


def _ws(ws):
    return (_ptr(ws), ws.numel() * ws.element_size()) if ws is not None else (None, 0)


def nf_layer_fwd(d, B, x, x_skip, p: LayerParams, y, ws, stream=None):
    wp, wn = _ws(ws)
    _check(lib().nf_layer_fwd(C.byref(d), B, _ptr(x), _ptr(x_skip), C.byref(p), _ptr(y), wp, wn, _stream(stream)),
           "nf_layer_fwd")


def nf_aux_fwd_loss(d, a, B, y, labels, ap: AuxParams, loss_out, ws, stream=None):
    wp, wn = _ws(ws)
    _check(lib().nf_aux_fwd_loss(C.byref(d), C.byref(a), B, _ptr(y), _ptr(labels), C.byref(ap), _ptr(loss_out), wp,
                                 wn, _stream(stream)), "nf_aux_fwd_loss")


def nf_local_bwd_wgrad(d, a, B, x, x_skip, y, p, ap, gp, ga, ws, stream=None):
    wp, wn = _ws(ws)
    _check(lib().nf_local_bwd_wgrad(C.byref(d), C.byref(a), B, _ptr(x), _ptr(x_skip), _ptr(y), C.byref(p),
                                    C.byref(ap), C.byref(gp), C.byref(ga), wp, wn, _stream(stream)),
           "nf_local_bwd_wgrad")


def nf_sgd_update(lr, momentum, w, g, v, stream=None):
    """w, g, v: lists of torch tensors (v None when momentum == 0)."""
    n = len(w)
    s = SgdDesc(lr, momentum)
    arr = lambda ts: (C.c_void_p * n)(*[_ptr(t) for t in ts])  # noqa: E731
    numel = (C.c_int64 * n)(*[t.numel() for t in w])
    _check(lib().nf_sgd_update(C.byref(s), n, arr(w), arr(g), arr(v) if v is not None else None, numel,
                               _stream(stream)), "nf_sgd_update")


def nf_cache_write(cache, cache_labels, capacity, sample_elems, first, B, y, labels, stream=None):
    _check(lib().nf_cache_write(_ptr(cache), _ptr(cache_labels), capacity, sample_elems, first, B, _ptr(y),
                                _ptr(labels), _stream(stream)), "nf_cache_write")


def nf_cache_read(cache, cache_labels, capacity, sample_elems, first, idx, B, x_out, labels_out, stream=None):
    _check(lib().nf_cache_read(_ptr(cache), _ptr(cache_labels), capacity, sample_elems, first, _ptr(idx), B,
                               _ptr(x_out), _ptr(labels_out), _stream(stream)), "nf_cache_read")


def nf_local_step(d, a, lr, momentum, B, x, x_skip, labels, p, ap, gp, ga, vp, va, y_out, loss_out, ws,
                  stream=None):
    s = SgdDesc(lr, momentum)
    wp, wn = _ws(ws)
    _check(lib().nf_local_step(C.byref(d), C.byref(a), C.byref(s), B, _ptr(x), _ptr(x_skip), _ptr(labels),
                               C.byref(p), C.byref(ap), C.byref(gp), C.byref(ga),
                               C.byref(vp) if vp is not None else None, C.byref(va) if va is not None else None,
                               _ptr(y_out), _ptr(loss_out), wp, wn, _stream(stream)), "nf_local_step")


def nf_local_step_static(d, a, lr, momentum, B, x, x_skip, labels, p, ap, gp, ga, vp, va, y_out, loss_out,
                         stream=None):
    """nf_local_step with the scratch in the library's static device array (allocates nothing)."""
    s = SgdDesc(lr, momentum)
    _check(lib().nf_local_step_static(C.byref(d), C.byref(a), C.byref(s), B, _ptr(x), _ptr(x_skip), _ptr(labels),
                                      C.byref(p), C.byref(ap), C.byref(gp), C.byref(ga),
                                      C.byref(vp) if vp is not None else None,
                                      C.byref(va) if va is not None else None,
                                      _ptr(y_out), _ptr(loss_out), _stream(stream)), "nf_local_step_static")


def nf_prof_begin():
    _check(lib().nf_prof_begin(), "nf_prof_begin")


def nf_prof_end(cap: int = 64):
    """list of dicts {kernel, launches, ms, flops, bytes}, sorted by total duration."""
    recs = (ProfRecord * cap)()
    n = C.c_int32()
    _check(lib().nf_prof_end(recs, cap, C.byref(n)), "nf_prof_end")
    return [dict(kernel=recs[i].kernel.decode(), launches=int(recs[i].launches), ms=float(recs[i].ms),
                 flops=float(recs[i].flops), bytes=float(recs[i].bytes)) for i in range(min(n.value, cap))]


def make_block(descs, auxs, skip_src, p, ap, gp=None, ga=None, vp=None, va=None) -> Block:
    """Packs per-layer descriptor / parameter structs (lists) into an nf_block.  The arrays are
    kept alive as attributes of the returned struct."""
    n = len(descs)
    blk = Block()
    blk.n_layers = n

    def arr(ctype, items):
        if items is None:
            return None
        a = (ctype * n)()
        for i, it in enumerate(items):
            C.memmove(C.byref(a, i * C.sizeof(ctype)), C.byref(it), C.sizeof(ctype))
        return a

    keep = dict(layers=arr(LayerDesc, descs), aux=arr(AuxDesc, auxs),
                skip_src=None if skip_src is None else (C.c_int32 * n)(*skip_src),
                p=arr(LayerParams, p), ap=arr(AuxParams, ap), gp=arr(LayerParams, gp), ga=arr(AuxParams, ga),
                vp=arr(LayerParams, vp), va=arr(AuxParams, va))
    for k, v in keep.items():
        if v is not None:
            setattr(blk, k, v)
    blk._keep = keep
    return blk


def nf_block_workspace_bytes(blk: Block, B: int) -> int:
    out = C.c_size_t()
    _check(lib().nf_block_workspace_bytes(C.byref(blk), B, C.byref(out)), "nf_block_workspace_bytes")
    return int(out.value)


def nf_block_train_epoch(blk: Block, lr, momentum, B, n_items, cache, cache_labels, capacity, idx, losses, ws,
                         stream=None, prefetch_stream=None):
    s = SgdDesc(lr, momentum)
    wp, wn = _ws(ws)
    _check(lib().nf_block_train_epoch(C.byref(blk), C.byref(s), B, n_items, _ptr(cache), _ptr(cache_labels), capacity,
                                      _ptr(idx), _ptr(losses), wp, wn, _stream(stream),
                                      None if prefetch_stream is None else _stream(prefetch_stream)),
           "nf_block_train_epoch")


def nf_block_graph_create(blk: Block, lr, momentum, B, n_items, cache, cache_labels, capacity, idx, losses, ws):
    """Returns the handle (an integer address) of the captured block pass."""
    s = SgdDesc(lr, momentum)
    wp, wn = _ws(ws)
    h = C.c_void_p()
    _check(lib().nf_block_graph_create(C.byref(blk), C.byref(s), B, n_items, _ptr(cache), _ptr(cache_labels), capacity,
                                       _ptr(idx), _ptr(losses), wp, wn, C.byref(h)), "nf_block_graph_create")
    return h.value


def nf_block_graph_launch(handle, stream=None):
    _check(lib().nf_block_graph_launch(C.c_void_p(handle), _stream(stream)), "nf_block_graph_launch")


def nf_block_graph_destroy(handle):
    _check(lib().nf_block_graph_destroy(C.c_void_p(handle) if handle else None), "nf_block_graph_destroy")


def nf_block_fill_cache(blk: Block, B, n_items, cache_in, labels_in, capacity_in, cache_out, labels_out,
                        capacity_out, ws, stream=None):
    wp, wn = _ws(ws)
    _check(lib().nf_block_fill_cache(C.byref(blk), B, n_items, _ptr(cache_in), _ptr(labels_in), capacity_in,
                                     _ptr(cache_out), _ptr(labels_out), capacity_out, wp, wn, _stream(stream)),
           "nf_block_fill_cache")


def nf_layer_step_bytes(d: LayerDesc, a: AuxDesc, B: int, with_momentum: bool) -> int:
    out = C.c_size_t()
    _check(lib().nf_layer_step_bytes(C.byref(d), C.byref(a), B, int(with_momentum), C.byref(out)),
           "nf_layer_step_bytes")
    return int(out.value)


def nf_fit_linear(batches, nbytes):
    n = len(batches)
    m = LinearModel()
    _check(lib().nf_fit_linear(n, (C.c_double * n)(*batches), (C.c_double * n)(*nbytes), C.byref(m)), "nf_fit_linear")
    return m.slope, m.intercept


def nf_profile_layer(d: LayerDesc, a: AuxDesc, with_momentum: bool, batches):
    n = len(batches)
    m = LinearModel()
    _check(lib().nf_profile_layer(C.byref(d), C.byref(a), int(with_momentum), n, (C.c_int32 * n)(*batches),
                                  C.byref(m)), "nf_profile_layer")
    return m.slope, m.intercept


def nf_partition(models, M: float, B_limit: int, rho: float):
    """models: list of (slope, intercept).  Returns (per-layer batch sizes, [(first layer, batch size), ...])."""
    n = len(models)
    R = (LinearModel * n)(*[LinearModel(s, c) for s, c in models])
    lb, bf, bb, nb = (C.c_int32 * n)(), (C.c_int32 * n)(), (C.c_int32 * n)(), C.c_int32()
    _check(lib().nf_partition(n, R, M, B_limit, rho, lb, bf, bb, C.byref(nb)), "nf_partition")
    return list(lb), [(int(bf[k]), int(bb[k])) for k in range(nb.value)]


def nf_aux_predict(d, a, B, y, labels, ap: AuxParams, pred_out, n_correct, accumulate, logits_out, ws, stream=None):
    wp, wn = _ws(ws)
    _check(lib().nf_aux_predict(C.byref(d), C.byref(a), B, _ptr(y), _ptr(labels), C.byref(ap), _ptr(pred_out),
                                _ptr(n_correct), int(accumulate), _ptr(logits_out), wp, wn, _stream(stream)),
           "nf_aux_predict")


def nf_block_evaluate(blk: Block, exit_layer, B, n_items, cache, cache_labels, capacity, pred_out, n_correct, ws,
                      stream=None):
    wp, wn = _ws(ws)
    _check(lib().nf_block_evaluate(C.byref(blk), exit_layer, B, n_items, _ptr(cache), _ptr(cache_labels), capacity,
                                   _ptr(pred_out), _ptr(n_correct), wp, wn, _stream(stream)), "nf_block_evaluate")


def nf_select_exit(n_correct, n_params) -> int:
    n = len(n_correct)
    out = C.c_int32()
    _check(lib().nf_select_exit(n, (C.c_int64 * n)(*n_correct), (C.c_int64 * n)(*n_params), C.byref(out)),
           "nf_select_exit")
    return int(out.value)


def nf_contraction(mode: int = -1) -> int:
    """Sets the process-wide contraction mode (NF_CONTRACT_F32 / NF_CONTRACT_BF16X6 / NF_CONTRACT_BF16X9) and returns the
    previous one; mode = -1 only queries."""
    rc = int(lib().nf_contraction(int(mode)))
    if rc < 0:
        _check(rc, "nf_contraction")
    return rc


def nf_device_info():
    """(compute units, peak shader clock in kHz) of the current device."""
    cu, khz = C.c_int32(), C.c_int32()
    _check(lib().nf_device_info(C.byref(cu), C.byref(khz)), "nf_device_info")
    return int(cu.value), int(khz.value)
