"""ctypes access to the CPU oracle (``oracle/nfo.cpp``).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's ``cpu_baseline`` leg may import this module.
It shares nothing with the GPU library: logical NCHW / OIHW numpy arrays in, numpy out.

Paper: Eq. 1 (layer), Eq. 2 (auxiliary head), Eq. 3 (loss), Algorithm 2 (local step; its
Worker loop over the batches and layers of a block), and the activation cache between blocks
(written by a forward-only sweep once a block is trained, read at the next block's batch size).

The block-level functions at the end are plain Python loops over the single-layer calls; they
are pinned by per-layer torch.optim.SGD / autograd runs of the same block and by the
equivalence "training from the cache == training on recomputed activations".
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnfo.so")
_lib = None


def build(verbose: bool = False) -> str:
    """Compile ``nfo.cpp`` into ``libnfo.so`` next to it (g++, OpenMP)."""
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           os.path.join(_HERE, "nfo.cpp"), "-o", _LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return _LIB_PATH


class LayerDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "C_in", "H_in", "W_in", "C_out", "R", "S", "stride", "pad",
        "pool_kind", "pool_k", "pool_stride", "pool_pad",
        "skip_kind", "skip_C", "skip_H", "skip_W", "skip_stride")]


class AuxDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "C_in", "H_in", "W_in", "A", "R", "S", "pad", "relu", "pool_oh", "pool_ow", "n_classes",
        "head_pool", "loss_kind")]


HEAD_POOL_AVG, HEAD_POOL_MAX = 0, 1
LOSS_CE, LOSS_MSE = 0, 1


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        _lib = C.CDLL(_LIB_PATH)
        _lib.nfo_layer_dims.restype = C.c_int32
        _lib.nfo_num_threads.restype = C.c_int32
    return _lib


def num_threads() -> int:
    return int(lib().nfo_num_threads())


def set_num_threads(n: int) -> None:
    lib().nfo_set_num_threads(C.c_int32(n))


def _suf(dtype) -> str:
    dtype = np.dtype(dtype)
    if dtype == np.float32:
        return "f32"
    if dtype == np.float64:
        return "f64"
    raise TypeError(f"oracle supports float32/float64, got {dtype}")


def _p(a):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"], "oracle arrays must be C-contiguous"
    return a.ctypes.data_as(C.c_void_p)


def layer_desc(C_in, H_in, W_in, C_out, R=3, S=3, stride=1, pad=1, pool_kind=0, pool_k=0,
               pool_stride=0, pool_pad=0, skip_kind=0, skip_C=0, skip_H=0, skip_W=0,
               skip_stride=0) -> LayerDesc:
    return LayerDesc(C_in, H_in, W_in, C_out, R, S, stride, pad, pool_kind, pool_k, pool_stride,
                     pool_pad, skip_kind, skip_C, skip_H, skip_W, skip_stride)


def aux_desc(C_in, H_in, W_in, A, n_classes, R=3, S=3, pad=1, relu=1, pool_oh=2, pool_ow=2, head_pool=0,
             loss_kind=0) -> AuxDesc:
    return AuxDesc(C_in, H_in, W_in, A, R, S, pad, relu, pool_oh, pool_ow, n_classes, head_pool, loss_kind)


def layer_dims(d: LayerDesc):
    """(Ho, Wo, Hp, Wp): conv output and emitted (post-pool) spatial sizes."""
    o = [C.c_int32() for _ in range(4)]
    rc = lib().nfo_layer_dims(C.byref(d), *[C.byref(v) for v in o])
    if rc != 0:
        raise ValueError("invalid layer descriptor")
    return tuple(int(v.value) for v in o)


def aux_out_hw(a: AuxDesc):
    return a.H_in + 2 * a.pad - a.R + 1, a.W_in + 2 * a.pad - a.S + 1


@dataclass
class LayerFwd:
    Z: np.ndarray
    Y: np.ndarray
    arg: np.ndarray | None


def layer_fwd(d: LayerDesc, x, x_skip, W, b, Wp=None) -> LayerFwd:
    """Eq. 1 for a batch ``x`` [B,C,H,W]."""
    dt = x.dtype
    B = x.shape[0]
    Ho, Wo, Hp, Wp_ = layer_dims(d)
    Z = np.empty((B, d.C_out, Ho, Wo), dt)
    Y = np.empty((B, d.C_out, Hp, Wp_), dt)
    arg = np.empty((B, d.C_out, Hp, Wp_), np.int32) if d.pool_kind else None
    getattr(lib(), "nfo_layer_fwd_" + _suf(dt))(
        C.byref(d), C.c_int32(B), _p(x), _p(x_skip), _p(W), _p(b), _p(Wp), _p(Z), _p(Y), _p(arg))
    return LayerFwd(Z, Y, arg)


@dataclass
class AuxFwd:
    U: np.ndarray
    Pq: np.ndarray
    z: np.ndarray
    loss: float
    dz: np.ndarray
    Upre: np.ndarray | None = None
    parg: np.ndarray | None = None


def aux_fwd_loss(a: AuxDesc, y, labels, Wa, ba, Wf, bf) -> AuxFwd:
    """Eq. 2 and Eq. 3 (batch mean of the head's loss) for the emitted activations ``y``."""
    dt = y.dtype
    B = y.shape[0]
    Hu, Wu = aux_out_hw(a)
    U = np.empty((B, a.A, Hu, Wu), dt)
    Pq = np.empty((B, a.A * a.pool_oh * a.pool_ow), dt)
    z = np.empty((B, a.n_classes), dt)
    dz = np.empty((B, a.n_classes), dt)
    Upre = np.empty_like(U)
    parg = np.zeros(Pq.shape, np.int32)
    loss = C.c_double()
    labels = np.ascontiguousarray(labels, np.int32)
    getattr(lib(), "nfo_aux_fwd_loss_" + _suf(dt))(
        C.byref(a), C.c_int32(B), _p(y), _p(labels), _p(Wa), _p(ba), _p(Wf), _p(bf),
        _p(U), _p(Pq), _p(z), C.byref(loss), _p(dz), _p(Upre), _p(parg))
    return AuxFwd(U, Pq, z, float(loss.value), dz, Upre, parg)


def local_bwd(d: LayerDesc, a: AuxDesc, x, x_skip, lf: LayerFwd, af: AuxFwd, Wa, Wf, mask_u=None, mask_z=None):
    """Gradients of the local loss w.r.t. the layer's and the head's parameters only.

    mask_u / mask_z (uint8, shapes of U / Z) optionally replace the ReLU decisions U>0 / Z>0;
    the head's max-pooling selection is taken from ``af.parg``."""
    parg = None if af.parg is None else np.ascontiguousarray(af.parg, np.int32)
    mask_u = None if mask_u is None else np.ascontiguousarray(mask_u, np.uint8)
    mask_z = None if mask_z is None else np.ascontiguousarray(mask_z, np.uint8)
    dt = x.dtype
    B = x.shape[0]
    F = a.A * a.pool_oh * a.pool_ow
    g = {
        "W": np.empty((d.C_out, d.C_in, d.R, d.S), dt),
        "b": np.empty((d.C_out,), dt),
        "Wp": np.empty((d.C_out, d.skip_C), dt) if d.skip_kind == 2 else None,
        "Wa": np.empty((a.A, a.C_in, a.R, a.S), dt),
        "ba": np.empty((a.A,), dt),
        "Wf": np.empty((a.n_classes, F), dt),
        "bf": np.empty((a.n_classes,), dt),
        "dY": np.empty_like(lf.Y),
        "dZ": np.empty_like(lf.Z),
    }
    getattr(lib(), "nfo_local_bwd_" + _suf(dt))(
        C.byref(d), C.byref(a), C.c_int32(B), _p(x), _p(x_skip), _p(lf.Z), _p(lf.Y), _p(lf.arg),
        _p(af.U), _p(af.Pq), _p(af.dz), _p(Wa), _p(Wf),
        _p(g["W"]), _p(g["b"]), _p(g["Wp"]), _p(g["Wa"]), _p(g["ba"]), _p(g["Wf"]), _p(g["bf"]),
        _p(g["dY"]), _p(g["dZ"]), _p(mask_u), _p(mask_z), _p(parg))
    return g


def sgd_update(w, g, v, lr, mu) -> None:
    """In place: v = mu*v + g; w = w - lr*v  (v None or mu == 0: w = w - lr*g)."""
    getattr(lib(), "nfo_sgd_update_" + _suf(w.dtype))(
        C.c_int64(w.size), _p(w), _p(g), _p(v), C.c_double(lr), C.c_double(mu))


def cache_write(cache, cache_labels, first, y, labels) -> None:
    B = y.shape[0]
    se = int(np.prod(y.shape[1:]))
    labels = None if labels is None else np.ascontiguousarray(labels, np.int32)
    getattr(lib(), "nfo_cache_write_" + _suf(cache.dtype))(
        _p(cache), _p(cache_labels), C.c_int64(se), C.c_int64(first), C.c_int32(B), _p(y), _p(labels))


def cache_read(cache, cache_labels, first, idx, B, sample_shape):
    se = int(np.prod(sample_shape))
    x = np.empty((B,) + tuple(sample_shape), cache.dtype)
    lab = np.empty((B,), np.int32) if cache_labels is not None else None
    idx = None if idx is None else np.ascontiguousarray(idx, np.int64)
    getattr(lib(), "nfo_cache_read_" + _suf(cache.dtype))(
        _p(cache), _p(cache_labels), C.c_int64(se), C.c_int64(first), _p(idx), C.c_int32(B), _p(x), _p(lab))
    return x, lab


PARAM_NAMES = ("W", "b", "Wp", "Wa", "ba", "Wf", "bf")


def local_step(d: LayerDesc, a: AuxDesc, x, x_skip, labels, params: dict, mom: dict | None,
               lr: float, mu: float):
    """One pass of the Algorithm 2 body.  ``params`` (and ``mom``) are updated in place.

    Returns (Y emitted with the pre-update weights, loss, dict of gradients).
    """
    dt = x.dtype
    B = x.shape[0]
    _, _, Hp, Wp_ = layer_dims(d)
    Y = np.empty((B, d.C_out, Hp, Wp_), dt)
    grads = {k: (None if params.get(k) is None else np.empty_like(params[k])) for k in PARAM_NAMES}
    loss = C.c_double()
    labels = np.ascontiguousarray(labels, np.int32)
    mom = mom or {}
    getattr(lib(), "nfo_local_step_" + _suf(dt))(
        C.byref(d), C.byref(a), C.c_int32(B), _p(x), _p(x_skip), _p(labels),
        *[_p(params.get(k)) for k in PARAM_NAMES],
        *[_p(grads[k]) for k in PARAM_NAMES],
        *[_p(mom.get(k)) for k in PARAM_NAMES],
        C.c_double(lr), C.c_double(mu), _p(Y), C.byref(loss))
    return Y, float(loss.value), grads


# ---- a block of consecutive local layers: the Worker loop of Algorithm 2 and the cache sweep ----
@dataclass
class BlockLayer:
    """One local layer inside a block.  ``skip_src`` is -1, or the position (inside the block)
    of the layer whose INPUT is this layer's shortcut tensor (0 = the block's input batch)."""
    d: LayerDesc
    a: AuxDesc
    params: dict
    mom: dict | None = None
    skip_src: int = -1


def _batches(n_items: int, B: int):
    return [(f, min(B, n_items - f)) for f in range(0, n_items, B)]


def block_train_epoch(layers, cache, cache_labels, idx, n_items, B, sample_shape, lr, mu, step=None):
    """One pass of a block over ``n_items`` cached samples in batches of ``B`` (the last batch
    may be smaller): for every batch, read it from the cache (rows ``idx[j]``, or the contiguous
    rows when ``idx`` is None), then run the Algorithm 2 body layer by layer — each layer is
    updated from its own local loss and hands on the activations it computed BEFORE its update.

    Parameters and momentum buffers of ``layers`` are updated in place.  Returns the losses as
    an array [n_batches, n_layers].  ``step(j, n, L, x, x_skip, labels) -> (y, loss)``, if given,
    stands in for ``local_step`` on layer ``L`` (a GPU comparison uses it to run the same step with
    the ReLU / max-pool decisions that are ties within rounding taken as the kernels took them)."""
    bl = _batches(n_items, B)
    losses = np.zeros((len(bl), len(layers)), np.float64)
    for j, (first, nb) in enumerate(bl):
        sel = None if idx is None else np.asarray(idx[first:first + nb], np.int64)
        x0, lab = cache_read(cache, cache_labels, first, sel, nb, sample_shape)
        inputs = [x0]
        for n, L in enumerate(layers):
            xs = None if L.skip_src < 0 else inputs[L.skip_src]
            if step is not None:
                y, loss = step(j, n, L, inputs[n], xs, lab)
            else:
                y, loss, _ = local_step(L.d, L.a, inputs[n], xs, lab, L.params, L.mom, lr, mu)
            losses[j, n] = loss
            inputs.append(y)
    return losses


def block_fill_cache(layers, cache_in, labels_in, n_items, B, sample_shape, cache_out, labels_out):
    """After a block has been trained: forward-only sweep with its final weights over the
    block's input set (contiguous batches of ``B``, last one partial), storing the last layer's
    emitted activations and the labels as rows ``[0, n_items)`` of the next cache."""
    for first, nb in _batches(n_items, B):
        x0, lab = cache_read(cache_in, labels_in, first, None, nb, sample_shape)
        inputs = [x0]
        for n, L in enumerate(layers):
            xs = None if L.skip_src < 0 else inputs[L.skip_src]
            p = L.params
            inputs.append(layer_fwd(L.d, inputs[n], xs, p["W"], p["b"], p.get("Wp")).Y)
        cache_write(cache_out, labels_out, first, inputs[-1], lab)


# ---- early-exit evaluation ("Trained Output CNN"): forward only, prediction, accuracy -----------
def aux_predict(a: AuxDesc, y, Wa, ba, Wf, bf):
    """Logits of the head on emitted activations ``y`` (Eq. 2) and the predicted class per
    sample: the class with the largest logit, the lowest index among equal maxima."""
    af = aux_fwd_loss(a, y, np.zeros((y.shape[0],), np.int32), Wa, ba, Wf, bf)
    pred = np.empty((y.shape[0],), np.int32)
    for n in range(y.shape[0]):
        best, bi = af.z[n, 0], 0
        for q in range(1, a.n_classes):
            if af.z[n, q] > best:
                best, bi = af.z[n, q], q
        pred[n] = bi
    return af.z, pred


def block_evaluate(layers, exit_layer, cache, cache_labels, n_items, B, sample_shape):
    """Early-exit model that leaves the block after layer ``exit_layer`` (0-based): forward
    through layers 0..exit_layer with their current weights, then that layer's head; rows
    [0, n_items) of the block's input cache in batches of B.  Returns (predictions [n_items],
    number of correct predictions)."""
    preds = np.empty((n_items,), np.int32)
    correct = 0
    for first, nb in _batches(n_items, B):
        x0, lab = cache_read(cache, cache_labels, first, None, nb, sample_shape)
        inputs = [x0]
        for n in range(exit_layer + 1):
            L = layers[n]
            xs = None if L.skip_src < 0 else inputs[L.skip_src]
            p = L.params
            inputs.append(layer_fwd(L.d, inputs[n], xs, p["W"], p["b"], p.get("Wp")).Y)
        p = layers[exit_layer].params
        _, pr = aux_predict(layers[exit_layer].a, inputs[-1], p["Wa"], p["ba"], p["Wf"], p["bf"])
        preds[first:first + nb] = pr
        correct += int((pr == lab).sum())
    return preds, correct


def select_exit(n_correct, n_params):
    """The output model: the exit with the highest validation accuracy; among equally accurate
    exits the one with the fewest parameters; among those the earliest.  ``n_correct[e]`` is the
    number of correct validation predictions of exit e, ``n_params[e]`` the parameter count of
    the model that ends there.  Returns the exit's index."""
    best = 0
    for e in range(1, len(n_correct)):
        if n_correct[e] > n_correct[best] or (n_correct[e] == n_correct[best] and n_params[e] < n_params[best]):
            best = e
    return best
