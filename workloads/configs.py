"""Network tables for the five benchmark configurations (shapes only, no arithmetic).

A network is a list of *local layers* in the sense of the paper's Eq. 1: one convolution
(+ bias, optional shortcut, ReLU, optional max-pool), each with its own auxiliary head
(Eq. 2) of ``A`` filters.  Consecutive layers are grouped into blocks, each with its own
batch size (the paper's partitioning into blocks with block-specific batch sizes).
"""
from __future__ import annotations

from dataclasses import dataclass, field


@dataclass
class LayerSpec:
    name: str
    C_in: int
    H_in: int
    W_in: int
    C_out: int
    R: int = 3
    S: int = 3
    stride: int = 1
    pad: int = 1
    pool_kind: int = 0      # 0 none, 1 max
    pool_k: int = 0
    pool_stride: int = 0
    pool_pad: int = 0
    skip_kind: int = 0      # 0 none, 1 identity, 2 1x1 strided projection
    skip_src: int = -1      # index of the layer whose INPUT is this layer's shortcut tensor
    skip_C: int = 0
    skip_H: int = 0
    skip_W: int = 0
    skip_stride: int = 0
    A: int = 0              # auxiliary-head filters
    block: int = 0          # index of the block this layer belongs to

    @property
    def Ho(self):
        return (self.H_in + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self):
        return (self.W_in + 2 * self.pad - self.S) // self.stride + 1

    @property
    def Hp(self):
        if not self.pool_kind:
            return self.Ho
        return (self.Ho + 2 * self.pool_pad - self.pool_k) // self.pool_stride + 1

    @property
    def Wp(self):
        if not self.pool_kind:
            return self.Wo
        return (self.Wo + 2 * self.pool_pad - self.pool_k) // self.pool_stride + 1

    def layer_desc_fields(self):
        return dict(C_in=self.C_in, H_in=self.H_in, W_in=self.W_in, C_out=self.C_out, R=self.R,
                    S=self.S, stride=self.stride, pad=self.pad, pool_kind=self.pool_kind,
                    pool_k=self.pool_k, pool_stride=self.pool_stride, pool_pad=self.pool_pad,
                    skip_kind=self.skip_kind, skip_C=self.skip_C, skip_H=self.skip_H,
                    skip_W=self.skip_W, skip_stride=self.skip_stride)

    def aux_desc_fields(self, n_classes):
        return dict(C_in=self.C_out, H_in=self.Hp, W_in=self.Wp, A=self.A, R=3, S=3, pad=1, relu=1,
                    pool_oh=2, pool_ow=2, n_classes=n_classes)


@dataclass
class Block:
    layers: list
    batch: int


@dataclass
class Config:
    name: str
    in_shape: tuple
    n_classes: int
    layers: list
    blocks: list
    lr: float
    momentum: float
    seed: int
    n_samples: int          # synthetic data-set size used for the cache streams
    notes: str = ""
    extra: dict = field(default_factory=dict)


def vgg_layers(channels, pool_after, in_shape=(3, 32, 32)):
    """3x3/pad-1 conv stack; ``pool_after`` holds 1-based layer indices followed by a 2x2/s2 max-pool."""
    C, H, W = in_shape
    layers = []
    for i, K in enumerate(channels, 1):
        ls = LayerSpec(f"conv{i}", C, H, W, K)
        if i in pool_after:
            ls.pool_kind, ls.pool_k, ls.pool_stride, ls.pool_pad = 1, 2, 2, 0
        layers.append(ls)
        C, H, W = K, ls.Hp, ls.Wp
    return layers


def resnet_layers(stage_blocks, widths=(64, 128, 256, 512), in_shape=(3, 32, 32), stem="3x3"):
    """Every convolution of a basic-block ResNet is its own local layer.  The second conv
    of a basic block adds the basic block's input (identity, or 1x1 strided projection when
    the shape changes) before the ReLU."""
    C, H, W = in_shape
    layers = []
    if stem == "3x3":
        ls = LayerSpec("stem", C, H, W, widths[0])
    else:  # 7x7 stride-2 stem followed by a 3x3 stride-2 pad-1 max-pool
        ls = LayerSpec("stem", C, H, W, widths[0], R=7, S=7, stride=2, pad=3,
                       pool_kind=1, pool_k=3, pool_stride=2, pool_pad=1)
    layers.append(ls)
    C, H, W = ls.C_out, ls.Hp, ls.Wp
    for si, (nb, K) in enumerate(zip(stage_blocks, widths)):
        for bi in range(nb):
            st = 2 if (si > 0 and bi == 0) else 1
            c1 = LayerSpec(f"s{si + 1}b{bi + 1}c1", C, H, W, K, stride=st)
            layers.append(c1)
            c2 = LayerSpec(f"s{si + 1}b{bi + 1}c2", K, c1.Ho, c1.Wo, K)
            c2.skip_src = len(layers) - 1
            if st == 1 and C == K:
                c2.skip_kind = 1
                c2.skip_C, c2.skip_H, c2.skip_W, c2.skip_stride = K, c1.Ho, c1.Wo, 1
            else:
                c2.skip_kind = 2
                c2.skip_C, c2.skip_H, c2.skip_W, c2.skip_stride = C, H, W, st
            layers.append(c2)
            C, H, W = K, c2.Ho, c2.Wo
    return layers


# The benchmark configurations name an optimizer only for the first two.  The deeper stacks
# have no normalisation layers, so on N(0,1) inputs with Kaiming-normal weights their
# activations grow with depth and lr = 0.05 diverges within a few steps; they use SGD with
# momentum 0.9 at lr = 0.001, which stays finite.
_LR_NOTE = "optimizer not given for this configuration: SGD momentum 0.9, lr 0.001 (stable without normalisation)"


def _assign(layers, block_sizes, batches, aux):
    blocks, i = [], 0
    for bi, (n, B) in enumerate(zip(block_sizes, batches)):
        idx = list(range(i, i + n))
        for j in idx:
            layers[j].block = bi
            layers[j].A = aux[bi] if isinstance(aux, (list, tuple)) else aux(layers[j])
        blocks.append(Block(idx, B))
        i += n
    assert i == len(layers), (i, len(layers))
    return blocks


def _cfg1():
    layers = [LayerSpec("conv1", 3, 32, 32, 16)]
    blocks = _assign(layers, [1], [8], [8])
    return Config("cfg1_single_layer", (3, 32, 32), 10, layers, blocks, 0.01, 0.0, 0, 8)


def _cfg2():
    layers = vgg_layers([64, 128, 256, 256, 512, 512, 512, 512], {1, 2, 4, 6, 8})
    blocks = _assign(layers, [8], [128], lambda l: l.C_out // 2)
    return Config("cfg2_vgg11", (3, 32, 32), 10, layers, blocks, 0.05, 0.9, 1, 8192)


def _cfg3():
    layers = resnet_layers([2, 2, 2, 2])
    blocks = _assign(layers, [5, 4, 4, 4], [64, 128, 256, 512], [32, 16, 8, 4])
    return Config("cfg3_resnet18", (3, 32, 32), 100, layers, blocks, 0.001, 0.9, 2, 8192, notes=_LR_NOTE)


def _cfg4():
    ch = [64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512]
    layers = vgg_layers(ch, {2, 4, 7, 10, 13}, (3, 64, 64))
    blocks = _assign(layers, [2, 2, 3, 3, 3], [32, 64, 128, 256, 512], [64, 32, 16, 8, 8])
    return Config("cfg4_vgg16", (3, 64, 64), 200, layers, blocks, 0.001, 0.9, 3, 8192, notes=_LR_NOTE)


def _cfg5():
    layers = resnet_layers([3, 4, 6, 3], in_shape=(3, 128, 128), stem="7x7")
    blocks = _assign(layers, [1, 6, 8, 6, 6, 6], [32, 64, 128, 256, 512, 512], [32, 32, 16, 8, 8, 4])
    # 33 un-normalised layers on 128x128 inputs: activations reach ~4e3 at the deepest heads and
    # lr = 0.001 still ends in inf/NaN there after a few steps (measured); 1e-5 stays finite
    return Config("cfg5_resnet34", (3, 128, 128), 200, layers, blocks, 1e-5, 0.9, 4, 16384,
                  notes=_LR_NOTE.replace("lr 0.001", "lr 1e-5"), extra={"memory_budget_bytes": 16 << 30})


def _aan_rule(layers):
    """The paper's own head widths (its "Adaptive Auxiliary Networks" rule): layers before the
    first down-sampling get half the narrowest layer width, all later ones half the widest."""
    lo, hi = min(l.C_out for l in layers) // 2, max(l.C_out for l in layers) // 2
    first_down = next((i for i, l in enumerate(layers) if l.stride > 1 or l.pool_kind), len(layers))
    for i, l in enumerate(layers):
        l.A = lo if i < first_down else hi


def _cfg3_aan():
    """cfg3's network and blocks with the paper's head widths (32 for the stem and stage 1,
    256 afterwards) instead of the benchmark configuration's 32/16/8/4: wide aux GEMMs."""
    c = _cfg3()
    _aan_rule(c.layers)
    c.name = "cfg3_resnet18_aan_heads"
    return c


def _cfg3_ll256():
    """cfg3's network with the fixed 256-filter heads of classic local learning."""
    c = _cfg3()
    for l in c.layers:
        l.A = 256
    c.name = "cfg3_resnet18_ll256_heads"
    return c


_BUILDERS = {"cfg1": _cfg1, "cfg2": _cfg2, "cfg3": _cfg3, "cfg4": _cfg4, "cfg5": _cfg5,
             "cfg3_aan": _cfg3_aan, "cfg3_ll256": _cfg3_ll256}


def config_names():
    return list(_BUILDERS)


def config(name: str) -> Config:
    return _BUILDERS[name]()
