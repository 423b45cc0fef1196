"""The benchmark configurations: which GEMMs, of which shapes, make up one
transformer layer's forward and backward pass.

Shapes follow the paper's per-layer GEMM inventory (Table "Representative
GEMMs ... in a single transformer layer": Q/K/V projections h x h, MLP
up-projection h x H; Sec. 5.2: four h x h matrices, one h x H and one H x h per
layer; Appendix A: Llama has three MLP matrices), with the tokens of a batch
merged into one row dimension T.

Storage convention (paper, Sec. 4.1: B_s is n x q, i.e. weights are stored
in x out):
    forward   Y  = X . W         A = X  (T x in),   B = W  (in x out)
    backward  dX = dY . W^T      A = dY (T x out),  B = W  read transposed
    backward  dW = X^T . dY      A = X  read transposed, B = dY (T x out)
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple


@dataclass(frozen=True)
class GemmSpec:
    name: str          # e.g. "q.fwd"
    kind: str          # "fwd" | "dx" | "dw"
    level: int         # DAG level: GEMMs of one level are independent (Sec. 4.1)
    M: int
    N: int
    K: int
    a: str             # name of the stored A tensor
    b: str             # name of the stored B tensor
    transA: int
    transB: int

    @property
    def flops(self):
        return 2 * self.M * self.N * self.K


@dataclass
class LayerConfig:
    name: str
    dtype: str                     # "f32" | "bf16"
    tile_m: int
    tile_n: int
    ksplit: int
    seed: int
    tensors: Dict[str, Tuple[Tuple[int, int], float]] = field(default_factory=dict)
    gemms: List[GemmSpec] = field(default_factory=list)

    @property
    def flops(self):
        return sum(g.flops for g in self.gemms)

    def levels(self):
        out = {}
        for g in self.gemms:
            out.setdefault(g.level, []).append(g)
        return [out[k] for k in sorted(out)]


def _layer(name, dtype, T, linears, tile, ksplit, seed):
    """linears: list of (name, in_features, out_features, level, input_name)."""
    cfg = LayerConfig(name, dtype, tile, tile, ksplit, seed)
    n_levels = 1 + max(l[3] for l in linears)
    for lname, fin, fout, level, xname in linears:
        cfg.tensors.setdefault(xname, ((T, fin), 1.0))        # activations ~ N(0,1)
        cfg.tensors["w_" + lname] = ((fin, fout), 0.02)       # weights ~ N(0, 0.02^2)
        cfg.tensors["dy_" + lname] = ((T, fout), 1.0)         # upstream gradients ~ N(0,1)
    for lname, fin, fout, level, xname in linears:
        cfg.gemms.append(GemmSpec(lname + ".fwd", "fwd", level, T, fout, fin,
                                  xname, "w_" + lname, 0, 0))
    for lname, fin, fout, level, xname in reversed(linears):
        blevel = 2 * n_levels - 1 - level
        cfg.gemms.append(GemmSpec(lname + ".dx", "dx", blevel, T, fin, fout,
                                  "dy_" + lname, "w_" + lname, 0, 1))
        cfg.gemms.append(GemmSpec(lname + ".dw", "dw", blevel, fin, fout, T,
                                  xname, "dy_" + lname, 1, 0))
    return cfg


def _c1():
    cfg = LayerConfig("c1_fp32_512", "f32", 128, 128, 2, 1001)
    cfg.tensors["a"] = ((512, 512), 1.0)
    cfg.tensors["b"] = ((512, 512), 1.0)
    cfg.gemms.append(GemmSpec("gemm", "fwd", 0, 512, 512, 512, "a", "b", 0, 0))
    return cfg


def _c2():
    T, h, F = 8192, 768, 3072
    return _layer("c2_gpt2_small", "bf16", T, [
        ("qkv", h, 3 * h, 0, "x_attn"),
        ("o", h, h, 1, "x_o"),
        ("fc1", h, F, 2, "x_mlp"),
        ("fc2", F, h, 3, "x_fc2"),
    ], 256, 2, 1002)


def _llama(name, T, h, F, tile, ksplit, seed):
    return _layer(name, "bf16", T, [
        ("q", h, h, 0, "x_attn"),
        ("k", h, h, 0, "x_attn"),
        ("v", h, h, 0, "x_attn"),
        ("o", h, h, 1, "x_o"),
        ("gate", h, F, 2, "x_mlp"),
        ("up", h, F, 2, "x_mlp"),
        ("down", F, h, 3, "x_down"),
    ], tile, ksplit, seed)


def _c3():
    return _llama("c3_llama7b", 4096, 4096, 11008, 512, 4, 1003)


def _c4():
    # Same tensors as c3 (same seed); the tiling is drawn per GEMM by
    # workloads.hetero with seed 1004 and the re-issue set with seed 2004.
    cfg = _llama("c4_llama7b_hetero", 4096, 4096, 11008, 0, 0, 1003)
    return cfg


def _c5():
    return _llama("c5_llama13b", 16384, 5120, 13824, 1024, 8, 1005)


_BUILDERS = {"c1": _c1, "c2": _c2, "c3": _c3, "c4": _c4, "c5": _c5}
CONFIG_NAMES = tuple(_BUILDERS)

C4_TILING_SEED = 1004
C4_REISSUE_SEED = 2004


def layer_config(name):
    return _BUILDERS[name]()
