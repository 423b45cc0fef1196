"""Seeded input tensors.  Values are drawn in fp32 on the CPU from a
per-tensor generator and, for bf16 configurations, rounded to bf16
(round-to-nearest-even); the oracle and the GPU then see byte-identical
stored values."""
import torch

_DTYPES = {"f32": torch.float32, "bf16": torch.bfloat16}


def make_tensor(cfg, name, integer_valued=False):
    """CPU tensor `name` of configuration `cfg` in the configuration's dtype.

    integer_valued=True draws uniform integers in [-4, 4] instead (exactly
    representable in bf16; sums of products stay exact in fp32 for the inner
    dimensions used here), for the bit-exact cross-check."""
    shape, std = cfg.tensors[name]
    index = list(cfg.tensors).index(name)
    g = torch.Generator(device="cpu")
    g.manual_seed(cfg.seed * 1000 + index)
    if integer_valued:
        t = torch.randint(-4, 5, shape, generator=g, dtype=torch.int32).to(torch.float32)
    else:
        t = torch.randn(shape, generator=g, dtype=torch.float32)
        if std != 1.0:
            t *= std
    return t.to(_DTYPES[cfg.dtype])


def make_gemm_operands(cfg, gemm, cache=None, integer_valued=False):
    """(A, B) stored tensors of one GemmSpec; `cache` (a dict) avoids redrawing
    tensors shared between GEMMs."""
    out = []
    for name in (gemm.a, gemm.b):
        if cache is not None and name in cache:
            out.append(cache[name])
            continue
        t = make_tensor(cfg, name, integer_valued)
        if cache is not None:
            cache[name] = t
        out.append(t)
    return tuple(out)


def make_matrix(seed, rows, cols, dtype="bf16", std=1.0, integer_valued=False):
    """Free-standing seeded matrix for ad-hoc test shapes."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    if integer_valued:
        t = torch.randint(-4, 5, (rows, cols), generator=g, dtype=torch.int32).to(torch.float32)
    else:
        t = torch.randn((rows, cols), generator=g, dtype=torch.float32) * std
    return t.to(_DTYPES[dtype])


def make_probe_vectors(seed, M, N, kind="normal"):
    """Seeded fp32 probe vectors r (M entries) and s (N entries) for the
    returned-block check: standard normal, or +-1 with equal probability."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    if kind == "normal":
        return (torch.randn(M, generator=g, dtype=torch.float32),
                torch.randn(N, generator=g, dtype=torch.float32))
    if kind == "sign":
        return (torch.randint(0, 2, (M,), generator=g, dtype=torch.int32).to(torch.float32) * 2 - 1,
                torch.randint(0, 2, (N,), generator=g, dtype=torch.int32).to(torch.float32) * 2 - 1)
    raise ValueError(kind)
