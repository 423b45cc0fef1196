"""Seeded synthetic workloads shared by the oracle-side tests and the GPU-side
tests / benchmark.  This package holds NONE of the method's arithmetic: it only
says which GEMMs a transformer layer consists of, draws the input tensors, and
draws the random choices of the test harness (heterogeneous tile edges, the
set of re-issued tasks).  Both the oracle and the HIP library receive these
values as plain inputs.
"""
from .configs import GemmSpec, LayerConfig, layer_config, CONFIG_NAMES  # noqa: F401
from .tensors import make_tensor, make_gemm_operands, make_probe_vectors  # noqa: F401
from .hetero import draw_explicit_tiling, draw_reissue, draw_fleet  # noqa: F401
