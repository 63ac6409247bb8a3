"""MI355X-native hot path of the semantic-parallel MoE layer (Sem-MoE, arxiv 2503.04398).

The product is libsemmoe.so (hand-written HIP kernels behind a C ABI, see include/semmoe.h);
`binding` marshals torch tensors into it.  There is no CPU fallback: a missing library is an error.
"""
from .binding import (SemMoE, SemMoEError, Config, lib_path, load_library, STATUS_NAMES)  # noqa: F401
