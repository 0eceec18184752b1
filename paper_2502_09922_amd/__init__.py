"""MI355X-native execute-while-load pipeline-stage executor (HIP kernels + C ABI).

`binding` loads libls_stage.so and exposes the entry points of include/ls_stage.h
under the same names; `build` compiles the library in-tree for gfx950.
"""
from . import binding  # noqa: F401  (raises ImportError if the library is not built)
from .binding import Stage, LsError, ls_cfg, ls_kv, make_cfg, pack_block  # noqa: F401
