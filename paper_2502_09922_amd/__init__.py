"""MI355X-native execute-while-load pipeline-stage executor (HIP kernels + C ABI).

`binding` loads libls_stage.so and exposes the entry points of include/ls_stage.h
under the same names; `build` compiles the library in-tree for gfx950.  The binding is
imported on first use, so that `python -m paper_2502_09922_amd.build` can run before the
library exists; a missing library is an ImportError, never a fallback.
"""
_LAZY = ("binding", "Stage", "Pipeline", "MicroBatch", "LsError", "ls_cfg", "ls_kv", "ls_microbatch", "make_cfg", "pack_block")


def __getattr__(name):
    if name in _LAZY:
        import importlib

        binding = importlib.import_module(".binding", __name__)
        return binding if name == "binding" else getattr(binding, name)
    raise AttributeError(name)
