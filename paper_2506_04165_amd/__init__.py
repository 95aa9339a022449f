"""MI355X-native generalized two-stage approximate Top-K (arXiv 2506.04165).

The compute path lives in ``libatk.so`` (hand-written HIP for gfx950 behind a
C ABI, see ``include/atk.h``); ``binding`` marshals arguments to it and
``workloads`` draws the seeded synthetic inputs.  Nothing here computes on the
CPU: if the library is missing, calls raise.
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    # the binding loads the shared library; import it lazily so CPU-only tools
    # (input generators, build) work before anything is compiled
    if name in ("binding", "approx_topk", "topk", "approx_topk_stage1", "expected_recall",
                "workspace_bytes", "status_string", "AtkError"):
        import importlib
        binding = importlib.import_module(__name__ + ".binding")
        return binding if name == "binding" else getattr(binding, name)
    raise AttributeError(name)
