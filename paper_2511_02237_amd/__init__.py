"""MI355X-native decode-time MoE layer with Opportunistic Expert Activation (arxiv 2511.02237).

The product is the C-ABI library built from csrc/ (declared in include/oea.h); `binding` is the thin
Python marshalling layer over it and `workloads` draws the seeded synthetic inputs.
"""
from . import workloads  # noqa: F401  (numpy only)


def __getattr__(name):
    # the binding (and torch) load on first use, so CPU-only tools can import `workloads` cheaply
    if name == "binding":
        import importlib

        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
