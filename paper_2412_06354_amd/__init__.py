"""MI355X-native message-passing hot path (CSR build, propagate, GCNConv, segment softmax,
GAT layer, GIN update, graph pooling) behind a C ABI; see include/gnn.h.

``paper_2412_06354_amd.binding`` is the Python face of the library (imports torch);
``paper_2412_06354_amd.synth`` draws the seeded synthetic workloads (numpy only).
Submodules are imported on first use so that the generators work without torch.
"""
import importlib

__all__ = ["binding", "synth", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
