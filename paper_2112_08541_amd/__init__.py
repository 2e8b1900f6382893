"""MI355X-native minibatch preparation for GNN training: k-hop neighbor
sampling and a GPU-resident FIFO feature cache (the data path of the BGL paper,
arXiv 2112.08541), as hand-written HIP kernels behind a C-ABI library.

``paper_2112_08541_amd.binding`` is the thin ctypes layer over that library;
``paper_2112_08541_amd.inputs`` generates seeded synthetic workloads.
Submodules are imported on first use so that the input generators can be used
without the HIP library being loaded.
"""
import importlib

__all__ = ["binding", "inputs", "buildlib", "pipeline"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
