"""Batched-lowering convolution for MI355X (gfx950): forward, data and weight gradients as
lowering + one MFMA GEMM per layer, col2im, and a fused momentum-SGD step.

`paper_1606_04487_amd.binding` is the ctypes binding over the C-ABI library built from
`csrc/`; it is imported on first attribute access so that the shape/workload helpers can be
used on machines without the built library.
"""
import importlib

__all__ = ["binding", "workloads"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
