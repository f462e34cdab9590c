"""fle: fused linear + epilogue for AMD MI355X (gfx950).

``fused_linear_epilogue(x, w, b, epilogue)`` runs entirely in the hand-written
HIP kernels of ``libfle.so`` (C ABI declared in ``include/fle.h``); this package
is argument marshalling only.  Nothing here falls back to a CPU or PyTorch
implementation: if the library is missing, calls raise.
"""
import importlib

__all__ = ["fused_linear_epilogue", "grouped_fused_linear_epilogue", "attention", "attention_block", "mlp_chain", "transformer_layer"]


def __getattr__(name):
    if name in __all__:
        return getattr(importlib.import_module(__name__ + ".binding"), name)
    raise AttributeError(name)
