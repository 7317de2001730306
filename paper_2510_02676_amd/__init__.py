"""MI355X-native ECF8: entropy-coded FP8 E4M3 weights, decoded by hand-written HIP kernels.

``paper_2510_02676_amd.ecf8`` is the thin Python binding of the C-ABI library
(loaded on first use; importing it fails loudly when the library is not built);
``paper_2510_02676_amd.ecfw`` binds the wide-alphabet (E5M2, BF16) calls;
``paper_2510_02676_amd.synth`` makes the seeded synthetic inputs.
"""

__all__ = ["ecf8", "ecfw", "synth"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
