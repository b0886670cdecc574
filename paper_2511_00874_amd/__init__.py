"""SR-quantized linear layer for MI355X: thin Python binding over the C-ABI library.

`paper_2511_00874_amd.lib` (loaded on first use) holds the binding; `synth` holds the
seeded input generators.  There is no CPU fallback: every compute call needs the
built HIP library and a GPU, and raises otherwise.
"""
__all__ = ["synth"]


def __getattr__(name):
    if name == "lib":
        import importlib
        return importlib.import_module(__name__ + ".lib")
    raise AttributeError(name)
