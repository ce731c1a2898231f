"""MI355X-native matrix-based bulk minibatch sampler (GraphSAGE and LADIES).

`paper_2311_02909_amd.bms` is the thin binding over the C-ABI library `libbms.so`
(hand-written HIP kernels for gfx950); `paper_2311_02909_amd.synth` makes the seeded
synthetic inputs.  The binding is imported lazily so that input generation works on
a machine without the built library.
"""
__all__ = ["bms", "synth"]


def __getattr__(name):
    if name in ("bms", "synth"):
        import importlib
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
