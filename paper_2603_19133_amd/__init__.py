"""MI355X-native implementation of PicoSpec's separate rejection sampling with sparse compression.

The work is done by hand-written gfx950 HIP kernels behind a C-ABI library (``include/picospec.h``);
``binding`` marshals torch device pointers into it, ``workloads`` draws the seeded synthetic inputs.
There is no CPU fallback: using ``compress`` / ``verify`` / ``sample_residual`` / ``sample_draft``
without the built library raises.
"""
__all__ = ["binding", "workloads"]


def __getattr__(name):
    # Loaded on first use so that the input generators can be imported without the HIP library.
    if name in ("compress", "verify", "sample_residual", "sample_draft", "binding"):
        import importlib
        _b = importlib.import_module(__name__ + ".binding")
        return _b if name == "binding" else getattr(_b, name)
    raise AttributeError(name)
