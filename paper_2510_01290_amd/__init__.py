"""ThinKV decode hot path for MI355X (gfx950): quantize-and-append into a paged,
thought-typed KV cache with in-place slot reuse, soft eviction, and decode attention over
the packed pages.  The compute lives in csrc/ (HIP, C ABI declared in include/thinkv.h);
`binding` marshals arguments; `synth` builds seeded synthetic workloads."""

__all__ = ["binding", "synth"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
