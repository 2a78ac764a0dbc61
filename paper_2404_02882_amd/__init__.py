"""MI355X-native hot path of LASP (arxiv 2404.02882): chunked causal linear
attention with decay and a carried KV state, forward and backward.

`paper_2404_02882_amd.lasp` is the thin ctypes binding over the C-ABI library
(hand-written HIP kernels for gfx950); `synth_inputs` draws the seeded
synthetic workloads. The binding is imported on first use so that the input
generator can be used on machines where the library has not been built.
"""

__all__ = ["lasp", "synth_inputs"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
