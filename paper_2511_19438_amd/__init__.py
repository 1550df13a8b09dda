"""MI355X-native W4A16 GPTQ matrix multiply (hand-written HIP for gfx950 behind a C ABI).

``paper_2511_19438_amd.binding`` wraps the C-ABI library (same function names, argument
marshalling only); ``paper_2511_19438_amd.workloads`` draws the seeded synthetic inputs.
Nothing here falls back to a CPU path: if the HIP library is missing the binding raises.
"""

__all__ = ["binding", "workloads", "build"]


def __getattr__(name):
    if name in __all__:
        import importlib

        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
