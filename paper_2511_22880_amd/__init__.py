"""Co-batched heterogeneous-rank LoRA delta for MI355X: Python binding over the C-ABI library.

``from paper_2511_22880_amd import binding`` loads ``liblora_gfx950.so`` (built in-tree by
``paper_2511_22880_amd.build``) and exposes the functions of ``include/lora.h`` under the same
names.  There is no fallback: if the library is missing or the GPU is absent, calls fail.
``workloads`` (seeded synthetic inputs) imports nothing from the binding.
"""
__all__ = ["binding", "workloads", "build"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
