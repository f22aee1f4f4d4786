"""MI355X-native rollout decode step (paged GQA decode attention + sampling).

``paper_2510_11345_amd.binding`` is the thin ctypes layer over the C ABI in
``include/roll_decode.h``; it is loaded on first use so that importing the
package (for ``workloads``) does not need the built library.
"""

__all__ = ["binding", "workloads"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
