"""MI355X-native train<->generation weight resharding (HybridFlow 3D-HybridEngine core).

`binding` mirrors the C ABI one to one; `Plan` is a thin convenience wrapper that only
marshals arguments into those calls.  Both load libhfreshard.so on first use and raise
if it has not been built (`python -m paper_2409_19256_amd.build`); there is no fallback.
"""
import importlib

__all__ = ["binding", "Plan", "build"]


def __getattr__(name):
    if name == "binding":
        return importlib.import_module(".binding", __name__)
    if name == "Plan":
        return importlib.import_module(".plan", __name__).Plan
    raise AttributeError(name)
