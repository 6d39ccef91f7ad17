"""MI355X-native hot path of Pyramid Attention Broadcast: broadcast schedule,
device-side broadcast cache and the spatial / temporal / cross attention
kernels behind the C-ABI library ``libpab.so``.

``paper_2408_12588_amd.workloads`` (shapes and seeded inputs) can be imported
without the library; everything else comes from ``paper_2408_12588_amd.pab``,
which loads ``libpab.so`` and raises if it has not been built.
"""
import importlib
import importlib.util


def __getattr__(name):
    # submodules (pab, workloads, build) import as themselves: build must be reachable before the library exists
    if not name.startswith("_") and importlib.util.find_spec(__name__ + "." + name) is not None:
        return importlib.import_module("." + name, __name__)
    pab = importlib.import_module(".pab", __name__)
    if hasattr(pab, name):
        return getattr(pab, name)
    raise AttributeError(name)
