"""MI355X (gfx950) hot path of Parallel Restarted SGD behind a C ABI.

`prsgd` mirrors include/prsgd.h one-to-one; `drivers` holds the host loops of the paper's
three algorithms on top of those calls.  Both need the built libprsgd.so
(`python -m paper_1807_06629_amd.build`) and, for every compute call, a GPU; they are loaded
on first use so that the build module can be imported before the library exists.
"""
import importlib

_LAZY = ("prsgd", "drivers", "build")


def __getattr__(name):
    if name in _LAZY:
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
