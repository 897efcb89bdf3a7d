"""MI355X (gfx950) hot path of Parallel Restarted SGD behind a C ABI.

`prsgd` mirrors include/prsgd.h one-to-one; `drivers` holds the host loops of the paper's
three algorithms on top of those calls.  The package needs the built libprsgd.so
(`python -m paper_1807_06629_amd.build`) and a GPU for every compute call.
"""
from . import prsgd  # noqa: F401
from . import drivers  # noqa: F401
