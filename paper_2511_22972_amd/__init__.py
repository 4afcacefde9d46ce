"""FLy verification step on MI355X: Python binding of the C-ABI library.

The HIP library (libfly.so, built in-tree by `python -m paper_2511_22972_amd.build`)
does all the work; there is no fallback path, and importing `binding` without the
library raises.
"""
from . import build  # noqa: F401  (build helper; does not need the library)


def load():
    """Import and return the binding module (raises if libfly.so is missing)."""
    from . import binding
    return binding
