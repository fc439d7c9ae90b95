"""MI355X-native hybrid decode path over asymmetric virtual-memory pools.

`binding` is the thin ctypes layer over the C-ABI library built from `csrc/`
(imported on demand); `session` drives steps through it; the seeded synthetic
workloads come from the separate top-level package `gen`.
"""

import os as _os
import sys as _sys

# the seeded input generators live beside this package, in gen/
_root = _os.path.dirname(_os.path.dirname(_os.path.abspath(__file__)))
if _root not in _sys.path:
    _sys.path.insert(0, _root)
