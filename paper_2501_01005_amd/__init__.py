"""fi355: paged (block-sparse-row) attention for AMD MI355X -- Python binding of the C-ABI library.

The compute lives in `lib/libfi355.so` (hand-written HIP for gfx950, built by `build.py`);
this package only marshals arguments.  Importing it without a built library fails loudly.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
