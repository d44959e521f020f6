"""fi355: paged (block-sparse-row) attention for AMD MI355X -- Python binding of the C-ABI library.

The compute lives in `lib/libfi355.so` (hand-written HIP for gfx950, built by `build.py`);
this package only marshals arguments.  The binding is loaded on first use and fails loudly
when the library is not built: there is no fallback path.
"""


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    import importlib
    binding = importlib.import_module(__name__ + ".binding")
    return getattr(binding, name)
