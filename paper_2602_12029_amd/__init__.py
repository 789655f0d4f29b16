"""Shared-prefix decode attention for MI355X: Python binding of the C-ABI library.

`binding` mirrors the C entry points name for name (argument marshalling only);
`runtime` holds the PyTorch plumbing (device buffers, streams) around them.
The HIP library must have been built (see `build.py`); nothing here falls back
to a CPU implementation.
"""
from . import binding  # noqa: F401
