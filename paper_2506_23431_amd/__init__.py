"""Pipelined decoder (arXiv 2506.23431, Section 3) for AMD MI355X.

The product is the C-ABI library `libpd.so` built from `csrc/` (declared in
`include/pd.h`); this package is its thin Python binding.  Importing the
package does not load the library; `binding.load()` does and raises if it has
not been built (there is no CPU fallback).
"""

from .binding import PipelinedDecoder, load, PdError  # noqa: F401
