"""MI355X-native hot path of one OPT-Tree decoding step (arxiv 2406.17276).

The product is the C-ABI library `libopttree.so` (include/opttree.h); this
package is its thin ctypes binding.  Importing the package loads nothing; the
library is opened on first use and its absence is an error, never a fallback.
"""
__all__ = ["api"]
