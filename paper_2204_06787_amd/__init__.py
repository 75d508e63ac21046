"""MI355X-native hot path of Marsit (arXiv 2204.06787): one-bit synchronisation for multi-hop
all-reduce.  See ``marsit`` for the binding over the C-ABI HIP library."""

__version__ = "0.1.0"
