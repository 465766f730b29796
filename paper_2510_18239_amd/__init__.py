"""MI355X-native LIME inference hot path (arXiv 2510.18239).

Importing the package loads nothing native; the HIP library is opened by
``paper_2510_18239_amd.binding`` on first use and its absence is an error
(there is no CPU fallback).
"""

__version__ = "0.1.0"
