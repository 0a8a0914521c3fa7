"""MI355X-native block-floating-point encode and matrix product (HBFP, arXiv 1804.01526).

``paper_1804_01526_amd.hbfp`` is the binding of the C ABI declared in ``include/hbfp.h``.
"""
from . import hbfp  # noqa: F401  (fails loudly when libhbfp.so has not been built)
