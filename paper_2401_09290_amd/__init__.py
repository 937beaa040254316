"""MI355X-native fenced-kernel library after Guardian (arXiv 2401.09290).

``paper_2401_09290_amd.binding`` is a thin ctypes layer over ``libguardian.so``
(C ABI in ``include/guardian.h``): argument marshalling only, every step of the
path runs in the library's own HIP kernels.  There is no CPU fallback: loading
fails loudly when the library has not been built.
"""
from .binding import *  # noqa: F401,F403
