"""Group-sparse convolution (fine-grained kernel group sparsity) for AMD MI355X.

Thin Python binding over the C ABI of libsbn.so (include/sbn.h): the functions
here carry the same names as the C entry points and only marshal arguments.
Every step of the method runs inside the library's C++/HIP code."""
from .api import *          # noqa: F401,F403
from .api import __all__    # noqa: F401
