"""MI355X-native KGE mini-batch training step (gather, chunked negative scoring, logistic loss, backward,
duplicate reduction, sparse Adagrad) behind the C ABI of include/kge.h.  This package is the thin Python
binding; all computation happens in the HIP kernels of libkge.so."""
from .binding import *  # noqa: F401,F403
from .binding import KgeContext, KgeError, kge_config  # noqa: F401
