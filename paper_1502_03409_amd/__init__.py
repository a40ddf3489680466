"""MI355X-native kernels for the locally connected (untied-weight) autoencoder layers of
"Large-Scale Deep Learning on the YFCC100M Dataset" (arXiv 1502.03409).

The product is ``liblc.so`` (hand-written HIP for gfx950 behind the C ABI in ``include/lc.h``);
this package is its thin Python binding.  PyTorch only provides device memory and streams.
"""
from .binding import *  # noqa: F401,F403
from .binding import lib, LcError, LcGeom, geom, geom_derive, workspace_bytes, plan_query, l2pool_lcn_plan_query  # noqa: F401
