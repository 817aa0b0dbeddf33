"""hgnn: half-precision sparse aggregation kernels (SpMM, discretized SpMM, SDDMM,
edge softmax) for AMD MI355X, after HalfGNN (HPDC'25).  The kernels live in
csrc/ (HIP, gfx950) behind the C ABI of include/hgnn.h; this package is the thin
ctypes binding."""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, HgnnError, Csr, Plan, load  # noqa: F401
