"""MI355X tensor-cache migration library: thin Python binding over libtc.so.

The binding marshals arguments only; every step of the hot path (decisions,
copies, pack/unpack) runs in the HIP kernels of the C-ABI library declared in
include/tc.h.
"""

from .binding import (  # noqa: F401
    TensorCache, TcError, lib, load_library, LIB_PATH,
    TENSOR_DESC, EVENT, POOL_CLASS, PLACEMENT, OP, STATS_FIELDS,
    copy_batch, exchange_batch, pack, unpack, pack_index, pack_tiles, pack_static, PACK_STATIC_MAX_BYTES,
    GPU, CPU, NVME, PRE, POST, END, END_CPU,
    OP_NAMES, LITERAL_ALG2, NO_PREFETCH, SMALLEST_FIRST, ALLOC_WRITE_ONLY, BIND_NULL_MOVER, BIND_FILE_DIRECT, BIND_HOST_TIER,
)
