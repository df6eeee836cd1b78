"""MI355X-native hot path of DELTA (arXiv 2203.15980): thin Python binding of libdelta.so.

Everything here is argument marshalling; planning, recomputation and swapping all run
inside the library (include/delta.h).  There is no CPU fallback: importing works without
a GPU, calling anything but `plan` needs one, and a missing library raises at load time.
"""
from .binding import (Delta, DeltaError, LayerDesc, BwdDesc, load_library, plan, layer_array,  # noqa: F401
                      OK, ERR_INVALID, ERR_INFEASIBLE, ERR_OOM_ARENA, ERR_OOM_PINNED, ERR_STATE,
                      ERR_BUFFER, ERR_HIP, F_UNCOMPUTABLE, F_EVICT_PINNED, F_OFFLOAD_PINNED,
                      FILTER_BASE, FILTER_LRU, FILTER_GREEDY, EV_EVICT, EV_OFFLOAD, EV_RECOMPUTE,
                      EV_RELOAD_PREFETCH, EV_RELOAD_DEMAND, EV_FREE, EV_DROP_TEMP, DTYPE_F32,
                      DTYPE_BF16, SYNC_D2H, SYNC_H2D, SYNC_COMPUTE, SYNC_ALL, DIR_D2H, DIR_H2D,
                      DIR_BOTH, NO_TENSOR, EXPORTS, OP_CONV, OP_MAXPOOL, OP_AVGPOOL, OP_SOFTMAX_CE, OP_ATTENTION,
                      OP_LAYERNORM, OP_BATCHNORM, OP_RELU, OP_ADD, ACT_NONE, ACT_RELU, ACT_GELU, FUSE_NONE, FUSE_BLOCK, FUSE_NO_STORE)
