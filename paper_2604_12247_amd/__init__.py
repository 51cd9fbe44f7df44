"""MI355X-native bounded self-speculative decoding (SpecBound): Python binding of
libspecbound.so.  The HIP library is the product; this package only marshals
arguments.  Importing it never falls back to a CPU path."""
from .binding import (Model, Session, Batch, Params, SbError, lib, query_sizes, packed_weight_bytes, make_config,
                      temperature_schedule, op_rmsnorm, op_gemv, op_gate_up, op_gemm, op_head, op_head_static, op_attention, op_prompt_attention, op_copy, op_read,
                      op_repack, rope_table, SYMBOLS, KERNEL_CLASSES, SB_MAX_W, SB_KV_BLOCK, FP32, BF16, EXITED,
                      WIDTH_BOUND, DEPTH_BOUND, PROJ_AUTO, PROJ_VALU, PROJ_MFMA, PROJ_MFMA_PACKED, OK, EINVAL, ENOMEM,
                      ECAPACITY, ESTATE, EDEVICE)
