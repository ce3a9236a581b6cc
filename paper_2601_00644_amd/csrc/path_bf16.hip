// placeholder until the bf16 kernels land
#include "fsv_internal.h"
int fsv_bf16_create(fsv_ctx *c, const fsv_weights *) { FSV_FAIL(c, FSV_E_UNSUPPORTED, "bf16 path not built yet"); }
int fsv_bf16_forward(fsv_ctx *c, const fsv_batch *, int, float *, hipStream_t) { FSV_FAIL(c, FSV_E_UNSUPPORTED, "bf16"); }
int fsv_bf16_linear(fsv_ctx *c, int, int, const void *, int, float *, hipStream_t) { FSV_FAIL(c, FSV_E_UNSUPPORTED, "bf16"); }
int fsv_bf16_attention(fsv_ctx *c, int, const void *, const fsv_batch *, int, float *, hipStream_t) { FSV_FAIL(c, FSV_E_UNSUPPORTED, "bf16"); }
int fsv_bf16_kv_copy(fsv_ctx *c, void *, void *, int, const int32_t *, int, int, void *, void *, bool, hipStream_t) { FSV_FAIL(c, FSV_E_UNSUPPORTED, "bf16"); }
