// Matrix-core (MFMA) kernels for bf16 models on gfx950.
#include "ssd_internal.h"

bool launch_gemm_mfma(const ssd_ctx*, int, const void*, const void*, void*, int, int, int, int*, hipStream_t) {
    return false;
}
bool launch_attn_mfma(const ssd_ctx*, int, int, hipStream_t) { return false; }
