// The fp32-partial-sum instantiations of the MFMA GEMM (QKV, attention output and down projections):
// a translation unit of their own so that they compile next to the other epilogues.
#include "gemm_mfma.h"

bool launch_gemm_mfma_f32(const ssd_ctx* c, const bf16_t* x, const uint4* wp, void* out, int M, int N, int K, int mt,
                          int m_chunks, int* n_split, hipStream_t st) {
    constexpr int WK = 2, KC = WK * 32;
    const size_t stride = (size_t)c->dm.max_rows * (size_t)c->part_cols;
    // Work-group shape and split along K: functions of the weight shape alone, chosen so that the
    // grid comes close to one work-group per CU (256) with at least 16 K chunks each where the
    // shape allows.  Wide outputs (the QKV projection): n-blocks of 96 rows, two k-slices; narrow
    // outputs with a short K (the attention output projection): 64 rows, four k-slices; narrow
    // outputs with a long K (the down projection): 128 rows, eight k-slices.
    int wn, want;
    if (N > 8192) {
        wn = (N / 32) % 3 == 0 ? 3 : 4;
        want = 2;
    } else if (K <= 4096) {
        wn = 2;
        want = 4;
    } else {
        wn = 4;
        want = 8;
    }
    if (want > SSD_MAX_SPLIT) want = SSD_MAX_SPLIT;
    const int split = pick_split(K, KC, want);
    *n_split = split;
    const int nch = K / split / KC;
    GemmArgs a{nch, mt, x, wp, out, M, N, K, split, stride, -1, 0, m_chunks, st};
    return wn == 3 ? gemm_f32_wn3(a) : wn == 2 ? gemm_f32_wn2(a) : gemm_f32_wn4(a);
}
