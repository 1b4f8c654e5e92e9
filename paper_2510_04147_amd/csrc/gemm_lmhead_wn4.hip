// LM head with the per-tile (max, arg-max, sum-exp) reduction, 128-row n-blocks: 64 chunks at d_model 4096
// (one instantiation unit of the MFMA GEMM template; see kernels_mfma.hip for the design)
#include "gemm_mfma.h"

bool gemm_lmhead_wn4(const GemmArgs& a) {
    return launch_shape<4, 2, EPI_LMHEAD, 64>(a.nch, a.mt, a.X, a.Wp, a.out, a.M, a.N, a.K, a.split, a.split_stride, a.mask_id,
                                         a.n_tiles_out, a.m_chunks, a.st);
}
