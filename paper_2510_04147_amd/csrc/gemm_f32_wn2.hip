// fp32 partial sums, 64-row n-blocks (the attention output projection): 16 chunks per k-slice at 4096
// (one instantiation unit of the MFMA GEMM template; see kernels_mfma.hip for the design)
#include "gemm_mfma.h"

bool gemm_f32_wn2(const GemmArgs& a) {
    return launch_shape<2, 2, EPI_F32, 16>(a.nch, a.mt, a.X, a.Wp, a.out, a.M, a.N, a.K, a.split, a.split_stride, a.mask_id,
                                         a.n_tiles_out, a.m_chunks, a.st);
}
