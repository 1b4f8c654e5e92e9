// gate/up projection with the SwiGLU epilogue, 128-row n-blocks (tile counts no multiple of three)
// (one instantiation unit of the MFMA GEMM template; see kernels_mfma.hip for the design)
#include "gemm_mfma.h"

bool gemm_swiglu_wn4(const GemmArgs& a) {
    return launch_shape<4, 2, EPI_SWIGLU, 0>(a.nch, a.mt, a.X, a.Wp, a.out, a.M, a.N, a.K, a.split, a.split_stride, a.mask_id,
                                         a.n_tiles_out, a.m_chunks, a.st);
}
