// Matrix-core (MFMA) kernels for bf16 models on gfx950.
//
// Skinny weight-streaming GEMM  out[M,N] = X[M,K] * W[N,K]^T  for M <= 160 rows
// per pass (the (N+1)*B rows of one verification forward, Eq. 5).  The weights
// are the HBM stream; the design is built around that:
//   * weights are repacked once, at context creation, into MFMA fragment
//     order: fragment (nt, ks) = rows [32nt, 32nt+32) x columns [16ks, 16ks+16)
//     is one contiguous 1 KiB block laid out lane by lane, so a wave's load
//     instruction reads 1 KiB of consecutive bytes and a wave streams a
//     contiguous region straight into registers (no LDS round trip);
//   * the weight fragment is the A operand of v_mfma_f32_32x32x16_bf16, the
//     activations are the B operand, so each lane ends up with 4 consecutive
//     output columns of one row: vector stores, lane-local SwiGLU and LM-head
//     reductions;
//   * activations are staged through LDS in K chunks, double buffered, shared
//     by all waves of the work-group;
//   * K can be split inside a work-group (waves reduce through LDS) and across
//     work-groups (partial sums to a workspace, summed in a fixed order by the
//     consumer).  Both splits depend on the weight shape only, never on M, and
//     a row's arithmetic never involves another row: a row is bit-identical in
//     a 1-node and an (N+1)-node forward.
#include <cstdlib>

#include "ssd_internal.h"

typedef uint16_t bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint16_t f2bf_m(float f) {
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40);
    x += 0x7fffu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}

// ------------------------------------------------------------------------
// One-time weight repack: W[N][K] row-major -> fragment order.
// dst uint4 index ((nt*KS + ks)*64 + lane) holds W[32nt + lane%32][16ks + 8(lane/32) .. +7].
// ------------------------------------------------------------------------
__global__ void k_pack_weights(const uint4* __restrict__ src, uint4* __restrict__ dst, int N, int K) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int KS = K >> 4;
    const size_t total = (size_t)(N >> 5) * KS * 64;
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    const size_t frag = idx >> 6;
    const int ks = (int)(frag % KS);
    const size_t nt = frag / KS;
    const size_t row = nt * 32 + (lane & 31);
    const int col = ks * 16 + 8 * (lane >> 5);
    dst[idx] = src[(row * K + col) >> 3];
}

void launch_pack_weights(const void* src, void* dst, int N, int K, hipStream_t st) {
    const size_t total = (size_t)(N / 32) * (K / 16) * 64;
    k_pack_weights<<<(unsigned)((total + 255) / 256), 256, 0, st>>>((const uint4*)src, (uint4*)dst, N, K);
}

// ------------------------------------------------------------------------
// GEMM.  Work-group = WN x WK waves.  Wave (wn, wk) owns R n-tiles of 32 rows
// and, of every K chunk of WK*KW columns, the KW columns [wk*KW, (wk+1)*KW).
// ------------------------------------------------------------------------
template <int WN, int WK, int R, int MT, int KW, int EPI>
__global__ __launch_bounds__(WN* WK * 64) void k_gemm_mfma(const bf16_t* __restrict__ X, const uint4* __restrict__ Wp,
                                                           void* __restrict__ outv, int M, int N, int K, int k_len,
                                                           size_t split_stride, int up_tile_off, int mask_id,
                                                           int n_tiles_out) {
    constexpr int T = WN * WK * 64, KC = WK * KW, KSTEPS = KW / 16, ROWS = MT * 32, LDW = KC + 8;
    constexpr int XSEG = ROWS * (KC / 8);               // 16-byte segments per X chunk
    constexpr int XPT = (XSEG + T - 1) / T;             // per thread
    extern __shared__ uint4 smem_u4[];
    bf16_t* xs = (bf16_t*)smem_u4;                      // [2][ROWS][LDW]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wn = wave % WN, wk = wave / WN;
    const int lm = lane & 31, lh = lane >> 5;
    const int m0 = blockIdx.y * ROWS;
    const int kbeg = blockIdx.z * k_len, nchunks = k_len / KC;
    const int KS = K >> 4, NT = N >> 5;

    // n-tiles of this wave.  SwiGLU: even waves take a gate tile, odd waves the up tile of
    // the same 32 channels (tile index + up_tile_off); R is 1 there.
    int nt[R];
    bool nt_ok[R];
    if (EPI == EPI_SWIGLU) {
        const int ch = blockIdx.x * (WN / 2) + (wn >> 1);
        nt_ok[0] = ch < up_tile_off;
        nt[0] = (nt_ok[0] ? ch : up_tile_off - 1) + ((wn & 1) ? up_tile_off : 0);
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            nt[r] = (blockIdx.x * WN + wn) * R + r;
            nt_ok[r] = nt[r] < NT;
            if (!nt_ok[r]) nt[r] = NT - 1;
        }
    }
    const uint4* wbase[R];
#pragma unroll
    for (int r = 0; r < R; ++r) wbase[r] = Wp + ((size_t)nt[r] * KS + (kbeg >> 4) + wk * KSTEPS) * 64 + lane;

    floatx16 acc[R][MT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[r][mt][i] = 0.f;

    uint4 wcur[R][KSTEPS], wnxt[R][KSTEPS], xreg[XPT];

    auto load_w = [&](uint4(&dst)[R][KSTEPS], int c) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) dst[r][ks] = wbase[r][((size_t)c * (KC / 16) + ks) * 64];
    };
    auto load_x = [&](int c) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int seg = tid + i * T;
            const int m = seg / (KC / 8), s = seg - m * (KC / 8);
            uint4 v = make_uint4(0, 0, 0, 0);
            if (seg < XSEG && m0 + m < M)
                v = *(const uint4*)(X + (size_t)(m0 + m) * K + kbeg + c * KC + s * 8);
            xreg[i] = v;
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int seg = tid + i * T;
            const int m = seg / (KC / 8), s = seg - m * (KC / 8);
            if (seg < XSEG) *(uint4*)(xs + ((size_t)buf * ROWS + m) * LDW + s * 8) = xreg[i];
        }
    };

    load_x(0);
    load_w(wcur, 0);
    store_x(0);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const bool more = c + 1 < nchunks;
        if (more) {
            load_x(c + 1);
            load_w(wnxt, c + 1);
        }
        const bf16_t* xb = xs + (size_t)(c & 1) * ROWS * LDW + wk * KW + lh * 8;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const bf16x8 xf = *(const bf16x8*)(xb + (size_t)(mt * 32 + lm) * LDW + ks * 16);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const uint4 wv = wcur[r][ks];
                    acc[r][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)&wv, xf, acc[r][mt], 0, 0, 0);
                }
            }
        }
        if (more) {
            store_x((c + 1) & 1);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) wcur[r][ks] = wnxt[r][ks];
        }
        __syncthreads();
    }

    // ---- reduce the WK k-slices of the work-group through LDS, in order wk = 1, 2, ...
    const bool lead = wk == 0;
    if (WK > 1) {
        float* red = (float*)smem_u4;                   // [(WK-1)][WN][R*MT*16][64]
        constexpr int VALS = R * MT * 16;
        if (!lead) {
            float* dst = red + ((size_t)((wk - 1) * WN + wn) * VALS) * 64 + lane;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) dst[((r * MT + mt) * 16 + i) * 64] = acc[r][mt][i];
        }
        __syncthreads();
        if (lead) {
#pragma unroll
            for (int w2 = 1; w2 < WK; ++w2) {
                const float* src = red + ((size_t)((w2 - 1) * WN + wn) * VALS) * 64 + lane;
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[r][mt][i] += src[((r * MT + mt) * 16 + i) * 64];
            }
        }
    }

    // ---- epilogues.  Lane (lm, lh) holds, per tile, rows n = 8*(i/4) + 4*lh + i%4 of column m = lm.
    if (EPI == EPI_F32) {
        float* out = (float*)outv + (size_t)blockIdx.z * split_stride;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (!lead || !nt_ok[r]) continue;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = m0 + mt * 32 + lm;
                if (m >= M) continue;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = nt[r] * 32 + g * 8 + lh * 4;
                    *(float4*)(out + (size_t)m * N + n) =
                        make_float4(acc[r][mt][g * 4], acc[r][mt][g * 4 + 1], acc[r][mt][g * 4 + 2], acc[r][mt][g * 4 + 3]);
                }
            }
        }
    } else if (EPI == EPI_SWIGLU) {
        // the up wave hands its tile to the gate wave of the same channels through LDS
        float* xch = (float*)smem_u4;                   // [WN/2][MT*16][64]
        if (WK > 1) __syncthreads();                    // the k-slice reduction has finished reading
        if (lead && (wn & 1)) {
            float* dst = xch + ((size_t)(wn >> 1) * MT * 16) * 64 + lane;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) dst[(mt * 16 + i) * 64] = acc[0][mt][i];
        }
        __syncthreads();
        bf16_t* out = (bf16_t*)outv;
        if (lead && !(wn & 1) && nt_ok[0]) {
            const float* src = xch + ((size_t)(wn >> 1) * MT * 16) * 64 + lane;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = m0 + mt * 32 + lm;
                if (m >= M) continue;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int f = nt[0] * 32 + g * 8 + lh * 4;
                    uint16_t o[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float gv = acc[0][mt][g * 4 + j], uv = src[(mt * 16 + g * 4 + j) * 64];
                        o[j] = f2bf_m(gv / (1.0f + expf(-gv)) * uv);
                    }
                    *(uint2*)(out + (size_t)m * (up_tile_off * 32) + f) =
                        make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
                }
            }
        }
    } else if (lead) {
        // LM head: per (row, wave) partial over the wave's R*32 vocabulary rows
        float* out = (float*)outv;
        const int tile_out = blockIdx.x * WN + wn;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float bm = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (!nt_ok[r]) continue;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int n = nt[r] * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
                    const float v = acc[r][mt][i];
                    if (n != mask_id && v > bm) { bm = v; bi = n; }
                }
            }
            {
                const float om = __shfl_xor(bm, 32, 64);
                const int oi = __shfl_xor(bi, 32, 64);
                if (om > bm || (om == bm && oi < bi)) { bm = om; bi = oi; }
            }
            float se = 0.f;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (!nt_ok[r]) continue;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int n = nt[r] * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
                    if (n != mask_id) se += expf(acc[r][mt][i] - bm);
                }
            }
            se += __shfl_xor(se, 32, 64);
            const int m = m0 + mt * 32 + lm;
            if (lh == 0 && m < M && tile_out < n_tiles_out && nt_ok[0]) {
                float* o = out + ((size_t)m * n_tiles_out + tile_out) * 3;
                o[0] = bm;
                o[1] = __int_as_float(bi);
                o[2] = se;
            }
        }
    }
}

// ------------------------------------------------------------------------
// launcher
// ------------------------------------------------------------------------
struct GemmPlan {
    int split;     // work-groups along K (global split, partial sums)
};

static int env_int(const char* name, int dflt) {
    const char* s = getenv(name);
    return s ? atoi(s) : dflt;
}

template <int WN, int WK, int R, int MT, int KW, int EPI>
static bool launch_one(const bf16_t* X, const uint4* Wp, void* out, int M, int N, int K, int split, size_t split_stride,
                       int up_tile_off, int mask_id, int n_tiles_out, int m_chunks, hipStream_t st) {
    constexpr int KC = WK * KW, ROWS = MT * 32, LDW = KC + 8;
    constexpr size_t xbytes = (size_t)2 * ROWS * LDW * 2;
    constexpr size_t rbytes = WK > 1 ? (size_t)(WK - 1) * WN * R * MT * 16 * 64 * 4 : 0;
    constexpr size_t smem = xbytes > rbytes ? xbytes : rbytes;
    static_assert(smem <= 160 * 1024, "LDS budget");
    auto kern = k_gemm_mfma<WN, WK, R, MT, KW, EPI>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return false;
        attr_done = true;
    }
    const int tiles = EPI == EPI_SWIGLU ? up_tile_off : N / 32;
    const int per_wg = EPI == EPI_SWIGLU ? WN / 2 : WN * R;
    dim3 grid((tiles + per_wg - 1) / per_wg, m_chunks, split);
    hipLaunchKernelGGL(kern, grid, dim3(WN * WK * 64), smem, st, X, Wp, out, M, N, K, K / split, split_stride,
                       up_tile_off, mask_id, n_tiles_out);
    return true;
}

template <int WN, int WK, int R, int KW, int EPI>
static bool launch_mt(int mt, const bf16_t* X, const uint4* Wp, void* out, int M, int N, int K, int split,
                      size_t split_stride, int up_tile_off, int mask_id, int n_tiles_out, int m_chunks,
                      hipStream_t st) {
#define SSD_MT_CASE(v)                                                                                          \
    case v:                                                                                                     \
        return launch_one<WN, WK, R, v, KW, EPI>(X, Wp, out, M, N, K, split, split_stride, up_tile_off, mask_id, \
                                                 n_tiles_out, m_chunks, st);
    switch (mt) {
        SSD_MT_CASE(1)
        SSD_MT_CASE(2)
        SSD_MT_CASE(3)
        SSD_MT_CASE(4)
        SSD_MT_CASE(5)
    }
#undef SSD_MT_CASE
    return false;
}

int lm_tiles_mfma(int V) { return V / 32; }

// Split along K across work-groups: a function of the weight shape only.
static int pick_split(int N, int K, int kc, int want) {
    int s = want;
    while (s > 1 && (K % (s * kc)) != 0) --s;
    (void)N;
    return s < 1 ? 1 : s;
}

bool launch_gemm_mfma(const ssd_ctx* c, int epi, const void* X, const Wt& W, void* out, int M, int* n_split,
                      hipStream_t st) {
    if (!W.packed) return false;
    const int N = W.N, K = W.K;
    constexpr int KW = 64, WN = 4, WK = 2, KC = WK * KW;
    if (K % KC) return false;
    // rows per pass: up to 160; more rows re-stream the weights per 160-row chunk
    const int mt = M >= 160 ? 5 : (M + 31) / 32;
    const int rows = mt * 32, m_chunks = (M + rows - 1) / rows;
    const bf16_t* x = (const bf16_t*)X;
    const uint4* wp = (const uint4*)W.packed;
    const size_t stride = (size_t)c->dm.max_rows * (size_t)c->part_cols;
    if (epi == EPI_SWIGLU) {
        // W = [2F, d]: gate rows then up rows; N is passed as F to the kernel's store
        const int F = N / 2;
        if (F % 32) return false;
        *n_split = 1;
        return launch_mt<WN, WK, 1, KW, EPI_SWIGLU>(mt, x, wp, out, M, F, K, 1, 0, F / 32, -1, 0, m_chunks, st);
    }
    if (epi == EPI_LMHEAD) {
        *n_split = lm_tiles_mfma(N);
        return launch_mt<WN, WK, 1, KW, EPI_LMHEAD>(mt, x, wp, out, M, N, K, 1, 0, 0, c->dm.mask_id, N / 32, m_chunks, st);
    }
    int want = 1;
    if (N <= 8192) want = env_int("SSD_SPLIT_SMALLN", 8);
    else want = env_int("SSD_SPLIT_LARGEN", 2);
    if (want > SSD_MAX_SPLIT) want = SSD_MAX_SPLIT;
    const int split = pick_split(N, K, KC, want);
    *n_split = split;
    return launch_mt<WN, WK, 1, KW, EPI_F32>(mt, x, wp, out, M, N, K, split, stride, 0, -1, 0, m_chunks, st);
}

// ------------------------------------------------------------------------
// a4: shared-prefix bidirectional attention on the matrix cores.
// One wave per (node, query head, 32-row query tile).  Keys are walked in
// tiles of 32, first the sequence's cached prefix [0,S), then the node's own
// rows; online softmax in fp32.
//   S^T[key][q] = K Q^T     : A = K fragment (rows = keys), B = Q fragment
//   O^T[d][q]  += V^T P^T   : A = V^T fragment (rows = d),  B = P^T fragment
// With q on the MFMA column axis every softmax statistic (running max, sum,
// rescale factor) is per lane, and the P^T values a lane computed are exactly
// its B-operand values for the second product, so nothing crosses lanes except
// one xor-32 exchange per tile.  The k index of the second product is the key;
// lane half lh supplies keys {8g + 4lh + 0..3 : g = 2st, 2st+1} of step st, which
// are two runs of 4 consecutive positions in the position-contiguous value
// layout (two 8-byte loads).
// The tile order depends on S and the block length only, so a row's result does
// not depend on how many nodes the forward holds.
// ------------------------------------------------------------------------
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

template <int DH>
__global__ __launch_bounds__(512) void k_attn_mfma(const FwdHeader* __restrict__ fw, const bf16_t* __restrict__ q,
                                                   const bf16_t* __restrict__ kown, const bf16_t* __restrict__ vt,
                                                   const bf16_t* __restrict__ kcache, const bf16_t* __restrict__ vcache,
                                                   bf16_t* __restrict__ out, int Hq, int Hkv, int layer, int max_seqs,
                                                   int seq_stride, int vt_rows, float scale) {
    constexpr int KST = DH / 16, DT = DH / 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int lm = lane & 31, lh = lane >> 5;
    const NodeDesc nd = fw->nodes[blockIdx.x];
    const int head = blockIdx.y, kvh = head / (Hq / Hkv);
    const int qt = blockIdx.z * waves + wave;
    if (qt * 32 >= nd.blen) return;
    const int nq = Hq * DH, nkv = Hkv * DH;
    const int qrow_in = qt * 32 + lm;
    const bool qvalid = qrow_in < nd.blen;
    const int qrow = nd.row0 + (qvalid ? qrow_in : 0);

    bf16x8 qf[KST];
#pragma unroll
    for (int ks = 0; ks < KST; ++ks) qf[ks] = *(const bf16x8*)(q + (size_t)qrow * nq + head * DH + ks * 16 + lh * 8);

    const size_t cbase = ((((size_t)layer * max_seqs + nd.seq) * Hkv) + kvh) * (size_t)seq_stride * DH;
    const bf16_t* kc = kcache + cbase;                      // [pos][DH]
    const bf16_t* vc = vcache + cbase;                      // [DH][seq_stride]
    const bf16_t* ko = kown + (size_t)nd.row0 * nkv + kvh * DH;   // [row][nkv]
    const bf16_t* vo = vt + (size_t)kvh * DH * vt_rows + nd.vrow0;   // [DH][vt_rows]

    floatx16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
    float m_run = -INFINITY, l_part = 0.f;

    const int pre_tiles = (nd.S + 31) >> 5, own_tiles = (nd.blen + 31) >> 5;
    for (int t = 0; t < pre_tiles + own_tiles; ++t) {
        const bool own = t >= pre_tiles;
        const int t0 = (own ? t - pre_tiles : t) * 32;     // first key of the tile, in its own index space
        const int n_valid = (own ? nd.blen : nd.S) - t0;   // keys of this tile that exist (may exceed 32)
        // ---- S^T = K Q^T
        const int krow = t0 + lm < (own ? nd.blen : nd.S) ? t0 + lm : 0;
        const bf16_t* kp = own ? ko + (size_t)krow * nkv : kc + (size_t)krow * DH;
        floatx16 sacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KST; ++ks) {
            const bf16x8 kf = *(const bf16x8*)(kp + ks * 16 + lh * 8);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc, 0, 0, 0);
        }
        // ---- values of this tile, position-contiguous: two 4-position runs per step
        const bf16_t* vp = own ? vo : vc;
        const size_t vstride = own ? (size_t)vt_rows : (size_t)seq_stride;
        bf16x8 vf[DT][2];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const bf16_t* a = vp + (size_t)(dt * 32 + lm) * vstride + t0 + 16 * st + 4 * lh;
                const bf16x4 lo = *(const bf16x4*)a, hi = *(const bf16x4*)(a + 8);
                vf[dt][st] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        // ---- online softmax over this lane's 16 keys (key = t0 + 8*(i/4) + 4*lh + i%4)
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = (i >> 2) * 8 + lh * 4 + (i & 3);
            sacc[i] = key < n_valid ? sacc[i] * scale : -INFINITY;
            mx = fmaxf(mx, sacc[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float corr = expf(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        bf16x8 pf[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = expf(sacc[i] - m_new);          // 0 for masked keys
            psum += p;
            pf[i >> 3][i & 7] = (__bf16)p;
        }
        l_part = l_part * corr + psum;
        if (n_valid < 32) {
            // keys past the end hold stale memory: zero them so 0 * garbage cannot produce NaN
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int st = 0; st < 2; ++st)
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int key = (2 * st + (j >> 2)) * 8 + lh * 4 + (j & 3);
                        if (key >= n_valid) vf[dt][st][j] = (__bf16)0.f;
                    }
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[dt][i] *= corr;
#pragma unroll
            for (int st = 0; st < 2; ++st)
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][st], pf[st], oacc[dt], 0, 0, 0);
        }
    }
    const float l = l_part + __shfl_xor(l_part, 32, 64);
    const float inv = 1.0f / l;
    if (qvalid) {
        bf16_t* op = out + (size_t)qrow * nq + head * DH;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint16_t o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = f2bf_m(oacc[dt][g * 4 + j] * inv);
                *(uint2*)(op + dt * 32 + g * 8 + lh * 4) =
                    make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
            }
    }
}

bool launch_attn_mfma(const ssd_ctx* c, int n_nodes, int max_blen, int layer, hipStream_t st) {
    const Dims& d = c->dm;
    const int qtiles = (max_blen + 31) / 32;
    const int waves = qtiles < 8 ? qtiles : 8;
    dim3 grid(n_nodes, d.Hq, (qtiles + waves - 1) / waves);
    const float scale = 1.0f / sqrtf((float)d.dh);
#define SSD_ATTN_ARGS                                                                                                  \
    c->b.fwd, (const bf16_t*)c->b.q, (const bf16_t*)c->b.k, (const bf16_t*)c->b.vt, (const bf16_t*)c->b.kcache,      \
        (const bf16_t*)c->b.vcache, (bf16_t*)c->b.attn, d.Hq, d.Hkv, layer, d.max_seqs, d.seq_stride(), d.vt_rows(), scale
    if (d.dh == 128)
        k_attn_mfma<128><<<grid, waves * 64, 0, st>>>(SSD_ATTN_ARGS);
    else if (d.dh == 64)
        k_attn_mfma<64><<<grid, waves * 64, 0, st>>>(SSD_ATTN_ARGS);
    else
        return false;
#undef SSD_ATTN_ARGS
    return true;
}
