// Plain (FMA, no matrix cores) kernels for every step of the forward, for fp32
// and bf16 storage.  They are the complete path for fp32 models and the
// fallback / cross-check for bf16.  Every reduction runs in a fixed order that
// depends only on the reduced extent, never on how many rows a launch holds,
// so a row's result is bit-identical whether it is computed in a 1-node or an
// (N+1)-node forward: that is what makes the batched verification (Eq. 5)
// reproduce stepwise decoding exactly.
#include "ssd_internal.h"

typedef uint16_t bf16_t;

__device__ __forceinline__ float ld_f(const float* p) { return *p; }
__device__ __forceinline__ float ld_f(const bf16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40);   // NaN stays NaN
    x += 0x7fffu + ((x >> 16) & 1u);                                            // round to nearest even
    return (uint16_t)(x >> 16);
}
__device__ __forceinline__ void st_f(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_f(bf16_t* p, float v) { *p = f2bf(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// ------------------------------------------------------------------------
// a0: tree build.  One work-group per node: node j of a decode group is the
// block state with drafts 1..j written in (Section 3.2.3).
// ------------------------------------------------------------------------
__global__ void k_build_rows(const FwdHeader* __restrict__ fw, SeqState* __restrict__ state,
                             const int* __restrict__ raw_tok, int* __restrict__ row_tok,
                             int* __restrict__ row_pos, int* __restrict__ row_node,
                             int* __restrict__ out_tok, int mask_id, int max_seq_len,
                             const float* __restrict__ ref_conf, const int* __restrict__ ref_arg) {
    const int ni = blockIdx.x;
    if (ni >= fw->n_nodes) return;
    const NodeDesc nd = fw->nodes[ni];
    const GroupDesc g = fw->groups[nd.group];
    SeqState* s = &state[nd.seq];
    // A block nobody has predicted yet, with drafts read off the last refresh (Section 3.2.2 with the cache of
    // Section 4.1): node j holds the j positions the refresh was most confident of.  One wave per node, one lane
    // per position.
    int ref_rank = 0x7fffffff, ref_tok = mask_id;
    if (g.mode == GM_DECODE && g.from_refresh) {             // uniform over the wave
        const int lane = threadIdx.x;
        const size_t base = (size_t)nd.seq * max_seq_len + nd.S;
        const float c = lane < nd.blen ? ref_conf[base + lane] : -1.f;
        int rank = 0;
        for (int qd = 0; qd < 64; ++qd) {
            const float cq = __shfl(c, qd, 64);
            if (qd < nd.blen && (cq > c || (cq == c && qd < lane))) ++rank;
        }
        ref_rank = rank;
        if (lane < nd.blen) ref_tok = ref_arg[base + lane];
    }
    for (int p = threadIdx.x; p < nd.blen; p += blockDim.x) {
        int tok;
        if (g.mode == GM_RAW) {
            tok = raw_tok[g.raw_off + p];
        } else if (g.mode == GM_APPEND) {
            tok = s->tok[p];
            if (g.out_off >= 0) out_tok[(size_t)nd.seq * max_seq_len + g.out_off + p] = tok;
        } else if (g.from_refresh) {
            tok = ref_rank < nd.j ? ref_tok : mask_id;       // a decode block has at most 64 positions: p is this lane
        } else if (g.fresh) {
            tok = mask_id;
        } else {
            tok = s->tok[p];
            for (int j = 0; j < nd.j; ++j)
                if (s->draft_pos[j] == p) tok = s->draft_tok[j];
            // a mix-order node skips draft j and holds draft j + 1 instead (Section 5.2)
            if (nd.extra >= 0 && s->draft_pos[nd.extra] == p) tok = s->draft_tok[nd.extra];
        }
        const int row = nd.row0 + p;
        row_tok[row] = tok;
        row_pos[row] = nd.S + p;
        row_node[row] = ni;
    }
}

// a1: embedding gather into the fp32 residual stream.
template <typename T>
__global__ void k_embed(const T* __restrict__ embed, const int* __restrict__ row_tok, float* __restrict__ h, int d,
                        int V) {
    const int row = blockIdx.x;
    // ids are validated on the host or produced by the arg-max; the clamp keeps the gather in
    // bounds whatever a corrupted state holds
    const int tok = min(max(row_tok[row], 0), V - 1);
    const T* e = embed + (size_t)tok * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)row * d + i] = ld_f(e + i);
}

// a2/a6/a9: h += sum of split-K partial sums (fixed order s = 0, 1, ...), then RMSNorm.
// One work-group of NORM_T threads per row; every thread owns up to NORM_J float4 groups of the
// row and issues all partial-sum loads of a group before the first add, so a 4096-wide row has
// its whole input (the row and every partial sum) in flight at once.
#define NORM_T 1024
#define NORM_J 2   // 1024 threads x 2 float4 = rows up to 8192 wide
__device__ __forceinline__ void st4(float* p, float a, float b, float c, float d) { *(float4*)p = make_float4(a, b, c, d); }
__device__ __forceinline__ void st4(bf16_t* p, float a, float b, float c, float d) {
    *(uint2*)p = make_uint2((uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16), (uint32_t)f2bf(c) | ((uint32_t)f2bf(d) << 16));
}

template <typename T, int NP>
__device__ __forceinline__ void norm_row(float* hr, const float* pr, size_t part_stride, const float* gain, T* xr,
                                         int d, float eps) {
    const int n4 = d >> 2;
    float4 v[NORM_J];
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < NORM_J; ++j) {
        const int i4 = threadIdx.x + j * NORM_T;
        if (i4 < n4) {
            v[j] = ((const float4*)hr)[i4];
            float4 pv[NP > 0 ? NP : 1];
#pragma unroll
            for (int s = 0; s < NP; ++s) pv[s] = ((const float4*)(pr + s * part_stride))[i4];
#pragma unroll
            for (int s = 0; s < NP; ++s) {
                v[j].x += pv[s].x; v[j].y += pv[s].y; v[j].z += pv[s].z; v[j].w += pv[s].w;
            }
            if (NP > 0) ((float4*)hr)[i4] = v[j];
            ss += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
        }
    }
    __shared__ float red[NORM_T / 64];
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < NORM_T / 64; ++w) tot += red[w];
    const float r = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int j = 0; j < NORM_J; ++j) {
        const int i4 = threadIdx.x + j * NORM_T;
        if (i4 < n4) {
            const float4 g = ((const float4*)gain)[i4];
            st4(xr + 4 * i4, v[j].x * r * g.x, v[j].y * r * g.y, v[j].z * r * g.z, v[j].w * r * g.w);
        }
    }
}

template <typename T>
__global__ __launch_bounds__(NORM_T) void k_norm(float* __restrict__ h, const float* __restrict__ part, int n_part,
                                              size_t part_stride, const float* __restrict__ gain,
                                              T* __restrict__ xn, int d, float eps) {
    const int row = blockIdx.x;
    float* hr = h + (size_t)row * d;
    const float* pr = part + (size_t)row * d;
    T* xr = xn + (size_t)row * d;
    switch (n_part) {
        case 0: norm_row<T, 0>(hr, pr, part_stride, gain, xr, d, eps); break;
        case 1: norm_row<T, 1>(hr, pr, part_stride, gain, xr, d, eps); break;
        case 2: norm_row<T, 2>(hr, pr, part_stride, gain, xr, d, eps); break;
        case 4: norm_row<T, 4>(hr, pr, part_stride, gain, xr, d, eps); break;
        case 8: norm_row<T, 8>(hr, pr, part_stride, gain, xr, d, eps); break;
        default: {
            // any other split count: fold the partial sums into h first, in order
            for (int i = threadIdx.x; i < d; i += NORM_T) {
                float v = hr[i];
                for (int s = 0; s < n_part; ++s) v += pr[s * part_stride + i];
                hr[i] = v;
            }
            __syncthreads();
            norm_row<T, 0>(hr, pr, part_stride, gain, xr, d, eps);
        }
    }
}

// Rotary embedding (rotate-half pairing) of Q and K from the fp32 projection (the sum of its
// split-K partial sums, in split order), conversion to the operand type, the fragment-order copies
// of the nodes' own keys and values, and the cache write for nodes that own finished tokens.
// One work-group per (node, 32-row tile, head of Q, K or V): 32 rows x 8 column groups.
template <typename T, int DH>
__global__ __launch_bounds__(256) void k_rope(const FwdHeader* __restrict__ fw, const float* __restrict__ part,
                                              int n_part, size_t part_stride, const float* __restrict__ cosT,
                                              const float* __restrict__ sinT, T* __restrict__ q,
                                              T* __restrict__ kown, T* __restrict__ vown, int vt_rows,
                                              T* __restrict__ kcache, T* __restrict__ vcache, int Hq, int Hkv,
                                              int layer, int max_seqs, int seq_stride) {
    constexpr int HALF = DH / 2, PT = HALF / 8;          // q/k: values of each rotary half per thread
    constexpr int VPT = DH / 8;                          // v: values per thread
    const NodeDesc nd = fw->nodes[blockIdx.x];
    const int r0 = blockIdx.y * 32;
    if (r0 >= nd.blen) return;
    const int hh = blockIdx.z, tid = threadIdx.x, r = tid >> 3, cg = tid & 7;
    const bool rvalid = r0 + r < nd.blen;
    const int row = nd.row0 + (rvalid ? r0 + r : 0);
    const int pos = nd.S + (rvalid ? r0 + r : 0);
    const int nq = Hq * DH, nkv = Hkv * DH, nqkv = nq + 2 * nkv;
    const float* src = part + (size_t)row * nqkv;
    const size_t cbase = (((size_t)layer * max_seqs + nd.seq) * Hkv) * (size_t)seq_stride * DH;
    auto load = [&](int col, float* dst, int n) {       // n values (multiple of 4) from column col
#pragma unroll
        for (int j = 0; j < n; j += 4) {
            float4 a = *(const float4*)(src + col + j);
            for (int sp = 1; sp < n_part; ++sp) {
                const float4 b = *(const float4*)(src + sp * part_stride + col + j);
                a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
            }
            dst[j] = a.x; dst[j + 1] = a.y; dst[j + 2] = a.z; dst[j + 3] = a.w;
        }
    };
    if (hh < Hq + Hkv) {
        const int i0 = cg * PT;
        float x1[PT], x2[PT], o1[PT], o2[PT];
        load(hh * DH + i0, x1, PT);
        load(hh * DH + i0 + HALF, x2, PT);
#pragma unroll
        for (int j = 0; j < PT; ++j) {
            const float c = cosT[(size_t)pos * HALF + i0 + j], sn = sinT[(size_t)pos * HALF + i0 + j];
            rope_pair(x1[j], x2[j], c, sn, o1[j], o2[j]);
        }
        if (rvalid) {
            if (hh < Hq) {
                T* dst = q + (size_t)row * nq + hh * DH;
#pragma unroll
                for (int j = 0; j < PT; j += 4) {
                    st4(dst + i0 + j, o1[j], o1[j + 1], o1[j + 2], o1[j + 3]);
                    st4(dst + i0 + HALF + j, o2[j], o2[j + 1], o2[j + 2], o2[j + 3]);
                }
            } else {
                // four consecutive channels starting at a multiple of four stay contiguous in fragment order
                const int kvh = hh - Hq;
                T* ko = kown + (size_t)kvh * vt_rows * DH;
                T* kc = kcache + cbase + (size_t)kvh * seq_stride * DH;
                const int prow = nd.vrow0 + r0 + r;
#pragma unroll
                for (int j = 0; j < PT; j += 4) {
                    st4(ko + kfrag_off(prow, i0 + j, DH), o1[j], o1[j + 1], o1[j + 2], o1[j + 3]);
                    st4(ko + kfrag_off(prow, i0 + HALF + j, DH), o2[j], o2[j + 1], o2[j + 2], o2[j + 3]);
                }
                if (nd.write_kv) {
#pragma unroll
                    for (int j = 0; j < PT; j += 4) {
                        st4(kc + kfrag_off(pos, i0 + j, DH), o1[j], o1[j + 1], o1[j + 2], o1[j + 3]);
                        st4(kc + kfrag_off(pos, i0 + HALF + j, DH), o2[j], o2[j + 1], o2[j + 2], o2[j + 3]);
                    }
                }
            }
        }
    } else {
        const int vh = hh - Hq - Hkv, c0 = cg * VPT;
        __shared__ float tile[32][DH + 1];
        float x[VPT];
        load(nq + nkv + vh * DH + c0, x, VPT);
#pragma unroll
        for (int j = 0; j < VPT; ++j) tile[r][c0 + j] = rvalid ? x[j] : 0.f;
        __syncthreads();
        // thread -> (channel, group of rows): four consecutive positions starting at a multiple of four
        // stay contiguous in fragment order; a node's rows start 64-aligned, rows past its end get zeros
        constexpr int TPC = 256 / DH, RPT = 32 / TPC;    // threads per channel, rows per thread
        const int col = tid / TPC, rg = (tid % TPC) * RPT;
        T* vd = vown + (size_t)vh * vt_rows * DH;
#pragma unroll
        for (int j = 0; j < RPT; j += 4)
            st4(vd + vfrag_off(nd.vrow0 + r0 + rg + j, col, DH), tile[rg + j][col], tile[rg + j + 1][col],
                tile[rg + j + 2][col], tile[rg + j + 3][col]);
        if (nd.write_kv) {
            T* vc = vcache + cbase + (size_t)vh * seq_stride * DH;
            for (int j = 0; j < RPT; ++j)
                if (r0 + rg + j < nd.blen) st_f(vc + vfrag_off(nd.S + r0 + rg + j, col, DH), tile[rg + j][col]);
        }
    }
}

// a4 (plain): one wave per (row, query head).  Keys = the sequence's cached
// prefix [0,S), its cached suffix behind the block if it has one, then the node's own rows; online softmax in fp32 over
// key tiles of 64 in position order.
template <typename T>
__global__ __launch_bounds__(64) void k_attn_plain(const FwdHeader* __restrict__ fw, const int* __restrict__ row_node,
                                                   const T* __restrict__ q, const T* __restrict__ kown,
                                                   const T* __restrict__ vown, const T* __restrict__ kcache,
                                                   const T* __restrict__ vcache, T* __restrict__ out, int Hq,
                                                   int Hkv, int dh, int layer, int max_seqs, int seq_stride,
                                                   int vt_rows) {
    const int row = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
    const NodeDesc nd = fw->nodes[row_node[row]];
    const int kvh = head / (Hq / Hkv);
    const int nq = Hq * dh;
    __shared__ float qs[128];
    for (int i = lane; i < dh; i += 64) qs[i] = ld_f(q + (size_t)row * nq + head * dh + i);
    __syncthreads();
    const size_t cbase = ((((size_t)layer * max_seqs + nd.seq) * Hkv) + kvh) * (size_t)seq_stride * dh;
    const T* kc = kcache + cbase;
    const T* vc = vcache + cbase;
    const T* ko = kown + (size_t)kvh * vt_rows * dh;
    const T* vo = vown + (size_t)kvh * vt_rows * dh;
    // keys: the cached prefix [0, S), the cached suffix [S + blen, T) if the sequence has one, the node's own rows
    const int n_suf = max(nd.T - (nd.S + nd.blen), 0), n_cache = nd.S + n_suf;
    const int n_keys = n_cache + nd.blen;
    auto cache_pos = [&](int j) { return j < nd.S ? j : j + nd.blen; };
    const float scale = 1.0f / sqrtf((float)dh);
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int t0 = 0; t0 < n_keys; t0 += 64) {
        const int j = t0 + lane;
        float s = -INFINITY;
        if (j < n_keys) {
            const bool pre = j < n_cache;
            const T* kp = pre ? kc : ko;
            const int p = pre ? cache_pos(j) : nd.vrow0 + j - n_cache;
            float acc = 0.f;
            for (int i = 0; i < dh; ++i) acc += qs[i] * ld_f(kp + kfrag_off(p, i, dh));
            s = acc * scale;
        }
        const float m_new = fmaxf(m, wave_max(s));
        const float p = j < n_keys ? expf(s - m_new) : 0.f;
        const float corr = expf(m - m_new);
        l = l * corr + wave_sum(p);
        o0 *= corr;
        o1 *= corr;
        const int cnt = min(64, n_keys - t0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj, 64);
            const int jk = t0 + jj;
            const bool pre = jk < n_cache;
            const T* vp = pre ? vc : vo;
            const int pp = pre ? cache_pos(jk) : nd.vrow0 + jk - n_cache;
            o0 += pj * ld_f(vp + vfrag_off(pp, lane, dh));
            if (dh > 64) o1 += pj * ld_f(vp + vfrag_off(pp, lane + 64, dh));
        }
        m = m_new;
    }
    T* op = out + (size_t)row * nq + head * dh;
    st_f(op + lane, o0 / l);
    if (dh > 64) st_f(op + lane + 64, o1 / l);
}

// ------------------------------------------------------------------------
// Plain tiled GEMM  out[M,N] = X[M,K] * W[N,K]^T, fp32 accumulation in
// ascending k.  64x64 tile per work-group, 4x4 outputs per thread.
// ------------------------------------------------------------------------
#define PBM 64
#define PBN 64
#define PBK 16

template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_gemm_plain(const T* __restrict__ X, const T* __restrict__ W,
                                                    void* __restrict__ outv, int M, int N, int K, int up_off,
                                                    int mask_id, int n_tiles) {
    __shared__ float Xs[PBK][PBM + 4];
    __shared__ float Ws[PBK][PBN + 4];
    __shared__ float Us[EPI == EPI_SWIGLU ? PBK : 1][PBN + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * PBM, n0 = blockIdx.x * PBN;
    const int lr = tid >> 2, lk = (tid & 3) * 4;
    float acc[4][4] = {}, accu[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += PBK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kk = k0 + lk + i;
            const bool kin = kk < K;
            Xs[lk + i][lr] = (kin && m0 + lr < M) ? ld_f(X + (size_t)(m0 + lr) * K + kk) : 0.f;
            Ws[lk + i][lr] = (kin && n0 + lr < N) ? ld_f(W + (size_t)(n0 + lr) * K + kk) : 0.f;
            if (EPI == EPI_SWIGLU)
                Us[lk + i][lr] = (kin && n0 + lr < N) ? ld_f(W + (size_t)(up_off + n0 + lr) * K + kk) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < PBK; ++kk) {
            float a[4], b[4], u[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = Xs[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Ws[kk][tx * 4 + j];
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int j = 0; j < 4; ++j) u[j] = Us[kk][tx * 4 + j];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] += a[i] * b[j];
                    if (EPI == EPI_SWIGLU) accu[i][j] += a[i] * u[j];
                }
        }
        __syncthreads();
    }
    if (EPI == EPI_F32) {
        float* out = (float*)outv;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
                if (m < M && n < N) out[(size_t)m * N + n] = acc[i][j];
            }
    } else if (EPI == EPI_SWIGLU) {
        T* out = (T*)outv;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
                if (m < M && n < N) {
                    const float g = acc[i][j];
                    st_f(out + (size_t)m * N + n, g / (1.0f + expf(-g)) * accu[i][j]);
                }
            }
    } else {
        // fused LM-head reduction: per row, over this tile's 64 vocabulary
        // columns: max logit, its lowest index, sum of exp(logit - max).  The
        // mask token takes no part.  The 16 threads of a row are 16 adjacent lanes.
        float* out = (float*)outv;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float bm = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + tx * 4 + j;
                if (n < N && n != mask_id && acc[i][j] > bm) { bm = acc[i][j]; bi = n; }
            }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                const float om = __shfl_xor(bm, off, 64);
                const int oi = __shfl_xor(bi, off, 64);
                if (om > bm || (om == bm && oi < bi)) { bm = om; bi = oi; }
            }
            float se = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + tx * 4 + j;
                if (n < N && n != mask_id) se += expf(acc[i][j] - bm);
            }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) se += __shfl_xor(se, off, 64);
            const int m = m0 + ty * 4 + i;
            if (tx == 0 && m < M) {
                float* o = out + ((size_t)m * n_tiles + blockIdx.x) * 3;
                o[0] = bm;
                o[1] = __int_as_float(bi);
                o[2] = se;
            }
        }
    }
}

// Merge the per-tile (max, arg, sumexp) triples of a row in a fixed order:
// each thread folds tiles tid, tid+256, ... in ascending order, then the 64
// lanes of a wave are folded by a butterfly and the four waves in order.
// Ties keep the lowest token id.
__device__ __forceinline__ void lm_fold(float& m, int& a, float& s, float om, int oa, float os) {
    if (os == 0.f) return;                 // empty partner
    if (s == 0.f) { m = om; a = oa; s = os; return; }
    const float nm = fmaxf(m, om);
    s = s * expf(m - nm) + os * expf(om - nm);
    if (om > m || (om == m && oa < a)) a = oa;
    m = nm;
}

__global__ __launch_bounds__(256) void k_lm_merge(const float* __restrict__ part, int n_tiles,
                                                  float* __restrict__ row_max, int* __restrict__ row_arg,
                                                  float* __restrict__ row_conf, int V, int mask_id) {
    // One work-group per row.  The fold order (tile t goes to thread t mod 256, then a butterfly
    // inside each wave, then waves 0..3 in order) depends on the tile count alone.
    __shared__ float sm[4], ss[4];
    __shared__ int sa[4];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float m = -INFINITY, s = 0.f;
    int a = 0x7fffffff;
    for (int t = tid; t < n_tiles; t += 256) {
        const float* p = part + ((size_t)row * n_tiles + t) * 3;
        lm_fold(m, a, s, p[0], __float_as_int(p[1]), p[2]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float om = __shfl_xor(m, off, 64), os = __shfl_xor(s, off, 64);
        const int oa = __shfl_xor(a, off, 64);
        // fold (lower lane, higher lane) in the same order on both sides
        if (lane & off) {
            float tm = om, ts = os;
            int ta = oa;
            lm_fold(tm, ta, ts, m, a, s);
            m = tm; a = ta; s = ts;
        } else {
            lm_fold(m, a, s, om, oa, os);
        }
    }
    if (lane == 0) { sm[wave] = m; sa[wave] = a; ss[wave] = s; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) lm_fold(m, a, s, sm[w], sa[w], ss[w]);
        // Non-finite logits (NaN weights) leave no arg-max: fall back to the lowest valid id and
        // confidence 0 so that every later step stays well defined and in bounds.
        if ((unsigned)a >= (unsigned)V) a = mask_id == 0 ? 1 : 0;
        float conf = 1.0f / s;             // softmax probability of the arg-max (Section 3.2.2)
        if (!(conf >= 0.f && conf <= 1.f)) conf = 0.f;
        row_max[row] = m;
        row_arg[row] = a;
        row_conf[row] = conf;
    }
}

// ------------------------------------------------------------------------
// a11: acceptance (Section 3.2.4).  One wave per decode group, one lane per
// block position.  Walks the chain: node m's stepwise choice (most confident
// masked position, ties to the lowest position) must equal draft m+1 in
// position and token; stops at the first mismatch; accepts the matched drafts
// plus the choice of the node it stopped at; ranks that node's remaining
// masked positions by confidence for the next drafts; commits to the state.
// With mix-order nodes in the group (Section 5.2) a mismatch whose choice is
// draft m+2 accepts that draft and ends at the node holding drafts 1..m, m+2.
// ------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_accept(const FwdHeader* __restrict__ fw, SeqState* __restrict__ state,
                                               const float* __restrict__ row_conf, const int* __restrict__ row_arg,
                                               const float* __restrict__ row_max, StepResult* __restrict__ result,
                                               int* __restrict__ out_tok, int max_seq_len, int blockB, int maxDraft,
                                               int mask_id, float* __restrict__ ref_conf, int* __restrict__ ref_arg) {
    const int gi = blockIdx.x, lane = threadIdx.x;
    const GroupDesc g = fw->groups[gi];
    const ssd_step_out out = fw->out;
    if (g.mode == GM_RAW && g.keep_ref) {
        // rows of a cache refresh behind the current block: their predictions are the drafts later blocks
        // start from (Section 3.2.2: candidates from the next block; Section 4.1: the refresh covers all positions)
        for (int p = lane; p < g.blen; p += 64) {
            ref_conf[(size_t)g.seq * max_seq_len + g.S + p] = row_conf[g.row0 + p];
            ref_arg[(size_t)g.seq * max_seq_len + g.S + p] = row_arg[g.row0 + p];
        }
        return;
    }
    if (g.mode != GM_DECODE || g.spec_of1 != 0) return;   // a speculative group is its master's business
    SeqState* s = &state[g.seq];
    // drafts = chain nodes - 1, or one per chain node if the node holding all of them was left out
    const int nd = g.leafless ? g.n_chain : g.n_chain - 1;
    const int blen = g.blen;
    __shared__ int sh_pos[64], sh_tok[64];
    // drafts read off the last refresh: the block's positions by descending confidence; lane k gets draft k
    auto drafts_from_refresh = [&](int S_blk, int blen_blk, int& dpos, int& dtok) {
        const size_t base = (size_t)g.seq * max_seq_len + S_blk;
        const float cr = lane < blen_blk ? ref_conf[base + lane] : -1.f;
        int rank = 0;
        for (int qd = 0; qd < 64; ++qd) {
            const float cq = __shfl(cr, qd, 64);
            if (qd < blen_blk && (cq > cr || (cq == cr && qd < lane))) ++rank;
        }
        __syncthreads();
        if (lane < blen_blk) { sh_pos[rank] = lane; sh_tok[rank] = ref_arg[base + lane]; }
        __syncthreads();
        dpos = lane < blen_blk ? sh_pos[lane] : -1;
        dtok = lane < blen_blk ? sh_tok[lane] : -1;
    };
    int my_dpos = lane <= SSD_MAX_DRAFT ? s->draft_pos[lane] : -1;
    int my_dtok = lane <= SSD_MAX_DRAFT ? s->draft_tok[lane] : -1;
    if (g.from_refresh) drafts_from_refresh(g.S, blen, my_dpos, my_dtok);
    // a fresh block starts all masked with no drafts (Algorithm 1, start of a block); its state is written here,
    // at the end of the forward, so that a KV-append group of the same sequence in the same forward
    // still reads the finished block's tokens
    unsigned long long cur = g.fresh ? (blen >= 64 ? ~0ull : ((1ull << blen) - 1ull)) : s->masked;
    __syncthreads();

    if (lane < blen) {
        for (int j = 0; j < g.n_chain && j <= maxDraft; ++j) {
            const int row = g.row0 + j * blen + lane;
            const size_t o = ((size_t)gi * (maxDraft + 1) + j) * blockB + lane;
            if (out.row_maxlogit) out.row_maxlogit[o] = row_max[row];
            if (out.row_argmax) out.row_argmax[o] = row_arg[row];
            if (out.row_conf) out.row_conf[o] = row_conf[row];
        }
    }

    // stepwise choice of a node (rows row0 + lane of a block of bl positions) over the positions still masked in
    // `cur`: highest confidence, ties to the lowest position; leaves this lane's confidence in c
    int pstar = 0, tstar = 0;
    float c = -1.f;
    auto choose_at = [&](int row0, int bl) {
        const bool valid = lane < bl && ((cur >> lane) & 1ull);
        c = valid ? row_conf[row0 + lane] : -1.f;
        float bc = c;
        int bp = lane;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float oc = __shfl_xor(bc, off, 64);
            const int op = __shfl_xor(bp, off, 64);
            if (oc > bc || (oc == bc && op < bp)) { bc = oc; bp = op; }
        }
        pstar = bp;
        tstar = row_arg[row0 + pstar];
    };
    auto choose = [&](int node) { choose_at(g.row0 + node * blen, blen); };
    int m = 0;
    bool complete = false;
    while (true) {
        if (cur == 0ull) { complete = true; break; }     // the drafts covered every masked position
        choose(m);
        const int dp = __shfl(my_dpos, m, 64), dt = __shfl(my_dtok, m, 64);
        if (m < nd && pstar == dp && tstar == dt) {
            cur &= ~(1ull << pstar);
            ++m;
            continue;
        }
        break;
    }
    StepResult* r = &result[g.seq];
    if (complete) {
        // Every draft verified and the block is finished (Section 3.2.2, the round across the block
        // boundary).  Its tokens go to the output (exact cache: its KV was written by the leaf in this
        // forward).  The group behind it, if any, holds the next block: all masked, then with the drafts
        // the last refresh gives it written in.  The walk goes on there: its matched drafts and the
        // choice of the node it stops at are further accepted tokens (positions counted on from this
        // block's length), and that node's other positions give the next drafts.
        if (g.fresh) s->tok[lane] = mask_id;
        __syncthreads();
        if (lane < m) {
            r->acc_pos[lane] = my_dpos;
            r->acc_tok[lane] = my_dtok;
            s->tok[my_dpos] = my_dtok;
            if (out.acc_pos) out.acc_pos[(size_t)gi * (maxDraft + 1) + lane] = my_dpos;
            if (out.acc_tok) out.acc_tok[(size_t)gi * (maxDraft + 1) + lane] = my_dtok;
        }
        __syncthreads();
        if (g.out_off >= 0 && lane < blen) out_tok[(size_t)g.seq * max_seq_len + g.out_off + lane] = s->tok[lane];
        __syncthreads();
        int n_acc = m, n_next = 0, n_in_next = 0;
        unsigned long long rem = 0ull;
        if (g.spec_next1 != 0) {
            const GroupDesc g2 = fw->groups[g.spec_next1 - 1];
            const int blen2 = g2.blen, nd2 = g2.n_chain - 1;
            int dpos2 = -1, dtok2 = -1;
            if (g2.from_refresh) drafts_from_refresh(g2.S, blen2, dpos2, dtok2);
            cur = blen2 >= 64 ? ~0ull : ((1ull << blen2) - 1ull);
            int k = 0;
            while (true) {
                choose_at(g2.row0 + k * blen2, blen2);
                const int dp = __shfl(dpos2, k, 64), dt = __shfl(dtok2, k, 64);
                if (k < nd2 && pstar == dp && tstar == dt) {
                    cur &= ~(1ull << pstar);
                    ++k;
                    continue;
                }
                break;
            }
            rem = cur & ~(1ull << pstar);
            const int n_rem = __popcll(rem);
            n_next = min(g2.n_draft_next, g2.allow_full ? n_rem : max(n_rem - 1, 0));
            const bool mine = (rem >> lane) & 1ull;
            int rank = 0;
            for (int qd = 0; qd < 64; ++qd) {
                const float cq = __shfl(c, qd, 64);
                if (((rem >> qd) & 1ull) && (cq > c || (cq == c && qd < lane))) ++rank;
            }
            const int my_tok = row_arg[g2.row0 + k * blen2 + (lane < blen2 ? lane : 0)];
            if (mine && rank < n_next) {
                r->next_pos[rank] = lane;
                r->next_tok[rank] = my_tok;
                s->draft_pos[rank] = lane;
                s->draft_tok[rank] = my_tok;
                if (out.next_pos) out.next_pos[(size_t)gi * maxDraft + rank] = lane;
                if (out.next_tok) out.next_tok[(size_t)gi * maxDraft + rank] = my_tok;
            }
            s->tok[lane] = mask_id;
            __syncthreads();
            if (lane <= k) {
                // the next block's matched drafts, then the choice of the node the walk stopped at
                const int ap = lane < k ? dpos2 : pstar, at = lane < k ? dtok2 : tstar;
                s->tok[ap] = at;
                r->acc_pos[m + lane] = blen + ap;
                r->acc_tok[m + lane] = at;
                if (out.acc_pos) out.acc_pos[(size_t)gi * (maxDraft + 1) + m + lane] = blen + ap;
                if (out.acc_tok) out.acc_tok[(size_t)gi * (maxDraft + 1) + m + lane] = at;
            }
            n_in_next = k + 1;
            n_acc = m + n_in_next;
        }
        if (lane == 0) {
            r->n_accept = n_acc;
            r->n_next = n_next;
            r->completed = 1;
            r->n_in_next = n_in_next;
            s->masked = rem;
            s->n_draft = n_next;
            if (out.n_accept) out.n_accept[gi] = n_acc;
            if (out.n_next) out.n_next[gi] = n_next;
        }
        return;
    }
    // mix order (Section 5.2): the choice is the draft after the expected one -> accept it and take
    // one more token from the node that holds drafts 1..m and m+2; that node has no children
    int last = m, res_pos = -1, res_tok = -1;
    if (g.n_nodes > g.n_chain && m + 1 < nd) {
        const int dp2 = __shfl(my_dpos, m + 1, 64), dt2 = __shfl(my_dtok, m + 1, 64);
        if (pstar == dp2 && tstar == dt2) {
            res_pos = pstar;
            res_tok = tstar;
            cur &= ~(1ull << pstar);
            last = g.n_chain + m;
            choose(last);
        }
    }
    const int n_acc = m + 1 + (res_pos >= 0 ? 1 : 0);
    const unsigned long long rem = cur & ~(1ull << pstar);
    const int n_rem = __popcll(rem);
    // the leaf keeps one masked position to predict, unless a next block exists for it to reach into
    const int n_next = min(g.n_draft_next, g.allow_full ? n_rem : max(n_rem - 1, 0));
    const bool mine = (rem >> lane) & 1ull;
    int rank = 0;
    for (int qd = 0; qd < 64; ++qd) {
        const float cq = __shfl(c, qd, 64);
        if (((rem >> qd) & 1ull) && (cq > c || (cq == c && qd < lane))) ++rank;
    }
    const int my_tok = row_arg[g.row0 + last * blen + (lane < blen ? lane : 0)];
    if (mine && rank < n_next) {
        r->next_pos[rank] = lane;
        r->next_tok[rank] = my_tok;
        s->draft_pos[rank] = lane;
        s->draft_tok[rank] = my_tok;
        if (out.next_pos) out.next_pos[(size_t)gi * maxDraft + rank] = lane;
        if (out.next_tok) out.next_tok[(size_t)gi * maxDraft + rank] = my_tok;
    }
    if (g.fresh) s->tok[lane] = mask_id;                  // SSD_MAX_BLOCK = 64 = one lane per position
    __syncthreads();
    if (lane < n_acc) {
        // the matched drafts, then (mix order) the out-of-order draft, then the last node's own choice
        const int ap = lane < m ? my_dpos : (lane == n_acc - 1 ? pstar : res_pos);
        const int at = lane < m ? my_dtok : (lane == n_acc - 1 ? tstar : res_tok);
        r->acc_pos[lane] = ap;
        r->acc_tok[lane] = at;
        s->tok[ap] = at;
        if (out.acc_pos) out.acc_pos[(size_t)gi * (maxDraft + 1) + lane] = ap;
        if (out.acc_tok) out.acc_tok[(size_t)gi * (maxDraft + 1) + lane] = at;
    }
    if (lane == 0) {
        r->n_accept = n_acc;
        r->n_next = n_next;
        r->completed = 0;
        r->n_in_next = 0;
        s->masked = rem;
        s->n_draft = n_next;
        if (out.n_accept) out.n_accept[gi] = n_acc;
        if (out.n_next) out.n_next[gi] = n_next;
    }
}

// ------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------
void launch_build_rows(const ssd_ctx* c, hipStream_t st, int n_nodes) {
    k_build_rows<<<n_nodes, 64, 0, st>>>(c->b.fwd, c->b.state, c->b.raw_tok, c->b.row_tok, c->b.row_pos,
                                         c->b.row_node, c->b.out_tok, c->dm.mask_id, c->dm.max_seq_len, c->b.ref_conf,
                                         c->b.ref_arg);
}

void launch_embed(const ssd_ctx* c, int M, hipStream_t st) {
    if (c->dm.dtype == SSD_F32)
        k_embed<float><<<M, 256, 0, st>>>((const float*)c->embed, c->b.row_tok, c->b.h, c->dm.d, c->dm.V);
    else
        k_embed<bf16_t><<<M, 256, 0, st>>>((const bf16_t*)c->embed, c->b.row_tok, c->b.h, c->dm.d, c->dm.V);
}

void launch_norm(const ssd_ctx* c, int M, const float* gain, int n_part, hipStream_t st) {
    const size_t stride = (size_t)c->dm.max_rows * c->part_cols;
    if (c->dm.dtype == SSD_F32)
        k_norm<float><<<M, NORM_T, 0, st>>>(c->b.h, c->b.part, n_part, stride, gain, (float*)c->b.xn, c->dm.d, c->dm.eps);
    else
        k_norm<bf16_t><<<M, NORM_T, 0, st>>>(c->b.h, c->b.part, n_part, stride, gain, (bf16_t*)c->b.xn, c->dm.d,
                                          c->dm.eps);
}

void launch_rope(const ssd_ctx* c, int n_nodes, int max_blen, int layer, int n_part, hipStream_t st) {
    const Dims& d = c->dm;
    const size_t ps = (size_t)d.max_rows * c->part_cols;
    dim3 grid(n_nodes, (max_blen + 31) / 32, d.Hq + 2 * d.Hkv);
#define SSD_ROPE_ARGS(T)                                                                                           \
    c->b.fwd, c->b.part, n_part, ps, c->b.rope_cos, c->b.rope_sin, (T*)c->b.q, (T*)c->b.kown, (T*)c->b.vown,        \
        d.vt_rows(), (T*)c->b.kcache, (T*)c->b.vcache, d.Hq, d.Hkv, layer, d.max_seqs, d.seq_stride()
    if (d.dtype == SSD_F32) {
        if (d.dh == 128) k_rope<float, 128><<<grid, 256, 0, st>>>(SSD_ROPE_ARGS(float));
        else k_rope<float, 64><<<grid, 256, 0, st>>>(SSD_ROPE_ARGS(float));
    } else {
        if (d.dh == 128) k_rope<bf16_t, 128><<<grid, 256, 0, st>>>(SSD_ROPE_ARGS(bf16_t));
        else k_rope<bf16_t, 64><<<grid, 256, 0, st>>>(SSD_ROPE_ARGS(bf16_t));
    }
#undef SSD_ROPE_ARGS
}

void launch_attn_plain(const ssd_ctx* c, int M, int layer, hipStream_t st) {
    const Dims& d = c->dm;
    dim3 grid(M, d.Hq);
    if (d.dtype == SSD_F32)
        k_attn_plain<float><<<grid, 64, 0, st>>>(c->b.fwd, c->b.row_node, (const float*)c->b.q,
                                                 (const float*)c->b.kown, (const float*)c->b.vown,
                                                 (const float*)c->b.kcache, (const float*)c->b.vcache,
                                                 (float*)c->b.attn, d.Hq, d.Hkv, d.dh, layer, d.max_seqs,
                                                 d.seq_stride(), d.vt_rows());
    else
        k_attn_plain<bf16_t><<<grid, 64, 0, st>>>(c->b.fwd, c->b.row_node, (const bf16_t*)c->b.q,
                                                  (const bf16_t*)c->b.kown, (const bf16_t*)c->b.vown,
                                                  (const bf16_t*)c->b.kcache, (const bf16_t*)c->b.vcache,
                                                  (bf16_t*)c->b.attn, d.Hq, d.Hkv, d.dh, layer, d.max_seqs,
                                                  d.seq_stride(), d.vt_rows());
}

template <typename T>
static void gemm_plain_t(const ssd_ctx* c, int epi, const T* X, const T* W, void* out, int M, int N, int K,
                         hipStream_t st) {
    dim3 grid((N + PBN - 1) / PBN, (M + PBM - 1) / PBM);
    if (epi == EPI_F32)
        k_gemm_plain<T, EPI_F32><<<grid, 256, 0, st>>>(X, W, out, M, N, K, 0, -1, 0);
    else if (epi == EPI_SWIGLU)
        k_gemm_plain<T, EPI_SWIGLU><<<grid, 256, 0, st>>>(X, W, out, M, N, K, N, -1, 0);
    else
        k_gemm_plain<T, EPI_LMHEAD><<<grid, 256, 0, st>>>(X, W, out, M, N, K, 0, c->dm.mask_id, (int)grid.x);
}

void launch_gemm_plain(const ssd_ctx* c, int epi, const void* X, const void* W, void* out, int M, int N, int K,
                       hipStream_t st) {
    if (c->dm.dtype == SSD_F32)
        gemm_plain_t<float>(c, epi, (const float*)X, (const float*)W, out, M, N, K, st);
    else
        gemm_plain_t<bf16_t>(c, epi, (const bf16_t*)X, (const bf16_t*)W, out, M, N, K, st);
}

int lm_tiles_plain(int V) { return (V + PBN - 1) / PBN; }

void launch_lm_merge(const ssd_ctx* c, int M, int n_tiles, hipStream_t st) {
    launch_lm_merge_to(c, M, n_tiles, c->b.lm_part, c->b.row_max, c->b.row_arg, c->b.row_conf, st);
}

void launch_lm_merge_to(const ssd_ctx* c, int M, int n_tiles, const float* part, float* row_max, int* row_arg,
                        float* row_conf, hipStream_t st) {
    k_lm_merge<<<M, 256, 0, st>>>(part, n_tiles, row_max, row_arg, row_conf, c->dm.V, c->dm.mask_id);
}

void launch_accept(const ssd_ctx* c, int n_groups, hipStream_t st) {
    k_accept<<<n_groups, 64, 0, st>>>(c->b.fwd, c->b.state, c->b.row_conf, c->b.row_arg, c->b.row_max, c->b.result,
                                      c->b.out_tok, c->dm.max_seq_len, c->dm.block, c->dm.max_draft, c->dm.mask_id,
                                      c->b.ref_conf, c->b.ref_arg);
}

// Helpers of the kernel-level entry points.
__global__ void k_sum_partials(const float* __restrict__ part, int n_part, size_t part_stride, float* __restrict__ out,
                               size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float v = part[i];
    for (int s = 1; s < n_part; ++s) v += part[s * part_stride + i];
    out[i] = v;
}

__global__ __launch_bounds__(256) void k_token_rank(const float* __restrict__ logits, int V, int mask_id, RankPairs pairs,
                                                    int* __restrict__ rank) {
    const int i = blockIdx.x;
    const float* row = logits + (size_t)pairs.pos[i] * V;
    const int t = pairs.tok[i];
    const float lt = row[t];
    int ahead = 0;
    for (int v = threadIdx.x; v < V; v += 256)
        ahead += v != mask_id && (row[v] > lt || (row[v] == lt && v < t));
    __shared__ int part[4];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ahead += __shfl_xor(ahead, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ahead;
    __syncthreads();
    if (threadIdx.x == 0) rank[i] = part[0] + part[1] + part[2] + part[3];
}

void launch_token_rank(const float* logits, int V, int mask_id, const RankPairs& pairs, int* rank, hipStream_t st) {
    if (pairs.n > 0) k_token_rank<<<pairs.n, 256, 0, st>>>(logits, V, mask_id, pairs, rank);
}

__global__ void k_int_to_float(const int* __restrict__ src, float* __restrict__ dst, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = (float)src[i];
}

void launch_sum_partials(const ssd_ctx* c, int M, int N, int n_part, float* out, hipStream_t st) {
    const size_t n = (size_t)M * N;
    k_sum_partials<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(c->b.part, n_part,
                                                                (size_t)c->dm.max_rows * c->part_cols, out, n);
}

// Kernel-level entry points: caller-supplied keys and values (row-major [n, Hkv, dh], keys after the
// rotary embedding) into a sequence's cache slot at positions [pos0, pos0 + n), fragment order.
template <typename T>
__global__ void k_write_cache(const T* __restrict__ k, const T* __restrict__ v, T* __restrict__ kcache,
                              T* __restrict__ vcache, int Hkv, int dh, int pos0, size_t slot_base, int seq_stride) {
    const int r = blockIdx.x, kvh = blockIdx.y;
    const size_t hb = slot_base + (size_t)kvh * seq_stride * dh;
    for (int ch = threadIdx.x; ch < dh; ch += blockDim.x) {
        const size_t src = ((size_t)r * Hkv + kvh) * dh + ch;
        kcache[hb + kfrag_off(pos0 + r, ch, dh)] = k[src];
        vcache[hb + vfrag_off(pos0 + r, ch, dh)] = v[src];
    }
}

void launch_write_cache(const ssd_ctx* c, int seq, int layer, int pos0, int n, const void* k, const void* v, hipStream_t st) {
    const Dims& d = c->dm;
    const size_t slot = (((size_t)layer * d.max_seqs + seq) * d.Hkv) * (size_t)d.seq_stride() * d.dh;
    dim3 grid(n, d.Hkv);
    if (d.dtype == SSD_F32)
        k_write_cache<float><<<grid, 128, 0, st>>>((const float*)k, (const float*)v, (float*)c->b.kcache, (float*)c->b.vcache,
                                                   d.Hkv, d.dh, pos0, slot, d.seq_stride());
    else
        k_write_cache<bf16_t><<<grid, 128, 0, st>>>((const bf16_t*)k, (const bf16_t*)v, (bf16_t*)c->b.kcache,
                                                    (bf16_t*)c->b.vcache, d.Hkv, d.dh, pos0, slot, d.seq_stride());
}

// The nodes' own keys and values of a forward, from fragment order back to row-major [M, Hkv, dh].
template <typename T>
__global__ void k_read_own_kv(const FwdHeader* __restrict__ fw, const int* __restrict__ row_node,
                              const T* __restrict__ kown, const T* __restrict__ vown, T* __restrict__ k,
                              T* __restrict__ v, int Hkv, int dh, int vt_rows) {
    const int row = blockIdx.x, kvh = blockIdx.y;
    const NodeDesc nd = fw->nodes[row_node[row]];
    const int prow = nd.vrow0 + (row - nd.row0);
    const size_t hb = (size_t)kvh * vt_rows * dh;
    for (int ch = threadIdx.x; ch < dh; ch += blockDim.x) {
        const size_t dst = ((size_t)row * Hkv + kvh) * dh + ch;
        k[dst] = kown[hb + kfrag_off(prow, ch, dh)];
        v[dst] = vown[hb + vfrag_off(prow, ch, dh)];
    }
}

void launch_read_own_kv(const ssd_ctx* c, int M, void* k, void* v, hipStream_t st) {
    const Dims& d = c->dm;
    dim3 grid(M, d.Hkv);
    if (d.dtype == SSD_F32)
        k_read_own_kv<float><<<grid, 128, 0, st>>>(c->b.fwd, c->b.row_node, (const float*)c->b.kown, (const float*)c->b.vown,
                                                   (float*)k, (float*)v, d.Hkv, d.dh, d.vt_rows());
    else
        k_read_own_kv<bf16_t><<<grid, 128, 0, st>>>(c->b.fwd, c->b.row_node, (const bf16_t*)c->b.kown,
                                                    (const bf16_t*)c->b.vown, (bf16_t*)k, (bf16_t*)v, d.Hkv, d.dh, d.vt_rows());
}

void launch_int_to_float(const int* src, float* dst, int n, hipStream_t st) {
    k_int_to_float<<<(n + 255) / 256, 256, 0, st>>>(src, dst, n);
}
