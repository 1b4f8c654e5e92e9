// The MFMA GEMM kernel template and its launchers, shared by the translation units that instantiate it
// (kernels_mfma.hip: SwiGLU and LM-head epilogues; kernels_mfma_f32.hip: fp32 partial sums), so that they
// compile in parallel.  See kernels_mfma.hip for the design.
#pragma once
#include <cstdlib>
#include <type_traits>

#include "ssd_internal.h"


typedef uint16_t bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// Compile-time loop: f(integral_constant<int, C>) for C in [BEGIN, END).  The ring slots of the
// GEMM pipeline are selected by these constants, so no register array is ever indexed by a
// run-time value (which would push it to scratch memory).
template <int BEGIN, int END, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}

// exp through the hardware's base-2 exponential (relative error about 1e-6): the epilogues and the softmax
// evaluate it once per output element, where the correctly rounded library routine costs as much as the
// arithmetic it follows; the results are rounded to bf16 or summed over a vocabulary afterwards.
__device__ __forceinline__ float fast_exp(float x) { return __expf(x); }

__device__ __forceinline__ uint16_t f2bf_m(float f) {
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40);
    x += 0x7fffu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}


// ------------------------------------------------------------------------
// GEMM.  Work-group = WN x WK waves.  Wave (wn, wk) owns one n-tile of 32
// weight rows and, of every K chunk of WK*32 columns, the 32 columns
// [32wk, 32wk+32) (two k16 steps).
//
// Software pipeline, all statically indexed:
//   weights      a ring of DW chunks in registers per wave: the fragment loads
//                of chunk c+DW-1 are issued while chunk c is multiplied;
//   activations  loads of chunk c+PX are issued into a register ring, chunk c+2
//                is written to the free stage of a three-stage LDS ring while
//                chunk c is multiplied, one barrier per chunk.
// With the chunk count known at compile time (NCH > 0) the loop is straight-line
// code, so the compiler's wait counts are exact; NCH = 0 is the same pipeline as
// a loop unrolled by DW with loads past the end clamped (in bounds, unused).
// Every work-group starts its K walk at a different chunk and wraps, which
// spreads the grid's weight streams over the HBM channels; the order depends
// on the n-tile only, so a row's summation order is the same in every forward.
// DBG is for measurement builds only (bit 0: no MFMA, bit 1: no activation
// loads, bit 2: no epilogue, bit 3: every chunk reads chunk 0's activations, bit 4: no weight
// loads, bit 5: weight loads with the default cache policy); the library
// instantiates DBG = 0.
// ------------------------------------------------------------------------
template <int WN, int WK, int R, int MT, int EPI, int NCH, int DBG = 0, int DW = 4, int PX = 4, int KSTEPS = 2>
__global__ __launch_bounds__(WN* WK * 64) void k_gemm_mfma(const bf16_t* X, const uint4* Wp, void* outv, int M, int N,
                                                           int K, int ldx, int k_len, size_t split_stride,
                                                           int mask_id, int n_tiles_out, int n_blocks, int n_split,
                                                           int m_chunks_total) {
    constexpr int T = WN * WK * 64, KW = 16 * KSTEPS, KC = WK * KW, ROWS = MT * 32, LDW = KC + 8;
    constexpr int NST = 3;                              // LDS stages
    static_assert(DW >= 2 && DW <= 6 && PX >= 3 && PX <= 4, "ring depths");
    static_assert(EPI != EPI_SWIGLU || (WK == 2 && R == 1), "the SwiGLU epilogue is written for two k-slice waves");
    constexpr int XSEG = ROWS * (KC / 8);               // 16-byte segments per X chunk
    constexpr int XPT = (XSEG + T - 1) / T;             // per thread
    constexpr int SPARE = NST * ROWS * LDW;             // LDS element offset of the per-thread spare slots
    extern __shared__ uint4 smem_u4[];
    bf16_t* xs = (bf16_t*)smem_u4;                      // [NST][ROWS][LDW] + spare

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wn = wave % WN, wk = wave / WN;
    const int lm = lane & 31, lh = lane >> 5;
    // The grid is one-dimensional; work-groups go to the 8 XCDs round-robin by their linear id, and every
    // XCD has an L2 of its own.  The id is decoded so that with split-K all work-groups of an XCD take the
    // same k-slice, i.e. read the same slice of the activations and find it in that XCD's L2, and so that
    // the row chunks of one n-block (forwards with more rows than one pass holds) are neighbours on one
    // XCD and stream the same weights at the same time.  A tile's result does not depend on where it runs.
    int bx, bz, by;
    {
        const int split = n_split, mch = m_chunks_total;
        const int id = blockIdx.x;
        if (split <= 8 && 8 % split == 0 && n_blocks % (8 / split) == 0) {
            const int xcd = id & 7, t = id >> 3, per = 8 / split;
            bz = xcd % split;
            by = t % mch;
            bx = (t / mch) * per + xcd / split;
        } else {
            bz = id % split;
            by = (id / split) % mch;
            bx = id / (split * mch);
        }
    }
    const int m0 = by * ROWS;
    const int kbeg = bz * k_len, nchunks = NCH > 0 ? NCH : k_len / KC;
    const int KS = K >> 4, NT = N >> 5;

    // n-tiles of this wave (tiles past the end are clamped and never stored)
    int nt[R];
    bool nt_ok[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        nt[r] = (bx * WN + wn) * R + r;
        nt_ok[r] = nt[r] < NT;
        if (!nt_ok[r]) nt[r] = NT - 1;
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

    const int rot = (int)((bx * 5u + bz * 3u) % (unsigned)nchunks);
    auto chunk_at = [&](int c) {
        c = c < nchunks - 1 ? c : nchunks - 1;
        c += rot;
        return c >= nchunks ? c - nchunks : c;
    };

    // per-thread activation segments (the same for every chunk); segments past the tile or
    // past row M load row 0 / write a spare slot or zeros, so nothing branches
    const bf16_t* xsrc[XPT];
    int xdst[XPT];
    bool xok[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        const int seg = tid + i * T;
        const int m = seg / (KC / 8), sg = seg - m * (KC / 8);
        xok[i] = seg < XSEG && m0 + m < M;
        xsrc[i] = X + (size_t)(xok[i] ? m0 + m : 0) * ldx + kbeg + sg * 8;
        xdst[i] = seg < XSEG ? m * LDW + sg * 8 : SPARE + tid * 8;
    }

    // the rings are separate arrays selected by compile-time constants only
    constexpr int WF = R * KSTEPS;                      // weight fragments per chunk per wave
    uint4 w0[WF], w1[WF], w2[WF], w3[WF], w4[WF], w5[WF];
    uint4 x0[XPT], x1[XPT], x2[XPT], x3[XPT];
#define SSD_WSLOT(i) ((i) % DW == 0 ? w0 : (i) % DW == 1 ? w1 : (i) % DW == 2 ? w2 : (i) % DW == 3 ? w3 : (i) % DW == 4 ? w4 : w5)
#define SSD_XSLOT(i) ((i) % PX == 0 ? x0 : (i) % PX == 1 ? x1 : (i) % PX == 2 ? x2 : x3)
    auto issue_w = [&](uint4* dst, int c) {
        const size_t off = (size_t)chunk_at(c) * (KC / 16) * 64;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                if (DBG & 16)
                    dst[r * KSTEPS + ks] = make_uint4((unsigned)off, (unsigned)ks, 0u, 0u);
                else if (DBG & 32)
                    dst[r * KSTEPS + ks] = wbase[r][off + ks * 64];
                else {
                    // weights are read once per launch: a non-temporal load keeps them from evicting the
                    // activations, which every work-group of the XCD re-reads, from L2
                    const u32x4 v = __builtin_nontemporal_load((const u32x4*)&wbase[r][off + ks * 64]);
                    dst[r * KSTEPS + ks] = make_uint4(v.x, v.y, v.z, v.w);
                }
            }
    };
    auto issue_x = [&](uint4* dst, int c) {
        const size_t off = (DBG & 8) ? (size_t)0 : (size_t)chunk_at(c) * KC;
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            if (DBG & 2)
                dst[i] = make_uint4(c, c, c, c);
            else
                dst[i] = *(const uint4*)(xsrc[i] + off);
        }
    };
    auto stage_x = [&](const uint4* src, int buf) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            uint4 v = src[i];
            if (!xok[i]) v = make_uint4(0, 0, 0, 0);
            const int off = xdst[i] < SPARE ? buf * ROWS * LDW + xdst[i] : xdst[i];
            *(uint4*)(xs + off) = v;
        }
    };
    // all activation fragments of the chunk are read from LDS first, then the MFMAs run back
    // to back: one exposed LDS latency per chunk instead of one per MFMA; a fragment serves
    // the wave's R weight tiles
    auto multiply = [&](const uint4* w, int buf) {
        const bf16_t* xb = xs + (size_t)buf * ROWS * LDW + wk * KW + lh * 8;
        bf16x8 xf[KSTEPS][MT];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xf[ks][mt] = *(const bf16x8*)(xb + (size_t)(mt * 32 + lm) * LDW + ks * 16);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint4 wv = w[r * KSTEPS + ks];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    if (DBG & 1)
                        acc[r][mt][0] += __uint_as_float(wv.x ^ wv.w) + __uint_as_float(((const uint4*)&xf[ks][mt])->x);
                    else
                        acc[r][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)&wv, xf[ks][mt], acc[r][mt], 0, 0, 0);
                }
            }
    };

    // Chunk c is multiplied in iteration c from LDS stage c % 3.  Its activations were written
    // to LDS in iteration c-2, before that iteration's MFMAs, so the write -> barrier -> read
    // chain of a chunk overlaps the arithmetic of the two chunks before it instead of sitting
    // between them.  A stage is rewritten in the iteration after its last read; the barrier
    // that ends every iteration separates the two.
    static_for<0, PX>([&](auto ic) { constexpr int u = decltype(ic)::value; issue_x(SSD_XSLOT(u), u); });
    static_for<0, DW - 1>([&](auto ic) { constexpr int u = decltype(ic)::value; issue_w(SSD_WSLOT(u), u); });
    stage_x(x0, 0);
    stage_x(x1, 1);
    __syncthreads();
    if constexpr (NCH > 0) {
        static_for<0, NCH>([&](auto ic) {
            constexpr int c = decltype(ic)::value;
            if constexpr (c + 2 < NCH) stage_x(SSD_XSLOT(c + 2), (c + 2) % NST);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (c + PX < NCH) issue_x(SSD_XSLOT(c + PX), c + PX);
            if constexpr (c + DW - 1 < NCH) issue_w(SSD_WSLOT(c + DW - 1), c + DW - 1);
            multiply(SSD_WSLOT(c), c % NST);
            __syncthreads();
        });
    } else {
        constexpr int UN = 12;                          // ring and stage slots repeat with this period
        static_assert(UN % DW == 0 && UN % PX == 0 && UN % NST == 0, "unroll period");
        for (int c0 = 0; c0 < nchunks; c0 += UN) {
            static_for<0, UN>([&](auto ic) {
                constexpr int u = decltype(ic)::value;
                const int c = c0 + u;
                if (c < nchunks) {
                    stage_x(SSD_XSLOT(u + 2), (u + 2) % NST);
                    __builtin_amdgcn_sched_barrier(0);
                    issue_x(SSD_XSLOT(u + PX), c + PX);
                    issue_w(SSD_WSLOT(u + DW - 1), c + DW - 1);
                    multiply(SSD_WSLOT(u), u % NST);
                    __syncthreads();
                }
            });
        }
    }
#undef SSD_WSLOT
#undef SSD_XSLOT
    if (DBG & 4) {
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += acc[r][mt][i];
        if (sum == 1.2345f) *(float*)outv = sum;
        return;
    }

    // ---- epilogues.  Lane (lm, lh) holds, per tile, rows n = 8*(i/4) + 4*lh + i%4 of column m = lm;
    // g = i/4 selects a group of four consecutive n.
    if constexpr (WK == 2 && R == 1 && EPI == EPI_F32) {
        // The two k-slice waves of an n-tile share the output: wave wk keeps groups 2wk, 2wk+1 and
        // hands the other two to its partner through LDS, so both waves add and store (k-slice 0
        // plus k-slice 1, the order of the sequential reduction).
        float4* ex = (float4*)smem_u4;                  // [WN][sender wk][MT][2][64]
        static_for<0, 2>([&](auto iw) {
            constexpr int w = decltype(iw)::value;
            if (wk == w) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int gq = 0; gq < 2; ++gq) {
                        constexpr int gbase = (1 - w) * 2;
                        const int g = gbase + gq;
                        ex[(((wn * 2 + w) * MT + mt) * 2 + gq) * 64 + lane] =
                            make_float4(acc[0][mt][g * 4], acc[0][mt][g * 4 + 1], acc[0][mt][g * 4 + 2], acc[0][mt][g * 4 + 3]);
                    }
            }
        });
        __syncthreads();
        float* out = (float*)outv + (size_t)bz * split_stride;
        static_for<0, 2>([&](auto iw) {
            constexpr int w = decltype(iw)::value;
            if (wk == w && nt_ok[0]) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int m = m0 + mt * 32 + lm;
#pragma unroll
                    for (int gq = 0; gq < 2; ++gq) {
                        constexpr int gbase = w * 2;
                        const int g = gbase + gq;
                        const float4 o = ex[(((wn * 2 + (1 - w)) * MT + mt) * 2 + gq) * 64 + lane];
                        const int n = nt[0] * 32 + g * 8 + lh * 4;
                        if (m < M)
                            *(float4*)(out + (size_t)m * N + n) =
                                make_float4(acc[0][mt][g * 4] + o.x, acc[0][mt][g * 4 + 1] + o.y,
                                            acc[0][mt][g * 4 + 2] + o.z, acc[0][mt][g * 4 + 3] + o.w);
                    }
                }
            }
        });
        return;
    }
    if constexpr (WK == 2 && R == 1 && EPI == EPI_SWIGLU) {
        // A tile holds 16 channels: rows 0..15 gate, rows 16..31 up, so groups g and g + 2 of a lane are
        // gate and up of the same four channels.  Wave wk finishes g = wk and receives the other
        // k-slice's values of groups wk and wk + 2 through LDS (k-slice 0 plus k-slice 1).
        float4* ex = (float4*)smem_u4;                  // [WN][sender wk][MT][gate, up][64]
        static_for<0, 2>([&](auto iw) {
            constexpr int w = decltype(iw)::value;
            if (wk == w) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        constexpr int gother = 1 - w;
                        const int g = gother + 2 * h;
                        ex[(((wn * 2 + w) * MT + mt) * 2 + h) * 64 + lane] =
                            make_float4(acc[0][mt][g * 4], acc[0][mt][g * 4 + 1], acc[0][mt][g * 4 + 2], acc[0][mt][g * 4 + 3]);
                    }
            }
        });
        __syncthreads();
        bf16_t* out = (bf16_t*)outv;
        const int F = N >> 1;                           // output channels = row stride of the output
        static_for<0, 2>([&](auto iw) {
            constexpr int w = decltype(iw)::value;
            if (wk == w && nt_ok[0]) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const float4 og = ex[(((wn * 2 + (1 - w)) * MT + mt) * 2 + 0) * 64 + lane];
                    const float4 ou = ex[(((wn * 2 + (1 - w)) * MT + mt) * 2 + 1) * 64 + lane];
                    const float gv[4] = {acc[0][mt][w * 4] + og.x, acc[0][mt][w * 4 + 1] + og.y,
                                         acc[0][mt][w * 4 + 2] + og.z, acc[0][mt][w * 4 + 3] + og.w};
                    const float uv[4] = {acc[0][mt][(w + 2) * 4] + ou.x, acc[0][mt][(w + 2) * 4 + 1] + ou.y,
                                         acc[0][mt][(w + 2) * 4 + 2] + ou.z, acc[0][mt][(w + 2) * 4 + 3] + ou.w};
                    uint16_t o[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) o[j] = f2bf_m(gv[j] * __builtin_amdgcn_rcpf(1.0f + fast_exp(-gv[j])) * uv[j]);   // result rounded to bf16
                    const int m = m0 + mt * 32 + lm;
                    const int f = nt[0] * 16 + w * 8 + lh * 4;
                    if (m < M)
                        *(uint2*)(out + (size_t)m * F + f) =
                            make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
                }
            }
        });
        return;
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
        float* out = (float*)outv + (size_t)bz * split_stride;
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
    } else if (lead) {
        // LM head: per (row, n-tile) partial over the tile's 32 vocabulary rows
        float* out = (float*)outv;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int tile_out = (bx * WN + wn) * R + r;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                float bm = -INFINITY;
                int bi = 0x7fffffff;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int n = nt[r] * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
                    const float v = acc[r][mt][i];
                    if (n != mask_id && v > bm) { bm = v; bi = n; }
                }
                {
                    const float om = __shfl_xor(bm, 32, 64);
                    const int oi = __shfl_xor(bi, 32, 64);
                    if (om > bm || (om == bm && oi < bi)) { bm = om; bi = oi; }
                }
                float se = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int n = nt[r] * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
                    if (n != mask_id) se += fast_exp(acc[r][mt][i] - bm);
                }
                se += __shfl_xor(se, 32, 64);
                const int m = m0 + mt * 32 + lm;
                if (lh == 0 && m < M && tile_out < n_tiles_out && nt_ok[r]) {
                    float* o = out + ((size_t)m * n_tiles_out + tile_out) * 3;
                    o[0] = bm;
                    o[1] = __int_as_float(bi);
                    o[2] = se;
                }
            }
        }
    }
}

// ------------------------------------------------------------------------
// launcher
// ------------------------------------------------------------------------

template <int WN, int WK, int R, int MT, int EPI, int NCH, int POLICY = 0>
static bool launch_one(const bf16_t* X, const uint4* Wp, void* out, int M, int N, int K, int split, size_t split_stride,
                       int mask_id, int n_tiles_out, int m_chunks, hipStream_t st) {
    constexpr int KC = WK * 32, ROWS = MT * 32, LDW = KC + 8;
    constexpr size_t xbytes = (size_t)3 * ROWS * LDW * 2 + (size_t)WN * WK * 64 * 16;   // three stages + spare slots
    // epilogue exchange areas: see the kernel's epilogues
    constexpr size_t rbytes = (WK == 2 && R == 1 && EPI != EPI_LMHEAD) ? (size_t)WN * 2 * MT * 2 * 1024
                              : WK > 1 ? (size_t)(WK - 1) * WN * R * MT * 16 * 64 * 4
                                       : (size_t)(WN / 2 + 1) * MT * 16 * 64 * 4;
    constexpr size_t smem = xbytes > rbytes ? xbytes : rbytes;
    static_assert(smem <= 160 * 1024, "LDS budget");
    auto kern = k_gemm_mfma<WN, WK, R, MT, EPI, NCH, POLICY>;
    static bool attr_done = false;
    if (!attr_done) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return false;
        attr_done = true;
    }
    const int tiles = N / 32, per_wg = WN * R;
    const int n_blocks = (tiles + per_wg - 1) / per_wg;
    dim3 grid(n_blocks * m_chunks * split);
    hipLaunchKernelGGL(kern, grid, dim3(WN * WK * 64), smem, st, X, Wp, out, M, N, K, K, K / split, split_stride,
                       mask_id, n_tiles_out, n_blocks, split, m_chunks);
    return true;
}

// Row tiles of 32 rows per pass: 1 (a stepwise forward of one block) to 6; other row counts round up
// (padding rows are zero and never stored).  The rows of a pass share nothing but the weight fragments,
// so a row's sums do not depend on the tile it is computed in.
template <int WN, int WK, int R, int EPI, int NCH>
static bool launch_mt(int mt, const bf16_t* X, const uint4* Wp, void* out, int M, int N, int K, int split,
                      size_t split_stride, int mask_id, int n_tiles_out, int m_chunks,
                      hipStream_t st) {
#define SSD_MT_CASE(v)                                                                                          \
    case v:                                                                                                     \
        return launch_one<WN, WK, R, v, EPI, NCH>(X, Wp, out, M, N, K, split, split_stride, mask_id,  \
                                               n_tiles_out, m_chunks, st);
    // more than one row chunk: every chunk re-reads the weights, so they are loaded with the default
    // cache policy (kernel option bit 5) and the later chunks find them in L2 / the Infinity Cache
    if (mt == 5 && m_chunks > 1)
        return launch_one<WN, WK, R, 5, EPI, NCH, 32>(X, Wp, out, M, N, K, split, split_stride, mask_id, n_tiles_out,
                                                      m_chunks, st);
    if (mt == 6 && m_chunks > 1)
        return launch_one<WN, WK, R, 6, EPI, NCH, 32>(X, Wp, out, M, N, K, split, split_stride, mask_id, n_tiles_out,
                                                      m_chunks, st);
    switch (mt) {
        SSD_MT_CASE(1)
        SSD_MT_CASE(2)
        SSD_MT_CASE(3)
        SSD_MT_CASE(4)
        SSD_MT_CASE(5)
        SSD_MT_CASE(6)
    }
#undef SSD_MT_CASE
    return false;
}

// One chunk count per work-group shape runs as straight-line code (NCH = the 8B-class shape's chunk
// count for that projection); every other chunk count takes the looped kernel (NCH = 0).
template <int WN, int WK, int EPI, int NCH>
static bool launch_shape(int nch, int mt, const bf16_t* X, const uint4* Wp, void* out, int M, int N, int K, int split,
                         size_t split_stride, int mask_id, int n_tiles_out, int m_chunks, hipStream_t st) {
    if (NCH > 0 && nch == NCH)
        return launch_mt<WN, WK, 1, EPI, NCH>(mt, X, Wp, out, M, N, K, split, split_stride, mask_id, n_tiles_out, m_chunks, st);
    return launch_mt<WN, WK, 1, EPI, 0>(mt, X, Wp, out, M, N, K, split, split_stride, mask_id, n_tiles_out, m_chunks, st);
}

// the launchers of the work-group shapes, one translation unit each (they compile in parallel)
struct GemmArgs {
    int nch, mt;
    const bf16_t* X;
    const uint4* Wp;
    void* out;
    int M, N, K, split;
    size_t split_stride;
    int mask_id, n_tiles_out, m_chunks;
    hipStream_t st;
};
bool gemm_f32_wn3(const GemmArgs& a);     // wide outputs (QKV): 96-row n-blocks
bool gemm_f32_wn2(const GemmArgs& a);     // narrow outputs, short K (attention output): 64-row n-blocks
bool gemm_f32_wn4(const GemmArgs& a);     // narrow outputs, long K (down) and everything else: 128-row n-blocks
bool gemm_swiglu_wn3(const GemmArgs& a);
bool gemm_swiglu_wn4(const GemmArgs& a);
bool gemm_lmhead_wn4(const GemmArgs& a);

// Split along K across work-groups: a function of the weight shape only.
static int pick_split(int K, int kc, int want) {
    int s = want;
    while (s > 1 && (K % (s * kc)) != 0) --s;
    return s < 1 ? 1 : s;
}
