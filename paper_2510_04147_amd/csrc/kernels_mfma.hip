// Matrix-core (MFMA) kernels for bf16 models on gfx950.
//
// Skinny weight-streaming GEMM  out[M,N] = X[M,K] * W[N,K]^T  for M <= 160 rows
// per pass (the (N+1)*B rows of one verification forward, Eq. 5).  The weights
// are the HBM stream; the design is built around that:
//   * weights are repacked once, at context creation, into MFMA fragment
//     order: fragment (nt, ks) = rows [32nt, 32nt+32) x columns [16ks, 16ks+16)
//     is one contiguous 1 KiB block laid out lane by lane, so a wave's load
//     instruction reads 1 KiB of consecutive bytes and a wave streams a
//     contiguous region straight into registers (no LDS round trip), with
//     non-temporal loads, so that the stream does not evict the activations
//     from L2; the gate/up matrix interleaves gate and up rows per 16 channels,
//     which makes SwiGLU lane-local;
//   * the weight fragment is the A operand of v_mfma_f32_32x32x16_bf16, the
//     activations are the B operand, so each lane ends up with 4 consecutive
//     output columns of one row: vector stores, lane-local SwiGLU and LM-head
//     reductions;
//   * activations are staged through LDS in K chunks (a three-stage ring),
//     shared by all waves of the work-group;
//   * grids aim at one work-group per CU (256) and are XCD-aware: with split-K
//     the work-groups of one XCD read the same k-slice of the activations;
//   * K can be split inside a work-group (waves reduce through LDS) and across
//     work-groups (partial sums to a workspace, summed in a fixed order by the
//     consumer).  Both splits depend on the weight shape only, never on M, and
//     a row's arithmetic never involves another row: a row is bit-identical in
//     a 1-node and an (N+1)-node forward.
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

__device__ __forceinline__ uint16_t f2bf_m(float f) {
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40);
    x += 0x7fffu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}

// ------------------------------------------------------------------------
// One-time weight repack: W[N][K] row-major -> fragment order.
// dst uint4 index ((nt*KS + ks)*64 + lane) holds row(nt, lane%32), columns [16ks + 8(lane/32), +8).
// Plain matrices: row(nt, r) = 32nt + r.  The gate/up matrix (F gate rows, then F up rows;
// gate_rows = F): tile nt holds 16 channels, row(nt, r) = gate row 16nt + r for r < 16 and
// up row F + 16nt + r - 16 for r >= 16, so that a lane of the 32x32 MFMA result, which holds
// rows r and r + 16 of a column, holds the gate and the up value of the same channel.
// ------------------------------------------------------------------------
__global__ void k_pack_weights(const uint4* __restrict__ src, uint4* __restrict__ dst, int N, int K, int gate_rows) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int KS = K >> 4;
    const size_t total = (size_t)(N >> 5) * KS * 64;
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    const size_t frag = idx >> 6;
    const int ks = (int)(frag % KS);
    const size_t nt = frag / KS;
    const int r = lane & 31;
    const size_t row = gate_rows > 0 ? (r < 16 ? nt * 16 + r : (size_t)gate_rows + nt * 16 + (r - 16)) : nt * 32 + r;
    const int col = ks * 16 + 8 * (lane >> 5);
    dst[idx] = src[(row * K + col) >> 3];
}

void launch_pack_weights(const void* src, void* dst, int N, int K, int gate_rows, hipStream_t st) {
    const size_t total = (size_t)(N / 32) * (K / 16) * 64;
    k_pack_weights<<<(unsigned)((total + 255) / 256), 256, 0, st>>>((const uint4*)src, (uint4*)dst, N, K, gate_rows);
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
                                                           int mask_id, int n_tiles_out) {
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
    // Work-groups go to the 8 XCDs round-robin by their linear id.  With split-K the low bits of
    // blockIdx.x pick the k-slice, so the work-groups of one XCD read the same slice of the
    // activations and find it in that XCD's L2; the n-block takes the remaining bits.
    int bx = blockIdx.x, bz = blockIdx.z;
    if (gridDim.z > 1 && gridDim.x % gridDim.z == 0) {
        bz = blockIdx.x % gridDim.z;
        bx = blockIdx.x / gridDim.z + (gridDim.x / gridDim.z) * blockIdx.z;
    }
    const int m0 = blockIdx.y * ROWS;
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
                    for (int j = 0; j < 4; ++j) o[j] = f2bf_m(gv[j] / (1.0f + expf(-gv[j])) * uv[j]);
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
                    if (n != mask_id) se += expf(acc[r][mt][i] - bm);
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
    dim3 grid((tiles + per_wg - 1) / per_wg, m_chunks, split);
    hipLaunchKernelGGL(kern, grid, dim3(WN * WK * 64), smem, st, X, Wp, out, M, N, K, K, K / split, split_stride,
                       mask_id, n_tiles_out);
    return true;
}

// Row tiles per pass: 1 (a stepwise forward of one block), 2, 5 (a 5-node tree) or 6;
// other row counts round up (padding rows are zero and never stored).
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
        SSD_MT_CASE(5)
        SSD_MT_CASE(6)
    }
#undef SSD_MT_CASE
    return false;
}

// Chunk counts with a straight-line kernel; anything else takes the looped one (NCH = 0).
template <int WN, int WK, int R, int EPI>
static bool launch_nch(int nch, int mt, const bf16_t* X, const uint4* Wp, void* out, int M, int N, int K, int split,
                       size_t split_stride, int mask_id, int n_tiles_out, int m_chunks,
                       hipStream_t st) {
#define SSD_NCH_CASE(v)                                                                                           \
    case v:                                                                                                       \
        return launch_mt<WN, WK, R, EPI, v>(mt, X, Wp, out, M, N, K, split, split_stride, mask_id,      \
                                         n_tiles_out, m_chunks, st);
    if (EPI == EPI_F32) {
        switch (nch) {
            SSD_NCH_CASE(8)
            SSD_NCH_CASE(16)
            SSD_NCH_CASE(24)
            SSD_NCH_CASE(32)
            SSD_NCH_CASE(64)
        }
    } else {
        switch (nch) { SSD_NCH_CASE(64) }
    }
#undef SSD_NCH_CASE
    return launch_mt<WN, WK, R, EPI, 0>(mt, X, Wp, out, M, N, K, split, split_stride, mask_id, n_tiles_out,
                                     m_chunks, st);
}

int lm_tiles_mfma(int V) { return V / 32; }

// Split along K across work-groups: a function of the weight shape only.
static int pick_split(int K, int kc, int want) {
    int s = want;
    while (s > 1 && (K % (s * kc)) != 0) --s;
    return s < 1 ? 1 : s;
}

#ifndef SSD_KERNELS_ONLY
bool launch_gemm_mfma(const ssd_ctx* c, int epi, const void* X, const Wt& W, void* out, int M, int* n_split,
                      hipStream_t st) {
    if (!W.packed) return false;
    const int N = W.N, K = W.K;
    constexpr int WN = 4, WK = 2, KC = WK * 32;
    if (K % KC) return false;
    // rows per pass: 32, 64 or 160 (a 5-node tree of 32-row blocks); forwards with more rows re-stream the
    // weights once per pass, in passes of 160 or 192 rows, whichever needs fewer.  The rows of a pass share
    // nothing but the weight fragments, so a row's sums do not depend on the choice.
    int mt = M <= 32 ? 1 : M <= 64 ? 2 : 5;
    if (M > 160 && (M + 191) / 192 < (M + 159) / 160) mt = 6;
    const int rows = mt * 32, m_chunks = (M + rows - 1) / rows;
    const bf16_t* x = (const bf16_t*)X;
    const uint4* wp = (const uint4*)W.packed;
    const size_t stride = (size_t)c->dm.max_rows * (size_t)c->part_cols;
    if (epi == EPI_SWIGLU) {
        // W = [2F, d] packed with gate and up rows interleaved per 16 channels: N/32 tiles of 16
        // channels each, any number of them per work-group; 96-row n-blocks give the 8B shape
        // (768 tiles) exactly one work-group per CU
        *n_split = 1;
        if ((N / 32) % 3 == 0)
            return launch_nch<3, WK, 1, EPI_SWIGLU>(K / KC, mt, x, wp, out, M, N, K, 1, 0, -1, 0, m_chunks, st);
        return launch_nch<WN, WK, 1, EPI_SWIGLU>(K / KC, mt, x, wp, out, M, N, K, 1, 0, -1, 0, m_chunks, st);
    }
    if (epi == EPI_LMHEAD) {
        *n_split = lm_tiles_mfma(N);
        return launch_nch<WN, WK, 1, EPI_LMHEAD>(K / KC, mt, x, wp, out, M, N, K, 1, 0, c->dm.mask_id, N / 32, m_chunks, st);
    }
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
    if (wn == 3) return launch_nch<3, WK, 1, EPI_F32>(nch, mt, x, wp, out, M, N, K, split, stride, -1, 0, m_chunks, st);
    if (wn == 2) return launch_nch<2, WK, 1, EPI_F32>(nch, mt, x, wp, out, M, N, K, split, stride, -1, 0, m_chunks, st);
    return launch_nch<WN, WK, 1, EPI_F32>(nch, mt, x, wp, out, M, N, K, split, stride, -1, 0, m_chunks, st);
}
#endif

// ------------------------------------------------------------------------
// a4: shared-prefix bidirectional attention on the matrix cores.
// One work-group of ATTN_WAVES waves per (node, query head, 32-row query tile).
// Keys are walked in tiles of 32, first the sequence's cached prefix [0,S), then
// the node's own rows; wave w takes tiles w, w + ATTN_WAVES, ...; online softmax
// in fp32; the waves' partial results are merged through LDS in wave order.
//   S^T[key][q] = K Q^T     : A = K fragment (rows = keys), B = Q fragment
//   O^T[d][q]  += V^T P^T   : A = V^T fragment (rows = d),  B = P^T fragment
// With q on the MFMA column axis every softmax statistic (running max, sum,
// rescale factor) is per lane, and the P^T values a lane computed are exactly
// its B-operand values for the second product, so nothing crosses lanes except
// one xor-32 exchange per tile.  The k index of the second product is the key;
// lane half lh supplies keys {8g + 4lh + 0..3 : g = 2st, 2st+1} of step st: the
// value layout stores exactly those eight next to each other, so keys and values
// both arrive as one 16-byte load per lane and fragment.
// The tile order depends on S and the block length only, so a row's result does
// not depend on how many nodes the forward holds.
// ------------------------------------------------------------------------
#define ATTN_WAVES 8   // waves per (node, head, query tile): wave w takes key tiles w, w+8, ...

// FUSED: the kernel starts from the QKV projection's fp32 partial sums instead of ready q / k / v: it
// adds the partial sums in split order, applies the rotary embedding to its head's queries and to
// the node's own keys and keeps the own key / value tile in LDS in fragment order.  For forwards whose
// nodes have at most 32 rows (one query tile) and append nothing to the cache, head size 128.
template <int DH, bool FUSED, bool SUFFIX>
__global__ __launch_bounds__(ATTN_WAVES * 64) void k_attn_mfma(const FwdHeader* __restrict__ fw,
                                                               const bf16_t* __restrict__ q,
                                                               const bf16_t* __restrict__ kown,
                                                               const bf16_t* __restrict__ vown,
                                                               const bf16_t* __restrict__ kcache,
                                                               const bf16_t* __restrict__ vcache,
                                                               bf16_t* __restrict__ out, int Hq, int Hkv, int layer,
                                                               int max_seqs, int seq_stride, int vt_rows, float scale,
                                                               const float* __restrict__ part, int n_part,
                                                               size_t part_stride, const float* __restrict__ cosT,
                                                               const float* __restrict__ sinT) {
    constexpr int KST = DH / 16, DT = DH / 32;
    constexpr int NE = DT * 16;                                      // O^T values per lane
    constexpr int EPW = NE / ATTN_WAVES;                             // of which each wave merges EPW
    static_assert(EPW % 4 == 0, "the merge writes groups of four head channels");
    static_assert(!FUSED || DH == 128, "the fused rotary stage is laid out for head size 128");
    __shared__ float mrg[ATTN_WAVES][NE + 2][64];                    // every wave's partial (O^T, max, sum)
    __shared__ __attribute__((aligned(16))) bf16_t qs[32][DH + 8];   // the query tile, shared by the waves
    // FUSED: the node's own key and value tile, fragment order, in the (not yet used) merge area
    bf16_t* ks_own = (bf16_t*)&mrg[0][0][0];
    bf16_t* vs_own = ks_own + 32 * DH;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lm = lane & 31, lh = lane >> 5;
    // Work-groups go to the 8 XCDs round-robin by their linear id, and every XCD has an L2 of its
    // own: all (node, query head) pairs that read one KV head are placed on the same XCD, so the
    // prefix is fetched from HBM once and the other nodes hit in L2.
    const int n_nodes = gridDim.x / Hq, G = Hq / Hkv;
    int node, head;
    if (Hkv % 8 == 0) {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        node = slot % n_nodes;
        const int rest = slot / n_nodes;
        head = ((rest / G) * 8 + xcd) * G + rest % G;
    } else {
        node = blockIdx.x % n_nodes;
        head = blockIdx.x / n_nodes;
    }
    const NodeDesc nd = fw->nodes[node];
    const int kvh = head / G;
    const int qt = blockIdx.y;
    if (qt * 32 >= nd.blen) return;                                  // uniform over the work-group
    const int nq = Hq * DH;
    const int qrow_in = qt * 32 + lm;
    const bool qvalid = qrow_in < nd.blen;
    const int qrow = nd.row0 + (qvalid ? qrow_in : 0);

    // keys and values of one KV head, fragment order: a tile of 32 positions is KST key pieces and
    // 2*DT value pieces of 64 lanes x 8 elements each, fetched with one 16-byte load per lane
    const size_t cbase = ((((size_t)layer * max_seqs + nd.seq) * Hkv) + kvh) * (size_t)seq_stride * DH;
    const bf16_t* kc = kcache + cbase;
    const bf16_t* vc = vcache + cbase;
    const size_t obase = ((size_t)kvh * vt_rows + nd.vrow0) * DH;   // the node's rows start on a tile boundary
    const bf16_t* ko = kown + obase;
    const bf16_t* vo = vown + obase;

    floatx16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
    float m_run = -INFINITY, l_part = 0.f;

    // Key tiles, in this order: the cached prefix [0, S); the cached suffix [S + blen, T) of a
    // sequence whose positions behind the block are cached too (T = 0: none); the node's own rows.
    // Cache tiles are whole 32-position tiles of the cache; a tile may hold the end of the prefix and
    // the start of the suffix at once, tiles that lie inside the block are skipped, and every tile
    // listed holds at least one valid key.
    // (SUFFIX = false: a forward none of whose nodes has a suffix; the suffix terms fold away)
    const int blk_end = nd.S + nd.blen, node_T = SUFFIX ? nd.T : 0;
    const int pre_tiles = (nd.S + 31) >> 5;
    const int suf_first = max(pre_tiles, blk_end >> 5);
    const int suf_tiles = SUFFIX && node_T > blk_end ? max(((node_T + 31) >> 5) - suf_first, 0) : 0;
    const int cache_tiles = pre_tiles + suf_tiles, n_tiles = cache_tiles + ((nd.blen + 31) >> 5);
    auto cache_tile = [&](int t) { return !SUFFIX || t < pre_tiles ? t : suf_first + (t - pre_tiles); };
    // positions that are not keys of this node hold other or stale data: masked (keys) or zeroed (values)
    auto load_k = [&](bf16x8(&kf)[KST], int t) {
        const bf16_t* kp;
        if (t >= cache_tiles)
            kp = (FUSED ? ks_own : ko + (size_t)(t - cache_tiles) * 32 * DH) + lane * 8;
        else
            kp = kc + (size_t)cache_tile(t) * 32 * DH + lane * 8;
#pragma unroll
        for (int ks = 0; ks < KST; ++ks) kf[ks] = *(const bf16x8*)(kp + ks * 512);
    };
    auto load_v = [&](bf16x8(&vf)[DT][2], int t) {
        const bf16_t* vp;
        if (t >= cache_tiles)
            vp = (FUSED ? vs_own : vo + (size_t)(t - cache_tiles) * 32 * DH) + lane * 8;
        else
            vp = vc + (size_t)cache_tile(t) * 32 * DH + lane * 8;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int st = 0; st < 2; ++st) vf[dt][st] = *(const bf16x8*)(vp + (dt * 2 + st) * 512);
    };
    bf16x8 kf[KST], kn[KST], vf[DT][2], vn[DT][2];
    // the first tile's loads go out before anything else (FUSED: unless it is the own tile, which is
    // not in LDS yet)
    const bool first_later = FUSED && wave >= cache_tiles;
    if (wave < n_tiles && !first_later) {
        load_k(kf, wave);
        load_v(vf, wave);
    }
    if constexpr (FUSED) {
        // 32 rows x 16 column groups.  q and k: thread (r, cg) owns channels [4cg, 4cg+4) of both rotary
        // halves; v: channels [8cg, 8cg+8).  Rows past the end of the block take row 0's values
        // (queries: never written back; keys: masked) or zeros (values).
        constexpr int HALF = DH / 2;
        const int tid = threadIdx.x, r = tid >> 4, cg = tid & 15;
        const bool rvalid = r < nd.blen;
        const int row = nd.row0 + (rvalid ? r : 0), pos = nd.S + (rvalid ? r : 0);
        const int nkv = Hkv * DH, nqkv = nq + 2 * nkv;
        const float* src = part + (size_t)row * nqkv;
        auto load4 = [&](int col, float* dst) {             // 4 values from column col, partial sums in split order
            float4 a = *(const float4*)(src + col);
            for (int sp = 1; sp < n_part; ++sp) {
                const float4 b = *(const float4*)(src + sp * part_stride + col);
                a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
            }
            dst[0] = a.x; dst[1] = a.y; dst[2] = a.z; dst[3] = a.w;
        };
        const int i0 = cg * 4;
        float qa[4], qb[4], ka[4], kb[4], vv[8], cs[4], sn[4];
        load4(head * DH + i0, qa);
        load4(head * DH + HALF + i0, qb);
        load4(nq + kvh * DH + i0, ka);
        load4(nq + kvh * DH + HALF + i0, kb);
        load4(nq + nkv + kvh * DH + cg * 8, vv);
        load4(nq + nkv + kvh * DH + cg * 8 + 4, vv + 4);
        {
            const float4 c4 = *(const float4*)(cosT + (size_t)pos * HALF + i0), s4 = *(const float4*)(sinT + (size_t)pos * HALF + i0);
            cs[0] = c4.x; cs[1] = c4.y; cs[2] = c4.z; cs[3] = c4.w;
            sn[0] = s4.x; sn[1] = s4.y; sn[2] = s4.z; sn[3] = s4.w;
        }
        uint16_t q1[4], q2[4], k1[4], k2[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float o1, o2;
            rope_pair(qa[j], qb[j], cs[j], sn[j], o1, o2);
            q1[j] = f2bf_m(o1); q2[j] = f2bf_m(o2);
            rope_pair(ka[j], kb[j], cs[j], sn[j], o1, o2);
            k1[j] = f2bf_m(o1); k2[j] = f2bf_m(o2);
        }
        auto pack4 = [](const uint16_t* h) {
            return make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
        };
        *(uint2*)&qs[r][i0] = pack4(q1);
        *(uint2*)&qs[r][HALF + i0] = pack4(q2);
        // four consecutive channels starting at a multiple of four stay contiguous in fragment order
        *(uint2*)&ks_own[kfrag_off(r, i0, DH)] = pack4(k1);
        *(uint2*)&ks_own[kfrag_off(r, HALF + i0, DH)] = pack4(k2);
        uint16_t vb[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            vb[j] = rvalid ? f2bf_m(vv[j]) : (uint16_t)0;
            vs_own[vfrag_off(r, cg * 8 + j, DH)] = vb[j];             // scattered 2-byte LDS stores, 8 per thread
        }
    } else {
        // the query tile, after the first key/value loads are on their way; rows past the end of the
        // block are read from row 0 and never written back
        for (int idx = threadIdx.x; idx < 32 * (DH / 8); idx += ATTN_WAVES * 64) {
            const int r = idx / (DH / 8), c8 = idx % (DH / 8);
            const int rin = qt * 32 + r;
            const int grow = nd.row0 + (rin < nd.blen ? rin : 0);
            *(bf16x8*)&qs[r][c8 * 8] = *(const bf16x8*)(q + (size_t)grow * nq + head * DH + c8 * 8);
        }
    }
    __syncthreads();                                                // the query tile (FUSED: and the own tile) is in LDS
    if (wave < n_tiles && first_later) {
        load_k(kf, wave);
        load_v(vf, wave);
    }
    for (int t = wave; t < n_tiles; t += ATTN_WAVES) {
        const bool own = t >= cache_tiles;
        // first key of the tile: a row of the node (own) or a cache position
        const int t0 = (own ? t - cache_tiles : cache_tile(t)) * 32;
        // keys t0 + [0, lim_a) and t0 + [lo_b, lim_b) of this tile exist
        const int lim_a = (own ? nd.blen : nd.S) - t0;
        const int lo_b = own ? 32 : blk_end - t0, lim_b = own ? 0 : node_T - t0;
        auto valid = [&](int key) { return key < lim_a || (SUFFIX && key >= lo_b && key < lim_b); };
        const bool all_valid = lim_a >= 32 || (SUFFIX && lo_b <= 0 && lim_b >= 32);
        // ---- this wave's next tile, in flight while this one is processed
        if (t + ATTN_WAVES < n_tiles) {
            load_k(kn, t + ATTN_WAVES);
            load_v(vn, t + ATTN_WAVES);
        }
        // ---- S^T = K Q^T
        floatx16 sacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KST; ++ks) {
            const bf16x8 qf = *(const bf16x8*)&qs[lm][ks * 16 + lh * 8];
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf, sacc, 0, 0, 0);
        }
        // ---- online softmax over this lane's 16 keys (key = t0 + 8*(i/4) + 4*lh + i%4)
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = (i >> 2) * 8 + lh * 4 + (i & 3);
            sacc[i] = valid(key) ? sacc[i] * scale : -INFINITY;
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
            const float p = expf(sacc[i] - m_new);                  // 0 for masked keys
            psum += p;
            pf[i >> 3][i & 7] = (__bf16)p;
        }
        l_part = l_part * corr + psum;
        if (!all_valid) {
            // positions that are not keys hold other data: zero them so 0 * garbage cannot produce NaN
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int st = 0; st < 2; ++st)
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int key = (2 * st + (j >> 2)) * 8 + lh * 4 + (j & 3);
                        if (!valid(key)) vf[dt][st][j] = (__bf16)0.f;
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
#pragma unroll
        for (int ks = 0; ks < KST; ++ks) kf[ks] = kn[ks];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int st = 0; st < 2; ++st) vf[dt][st] = vn[dt][st];
    }
    // ---- merge the waves' partial results: every wave publishes its partial, then wave w folds
    // values [w*EPW, (w+1)*EPW) of all waves in wave order (fixed, independent of the forward's shape)
    if constexpr (FUSED) __syncthreads();                           // the own tile shared the merge area
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) mrg[wave][dt * 16 + i][lane] = oacc[dt][i];
    mrg[wave][NE][lane] = m_run;
    mrg[wave][NE + 1][lane] = l_part;
    __syncthreads();
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < ATTN_WAVES; ++w) m_all = fmaxf(m_all, mrg[w][NE][lane]);
    float cw[ATTN_WAVES], l = 0.f;
#pragma unroll
    for (int w = 0; w < ATTN_WAVES; ++w) {
        const float mw = mrg[w][NE][lane];
        cw[w] = mw == -INFINITY ? 0.f : expf(mw - m_all);            // a wave without a tile counts for nothing
        l += mrg[w][NE + 1][lane] * cw[w];
    }
    l += __shfl_xor(l, 32, 64);
    const float inv = 1.0f / l;
    float o[EPW];
#pragma unroll
    for (int e = 0; e < EPW; ++e) {
        float acc = 0.f;
#pragma unroll
        for (int w = 0; w < ATTN_WAVES; ++w) acc += mrg[w][wave * EPW + e][lane] * cw[w];
        o[e] = acc * inv;
    }
    if (qvalid) {
        bf16_t* op = out + (size_t)qrow * nq + head * DH;
#pragma unroll
        for (int g4 = 0; g4 < EPW / 4; ++g4) {
            const int e = wave * EPW + g4 * 4;                       // first of four consecutive values
            const int dt = e >> 4, g = (e & 15) >> 2;                // head channel = dt*32 + g*8 + lh*4 + j
            uint16_t ob[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) ob[j] = f2bf_m(o[g4 * 4 + j]);
            *(uint2*)(op + dt * 32 + g * 8 + lh * 4) =
                make_uint2((uint32_t)ob[0] | ((uint32_t)ob[1] << 16), (uint32_t)ob[2] | ((uint32_t)ob[3] << 16));
        }
    }
}

bool attn_mfma_can_fuse_rope(const ssd_ctx* c, int max_blen) {
    return c->dm.dtype == SSD_BF16 && c->dm.dh == 128 && max_blen <= 32;
}

bool launch_attn_mfma(const ssd_ctx* c, int n_nodes, int max_blen, int layer, int n_part, bool suffix, hipStream_t st) {
    const Dims& d = c->dm;
    dim3 grid(n_nodes * d.Hq, (max_blen + 31) / 32);
    const float scale = 1.0f / sqrtf((float)d.dh);
    const size_t ps = (size_t)d.max_rows * c->part_cols;
#define SSD_ATTN_ARGS                                                                                                  \
    c->b.fwd, (const bf16_t*)c->b.q, (const bf16_t*)c->b.kown, (const bf16_t*)c->b.vown, (const bf16_t*)c->b.kcache, \
        (const bf16_t*)c->b.vcache, (bf16_t*)c->b.attn, d.Hq, d.Hkv, layer, d.max_seqs, d.seq_stride(), d.vt_rows(), scale, \
        c->b.part, n_part, ps, c->b.rope_cos, c->b.rope_sin
#define SSD_ATTN_LAUNCH(DH_, FUSED_)                                                                       \
    do {                                                                                                   \
        if (suffix) k_attn_mfma<DH_, FUSED_, true><<<grid, ATTN_WAVES * 64, 0, st>>>(SSD_ATTN_ARGS);      \
        else k_attn_mfma<DH_, FUSED_, false><<<grid, ATTN_WAVES * 64, 0, st>>>(SSD_ATTN_ARGS);            \
    } while (0)
    if (n_part >= 0) {
        if (!attn_mfma_can_fuse_rope(c, max_blen)) return false;
        SSD_ATTN_LAUNCH(128, true);
    } else if (d.dh == 128)
        SSD_ATTN_LAUNCH(128, false);
    else if (d.dh == 64)
        SSD_ATTN_LAUNCH(64, false);
    else
        return false;
#undef SSD_ATTN_LAUNCH
#undef SSD_ATTN_ARGS
    return true;
}

// ------------------------------------------------------------------------
// Measurement aid: a pure read of `bytes` with the access pattern of the
// GEMM's weight stream (each wave walks its own contiguous region with
// 16-byte loads, DEPTH independent loads in flight).  It gives the HBM read
// rate the chip sustains for that pattern: the practical ceiling the GEMM is
// measured against.
// ------------------------------------------------------------------------
template <int DEPTH>
__global__ __launch_bounds__(512) void k_stream_read(const uint4* src, size_t n16_per_wave, unsigned* sink) {
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const uint4* p = src + wave * n16_per_wave + lane;
    unsigned acc = 0;
    for (size_t i = 0; i < n16_per_wave; i += 64 * DEPTH) {
        uint4 v[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) v[d] = p[i + (size_t)d * 64];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) acc ^= v[d].x ^ v[d].y ^ v[d].z ^ v[d].w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;      // practically never true; keeps the loads alive
}

extern "C" __attribute__((visibility("default"))) int ssd_debug_stream_read(const void* src, size_t bytes,
                                                                            int work_groups, int waves_per_wg,
                                                                            int depth, void* sink, void* stream) {
    if (!src || !sink || work_groups < 1 || waves_per_wg < 1 || waves_per_wg > 8) return SSD_EINVAL;
    const size_t waves = (size_t)work_groups * waves_per_wg;
    size_t per = bytes / 16 / waves;
    per -= per % (64 * 16);                      // whole unrolled steps for every depth
    if (per == 0) return SSD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if (depth == 16)
        k_stream_read<16><<<work_groups, waves_per_wg * 64, 0, st>>>((const uint4*)src, per, (unsigned*)sink);
    else if (depth == 8)
        k_stream_read<8><<<work_groups, waves_per_wg * 64, 0, st>>>((const uint4*)src, per, (unsigned*)sink);
    else if (depth == 4)
        k_stream_read<4><<<work_groups, waves_per_wg * 64, 0, st>>>((const uint4*)src, per, (unsigned*)sink);
    else
        return SSD_EINVAL;
    return hipGetLastError() == hipSuccess ? SSD_OK : SSD_EHIP;
}
