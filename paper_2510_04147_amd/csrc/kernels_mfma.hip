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
#include "gemm_mfma.h"

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

int lm_tiles_mfma(int V) { return V / 32; }

bool launch_gemm_mfma(const ssd_ctx* c, int epi, const void* X, const Wt& W, void* out, int M, int* n_split,
                      hipStream_t st) {
    if (!W.packed) return false;
    const int N = W.N, K = W.K;
    constexpr int WK = 2, KC = WK * 32;
    if (K % KC) return false;
    // rows per pass: 32 ... 192 in steps of 32; forwards with more rows re-stream the weights once per pass,
    // in passes of 160 or 192 rows, whichever needs fewer.  The rows of a pass share nothing but the weight
    // fragments, so a row's sums do not depend on the choice.
    int mt = (M + 31) / 32;
    if (mt > 6) mt = (M + 191) / 192 < (M + 159) / 160 ? 6 : 5;
    const int rows = mt * 32, m_chunks = (M + rows - 1) / rows;
    const bf16_t* x = (const bf16_t*)X;
    const uint4* wp = (const uint4*)W.packed;
    GemmArgs a{K / KC, mt, x, wp, out, M, N, K, 1, 0, -1, 0, m_chunks, st};
    if (epi == EPI_SWIGLU) {
        // W = [2F, d] packed with gate and up rows interleaved per 16 channels: N/32 tiles of 16
        // channels each, any number of them per work-group; 96-row n-blocks give the 8B shape
        // (768 tiles) exactly one work-group per CU
        *n_split = 1;
        return (N / 32) % 3 == 0 ? gemm_swiglu_wn3(a) : gemm_swiglu_wn4(a);
    }
    if (epi == EPI_LMHEAD) {
        *n_split = lm_tiles_mfma(N);
        a.mask_id = c->dm.mask_id;
        a.n_tiles_out = N / 32;
        return gemm_lmhead_wn4(a);
    }
    return launch_gemm_mfma_f32(c, x, wp, out, M, N, K, mt, m_chunks, n_split, st);
}

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
                                                               const float* __restrict__ sinT, int nodes_per_seq) {
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
    // Work-groups go to the 8 XCDs round-robin by their linear id, and every XCD has an L2 of its own.
    // The (node, query head) pairs that read the same keys and values form a class: the nodes of one
    // sequence (nodes_per_seq consecutive nodes; 0: all nodes of the launch) times the query heads of one
    // KV head.  Whole classes are placed on one XCD, so a sequence's prefix crosses the fabric once per
    // KV head and the other members of the class hit in that L2.  Needs a class count divisible by 8;
    // otherwise the plain order.
    const int n_nodes = gridDim.x / Hq, G = Hq / Hkv;
    const int nps = nodes_per_seq > 0 ? nodes_per_seq : n_nodes;
    const int n_classes = (n_nodes / nps) * Hkv, members = nps * G;
    int node, head;
    if (n_classes % 8 == 0) {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int cls = (slot / members) * 8 + xcd, mem = slot % members;
        node = (cls / Hkv) * nps + mem % nps;
        head = (cls % Hkv) * G + mem / nps;
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
        const float corr = fast_exp(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        bf16x8 pf[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = fast_exp(sacc[i] - m_new);                  // 0 for masked keys
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
        cw[w] = mw == -INFINITY ? 0.f : fast_exp(mw - m_all);            // a wave without a tile counts for nothing
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

bool launch_attn_mfma(const ssd_ctx* c, int n_nodes, int nodes_per_seq, int max_blen, int layer, int n_part, bool suffix,
                      hipStream_t st) {
    if (nodes_per_seq <= 0 || n_nodes % nodes_per_seq) nodes_per_seq = 0;
    const Dims& d = c->dm;
    dim3 grid(n_nodes * d.Hq, (max_blen + 31) / 32);
    const float scale = 1.0f / sqrtf((float)d.dh);
    const size_t ps = (size_t)d.max_rows * c->part_cols;
#define SSD_ATTN_ARGS                                                                                                  \
    c->b.fwd, (const bf16_t*)c->b.q, (const bf16_t*)c->b.kown, (const bf16_t*)c->b.vown, (const bf16_t*)c->b.kcache, \
        (const bf16_t*)c->b.vcache, (bf16_t*)c->b.attn, d.Hq, d.Hkv, layer, d.max_seqs, d.seq_stride(), d.vt_rows(), scale, \
        c->b.part, n_part, ps, c->b.rope_cos, c->b.rope_sin, nodes_per_seq
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
