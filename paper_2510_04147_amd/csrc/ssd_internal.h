// Internal declarations shared by the host driver and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/ssd.h"

#define SSD_MAX_SEQS 16
// per sequence: the largest tree (2 * draft length nodes with mix order) plus a KV-append node
#define SSD_MAX_NODES (SSD_MAX_SEQS * (2 * SSD_MAX_DRAFT + 1))
// per sequence: a block's chain, the next block behind its leaf or a KV append; a cache refresh's segments (the
// block, the positions behind it whose predictions are kept, the rest behind, everything before)
#define SSD_MAX_GROUPS (4 * SSD_MAX_SEQS)
#define SSD_MAX_SPLIT 8

// ---- forward descriptor (host-built, copied to the device before each forward)
enum GroupMode : int {
    GM_DECODE = 0,   // chain of nodes from the device-side block state; logits + acceptance
    GM_APPEND = 1,   // one node = the finished block from the block state; writes KV
    GM_RAW = 2,      // one node of raw tokens (prompt prefill); writes KV
};

struct GroupDesc {
    int seq, row0, blen, S;
    int n_nodes, mode, raw_off, n_draft_next;
    int fresh;      // GM_DECODE: block starts now, state = all masked, no drafts
    int out_off;    // GM_APPEND: offset into the device token output, or -1
    int node0;      // index of the group's first node
    int n_chain;    // GM_DECODE: nodes 0 .. n_chain-1 are the chain, the rest mix-order nodes
    // A round that reaches across the block boundary (Section 3.2.2): the chain's drafts cover every
    // masked position, so its leaf holds the finished block (and writes its KV); group spec_next1 - 1
    // evaluates the next block behind that leaf.  0 = none.  The speculative group has spec_of1 =
    // its master's index + 1 and is handled by the master's work-group of the acceptance kernel.
    int spec_next1, spec_of1;
    int allow_full; // next drafts may cover every remaining masked position (a next block exists)
    // Spill-over with the dual cache (Section 3.2.2 + Section 4.1).  from_refresh: the block is all masked and
    // nobody has predicted it yet; its drafts are its positions by descending confidence of the last refresh
    // (ref_conf / ref_arg), n_chain - 1 of them (n_chain if leafless).  leafless: the chain's drafts cover every
    // masked position and the node holding all of them is left out (between refreshes nothing reads it).
    // keep_ref (a raw group of a refresh): the rows' predictions are kept as that refresh's drafts.
    int from_refresh, leafless, keep_ref;
    int pad[2];
};

struct NodeDesc {
    int seq, row0, blen, S;
    int group, j;   // j = number of leading drafts written in (= the node's index along the chain)
    int extra;      // mix-order node: index of the one further draft written in (j + 1), else -1
    int write_kv;
    int vrow0;      // 64-aligned start of the node's rows in the own-key / own-value buffers
    int T;          // dual cache (Section 4.1): positions [S + blen, T) are cached too and visible; 0 = prefix only
};

struct FwdHeader {
    int n_groups, n_nodes, M, M_logits;
    ssd_step_out out;            // where the acceptance kernel writes a step call's outputs (null pointers: nowhere)
    GroupDesc groups[SSD_MAX_GROUPS];
    NodeDesc nodes[SSD_MAX_NODES];
};

// Device-side block state of one sequence slot (Algorithm 1's x restricted to
// the current block, its masked set, and the drafts d for the next round).
struct SeqState {
    unsigned long long masked;
    int n_draft;
    int pad;
    int tok[SSD_MAX_BLOCK];
    int draft_pos[SSD_MAX_DRAFT + 1];
    int draft_tok[SSD_MAX_DRAFT + 1];
};

// Per-forward results of the acceptance kernel (device), mirrored to the host
// by ssd_generate.
struct StepResult {
    int n_accept, n_next;
    int completed;  // the round verified drafts for every masked position: the block is finished (exact cache: and its KV cached)
    int n_in_next;  // of the accepted tokens, those that lie in the next block (their acc_pos count on from this block's length)
    int acc_pos[SSD_MAX_DRAFT + 1], acc_tok[SSD_MAX_DRAFT + 1];
    int next_pos[SSD_MAX_DRAFT + 1], next_tok[SSD_MAX_DRAFT + 1];
};

// ---- kernel classes for profiling
enum KClass : int {
    KC_ROWS = 0, KC_NORM, KC_GEMM_QKV, KC_ROPE, KC_ATTN, KC_GEMM_O, KC_GEMM_GU, KC_GEMM_DOWN,
    KC_LMHEAD, KC_LMMERGE, KC_ACCEPT, KC_COUNT
};

struct Dims {
    int L, d, Hq, Hkv, dh, F, V, mask_id, dtype;
    float eps;
    int max_seqs, max_seq_len, block, max_draft, max_rows;
    int nq() const { return Hq * dh; }
    int nkv() const { return Hkv * dh; }
    int nqkv() const { return (Hq + 2 * Hkv) * dh; }
    size_t esz() const { return dtype == SSD_F32 ? 4 : 2; }
    // positions allocated per cache slot: whole 64-position tiles, so tile loads stay in bounds
    int seq_stride() const { return (max_seq_len + 63) & ~63; }
    // most nodes one forward of this context can hold
    int max_nodes() const {
        const int tree = 2 * max_draft > max_draft + 1 ? 2 * max_draft : max_draft + 1;
        return max_seqs * (tree + 1 > 4 ? tree + 1 : 4);           // a cache refresh takes up to four nodes
    }
    // rows of the own-key / own-value buffers: every node starts on a 64-row boundary
    int vt_rows() const { return ((max_rows + 63) & ~63) + 64 * max_nodes(); }
};

// Keys and values, cached or of the forward's own rows, are stored per KV head in the order the
// attention kernel's matrix instructions consume them, so that a wave fetches each operand
// fragment as one contiguous 64 x 8 element piece.  Position p, head channel c, head size dh:
//   keys:   [p/32][c/16][lane = (c/8 % 2)*32 + p%32][c%8]
//           (fragment ks = c/16 of S^T = K Q^T: lane (p%32, half) holds 8 consecutive channels);
//   values: [p/32][c/32][p/16 % 2][lane = (p/4 % 2)*32 + c%32][(p/8 % 2)*4 + p%4]
//           (fragment of O^T = V^T P^T: lane (c%32, half) holds the 8 keys whose probabilities
//           the same lane half holds after the S^T product).
// A head's region of n positions (n a multiple of 32) holds n*dh elements in either order.
// Rotary embedding of one (x1, x2) = (channel i, channel i + dh/2) pair, with the roundings spelled
// out so that every kernel that applies it produces the same bits.
__device__ __forceinline__ void rope_pair(float x1, float x2, float c, float sn, float& o1, float& o2) {
    o1 = __fmaf_rn(x1, c, -__fmul_rn(x2, sn));
    o2 = __fmaf_rn(x2, c, __fmul_rn(x1, sn));
}

__host__ __device__ inline size_t kfrag_off(int p, int c, int dh) {
    return ((((size_t)(p >> 5) * (dh >> 4) + (c >> 4)) * 64 + ((c >> 3) & 1) * 32 + (p & 31)) << 3) + (c & 7);
}
__host__ __device__ inline size_t vfrag_off(int p, int c, int dh) {
    return (((((size_t)(p >> 5) * (dh >> 5) + (c >> 5)) * 2 + ((p >> 4) & 1)) * 64 + ((p >> 2) & 1) * 32 + (c & 31)) << 3) +
           ((p >> 3) & 1) * 4 + (p & 3);
}

// Workspace carve-up (all device pointers into the caller's workspace).
struct Buffers {
    float* h;            // [max_rows, d] residual stream, fp32
    void* xn;            // [max_rows, d] normed rows, T
    void* q;             // [max_rows, nq] T, after rotary
    void* kown;          // [Hkv][vt_rows * dh] T: the nodes' own keys after rotary, fragment order (kfrag_off)
    void* vown;          // [Hkv][vt_rows * dh] T: the nodes' own values, fragment order (vfrag_off)
    void* attn;          // [max_rows, nq] T
    void* act;           // [max_rows, F] T
    float* part;         // [SSD_MAX_SPLIT, max_rows, max(d, nqkv)] fp32 split-K partial sums of the
                         // QKV, O and down projections (summed in order by the consumer)
    void* packed;        // fragment-order copies of the weights (bf16 models)
    float* lm_part;      // [max_rows, n_vtiles, 3] (max, arg as float bits, sumexp)
    float* row_max;      // [max_rows]
    int* row_arg;        // [max_rows]
    float* row_conf;     // [max_rows]
    int* row_tok;        // [max_rows]
    int* row_pos;        // [max_rows]
    int* row_node;       // [max_rows]
    int* raw_tok;        // [max_rows]
    void* kcache;        // [L][max_seqs][Hkv][seq_stride * dh] T, keys after rotary, fragment order
    void* vcache;        // [L][max_seqs][Hkv][seq_stride * dh] T, values, fragment order
    float* rope_cos;     // [max_seq_len, dh/2]
    float* rope_sin;
    FwdHeader* fwd;      // device copy of the descriptor
    SeqState* state;     // [max_seqs]
    StepResult* result;  // [max_seqs]
    int* out_tok;        // [max_seqs, max_seq_len] device token output of ssd_generate
    float* ref_conf;     // [max_seqs, max_seq_len] confidence per position at the sequence's last cache refresh
    int* ref_arg;        // [max_seqs, max_seq_len] arg-max token per position at that refresh
    float* probe_logits; // [block, V] logits of a round's first forward (ssd_acceptance_limit)
    int* probe_rank;     // [SSD_MAX_DRAFT + 1]
    int lm_tiles;        // vocab tiles of the LM-head reduction
};

// A linear weight: the caller's row-major [N, K] matrix and, for bf16 models
// whose shape allows it, the library's copy in MFMA fragment order.
struct Wt {
    const void* raw;
    const void* packed;
    int N, K;
};

struct LayerW {
    Wt wqkv, wo, wgu, wdown;
    const float *norm1, *norm2;
};

struct ssd_ctx {
    Dims dm;
    Buffers b;
    std::vector<LayerW> lw;
    const void* embed;
    Wt lm_head;
    const float* final_norm;
    int part_cols;             // columns of one split-K partial buffer = max(d, nqkv)
    hipStream_t stream;
    int device;                // HIP device the context was created on
    int kernel_path;
    int fuse_boundary;   // ssd_generate: KV append + next block's draft in one forward
    int tree_mode;       // 0 = greedy chain (Section 3.2.3), 1 = mix-order tree (Section 5.2)
    int cross_block;     // ssd_generate: the last round of a block may reach into the next block (Section 3.2.2)
    int spill_over;      // ssd_generate with the dual cache: the chain continues into the next block (Section 3.2.2)
    // HIP graphs of the forward's kernel sequence, one per launch shape.  Everything that changes
    // between forwards of one shape (tokens, prefix lengths, drafts, output pointers) lives in
    // device memory, so a shape's second forward is captured and later ones replay the graph.
    int use_graphs;
    struct FwdGraph {
        int M, ML, n_nodes, n_groups, max_blen, kernel_path;
        int flags;       // bit 0: some node appends KV, bit 1: some node reads a cached suffix (other kernels)
        int seen;
        hipGraphExec_t exec;
    };
    std::vector<FwdGraph> graphs;
    // Cache of the paper's experiments (Section 4.1), 0 = exact block-causal prefix cache: 1 = dual
    // cache, keys and values of ALL positions renewed by a full forward every refresh_interval
    // decoded tokens (0 = once per block).  total_len[seq] > 0: positions up to there are cached.
    int cache_mode, refresh_interval;
    int total_len[SSD_MAX_SEQS];
    int cached_len[SSD_MAX_SEQS];
    // host staging ring for descriptors / small uploads
    static const int kSlots = 4;
    char* stage[kSlots];
    hipEvent_t stage_ev[kSlots];
    bool stage_used[kSlots];
    int stage_next;
    size_t stage_bytes;
    StepResult* host_result;   // pinned
    // profiling
    bool profiling;
    std::vector<hipEvent_t> ev_pool;
    std::vector<int> ev_class;
    size_t ev_used;
    double prof_ms[KC_COUNT];
    long long prof_n[KC_COUNT];
    std::string err;
};

// ---- launchers implemented in the kernel files (all asynchronous on `st`)
// T-typed buffers are passed as void* with the dtype flag.
void launch_build_rows(const ssd_ctx* c, hipStream_t st, int n_nodes);
void launch_embed(const ssd_ctx* c, int M, hipStream_t st);
void launch_norm(const ssd_ctx* c, int M, const float* gain, int n_part, hipStream_t st);
// gate_rows > 0: the matrix is gate rows then up rows; interleave them per 16 channels
void launch_pack_weights(const void* src, void* dst, int N, int K, int gate_rows, hipStream_t st);
void launch_rope(const ssd_ctx* c, int n_nodes, int max_blen, int layer, int n_part, hipStream_t st);
void launch_attn_plain(const ssd_ctx* c, int M, int layer, hipStream_t st);
void launch_accept(const ssd_ctx* c, int n_groups, hipStream_t st);
void launch_lm_merge(const ssd_ctx* c, int M, int n_tiles, hipStream_t st);
// the same merge on caller-chosen buffers: part [M, n_tiles, 3] -> row_max / row_arg / row_conf [M]
void launch_lm_merge_to(const ssd_ctx* c, int M, int n_tiles, const float* part, float* row_max, int* row_arg,
                        float* row_conf, hipStream_t st);
int lm_tiles_plain(int V);
// out[M,N] = sum over the first n_part split-K partial buffers, in split order
void launch_sum_partials(const ssd_ctx* c, int M, int N, int n_part, float* out, hipStream_t st);
void launch_int_to_float(const int* src, float* dst, int n, hipStream_t st);
// kernel-level entry points: caller-supplied keys / values into the cache; a forward's own keys / values back out
void launch_write_cache(const ssd_ctx* c, int seq, int layer, int pos0, int n, const void* k, const void* v, hipStream_t st);
void launch_read_own_kv(const ssd_ctx* c, int M, void* k, void* v, hipStream_t st);
// rank[i] = number of tokens ahead of tok[i] in row pos[i] of logits [*, V]: higher logit, or equal and
// lower id; the mask token never counts
struct RankPairs { int n; int pos[SSD_MAX_DRAFT + 1]; int tok[SSD_MAX_DRAFT + 1]; };
void launch_token_rank(const float* logits, int V, int mask_id, const RankPairs& pairs, int* rank, hipStream_t st);

enum GemmEpi : int { EPI_F32 = 0, EPI_SWIGLU = 1, EPI_LMHEAD = 2 };
// out[M,N] = X[M,K] * W[N,K]^T with the plain FMA kernel.
void launch_gemm_plain(const ssd_ctx* c, int epi, const void* X, const void* W, void* out, int M, int N, int K,
                       hipStream_t st);

// MFMA path (bf16 only).  Return false if the shape is not supported.
bool launch_gemm_mfma(const ssd_ctx* c, int epi, const void* X, const Wt& W, void* out, int M, int* n_split,
                      hipStream_t st);
int lm_tiles_mfma(int V);
// the fp32-partial-sum GEMMs (QKV, attention output, down), instantiated in a translation unit of their own;
// mt row tiles of 32 rows per pass, m_chunks passes
bool launch_gemm_mfma_f32(const ssd_ctx* c, const uint16_t* x, const uint4* wp, void* out, int M, int N, int K, int mt,
                          int m_chunks, int* n_split, hipStream_t st);
// n_part >= 0: the kernel also sums the QKV projection's n_part partial sums and applies the rotary
// embedding itself (nodes of at most 32 rows, head size 128, no cache append); n_part < 0: q / kown / vown are ready
// suffix: some node of the forward sees cached positions behind its block (NodeDesc::T)
// nodes_per_seq: nodes of every sequence of the forward if all have equally many (consecutive in the node list), else 0
bool launch_attn_mfma(const ssd_ctx* c, int n_nodes, int nodes_per_seq, int max_blen, int layer, int n_part, bool suffix,
                      hipStream_t st);
bool attn_mfma_can_fuse_rope(const ssd_ctx* c, int max_blen);
