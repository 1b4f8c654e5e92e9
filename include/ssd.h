/*
 * ssd.h - C ABI of the MI355X (gfx950) hot path of Self Speculative Decoding
 * (SSD) for masked-diffusion language models.
 *
 * One call of ssd_verify_tree runs the paper's batched verification forward
 * (Section 3.2.4, Eq. 5): the greedy chain of N+1 candidate states of the
 * current block (Section 3.2.3) goes through the bidirectional transformer
 * f_theta (Section 3.1, Eq. 2) against a shared, exact prefix KV cache; a fused
 * LM-head reduction yields per masked position the arg-max token, its logit
 * and its softmax confidence (Section 3.2.2, Eq. 4); an acceptance kernel walks
 * the chain and keeps the longest draft prefix that greedy stepwise decoding
 * would have produced, plus the last valid node's own prediction, and reads
 * the next drafts off that node (Section 3.2.4; Algorithm 1).
 *
 * Conventions
 *   - Every function returns 0 (SSD_OK) or a negative SSD_E* code; nothing
 *     throws across this boundary.  ssd_strerror() names a code and
 *     ssd_last_error() gives the detail of the last failure on this ctx.
 *   - "device" pointers are HIP device memory owned by the caller; "host"
 *     pointers are ordinary host memory.  The library allocates no device
 *     memory: the caller hands in one workspace (ssd_workspace_bytes) that
 *     holds the KV cache, activations and partial results, and it must
 *     outlive the context.  Weights are borrowed read-only and must outlive
 *     the context too.
 *   - All arguments are validated on the host before any kernel is launched;
 *     a call that fails validation launches nothing.
 *   - Kernels run on the HIP stream given to ssd_create.  ssd_prefill_kv,
 *     ssd_draft and ssd_verify_tree are asynchronous: their outputs are device
 *     buffers that are valid once the stream has been synchronised.
 *     ssd_generate synchronises internally and writes host memory.
 *   - A context is not thread safe; calls on one context must not overlap.
 *
 * Model (all shapes from ssd_config): pre-norm transformer, RMSNorm (fp32
 * gain), rotary embedding with rotate-half pairing (i, i + head_dim/2),
 * grouped-query attention (query head h reads kv head h / (n_q_heads /
 * n_kv_heads)), SwiGLU feed-forward, untied LM head, no biases.  The mask
 * token (mask_id) is never predicted: it is excluded from max, arg-max and
 * the softmax sum.  Ties: lowest token id, lowest position.
 *
 * Attention scope (exact block-causal cache): a row of a node attends to the
 * cached prefix [0, pos0) of its sequence and to the rows of its own node,
 * never to other nodes and never to later blocks.
 */
#ifndef SSD_H
#define SSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SSD_OK        0
#define SSD_EINVAL   -1   /* bad argument (null pointer, inconsistent values)     */
#define SSD_ERANGE   -2   /* a size or index exceeds what the context was made for */
#define SSD_ENOMEM   -3   /* workspace too small                                  */
#define SSD_EHIP     -4   /* a HIP runtime call failed                            */
#define SSD_ESTATE   -5   /* call does not fit the cached prefix of the sequence  */

#define SSD_F32  0
#define SSD_BF16 1

#define SSD_MAX_BLOCK 64   /* a block's masked set is one 64-bit word; one lane per position */
#define SSD_MAX_DRAFT 15

typedef struct ssd_ctx ssd_ctx;   /* opaque */

typedef struct {
    int n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, mask_id;
                               /* d_model <= 8192, a multiple of 8; head_dim 64 or 128           */
    int dtype;                 /* SSD_F32 or SSD_BF16: type of weights, KV cache, GEMM operands */
    float rope_theta, rms_eps;
    int max_seqs;              /* sequence slots in the KV cache                               */
    int max_seq_len;           /* positions per sequence slot (prompt + generation)            */
    int block;                 /* largest block length B, <= SSD_MAX_BLOCK                     */
    int max_draft;             /* largest draft length N, <= SSD_MAX_DRAFT                     */
    int max_rows;              /* most rows in one forward: >= the longest prefill segment and
                                  >= max_seqs * (max_draft + 1) * block                        */
} ssd_config;

/* Device pointers.  Linear weights are row-major [out_features, in_features]
 * in cfg.dtype; norm gains are fp32 [d_model].  Arrays of per-layer pointers
 * are host arrays of n_layers device pointers (copied at ssd_create). */
typedef struct {
    const void* embed;               /* [vocab, d_model]                                   */
    const void* lm_head;             /* [vocab, d_model]                                   */
    const float* final_norm;         /* [d_model]                                          */
    const void* const* wqkv;         /* [(Hq + 2 Hkv) * dh, d_model]: Q heads, K heads, V heads */
    const void* const* wo;           /* [d_model, Hq * dh]                                 */
    const void* const* wgu;          /* [2 * d_ffn, d_model]: gate rows, then up rows      */
    const void* const* wdown;        /* [d_model, d_ffn]                                   */
    const float* const* norm1;       /* [d_model] gain before attention                   */
    const float* const* norm2;       /* [d_model] gain before the feed-forward            */
} ssd_weights;

/* Outputs of one decode forward, all device pointers, any may be NULL.
 * Row strides use the context's block and max_draft, whatever the call used. */
typedef struct {
    int32_t* n_accept;     /* [n]               tokens accepted, 1 .. n_draft+1              */
    int32_t* acc_pos;      /* [n, max_draft+1]  accepted positions within the block, in order */
    int32_t* acc_tok;      /* [n, max_draft+1]  accepted tokens                              */
    int32_t* n_next;       /* [n]               drafts for the next round                    */
    int32_t* next_pos;     /* [n, max_draft]    their positions, highest confidence first    */
    int32_t* next_tok;     /* [n, max_draft]    their tokens                                 */
    float*   row_maxlogit; /* [n, max_draft+1, block]  per node and position: max logit      */
    int32_t* row_argmax;   /* [n, max_draft+1, block]  arg-max token                         */
    float*   row_conf;     /* [n, max_draft+1, block]  softmax probability of the arg-max    */
} ssd_step_out;

typedef struct {
    int64_t forwards;          /* decode forwards (each accepts >= 1 token per live sequence) */
    int64_t kv_passes;         /* forwards that only append a finished segment's KV          */
    int64_t tokens;            /* generated tokens over all sequences                        */
    int64_t accept_hist[SSD_MAX_DRAFT + 2];   /* [a] = (sequence, forward) pairs accepting a */
    double  decode_ms;         /* stream time spent in decode forwards (HIP events)          */
    double  kv_ms;             /* stream time spent in KV passes, prompt prefill included    */
    double  total_ms;          /* wall time of the call                                      */
} ssd_stats;

/* Bytes of device workspace a context with this config needs (0 on a bad config). */
size_t ssd_workspace_bytes(const ssd_config* cfg);

/* Create a context.  `workspace` is device memory of at least ssd_workspace_bytes(cfg),
 * 256-byte aligned; `hip_stream` is a hipStream_t (NULL = the default stream).
 * bf16 weights are repacked into the workspace by kernels on `hip_stream`; the call first waits
 * for the device (hipDeviceSynchronize), so weights written on any stream of it are complete.
 * Errors: SSD_EINVAL (null / inconsistent config), SSD_ERANGE (block, draft,
 * d_model or head_dim beyond the supported limits), SSD_ENOMEM, SSD_EHIP. */
int ssd_create(const ssd_config* cfg, const ssd_weights* weights, void* workspace,
               size_t workspace_bytes, void* hip_stream, ssd_ctx** out);
int ssd_destroy(ssd_ctx* ctx);

/* Forget the cached prefix of sequence slot `seq` (length becomes 0). */
int ssd_reset(ssd_ctx* ctx, int seq);
/* Cached prefix length of a slot, or a negative error code. */
int ssd_cached_len(ssd_ctx* ctx, int seq);

/* Segment KV (Section 3.1: a finished segment's keys and values are final).
 * Runs tokens[0..n) (host) of sequence `seq` at positions [pos0, pos0+n): every
 * row attends to cache[0, pos0) and to all n rows; their keys (after rotary
 * embedding) and values are written to the cache, whose length becomes pos0+n.
 * pos0 must not exceed the current cached length (a smaller pos0 rewinds).
 * Errors: SSD_ERANGE (n > max_rows, pos0+n > max_seq_len, token id out of range). */
int ssd_prefill_kv(ssd_ctx* ctx, int seq, const int32_t* tokens, int n, int pos0);

/* Self-draft (Section 3.2.2, Eq. 4; the self-draft step of Algorithm 1): a one-node forward for
 * each listed sequence on its current block.  Accepts the stepwise choice (most
 * confident masked position) and returns up to n_draft_next drafts, the other
 * masked positions by descending confidence, always one fewer than remain
 * masked (see ssd_verify_tree).  Equivalent to ssd_verify_tree with no drafts.
 *   seqs      [n] host   sequence slots, distinct
 *   block_tok [n, cfg.block] host   tokens of the block (mask_id where masked)
 *   masked    [n] host   bit p set = position p is masked; bits >= block_len clear
 *   pos0      [n] host   absolute position of the block = cached prefix length
 *   block_len [n] host   or NULL (= cfg.block)
 */
int ssd_draft(ssd_ctx* ctx, int n, const int* seqs, const int32_t* block_tok,
              const uint64_t* masked, const int* pos0, const int* block_len,
              int n_draft_next, const ssd_step_out* out);

/* Hierarchical verification (Sections 3.2.3-3.2.4, Eq. 5): builds, for each
 * listed sequence, the chain of n_draft[i]+1 nodes (node j = block state with
 * drafts 1..j written in), runs all nodes of all sequences in one forward,
 * and accepts per sequence the longest prefix of drafts such that draft j+1
 * equals (position and token) node j's stepwise choice, plus the choice of the
 * node where the walk stops.  Next drafts: that node's remaining masked
 * positions by descending confidence, at most n_draft_next and at most one
 * fewer than remain masked (so the next leaf still has a position to predict).
 *   draft_pos, draft_tok [n, cfg.max_draft] host   drafts in priority order
 *   n_draft   [n] host   0 .. min(max_draft, popcount(masked)-1)
 * Draft positions must be distinct, masked and < block_len.
 * The accepted tokens are also committed to the context's device-side block
 * state (used by ssd_generate); the caller's host arrays are not modified. */
int ssd_verify_tree(ssd_ctx* ctx, int n, const int* seqs, const int32_t* block_tok,
                    const uint64_t* masked, const int* pos0, const int* block_len,
                    const int32_t* draft_pos, const int32_t* draft_tok, const int* n_draft,
                    int n_draft_next, const ssd_step_out* out);

/* Algorithm 1 end to end for n sequences (slots 0..n-1): prefill each prompt,
 * then per block: self-draft, verify/accept rounds until the block is full,
 * append the block's KV.  draft_depth = 0 is greedy stepwise decoding (one
 * token per forward), the result SSD reproduces token for token (Abstract).
 *   prompts     [n] host pointers to prompt_len[i] token ids
 *   out_tokens  [n, gen_len] host
 *   stats       host, may be NULL
 */
int ssd_generate(ssd_ctx* ctx, int n, const int32_t* const* prompts, const int* prompt_len,
                 int gen_len, int block, int draft_depth, int32_t* out_tokens, ssd_stats* stats);

/* Kernel selection: 0 = plain FMA kernels (any dtype), 1 = MFMA kernels where
 * available (bf16), the rotary stage fused into the attention kernel where the
 * forward's shape allows, 2 = as 1 with the rotary stage always a kernel of
 * its own (same results; for measurement).  Default 1.  Returns the previous
 * value or an error. */
int ssd_set_kernel_path(ssd_ctx* ctx, int path);

/* Block-boundary fusion in ssd_generate (Section 3.1: blocks are decoded in
 * order, each against the cache of all earlier ones): 1 = the KV append of a
 * finished block and the block-start draft of the next block share one
 * forward (one weight pass instead of two per block), 0 = separate forwards.
 * The generated tokens are the same either way.  Default 1.  Returns the
 * previous value or an error. */
int ssd_set_boundary_fusion(ssd_ctx* ctx, int on);

/* A round across the block boundary in ssd_generate (Section 3.2.2: once fewer than N positions
 * remain in the current block, candidates come from the next block).  1 = while a next block
 * exists the drafts may cover every remaining position of the current block; the chain's leaf
 * then holds the finished block, and the same forward runs the next block, all masked, behind it.
 * If every draft verifies, the block is finished, its KV stays in the cache, and the next block
 * starts with one token and its drafts: the boundary costs no forward of its own.  Otherwise the
 * round ends like any other.  Needs max_rows >= (draft_depth + 2) * block rows per sequence to
 * take effect; greedy chain only.  The generated tokens are the same.  Default 0.  Returns the
 * previous value or an error. */
int ssd_set_cross_block(ssd_ctx* ctx, int on);

/* Cache of the paper's experiments (Section 4.1: the prefix and suffix cache, refreshed every fixed
 * number of decoded tokens).  mode 0 (default) = the exact block-causal prefix cache: a block sees
 * the prompt, the finished blocks and itself.  mode 1 = dual cache: a refresh is one forward over
 * the WHOLE sequence (prompt, decoded tokens, every still masked position up to the generation
 * length) with full bidirectional attention; it renews the keys and values of all positions and is
 * itself the decoding step of that moment.  Between refreshes only the current block is computed,
 * against the cached keys and values of all other positions, before and behind it.  ssd_generate
 * refreshes at the start and whenever refresh_interval tokens have been decoded since the last
 * refresh (0 = the block length); a chain never carries more drafts than fit before the next
 * refresh, so SSD and stepwise decoding (draft_depth 0) refresh at the same states and generate the
 * same tokens.  Needs max_rows >= the sum of prompt + generation lengths of the sequences decoded
 * together.  In mode 1 ssd_generate uses the greedy chain inside the block (tree mode, boundary
 * fusion and cross-block rounds do not apply); stats.kv_passes counts the refreshes, each of which
 * is also counted in stats.forwards.  Returns the previous mode or an error. */
int ssd_set_cache_mode(ssd_ctx* ctx, int mode, int refresh_interval);

/* Spill-over selection in ssd_generate with the dual cache (Section 3.2.2: once the current block has fewer
 * positions left than the draft length, further candidates come from the next block).  1 = while a next block
 * exists the chain may hold drafts for every remaining position of the current block and then goes on in the
 * next block: that block all masked, then with its drafts written in, in the same forward (between refreshes a
 * block sees all other positions through the cache, so those are the states stepwise decoding reaches once the
 * current block is complete).  The next block's drafts, and those of any block nobody has predicted yet, are
 * its positions by descending confidence of the last refresh, whose forward covers every masked position: a
 * block then starts with a full chain instead of a one-node forward.  A round still never decodes past the
 * next refresh, so the generated tokens are those of stepwise decoding; at most one block boundary per round.
 * Only with cache mode 1 and the greedy chain; the step calls (ssd_refresh_kv, ssd_verify_tree) are not
 * affected.  Default 0.  Returns the previous value or an error. */
int ssd_set_spill_over(ssd_ctx* ctx, int on);

/* One cache refresh of the dual cache (Section 4.1) for sequence `seq`, as a call of its own:
 * tokens[0..total_len) (host) is the whole sequence, mask id at every position not decoded yet;
 * the current block is [pos0, pos0 + block_len) and must hold at least one mask.  Runs all
 * total_len rows with full bidirectional attention, writes every position's keys and values to the
 * cache, and treats the block's rows like ssd_draft does: per-row outputs, the stepwise choice and
 * n_draft_next next drafts go to `out` (slot 0) and to the sequence's device state.  Afterwards the
 * slot's prefix length is pos0 and positions [pos0 + block_len, total_len) count as cached suffix:
 * ssd_draft / ssd_verify_tree on this block (pos0 unchanged) attend to both.  ssd_prefill_kv and
 * ssd_reset drop the suffix again.  Asynchronous.  Errors: SSD_ERANGE (total_len > max_rows or
 * max_seq_len, block outside the sequence, token id out of range), SSD_EINVAL (no mask in the block). */
int ssd_refresh_kv(ssd_ctx* ctx, int seq, const int32_t* tokens, int total_len, int pos0, int block_len,
                   int n_draft_next, const ssd_step_out* out);

/* Acceptance-rate limit of self-drafting (Section 5.1, the procedure behind Table 2), an analysis
 * call.  Decodes prompt (host, prompt_len tokens) stepwise in sequence slot 0 with the exact prefix
 * cache: gen_len tokens in blocks of `block`.  The steps are cut into rounds of n_draft + 1 (a new
 * round at every block start); the logits of a round's first forward are kept, and every token the
 * round decodes is ranked in them at its position (tokens with a higher logit, or an equal logit and
 * a lower id, are ahead; the mask token is no candidate).  For k = 1 .. k_max (host arrays of k_max
 * entries): matched[k-1] = tokens with rank < k, i.e. found among the k best candidates a draft made
 * at the round's start would hold; forwards[k-1] = sum over rounds of (steps - matched + 1), the
 * forwards an ideal verification tree would need; 1 - forwards / gen_len is the table's reduction,
 * n_draft / (n_draft + 1) its upper bound; reduction[k-1] (optional, host, k_max entries) receives
 * 1 - forwards[k-1] / gen_len.  *rounds (optional) = number of rounds; out_tokens (optional, host,
 * gen_len entries) = the decoded tokens.  Synchronous.  Errors as ssd_generate. */
int ssd_acceptance_limit(ssd_ctx* ctx, const int32_t* prompt, int prompt_len, int gen_len, int block, int n_draft,
                         int k_max, int32_t* out_tokens, int64_t* matched, int64_t* forwards, int64_t* rounds,
                         double* reduction);

/* Shape of the verification tree of ssd_verify_tree / ssd_generate:
 * 0 = the greedy chain of n_draft + 1 nodes (Section 3.2.3), 1 = the mix-order
 * tree (Section 5.2, Table 3): the chain plus, for every chain node but the last
 * two, a node that skips the next draft and holds the one after it, 2 * n_draft
 * nodes in all.  When a chain node's stepwise choice is the draft after the
 * expected one (same candidates, different order) that draft is accepted and
 * the extra node supplies one more token.  A forward then has up to
 * 2 * n_draft * block rows per sequence: max_rows must allow for it.  The
 * per-row debug outputs of ssd_step_out cover the chain nodes only.  The
 * generated tokens are the same in both modes.  Default 0.  Returns the
 * previous value or an error. */
int ssd_set_tree_mode(ssd_ctx* ctx, int mode);

/* HIP graphs: 1 = the kernel sequence of a forward is captured the second time
 * a launch shape (row count, node count, block length) occurs and replayed from
 * then on; 0 = every forward launches its kernels one by one.  Results are the
 * same; a context keeps at most 64 graphs and runs further shapes ungraphed,
 * as it does every forward of a context on the default (NULL) stream, which
 * cannot be captured.  Default 0: on MI355X a replayed graph of the ~270 dependent
 * kernels of an 8B forward took the same time as launching them one by one (the
 * host stays ahead of the GPU either way).  Returns the previous value or an error. */
int ssd_set_graphs(ssd_ctx* ctx, int on);

/* Per-kernel-class timing with HIP events on the context's stream.
 * ssd_profile_begin() turns it on and clears the counters; ssd_profile_read()
 * synchronises the stream and fills, for class c < *n_classes: launches[c],
 * ms[c] (summed event time) and names[c] (static strings).  On return
 * *n_classes is the number of classes.  Profiling serialises launches; it is
 * meant for measurement runs only.  ssd_profile_end() turns it off. */
int ssd_profile_begin(ssd_ctx* ctx);
int ssd_profile_read(ssd_ctx* ctx, int* n_classes, const char** names, int64_t* launches, double* ms);
int ssd_profile_end(ssd_ctx* ctx);

const char* ssd_strerror(int code);
const char* ssd_last_error(const ssd_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* SSD_H */
