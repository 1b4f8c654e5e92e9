/*
 * ssd_kernels.h - kernel-level entry points of the SSD library, for unit
 * parity tests.  They run exactly the kernels the forward
 * (ssd.h) runs for one step of Section 3.1's transformer f_theta, on operands
 * the caller supplies, so a single step can be checked against a definition
 * with nothing upstream to blur it.
 */
#ifndef SSD_KERNELS_H
#define SSD_KERNELS_H

#include "ssd.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SSD_LIN_QKV  0   /* x [M, d_model]      -> out fp32 [M, (Hq+2Hkv)*dh]                  */
#define SSD_LIN_O    1   /* x [M, Hq*dh]        -> out fp32 [M, d_model]                        */
#define SSD_LIN_GU   2   /* x [M, d_model]      -> out cfg.dtype [M, d_ffn] = silu(gate)*up     */
#define SSD_LIN_DOWN 3   /* x [M, d_ffn]        -> out fp32 [M, d_model]                        */
#define SSD_LIN_LM   4   /* x [M, d_model]      -> out fp32 [3, M]: max logit, arg-max (as float), confidence */

/* One linear step of layer `layer` (ignored for SSD_LIN_LM) with the kernel path the context
 * currently selects: x and out are device pointers, x in cfg.dtype, row-major, M <= max_rows.
 * Split-K partial sums are added in split order, as the forward's consumers do.
 * Asynchronous on the context's stream.  Errors: SSD_EINVAL, SSD_ERANGE. */
int ssd_k_linear(ssd_ctx* ctx, int which, int layer, const void* x, int M, void* out);

/* One node of a kernel-level attention call: rows [sum of earlier blen, +blen) of the call belong to
 * sequence slot `seq`, sit at positions [S, S + blen) and attend to the slot's cached positions
 * [0, S), to their own node's rows and, if T > S + blen, to the cached positions [S + blen, T)
 * (the dual cache of Section 4.1); T = 0: no cached suffix. */
typedef struct { int seq, S, blen, T; } ssd_k_node;

/* Writes caller-supplied keys and values into the cache of sequence slot `seq`, layer `layer`, at
 * positions [pos0, pos0 + n): k, v device, cfg.dtype, row-major [n, n_kv_heads, head_dim], keys
 * already rotated.  The slot's cached length (ssd_cached_len) is not changed: the kernel-level
 * attention call names the prefix length itself.  Asynchronous.  Errors: SSD_EINVAL, SSD_ERANGE. */
int ssd_k_write_cache(ssd_ctx* ctx, int seq, int layer, int pos0, int n, const void* k, const void* v);

/* The attention step of layer `layer` (Section 3.1's f_theta restricted to the scope of Eq. 5: cached
 * prefix + the node's own rows, bidirectional) with exactly the kernels the forward runs, on a
 * caller-supplied QKV projection: qkv device fp32 [n_part, M, (Hq + 2 Hkv) * dh], the projection's
 * split-K partial sums (added in split order; n_part = 1: the projection itself), M = sum of the
 * nodes' blen, `nodes` a host array.  fused = 0: the rotary stage runs as a kernel of its own, then
 * the attention kernel of the context's kernel path; out_q (cfg.dtype [M, Hq * dh]) and out_k / out_v
 * (cfg.dtype [M, Hkv, dh]; both or neither) optionally receive the rotary stage's outputs, i.e. the
 * attention kernel's operands.  fused = 1: the attention kernel sums, rotates and converts itself
 * (bf16, kernel path 1, head size 128, nodes of at most 32 rows; out_q / out_k / out_v must be
 * NULL).  out_attn: cfg.dtype [M, Hq * dh].  Nothing is appended to the cache.  Asynchronous.
 * Errors: SSD_EINVAL, SSD_ERANGE. */
int ssd_k_attention(ssd_ctx* ctx, int layer, int n_nodes, const ssd_k_node* nodes, const float* qkv, int n_part,
                    int fused, void* out_attn, void* out_q, void* out_k, void* out_v);

/* The residual + RMSNorm step (Section 3.1's f_theta): h (device fp32 [M, d_model], in and out) += the
 * n_part split-K partial sums `partials` (device fp32 [n_part, M, d_model], added in order; n_part may be
 * 0), then out (cfg.dtype [M, d_model]) = h / sqrt(mean(h^2) + rms_eps) * gain (device fp32 [d_model]).
 * Asynchronous.  Errors: SSD_EINVAL, SSD_ERANGE. */
int ssd_k_norm(ssd_ctx* ctx, float* h, const float* partials, int n_part, const float* gain, int M, void* out);

/* SSD_LIN_LM of ssd_k_linear for callers that cannot allocate device memory or hand over a region
 * for partial results of their own: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  The per-tile partial results of the LM-head reduction and the integer
 * arg-max live in a static device array of SSD_STATIC_SCRATCH_BYTES that each GPU the library runs
 * on holds until the process ends (its address is resolved once per device in ssd_create); the call
 * itself allocates nothing and uses nothing of the context's workspace but the weights.
 *   x   device, cfg.dtype [M, d_model], row-major        out  device, fp32 [3, M] as for SSD_LIN_LM
 * Same kernels, same results as ssd_k_linear(ctx, SSD_LIN_LM, 0, x, M, out).  M * ceil(vocab / 32)
 * * 12 + M * 4 bytes must fit the array (M <= 176 for a 126464-token vocabulary), else SSD_ERANGE and
 * nothing is launched.  Nothing in the array has to start at zero: every entry that is read was
 * written by the same call.  All calls on one GPU share that GPU's array, from every context and
 * stream: calls that overlap in time on one GPU race; on one stream they are ordered.
 * Asynchronous on the context's stream.  Errors: SSD_EINVAL, SSD_ERANGE, SSD_EHIP. */
#define SSD_STATIC_SCRATCH_BYTES (8u << 20)
int ssd_k_lm_head_static(ssd_ctx* ctx, const void* x, int M, void* out);

/* The acceptance step alone (Section 3.2.4; with ssd_set_tree_mode(ctx, 1) the mix-order walk of
 * Section 5.2) on caller-supplied model outputs.  Arguments as ssd_verify_tree, without prefix
 * lengths; row_conf / row_argmax are device arrays with one entry per row of the forward the call
 * describes: sequences in call order, per sequence the chain nodes 0 .. n_draft[i] and then the
 * mix-order nodes, block_len (default: the context's block) rows per node.  Writes `out` and the
 * context's block state exactly as the forward's last kernel does.  Asynchronous on the
 * context's stream.  Errors as ssd_verify_tree. */
int ssd_k_accept(ssd_ctx* ctx, int n, const int* seqs, const int32_t* block_tok, const uint64_t* masked,
                 const int* block_len, const int32_t* draft_pos, const int32_t* draft_tok, const int* n_draft,
                 int n_draft_next, const float* row_conf, const int32_t* row_argmax, const ssd_step_out* out);

#ifdef __cplusplus
}
#endif
#endif /* SSD_KERNELS_H */
