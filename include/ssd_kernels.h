/*
 * ssd_kernels.h - kernel-level entry points of the SSD library, for unit
 * parity tests and measurement.  They run exactly the kernels the forward
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

/* Streams `bytes` of device memory with the access pattern of the GEMM's weight stream
 * (work_groups x waves_per_wg waves, `depth` 16-byte loads in flight per lane: 4, 8 or 16):
 * the HBM read rate the chip sustains, i.e. the practical ceiling of the roofline.
 * `sink` is 16 bytes of device scratch.  Asynchronous on `hip_stream`. */
int ssd_debug_stream_read(const void* src, size_t bytes, int work_groups, int waves_per_wg, int depth,
                          void* sink, void* hip_stream);

/* Measurement aid: while on (1), every forward of the context leaves out the gate/up GEMM launch of each
 * layer (the feed-forward block then reads stale activations: the results of such forwards are invalid, their
 * kernels and launch order otherwise unchanged).  The difference between the duration of a forward with and
 * without it, divided by the layer count, is what one gate/up launch costs inside the forward, measured with
 * two events per forward instead of two per kernel.  Returns the previous setting or an error. */
int ssd_debug_skip_gate_up(ssd_ctx* ctx, int on);

/* The loads of a weight-streaming GEMM and nothing else: each of `work_groups` work-groups (512
 * threads) reads all shared_bytes of `shared` (the activations every work-group needs) and its own
 * priv_bytes_per_wg of `priv` (work-group g reads [g, g+1) * priv_bytes_per_wg: its share of the
 * weights, non-temporal), evenly interleaved, with `threads` (512 or 1024) lanes and `depth` (4 or 8)
 * 16-byte loads in flight per lane.  Both sizes must be multiples of threads * depth * 16 bytes; `priv`
 * must hold work_groups * priv_bytes_per_wg bytes.  The duration is what the load path alone needs for
 * that GEMM's bytes.  `sink` is 16 bytes of device scratch.  Asynchronous on `hip_stream`. */
int ssd_debug_mixed_read(const void* shared, size_t shared_bytes, const void* priv, size_t priv_bytes_per_wg,
                         int work_groups, int threads, int depth, void* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SSD_KERNELS_H */
