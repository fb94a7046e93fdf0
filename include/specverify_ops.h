/*
 * specverify_ops -- single-operation entry points of the verification library.
 *
 * Each runs one stage of the verification pass (see specverify.h for the pass as a whole) on
 * caller-provided device buffers, so that a stage can be checked against the oracle and timed
 * on its own.  All pointers are DEVICE pointers unless stated; `stream` is a hipStream_t
 * (NULL = null stream); calls return after enqueueing.  Return values are sv_status codes.
 */
#ifndef SPECVERIFY_OPS_H
#define SPECVERIFY_OPS_H

#include <stddef.h>
#include <stdint.h>
#include "specverify.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Dense projection of the forward pass (the part of parallel verification that is bound by matrix
 * throughput at large per-worker batch, Section 3 "Challenge #1"):
 *   out[s][m][n] = sum over k in split s of A[m][k] * W[n][k],   s = 0 .. splits-1
 * A [M,K] bf16, W [N,K] bf16, out [splits,M,N] fp32 (the consumer adds the splits).
 * N % 128 == 0, K % (64*splits) == 0.  Row-major operands (the path of models whose weights are not packed);
 * variant selects the work-group tile (tokens x features): 0: 128x128, 1: 64x128, 2: 256x128. */
int sv_op_gemm_bf16(const void *A, const void *W, float *out, int M, int N, int K, int splits, int variant,
                    void *stream);

/* The same projection with both operands in packed order, by the weight-streaming kernel: Ap = activations
 * packed by sv_op_pack_rows, Wp = weights packed by sv_op_pack_weight, out [splits, M, N] fp32.
 * wide != 0: 256 output features per work-group (N % 256 == 0), else 128.  K % (64*splits) == 0.
 * row_tiles: 32-row tiles per work-group, 1..5, or 0 = as few work-groups along the rows as five tiles each allow;
 * 8 = the second packed-operand kernel instead (256 rows x 256 features per work-group, both operands through LDS:
 * what the step uses from about a thousand rows on where its launch fills the chip; needs wide != 0). */
int sv_op_gemm_bf16_ws(const void *Ap, const void *Wp, float *out, int M, int N, int K, int splits, int wide,
                       int row_tiles, void *stream);

/* The launch shape verify_step gives the weight-streaming projection of M rows onto N features over K inputs
 * (HOST pointers out: reduction splits, 256- or 128-feature strips, 32-row tiles per work-group -- 8 = the 256 x 256
 * kernel).  Host arithmetic only.  N % 128 == 0, K % 64 == 0. */
int sv_op_gemm_plan(int M, int N, int K, int *splits, int *wide, int *row_tiles);

/* Reorder row-major bf16 activations src [M, K] into dst (ceil(M/32)*32*K elements) in the order the
 * weight-streaming kernel reads them: [ceil(M/32)][K/16][64 lanes][8 elements], lane 32*g + r of a fragment
 * holding row r of the 32-row tile, elements 8*g .. 8*g+7 of the 16-wide k slice; padding rows are zero. */
int sv_op_pack_rows(const void *src, void *dst, int M, int K, void *stream);

/* Reorder a row-major bf16 matrix src [N, K] into dst (N*K elements, distinct from src) in the order the
 * projection kernels stream it: [N/128][K/16][4 tiles of 32 rows][64 lanes][8 elements], where lane 32*g + r
 * of a tile holds row r, elements 8*g .. 8*g+7 of the 16-wide k slice.  N % 128 == 0, K % 32 == 0. */
int sv_op_pack_weight(const void *src, void *dst, int N, int K, void *stream);

/* Accept/reject + replacement/bonus draw + chain choice on given target logits (the rule restated at
 * verify_step).  logits fp32 [B*(1+N*k), V] in verify_step's row order; other arguments as in
 * verify_step / sv_batch / sv_out.  scratch: sv_op_sample_scratch_bytes(B,N,k) bytes. */
size_t sv_op_sample_scratch_bytes(int B, int N, int k);
int sv_op_sample(const float *logits, const int32_t *drafts, const float *draft_probs, const float *uniforms,
                 const int32_t *draft_lens, int B, int N, int k, int V, int verify_mode, int sample_mode,
                 float temperature, void *scratch, int32_t *accepted_len, int32_t *out_tokens,
                 int32_t *best_chain, void *stream);

/* sv_op_sample for callers that cannot allocate device memory or bring a scratch buffer: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * sv_op_sample without `scratch`: the scratch lives in a static device array of the library (624 KiB, held on
 * every GPU the library runs on until the process ends).  Limits: B * (1 + N * k) <= 4096 logits rows and
 * B * N <= 4096 chains; beyond them SV_EINVAL and nothing is enqueued.  The call allocates nothing (no
 * hipMalloc / hipFree, no allocating library routine); the caller still provides inputs and outputs.  All
 * calls on one GPU share the one array, which keeps the previous call's contents (no field is read before the
 * same call has written it, so nothing is cleared): calls that overlap on one GPU -- different streams,
 * different threads -- race on it; calls on one stream are ordered and safe. */
int sv_op_sample_static(const float *logits, const int32_t *drafts, const float *draft_probs, const float *uniforms,
                        const int32_t *draft_lens, int B, int N, int k, int V, int verify_mode, int sample_mode,
                        float temperature, int32_t *accepted_len, int32_t *out_tokens, int32_t *best_chain,
                        void *stream);

/* Verify attention alone (the part of parallel verification bound by HBM: every cached K/V byte is read
 * once for all n rows of a request).  For each listed sequence (HOST array seq_ids[B], live length L_b) the
 * n query rows q [B*n, n_q_heads, head_dim] (storage type) attend cache entries 0 .. L_b-1 and, of the
 * entries L_b .. L_b+n-1 (which the caller has written with verify_kv_write: x0, then chain 0's k drafts,
 * chain 1's ...), x0 and the earlier drafts of their own chain.  out [B*n, n_q_heads*head_dim] (storage
 * type).  n = 1 + N*k.  Lengths are not changed. */
int sv_op_attention(sv_ctx *, const int32_t *seq_ids, int B, int n, int k, int layer, const void *q, void *out);

/* One decoder layer of the parallel verification pass on given residual rows (Section 3, "Opportunity": the
 * pass of the trained model over the drafted tokens, here one layer of it at a time so that every layer can be
 * held to the oracle on the oracle's own input).  For the listed sequences (HOST array seq_ids[B], live length
 * L_b) and n = 1 + N*k new rows per request in verify_step's row order, h_in [B*n, d_model] fp32 is the residual
 * stream entering layer `layer`; h_out [B*n, d_model] fp32 (may alias h_in) receives it after the layer's
 * attention and feed-forward blocks, through exactly the launches verify_step makes for that layer: the rows'
 * K/V entries of this layer are written to cache slots L_b .. L_b+n-1 as in a step, lengths are not changed.
 * Mixture-of-experts models: top_ids / top_w (device [B*n, top_k], optional) receive the routing of the rows. */
int sv_op_layer(sv_ctx *, const int32_t *seq_ids, int B, int n, int k, int layer, const float *h_in, float *h_out,
                int32_t *top_ids, float *top_w);

/* The rollback stage alone (the last step of a verification: the first rejected draft and everything after it
 * are dropped, Section 3 "Opportunity"): for the listed sequences (HOST array seq_ids[B], live length L_b), whose
 * cache slots L_b .. L_b + N*k hold x0 and N chains of k drafts as a pass leaves them, the accepted_len[b] (DEVICE,
 * 0..k) first entries of chain best_chain[b] (DEVICE, 0..N-1) are moved next to x0, to slots L_b+1 .. L_b+a, in
 * every layer; verdicts outside those ranges move nothing.  commit != 0: the live lengths advance by a_b + 1 as
 * at the end of verify_step; commit == 0: lengths stay (the same verdicts can be applied again, for timing). */
int sv_op_rollback(sv_ctx *, const int32_t *seq_ids, int B, int N, int k, const int32_t *accepted_len,
                   const int32_t *best_chain, int commit);

/* The mixture-of-experts feed-forward on its own (the MoE model the paper evaluates, Section 5.3): softmax
 * router over E experts, top_k largest probabilities (lowest id among equals), renormalised; per selected
 * expert (silu(x Wg^T) * (x Wu^T)) Wd^T with the product silu * up rounded to bf16; out[t] = weighted sum.
 * All pointers device.  a_packed: activations [T, d] bf16 in the order sv_op_pack_rows() writes;
 * w_router [E, d] bf16 row-major; w_gate_up_packed: the [E, 2F, d] tensor (gate rows, then up rows, per expert)
 * packed by sv_op_pack_weight() as one (E*2F) x d matrix; w_down_packed: [E, d, F] packed as (E*d) x F.
 * scratch: sv_op_moe_scratch_bytes() bytes, 256-byte aligned.  out [T, d] fp32; top_ids / top_w [T, top_k]
 * (optional) receive the routing.  SV_EUNSUPPORTED unless E is a multiple of 64 up to 256 and d, F are
 * multiples of 128. */
size_t sv_op_moe_scratch_bytes(int T, int d, int E, int top_k, int F);
int sv_op_moe_ffn(const void *a_packed, const void *w_router, const void *w_gate_up_packed, const void *w_down_packed,
                  int T, int d, int E, int top_k, int F, void *scratch, size_t scratch_bytes, float *out,
                  int32_t *top_ids, float *top_w, void *stream);

/* Set the live lengths of n sequences at once (HOST arrays; same meaning as verify_seq_set_len, one
 * small copy and one launch instead of n).  Used to put a batch back to a saved state between steps. */
int sv_seq_set_lens(sv_ctx *, const int32_t *seq_ids, const int32_t *lens, int n);

/* Per-kind kernel timing inside verify_step / verify_prefill.  While bit k of kind_mask is set, every
 * launch group of kind k is bracketed by a pair of HIP events on the context's stream.
 * sv_profile_read synchronises the stream, returns the summed elapsed time and the number of
 * bracketed groups of that kind since the last read, and forgets them. */
enum { SV_PROF_GEMM = 0, SV_PROF_ATTENTION = 1, SV_PROF_SAMPLER = 2, SV_PROF_ROLLBACK = 3, SV_PROF_MOE = 4, SV_PROF_KINDS = 5 };
int sv_profile_enable(sv_ctx *, unsigned kind_mask);
int sv_profile_read(sv_ctx *, int kind, double *total_ms /* host */, int *launches /* host */);

/* Rooflines of this very GPU, measured (all pointers DEVICE unless stated; both calls synchronise `stream`).
 * sv_probe_mfma_bf16: 256 work-groups of four waves run `iters` rounds of eight independent
 *   v_mfma_f32_32x32x16_bf16 on operands held in registers (read once from `operands`, at least 256*256*128
 *   bytes: random bf16 values give the rate on real data, zeros the unthrottled one); `sink` takes 65536 floats;
 *   *tflops (HOST) = achieved dense bf16 rate.
 * sv_probe_hbm_copy: plain copies of `bytes` (a multiple of 16, at least 1 MiB, both buffers 16-byte aligned, choose
 *   it far larger than the caches), `reps` of them (after a warm-up) for each of five grid sizes;
 *   *gbs_each_way (HOST) = bytes copied per second in GB/s at the best grid, i.e. that much read and as much written.
 * sv_probe_hbm_read: the same for plain read-only passes over `bytes`; `sink` takes 4 bytes;
 *   *gbs (HOST) = bytes read per second in GB/s at the best grid. */
int sv_probe_mfma_bf16(const void *operands, size_t operand_bytes, float *sink, int iters, void *stream, double *tflops);
int sv_probe_hbm_copy(const void *src, void *dst, size_t bytes, int reps, void *stream, double *gbs_each_way);
int sv_probe_hbm_read(const void *src, size_t bytes, int reps, void *sink, void *stream, double *gbs);
/* Whether the matrix unit and the vector ALU overlap: 256 work-groups of 4 * waves_per_simd (1 or 2) waves run
 * `iters` rounds of (a) eight independent v_mfma_f32_16x16x32_bf16, (b) 8 * valu_per_mfma (2, 4 or 6) independent
 * v_fma_f32, (c) both, the FMAs placed after each MFMA; operands in registers.  sink (DEVICE, 256 * 512 floats) takes
 * a checksum; out_ms (HOST, 3 doubles) the three times in milliseconds.  Synchronises the stream. */
int sv_probe_mfma_valu(float *sink, int iters, int valu_per_mfma, int waves_per_simd, void *stream, double *out_ms);

/* Tuning / diagnostic knobs of a context.
 *   SV_OPT_GEMM_VARIANT  work-group tile of the row-major bf16 projections (0..2; -1 = per shape, default)
 *   SV_OPT_GEMM_TILE  the 256 x 256 kernel for packed projections: -1 = where the launch plan expects it to pay
 *                     (default), 0 = never, 1 = wherever the shape allows (output features a multiple of 256)
 *   SV_OPT_ATTN_GENERIC  1 = always use the untuned one-wave-per-row attention (default 0)
 *   SV_OPT_ATTN_MIN_ROW_TILES  lower bound (1..4) on the 16-row tiles the bf16 attention is built for
 *   SV_OPT_ATTN_MAX_ROW_TILES  most 16-row tiles (1..4, default 4) one work-group of the bf16 attention takes;
 *                           more stacked rows are split over row groups that stream the same keys
 *   SV_OPT_GRAPH  1 = verify_step replays its device work from a HIP graph captured on the second step with the
 *                 same batch shape and the same caller buffers (the first runs as plain launches); needs a context
 *                 stream other than the null stream; not used while sv_profile_enable brackets are on.  Default 0
 *   SV_OPT_ATTN_CHUNK_KEYS  keys per split-KV chunk of the bf16 attention (multiple of 128, at least 1024; 0 = chosen per
 *                           batch from the lengths, default) */
enum { SV_OPT_GEMM_VARIANT = 1, SV_OPT_ATTN_GENERIC = 2, SV_OPT_ATTN_MIN_ROW_TILES = 3, SV_OPT_ATTN_CHUNK_KEYS = 4,
       SV_OPT_ATTN_MAX_ROW_TILES = 5, SV_OPT_GRAPH = 6, SV_OPT_GEMM_TILE = 7 };
int sv_set_option(sv_ctx *, int option, int value);

#ifdef __cplusplus
}
#endif
#endif /* SPECVERIFY_OPS_H */
