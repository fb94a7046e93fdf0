// Host-callable launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "common.h"

namespace sv {

// ---- gemm.hip ----
int gemm_bf16_shape_ok(int N, int K, int splits);
int gemm_bf16_variant_ok(int variant, int N);
hipError_t gemm_bf16(const bf16_t* A, const bf16_t* W, float* out, int M, int N, int K, int splits, int variant,
                     hipStream_t st);
hipError_t pack_weight(const bf16_t* src, bf16_t* dst, int N, int K, hipStream_t st);
hipError_t pack_rows(const bf16_t* src, bf16_t* dst, int M, int K, hipStream_t st);
// row_tiles: 32-row tiles per work-group (1..5; 0 = as few work-groups along the rows as five tiles each allow)
hipError_t gemm_bf16_ws(const bf16_t* Ap, const bf16_t* Wp, float* out, int M, int N, int K, int splits, bool wide,
                        hipStream_t st, int row_tiles = 0);
int gemm_bf16_ws_row_tiles(int M);
// 256 x 256 tiles, both operands through LDS (for a thousand rows and more).  glu: N = 2 F gate and up rows, out =
// packed bf16 activations [ceil(M/32)*32, F]
hipError_t gemm_bf16_tile(const bf16_t* Ap, const bf16_t* Wp, float* out, int M, int N, int K, int splits, bool glu, hipStream_t st);
// what a CU sustains on 256 x 256 tiles with the gated bf16 output, TFLOP/s (measured inside a step on MI355X)
constexpr double kTileRateGlu = 4.85;
// tile_mode: -1 = the 256 x 256 kernel where it pays, 0 = never, 1 = whenever the shape allows
hipError_t gemm_bf16_ws_glu(const bf16_t* Ap, const bf16_t* Wp, bf16_t* act_out, int M, int F, int K, hipStream_t st, int tile_mode = -1);
hipError_t gemm_f32(const float* A, const float* W, float* out, int M, int N, int K, hipStream_t st);

// ---- elementwise.hip ----
struct RowPrep {
    const int32_t* batch_seq;   // [B] sequence id per request
    const int32_t* seq_len;     // [max_seqs] live lengths
    const int32_t* last_tokens; // [B]
    const int32_t* drafts;      // [B, N*k] (may be null when k == 0)
    int32_t* row_tok;           // [T]
    int32_t* row_pos;           // [T]
    int32_t* row_slot;          // [T]
    float* rope;                // [T, head_dim/2, 2] cos, sin
    int B, n, k, head_dim, vocab;
    float rope_theta;
    // when set, the tokens come from a matrix of prompts instead: row t = b*n + j holds tok_matrix[b*tok_ld + tok_col0 + j],
    // or, past the end of prompt b (tok_len[b] tokens), its last token (a padding row whose results are never used)
    const int32_t* tok_matrix; const int32_t* tok_len; int tok_ld, tok_col0;
};
hipError_t prep_rows(const RowPrep& p, hipStream_t st);
hipError_t embed_rows(const void* embed, int dtype, const int32_t* row_tok, float* h, int T, int d, hipStream_t st);
// h[t,:] += sum_s part[s][t,:] (S may be 0), then a[t,:] = storage(h * rsqrt(mean(h^2)+eps) * w)
hipError_t add_rmsnorm(float* h, const float* part, int S, const void* w, void* a, int dtype, int T, int d, float eps,
                       bool packed, hipStream_t st);
// the same with the addend = weighted sum of the row's top_k expert outputs y[inv[t*top_k + j]] (bf16 models)
hipError_t add_rmsnorm_experts(float* h, const float* y, const int32_t* inv, const float* wts, int top_k, const void* w, void* a,
                               int T, int d, float eps, bool packed, hipStream_t st);
struct RopeAppend {
    const float* qkv_part; int S;       // [S][T][(Hq+2Hkv)*hd]
    const float* rope;                  // [T][hd/2][2]
    const int32_t* row_slot;            // [T]
    const int32_t* batch_seq;           // [B]
    const int32_t* page_table; int max_pages_per_seq;
    void* q_out;                        // [T][Hq][hd] storage type
    void* pool; KvGeom geom; int layer;
    int T, n, Hq, Hkv, hd, dtype;
};
hipError_t rope_append(const RopeAppend& p, hipStream_t st);
hipError_t swiglu(const float* gu_part, int S, void* act, int dtype, int T, int F, bool packed, hipStream_t st);
hipError_t kv_copy(void* pool, const KvGeom& geom, int layer, const int32_t* page_table_row, int pos0, int n,
                   void* k, void* v, int dtype, bool to_pool, hipStream_t st);
hipError_t set_i32(int32_t* p, int32_t v, hipStream_t st);
hipError_t add_len(int32_t* seq_len, const int32_t* batch_seq, int B, int delta, hipStream_t st);
// seq_len[batch_seq[b]] += min(width, len[b] - col0): what request b really holds of a pass over columns col0 .. col0+width-1
hipError_t add_len_ragged(int32_t* seq_len, const int32_t* batch_seq, int B, const int32_t* len, int col0, int width, hipStream_t st);

// ---- attention.hip ----
struct AttnArgs {
    const void* q;                      // [T][Hq][hd] storage type
    const void* pool; KvGeom geom; int layer;
    const int32_t* page_table; int max_pages_per_seq;
    const int32_t* batch_seq;           // [B]
    const int32_t* seq_len;             // [max_seqs]
    void* out;                          // [T][Hq*hd] storage type
    float* part_o;                      // [B][Hkv][max_chunks][rows_pad][hd]
    int rows_pad;                       // row pitch of the partials (a multiple of 16, >= stacked rows for the MFMA path)
    int row_groups;                     // set by attention(): work-groups that share one (item, head)
    float* part_ml;                     // [B][Hkv][max_chunks][rows_pad][2]
    int B, n, k, Hq, Hkv, hd, dtype;
    int chunk_keys, max_chunks;
    const int32_t* work; int n_work;    // items of the bf16 kernel, 4 ints each: request << 16 | chunk, sequence id, first key, end
    const int32_t* req_chunk;           // [B][2] keys per piece, pieces (from the host's upper bounds of the lengths)
    const int32_t* n_work_dev;          // when set: the item count lives here (a captured launch cannot carry it)
    int grid_items;                     // when > 0: items the grid is sized for (an upper bound of the item count)
    int min_row_tiles;                  // lower bound on the 16-row tiles of the bf16 kernel (tuning)
    int max_row_tiles;                  // most 16-row tiles one work-group takes (1..4); more rows -> row groups
    bool out_packed;                    // write `out` in the packed activation order (see act_index)
    bool force_generic;                 // take the untuned one-wave-per-row path whatever the shape
};
int attn_rows_pad(int n, int group);        // padded query rows per (request, kv head); 0 = MFMA path not applicable
hipError_t attention(const AttnArgs& a, hipStream_t st);

// ---- moe.hip ----
struct MoeArgs {
    const bf16_t* a;          // activations, packed [ceil(T/32)][d/16][64][8]
    const bf16_t* w_router;   // [E][d] row-major
    const bf16_t* w_gate_up;  // [E][2F][d] packed as one (E*2F) x d matrix
    const bf16_t* w_down;     // [E][d][F] packed as one (E*d) x F matrix
    float* router_logits;     // [4][T][E] partial router logits (up to four parts of the reduction)
    int32_t* top_ids;         // [T][top_k] experts in descending probability
    float* top_w;             // [T][top_k] renormalised weights
    int32_t* cnt;             // [E] rows per expert
    int32_t* tile_off;        // [E+1] first 32-row tile of each bucket
    int32_t* perm;            // [32 * max_tiles] source row of a padded row
    int32_t* inv;             // [T * top_k] padded row of an assignment
    bf16_t* act;              // [max_tiles][F/16][64][8] SwiGLU outputs as operand tiles
    float* y;                 // [32 * max_tiles][d] expert outputs (until the first product has read them: the buckets' rows as bf16 operand tiles)
    float* out;               // [T][d] combined result
    int T, d, E, top_k, F;
};
int moe_shape_ok(int T, int d, int E, int top_k, int F);
size_t moe_group_lds_bytes(int T, int E);
int moe_max_tiles(int T, int E, int top_k);
hipError_t moe_ffn(const MoeArgs& a, hipStream_t st);

// ---- sampler.hip ----
struct SampleArgs {
    const float* logits;                // [T][V]
    const int32_t* drafts;              // [B][N][k]
    const float* draft_probs;           // [B][N][k][V] or null
    const float* uniforms;              // [B][N][k+1] or null (greedy)
    const int32_t* draft_lens;          // [B] or null
    float* row_stat;                    // [T][4]: max logit, sum exp((x-max)/temp), argmax id (as int bits), unused
    int32_t* chain_acc;                 // [B][N]
    int32_t* chain_tok;                 // [B][N]
    int32_t* chain_row;                 // [B][N] scratch
    float* draw_part;                   // [B][N][kDrawParts][4] winners of the parts of the exponential race
    int32_t* accepted_len;              // [B]
    int32_t* out_tokens;                // [B][k+1]
    int32_t* best_chain;                // [B]
    int B, N, k, V, verify_mode, sample_mode;
    float temperature;
};
constexpr int kDrawParts = 8;
hipError_t sample_verify(const SampleArgs& a, hipStream_t st);
struct RollbackArgs {
    void* pool; KvGeom geom; int n_layers, dtype;
    const int32_t* page_table; int max_pages_per_seq;
    const int32_t* batch_seq;
    int32_t* seq_len;
    const int32_t* accepted_len;
    const int32_t* best_chain;
    int B, N, k;
};
// move the kept chain's accepted K/V entries next to x0 (N > 1 only); commit: also advance the live lengths by a + 1
hipError_t rollback(const RollbackArgs& a, hipStream_t st, bool commit = true);

}  // namespace sv
