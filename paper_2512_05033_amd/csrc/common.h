// Internal declarations shared by the libarb translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "arb.h"

typedef __bf16 bf16;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define ARB_WAVE 64
#define ARB_KV_BLOCK 16

// Records a message for arb_last_error() and returns `st`.
arb_status arb_fail(arb_status st, const char *fmt, ...);

#define ARB_CHECK_HIP(expr)                                                               \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) return arb_fail(ARB_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

#define ARB_CHECK_LAUNCH(name)                                                            \
  do {                                                                                    \
    hipError_t e_ = hipGetLastError();                                                    \
    if (e_ != hipSuccess) return arb_fail(ARB_EHIP, "launch %s: %s", name, hipGetErrorString(e_)); \
  } while (0)

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- tile order shared by the GEMM kernels ----

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Give
// every XCD a contiguous range of logical tiles so that the m-tiles that share a
// weight tile run on the same L2.
static __device__ __forceinline__ int xcd_remap(int bid, int total) {
  const int per = total / 8, rem = total % 8;
  const int xcd = bid % 8, j = bid / 8;
  // XCDs [0, rem) hold per+1 tiles, the rest hold per
  const int base = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
  return base + j;
}

// Logical tile index -> (tile_m, tile_n): m-tiles in groups of GM, n fastest across groups, so that the
// tiles an XCD runs at the same time form a compact block (few distinct A and B tiles for its L2).  What
// an XCD fetches is (block height) A tiles + (block width) B tiles, least for a square block of rows:
// groups of 512 rows (GM = 4 tiles of 128 rows, 8 of 64) measured 1-3 % faster than groups of 1024 rows on the
// narrow projections of the 1.5B shape (an XCD then reads half of the activations instead of all of them).
template <int GM>
static __device__ __forceinline__ void tile_of(int logical, int tiles_m, int tiles_n, int &tile_m, int &tile_n) {
  const int per_group = GM * tiles_n, g = logical / per_group, idx = logical - g * per_group;
  const int rows = min(GM, tiles_m - g * GM);
  tile_n = idx / rows;
  tile_m = g * GM + (idx - tile_n * rows);
}

// ---- launchers implemented in the kernel files (all asynchronous on `st`) ----

// gemm.hip
// With splits > 1 (residual and fp32-store epilogues) C is not accumulated into: split s writes its fp32
// partial product to C + s*M*N and the consumer adds the partials up (the norm kernels for the residual
// stream, rope_append for q/k/v).
// A launch is up to two kernels: n-tile columns [0, gemm_large_cols) in 256x256 tiles, the rest in
// 128x128 tiles; `part` restricts the call to one of them.
enum { GEMM_PART_ALL = 0, GEMM_PART_LARGE = 1, GEMM_PART_SMALL = 2 };
// B_blocked: optional K-blocked copy of B (launch_pack_k_blocked); the 256x256-tile part of the launch reads it instead of B.
arb_status launch_gemm(const bf16 *A, const bf16 *B, void *C, int M, int N, int K, int epilogue, hipStream_t st,
                       int splits = 1, int part = GEMM_PART_ALL, const bf16 *B_blocked = nullptr);
arb_status launch_pack_k_blocked(const bf16 *W, size_t rows, int K, bf16 *packed, hipStream_t st);
int gemm_large_cols(int M, int N, int K, int epilogue, int splits);   // in units of 256 columns (128 SwiGLU features)
int gemm_residual_splits(int M, int N, int K);

// attention.hip
struct AttnPlan {
  int kv_chunk;      // keys per split (multiple of 64)
  int max_splits;    // ceil(max_ctx / kv_chunk) over the batch
  int max_qtiles;    // ceil(max_step * G / 128)
};
AttnPlan plan_attention(int batch, const int32_t *prefix_host, const int32_t *cu_host, int G, int n_kv_heads);
size_t attention_ws_bytes(int max_splits_cap, int total_tokens, int n_q_heads, int head_dim);
int attention_splits_cap(int max_ctx);   // largest max_splits plan_attention can return for contexts <= max_ctx
arb_status launch_attention(const bf16 *q, int q_row_stride, const bf16 *k_pool, const bf16 *v_pool,
                            const int32_t *block_tables, int max_blocks_per_seq, const int32_t *prefix_lens,
                            const int32_t *cu_step_lens, int batch, int total_tokens, int n_q_heads, int n_kv_heads,
                            int head_dim, const AttnPlan &plan, const int32_t *tok_pos_in, bf16 *out, void *ws, size_t ws_bytes,
                            hipStream_t st, bool q_prescaled);
// log2(e) / sqrt(head_dim): the factor the attention kernel wants folded into the queries (q_prescaled), so that
// its score products are logits in log2 units; launch_rope_append applies it (q_scale) before it rounds q.
float attention_q_scale(int head_dim);

// elementwise.hip
arb_status launch_token_meta(const int32_t *prefix_lens, const int32_t *cu_step_lens, const int32_t *block_tables,
                             int batch, int total_tokens, int max_blocks_per_seq, int kv_block, int32_t *tok_pos,
                             int32_t *tok_slot, hipStream_t st);
// Debug range check of token ids and of the block ids a batch references; err: device int32 [4].
arb_status launch_check_ids(const int32_t *token_ids, int T, int vocab, const int32_t *block_tables, int batch,
                            int max_blocks_per_seq, const int32_t *prefix_lens, const int32_t *cu_step_lens,
                            int kv_block, int n_blocks, int32_t *err, hipStream_t st);
arb_status launch_rope_table(const int32_t *tok_pos, int total_tokens, int head_dim, float rope_base, f32x2 *cs,
                             hipStream_t st);
arb_status launch_embed_rmsnorm(const bf16 *embed, const int32_t *token_ids, const float *g, float eps, int T, int d,
                                float *h, bf16 *x, hipStream_t st);
// parts/n_parts: fp32 partial products [n_parts, T, d] that are first added to h (and h is updated).
arb_status launch_rmsnorm(float *h, const float *parts, int n_parts, const float *g, float eps, int T, int d, bf16 *x,
                          hipStream_t st);
// parts/n_parts: when n_parts > 0 the projection is read as the sum of fp32 partial products
// [n_parts, T, (Hq+2Hkv)*hd] instead of from qkv; the rotated q is written to qkv (bf16) either way.
arb_status launch_rope_append(bf16 *qkv, const float *parts, int n_parts, const f32x2 *cs, const int32_t *tok_slot,
                              bf16 *k_pool, bf16 *v_pool, int T, int n_q_heads, int n_kv_heads, int head_dim,
                              float q_scale, hipStream_t st);
arb_status launch_final_norm_head(const float *h, const float *parts, int n_parts, const float *g, float eps, int T,
                                  int d, const float *w_head, const float *w_head1, bf16 *hidden_out, float *tok_dot,
                                  hipStream_t st);     // w_head1: class-1 row of a two-class head, else null
arb_status launch_pool_route(const float *tok_dot, const int32_t *cu_step_lens, int batch, float b_head, int pool,
                             int probability, float tau, float *scores, uint8_t *escalate, hipStream_t st);
arb_status launch_route(const float *scores, int n, float tau, int sense, uint8_t *escalate, hipStream_t st);
arb_status launch_advantage_route(const float *s_t, const float *s_d, int n, float tau, const float *tau_device,
                               float *delta, uint8_t *escalate, float *realized, hipStream_t st);
arb_status launch_budget_threshold(const float *delta, int n, int budget, float *tau_out, hipStream_t st);
arb_status launch_gather_rows(const bf16 *src, const int32_t *rows, int n, int d, bf16 *dst, hipStream_t st);
arb_status launch_sample_token(const float *logits, int n, int V, float temperature, const float *uniforms,
                               int32_t *token, float *chosen, hipStream_t st);
arb_status launch_first_stop(const int32_t *tokens, int n, int S, int sep, int eos, int32_t *len, uint8_t *ended,
                             hipStream_t st);
arb_status launch_step_advance(const int32_t *open_rows, const int32_t *chosen, int n_open, int S, int sep, int eos,
                               int32_t *steps, int32_t *len, uint8_t *done, int32_t *next_rows, int32_t *next_ids,
                               int32_t *n_next, hipStream_t st);
arb_status launch_pack_steps(const int32_t *steps, int S, const int32_t *rows, const int32_t *cu, int n_rows, int32_t *ids,
                             hipStream_t st);

// gemm_w4.hip: 4-bit weights (offset-binary nibbles, eight k per uint32, bf16 scale per row and 128 k)
arb_status launch_w4_quantize(const bf16 *W, int N, int K, uint32_t *packed, bf16 *scales, int bits, hipStream_t st);
arb_status launch_gemm_w4(const bf16 *A, const uint32_t *Bq, const bf16 *Bscale, void *C, int M, int N, int K,
                          int epilogue, hipStream_t st, int splits = 1);
