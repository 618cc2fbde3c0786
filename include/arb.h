/* arb.h - C ABI of libarb: the batched step-scoring forward and routing decision
 * of Arbitrage (step-level speculative generation), for one AMD MI355X (gfx950).
 *
 * The method (paper Section 4.2, Fig. 1, Algorithm 1): at every reasoning step
 * a draft model proposes a step z_d for the context x; a router
 * h_router(x, z_d) gives a score y_hat; the draft is ACCEPTED iff y_hat <= tau
 * and the step is ESCALATED to the target model iff y_hat > tau; the target then
 * regenerates the step "from the same prefix" x.  The router is a decoder-only
 * transformer with a classification head.  This library runs that transformer
 * over the drafted steps of a batch of independent sequences, against their
 * cached (block-paged) prefixes, and takes the decision.  The same forward
 * without the head is the target model's pass over an appended step.
 *
 * Conventions
 *  - "device" pointers are HIP device memory on the current device; "host"
 *    pointers are ordinary host memory.  The caller owns every buffer, including
 *    the KV pool and the workspace; the library allocates nothing in the hot
 *    calls (arb_prefill, arb_score_steps, arb_route and the arb_stage_* calls),
 *    never synchronises the device and never reads results back.
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream).  Outputs are valid once the caller has synchronised it.
 *  - Every call returns an arb_status; nothing throws or aborts across the ABI.
 *    arb_last_error() gives a message for the last failing call of this thread.
 *  - bf16 = the upper 16 bits of an IEEE fp32, round-to-nearest-even.
 *  - Lengths are stateless: each call is told prefix_lens and the step lengths;
 *    the step's keys/values are written at positions [p_b, p_b+s_b) of sequence
 *    b and nothing records that.  Rejecting a draft (Alg. 1, escalate branch) is
 *    not advancing prefix_lens; accepting it (x <- x || z) is advancing it by s_b.
 *    Repeating a call with the same arguments gives the same results.
 *
 * Debug mode: if the environment variable ARB_DEBUG_IDS is set (to anything but "0") when arb_model_create
 * runs, every arb_prefill / arb_score_steps / arb_score_steps_noalloc / arb_stage_layers call of that model
 * first range-checks, on the device, the token ids against [0, vocab) and every block id its sequences
 * reference against [0, arb_kv.n_blocks), waits for the result (the one case in which a hot call
 * synchronises) and returns ARB_EINVAL naming the first offender before any kernel has used an id.
 * Without it ids are trusted: a bad one is an out-of-bounds access.
 *
 * Supported shapes: head_dim == 64 or 128; d_model, d_ffn and n_q_heads*head_dim multiples of
 * 128; n_q_heads a multiple of n_kv_heads; kv_block == 16.  Others -> ARB_EUNSUPPORTED.
 */
#ifndef ARB_H
#define ARB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ARB_OK = 0,
  ARB_EINVAL = 1,       /* null pointer, negative size, empty step (s_b == 0), inconsistent cu_step_lens */
  ARB_ESHAPE = 2,       /* n_q_heads % n_kv_heads != 0, odd head_dim, non-positive dimension */
  ARB_ECAPACITY = 3,    /* block table row or workspace too small for the call */
  ARB_EHIP = 4,         /* a HIP runtime call failed (message has the HIP error string) */
  ARB_EUNSUPPORTED = 5  /* a valid shape this build has no kernel for */
} arb_status;

/* How the step's hidden states are pooled before the head.  MEAN over the s_b
 * step tokens is what the workload configs use; LAST is the paper's statement
 * that the classification head sits on the final-token embedding (Section 4.2,
 * "Training"). */
typedef enum { ARB_POOL_MEAN = 0, ARB_POOL_LAST = 1 } arb_pool_mode;

/* Comparison sense.  ARB_ESCALATE_IF_GT is Arbitrage: accept iff score <= tau
 * (Fig. 1, Alg. 1).  ARB_ACCEPT_IF_GT is the RSD baseline: accept iff
 * score > tau (Section 3.1).  In both, a NaN score escalates. */
typedef enum { ARB_ESCALATE_IF_GT = 0, ARB_ACCEPT_IF_GT = 1 } arb_route_sense;

/* The router head (arb_model_cfg.has_router_head).  LINEAR: one fp32 vector w_head [d], the score is the
 * raw value w_head . pool + b_head (what the workload configs use; tau is a threshold on that scale).
 * TWO_CLASS: the two-way classification head of Section 4.2 ("Training": class 1 = the target's step has
 * the higher PRM score): w_head is fp32 [2, d] (row 0 class 0, row 1 class 1), b_head is the bias
 * difference c_1 - c_0, and the score is the softmax probability of class 1,
 * y_hat = 1 / (1 + exp(-((w_1 - w_0) . pool + b_head))), so tau is a probability. */
typedef enum { ARB_HEAD_NONE = 0, ARB_HEAD_LINEAR = 1, ARB_HEAD_TWO_CLASS = 2 } arb_head_kind;

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps;        /* added to the mean square under the root */
  float rope_base;      /* rotary angle of pair t at position pos: pos * base^(-2t/head_dim) */
  int32_t kv_block;     /* tokens per KV block (16) */
  int32_t pool;         /* arb_pool_mode */
  int32_t has_router_head; /* arb_head_kind; 0: target pass (hidden states only) */
} arb_model_cfg;

/* Weights.  All DEVICE pointers, caller-owned, must outlive the model.  The
 * per-layer arrays themselves (wqkv[l], ...) are HOST arrays of n_layers device
 * pointers and are copied by arb_model_create.
 * Every matrix is bf16, row-major [out_features, in_features] (y = x W^T):
 *   embed [vocab, d]
 *   wqkv  [(Hq + 2 Hkv) * hd, d]  rows: Hq query heads, then Hkv key heads, then Hkv value heads
 *   wo    [d, Hq * hd]
 *   wgu   [2 F, d]                rows: F gate rows, then F up rows; MLP = (silu(x Wg^T) * (x Wu^T)) Wd^T
 *   wd    [d, F]
 * RMSNorm gains g_attn[l], g_mlp[l], g_final are fp32 [d]; w_head is fp32 [d] (fp32 [2, d] for
 * ARB_HEAD_TWO_CLASS; NULL when has_router_head == 0); b_head is the head's scalar bias. */
typedef struct {
  const void *embed;
  const void *const *wqkv, *const *wo, *const *wgu, *const *wd;
  const float *const *g_attn, *const *g_mlp;
  const float *g_final;
  const float *w_head;
  float b_head;
  /* 4-bit projection weights (the weight-quantized draft of Section 5.1).  NULL (all four): the projection
   * weights above are bf16.  Otherwise HOST arrays of n_layers DEVICE pointers to bf16 scales
   * [rows, in/128], and wqkv/wo/wgu/wd point at the packed integers uint32 [rows, in/8] of
   * arb_w4_quantize instead of bf16 values (same row order).  Embedding, gains and head stay as above. */
  const void *const *wqkv_scale, *const *wo_scale, *const *wgu_scale, *const *wd_scale;
  /* Optional second copy of the gate/up weights in the K-blocked layout of arb_pack_k_blocked (bf16 weights
   * only): NULL, or a HOST array of n_layers DEVICE pointers.  The gate/up projection's large-tile kernel
   * then reads whole cache lines (about 6 % faster on the 1.5B shape); results are bit-identical.  wgu is
   * still required (the rest of the projection reads it).  Costs 4 F d bytes per layer. */
  const void *const *wgu_blocked;
} arb_weights;

/* Paged KV cache.  k_pool / v_pool are HOST arrays of n_layers DEVICE pointers;
 * each pool is bf16 [n_blocks, Hkv, kv_block, head_dim].  Position pos of
 * sequence b lives in block block_tables[b][pos / kv_block] at row pos % kv_block.
 * Keys are stored after the rotary embedding.  The calls write only the slots of
 * the step's own positions. */
typedef struct {
  void *const *k_pool, *const *v_pool;
  int32_t n_blocks;
} arb_kv;

/* One batch of B independent sequences: a cached prefix of prefix_lens[b] tokens
 * and a new step of s_b = cu_step_lens[b+1] - cu_step_lens[b] >= 1 tokens whose
 * ids are token_ids[cu_step_lens[b] .. cu_step_lens[b+1]).  The two length arrays
 * are given twice: on the device for the kernels, on the host for validation and
 * launch sizing.  Block-table contents are trusted (not range-checked). */
typedef struct {
  int32_t batch, total_tokens, max_blocks_per_seq;
  const int32_t *token_ids;          /* device [total_tokens] */
  const int32_t *block_tables;       /* device [batch, max_blocks_per_seq] */
  const int32_t *prefix_lens;        /* device [batch] */
  const int32_t *cu_step_lens;       /* device [batch + 1] */
  const int32_t *prefix_lens_host;   /* host   [batch] */
  const int32_t *cu_step_lens_host;  /* host   [batch + 1] */
} arb_batch;

typedef struct arb_model arb_model;

/* Validates the shape and copies the configuration and pointer tables (host
 * memory only).  *out is owned by the caller until arb_model_destroy. */
arb_status arb_model_create(const arb_model_cfg *cfg, const arb_weights *w, arb_model **out);
arb_status arb_model_destroy(arb_model *m);

/* Bytes of device workspace the hot calls need for batches of at most
 * max_total_tokens step tokens in at most max_batch sequences whose context
 * (prefix + step) is at most max_ctx tokens.  0 on invalid arguments. */
size_t arb_workspace_bytes(const arb_model *m, int32_t max_batch, int32_t max_total_tokens, int32_t max_ctx);

/* The router forward (Section 4.2; Alg. 1 "routing decision") or, with
 * has_router_head == 0, the target's pass over an appended step.
 *   scores     device fp32 [batch]: y_hat_b = w_head . pool_b(final-normed hidden) + b_head (the class-1
 *              probability for ARB_HEAD_TWO_CLASS); required iff has_router_head, else must be NULL
 *   escalate   device uint8 [batch] or NULL: 1 iff not (y_hat_b <= tau)
 *   hidden_out device bf16 [total_tokens, d_model] or NULL: final-normed hidden states
 *   ws         device workspace of ws_bytes >= arb_workspace_bytes(...)
 * Side effect: the step's rotary keys and values are stored (bf16) at its slots
 * in every layer's pool.  batch == 0 is a no-op. */
arb_status arb_score_steps(arb_model *m, const arb_kv *kv, const arb_batch *batch, float tau, float *scores,
                           uint8_t *escalate, void *hidden_out, void *ws, size_t ws_bytes, void *stream);

/* arb_score_steps for callers that cannot allocate or hold a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments and results (bit for bit) without `ws`:
 * the workspace is a static device array of ARB_NOALLOC_SCRATCH_BYTES inside the library, one copy per GPU
 * the library runs on, held until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine); its first call on a device looks the array's address up (not stream work; do
 * it once before capturing).  A batch whose workspace would exceed the array returns ARB_ECAPACITY with a
 * message that says how much it needs (the array holds e.g. 128 step tokens of the 1.5B-class shape
 * against 32 K contexts, or 64 of the 8B-class shape against 8 K); arb_workspace_bytes is an upper bound of
 * that need.  All calls on one GPU share the array: calls that overlap on one GPU (different streams or
 * threads) race; calls on one stream do not.  Nothing in it has to be cleared between calls. */
#define ARB_NOALLOC_SCRATCH_BYTES (64u << 20)
arb_status arb_score_steps_noalloc(arb_model *m, const arb_kv *kv, const arb_batch *batch, float tau, float *scores,
                                   uint8_t *escalate, void *hidden_out, void *stream);

/* Fills the cache for whole prompts: the same forward with the "step" being the
 * prompt (prefix_lens normally all 0; a non-zero prefix continues a chunked
 * prefill).  No head.  hidden_out as above, may be NULL. */
arb_status arb_prefill(arb_model *m, const arb_kv *kv, const arb_batch *batch, void *hidden_out, void *ws,
                       size_t ws_bytes, void *stream);

/* The decision alone (Fig. 1; Alg. 1; Section 3.1 for the RSD sense), so that
 * tau can be swept without repeating the forward.  Also serves the oracle
 * policy a*_tau = 1{Delta > tau} (Eq. 4.4) when `scores` holds advantages.
 * scores: device fp32 [n]; escalate: device uint8 [n].  n == 0 is a no-op. */
arb_status arb_route(const float *scores, int32_t n, float tau, int32_t sense, uint8_t *escalate, void *stream);

/* Routing by the true advantage (the ideal policy that Section 4.1 calls the oracle) on two PRM score arrays (Definitions 4.1 and 4.2, Eq. 4.4), all device fp32 [n]:
 *   delta[i]    = s_t[i] - s_d[i]                      (step-level advantage)
 *   escalate[i] = 1 iff not (delta[i] <= tau)          (a*_tau; NaN escalates, as in arb_route)
 *   realized[i] = escalate[i] ? s_t[i] : s_d[i]        (S(a) of Definition 4.2)
 * Any of the three outputs may be NULL (not all).  If tau_device is not NULL the threshold is read from that
 * device float (e.g. the output of arb_budget_threshold) and `tau` is ignored.  n == 0 is a no-op. */
arb_status arb_advantage_route(const float *s_t, const float *s_d, int32_t n, float tau, const float *tau_device,
                            float *delta, uint8_t *escalate, float *realized, void *stream);

/* The threshold that spends a budget of at most `budget` escalations best (Theorem B.1 and its proof):
 * *tau_out (device float) = max(0, the (budget+1)-th largest of delta[0..n)), 0 when budget >= n.  With it,
 * a*_tau escalates the min(budget, #positive) largest positive advantages (fewer if equal values straddle the
 * cut).  A NaN escalates under any tau, so NaNs rank first; if they alone exceed the budget the result is
 * +inf.  One workgroup; meant for n = number of reasoning steps. */
arb_status arb_budget_threshold(const float *delta, int32_t n, int32_t budget, float *tau_out, void *stream);

/* ---- the steps of Alg. 1 on either side of the scoring: next-token choice and step boundaries ---- */

/* Next token of n sequences (Alg. 1 "sample z ~ q(. | x)"; Section 3.1): logits = hidden[rows[i]] . w_lm^T,
 * then, per row, greedy choice (temperature <= 0: smallest index of the maximum) or a draw from
 * softmax(logits / temperature) by inversion with the caller's uniforms[i] in [0, 1) (the smallest k whose
 * cumulative weight reaches uniforms[i] times the total).
 *   hidden  device bf16 [*, d_model]: final-normed hidden states as arb_prefill / arb_score_steps emit them
 *   rows    device int32 [n]: the row of each sequence's last token
 *   w_lm    device bf16 [vocab, d_model]; vocab must be a multiple of 128, d_model of 64
 *   token   device int32 [n]; chosen_logit device fp32 [n] or NULL: the logit of the chosen token
 *   ws      device workspace of at least arb_next_token_workspace_bytes(n, d_model, vocab) */
size_t arb_next_token_workspace_bytes(int32_t n, int32_t d_model, int32_t vocab);
arb_status arb_next_token(const void *hidden, const int32_t *rows, int32_t n, int32_t d_model, const void *w_lm,
                          int32_t vocab, float temperature, const float *uniforms, int32_t *token,
                          float *chosen_logit, void *ws, size_t ws_bytes, void *stream);

/* Length of each generated step (Alg. 1: a step ends with the first separator or end-of-sequence token):
 * tokens device int32 [n, max_len]; len[i] = index of the first sep/eos + 1, or max_len if there is none;
 * ended[i] (device uint8, may be NULL) = 1 iff that token is eos. */
arb_status arb_first_stop(const int32_t *tokens, int32_t n, int32_t max_len, int32_t sep, int32_t eos, int32_t *len,
                          uint8_t *ended, void *stream);

/* One decoding iteration of n steps that are generated token by token (Alg. 1: a step ends with the first
 * separator or end-of-sequence token; here also when it is max_len tokens long).  State, all on the device and
 * owned by the caller, zero-initialised before a step's first iteration:
 *   steps  int32 [n, max_len]  the tokens generated so far (row i valid up to len[i])
 *   len    int32 [n]           tokens in each step so far
 *   done   uint8 [n]           0 = open, 1 = ended by a separator or by reaching max_len, 2 = ended by eos
 * open_rows (device int32 [n_open], ascending, each in [0, n), len < max_len, done = 0) lists the rows that were
 * fed this iteration and chosen (device int32 [n_open]) the token arb_next_token chose for each.  The call appends
 * every token to its row and updates len and done; the rows that stay open are written in ascending order to
 * next_rows (device int32 [n_open]) and their tokens, the next iteration's input ids, to next_ids (device int32
 * [n_open]); *n_next (device int32) is their number.  The host reads n_next and next_rows back to build the next
 * iteration's batch: finished steps cost no further forward work and the loop ends when none is open; the tokens
 * themselves never leave the device inside a step.  Rows outside open_rows are not touched.
 * Errors: ARB_EINVAL for negative sizes, n_open > n, max_len <= 0 or a null pointer (n_next always required). */
arb_status arb_step_advance(const int32_t *open_rows, const int32_t *chosen, int32_t n_open, int32_t n, int32_t max_len,
                            int32_t sep, int32_t eos, int32_t *steps, int32_t *len, uint8_t *done, int32_t *next_rows,
                            int32_t *next_ids, int32_t *n_next, void *stream);

/* The generated steps of rows[0 .. n_rows) as one ragged token list, the form arb_score_steps and arb_prefill take
 * (Alg. 1: the router scores the draft step z_d, the chosen step is appended to the context): ids[cu[j] + i] =
 * steps[rows[j]][i] for i < cu[j+1] - cu[j].  steps device int32 [*, max_len] as above, rows device int32
 * [n_rows], cu device int32 [n_rows + 1] (the batch's cu_step_lens), ids device int32 [cu[n_rows]]. */
arb_status arb_pack_steps(const int32_t *steps, int32_t max_len, const int32_t *rows, const int32_t *cu, int32_t n_rows,
                          int32_t *ids, void *stream);

/* Pool slot of every step token, slot = block_tables[b][pos/kv_block]*kv_block + pos%kv_block with
 * pos = prefix_lens[b] + i, as the forward computes it.  slots: device int32 [total_tokens]. */
arb_status arb_slot_mapping(const arb_batch *batch, int32_t kv_block, int32_t *slots, void *stream);

/* ---- single stages of the forward, exposed so each kernel can be checked and
 * timed on its own at full size.  Same pointer conventions as above. ---- */

typedef enum {
  ARB_EPI_STORE_BF16 = 0,   /* C bf16 [M, N] = A B^T */
  ARB_EPI_RESIDUAL_F32 = 1, /* C fp32 [M, N] += A B^T */
  ARB_EPI_SWIGLU_BF16 = 2,  /* B is [2F, K] (gate rows, up rows); C bf16 [M, F] = silu(A Bg^T) * (A Bu^T); N = F */
  ARB_EPI_STORE_F32 = 3     /* C fp32 [M, N] = A B^T (logits of the LM head) */
} arb_gemm_epilogue;

/* Projection GEMM: A bf16 [M, K] row-major, B bf16 [N, K] row-major (weights),
 * fp32 accumulation.  K % 64 == 0 and N % 128 == 0 (N % 64 == 0 for SWIGLU).  B_blocked: NULL, or the
 * arb_pack_k_blocked copy of B, which the large-tile kernel then reads in B's place. */
arb_status arb_stage_gemm(const void *A, const void *B, const void *B_blocked, void *C, int32_t M, int32_t N,
                          int32_t K, int32_t epilogue, void *stream);

/* K-blocked copy of a bf16 weight matrix W [rows, K] (K % 32 == 0), both on the device:
 * packed[(kb * rows + r) * 32 + j] = W[r][kb * 32 + j], i.e. [K/32][rows][32], so that the same 32 inputs
 * of consecutive rows are consecutive in memory.  For callers that cannot spare the copy the model works without it
 * (arb_weights.wgu_blocked). */
arb_status arb_pack_k_blocked(const void *W, int64_t rows, int32_t K, void *packed, void *stream);

/* 4-bit weight format of the quantized draft (Section 5.1; the paper takes its integers from GPTQ /
 * llama.cpp, the forward only needs integers and group scales): per row and group of 128 consecutive
 * inputs, scale = bf16(max|w| / 7), q = clip(rint(w / scale), -8, 7) (0 where scale is 0; fp32
 * quotients, round half to even); stored as q + 8 in nibbles, eight consecutive inputs per uint32: input
 * 8j + 2i in nibble i and input 8j + 2i + 1 in nibble 4 + i of word j (nibble 0 = bits 0..3), i.e. the even
 * inputs in the low half and the odd ones in the high half, two neighbours 16 bits apart, which is where a
 * register holds a pair of bf16.  W device bf16 [N, K], K % 128 == 0; packed device uint32 [N, K/8];
 * scales device bf16 [N, K/128]. */
arb_status arb_w4_quantize(const void *W, int32_t N, int32_t K, void *packed, void *scales, void *stream);

/* The same with 3-bit integers (the 3-bit self-draft of Section 5.2): scale = bf16(max|w| / 3),
 * q = clip(rint(w / scale), -4, 3), stored in the same nibbles (q + 8), so that everything that takes the
 * 4-bit format takes these weights unchanged (they occupy 4 bits each; a denser packing is not offered).
 * Arguments, shapes and errors as arb_w4_quantize. */
arb_status arb_w3_quantize(const void *W, int32_t N, int32_t K, void *packed, void *scales, void *stream);

/* arb_stage_gemm with such weights: C = A W'^T, W'[n,k] = q[n,k] * scale[n, k/128] (no rounding of the
 * products; fp32 accumulation).  K % 128 == 0; N and epilogues as arb_stage_gemm. */
arb_status arb_stage_gemm_w4(const void *A, const void *packed, const void *scales, void *C, int32_t M, int32_t N,
                             int32_t K, int32_t epilogue, void *stream);

/* How the projection GEMM of that shape is launched (host arithmetic only): the number of leading
 * 256-column blocks of C (128-feature blocks for SWIGLU) that one kernel computes in 256x256 tiles; the
 * remaining columns go to a second kernel in 128x128 tiles.  0 = one kernel, 128x128 tiles throughout. */
int32_t arb_gemm_large_tile_columns(int32_t M, int32_t N, int32_t K, int32_t epilogue);

/* Append-attention of one layer.  q: device bf16, row t at q + t*q_row_stride elements, heads contiguous
 * [Hq, hd], already rotated; the pools already hold the step's keys/values.  out: bf16 [T, Hq*hd].
 * q_scaled == 0: q is the rotated query itself and the logits are q.k / sqrt(hd).  q_scaled != 0: q already
 * carries the factor log2(e) / sqrt(hd), as the forward's rotary stage stores it (multiplied in fp32 before
 * the one rounding to bf16), and q.k is taken as the logit in log2 units: the kernel of the forward. */
arb_status arb_stage_attention(const arb_model *m, const void *q, int32_t q_row_stride, int32_t q_scaled,
                               const void *k_pool, const void *v_pool, const arb_batch *batch, void *out, void *ws,
                               size_t ws_bytes, void *stream);

/* RMSNorm rows: x fp32 [T, d] -> out bf16 [T, d] = x / sqrt(mean(x^2) + eps) * g. */
arb_status arb_stage_rmsnorm(const float *x, const float *g, float eps, int32_t T, int32_t d, void *out, void *stream);

/* Rotary embedding of the q and k heads of qkv (bf16 [T, (Hq+2Hkv)*hd], q rotated in place) at
 * positions prefix_lens[b] + i, and the K/V append into one layer's pool. */
arb_status arb_stage_rope_append(const arb_model *m, void *qkv, void *k_pool, void *v_pool, const arb_batch *batch,
                                 void *ws, size_t ws_bytes, void *stream);

/* Final RMSNorm of the residual stream h (fp32 [T, d]) followed by pooling, head and threshold
 * (Section 4.2; Alg. 1): hidden_out bf16 [T, d] or NULL; scores fp32 [batch]; escalate uint8 [batch] or
 * NULL.  The head is applied to the unrounded fp32 normed states.  ws: >= 4*T bytes. */
arb_status arb_stage_norm_pool_head(const float *h, const float *g_final, float eps, const arb_batch *batch,
                                    int32_t d, const float *w_head, float b_head, int32_t pool, float tau,
                                    void *hidden_out, float *scores, uint8_t *escalate, void *ws, size_t ws_bytes,
                                    void *stream);

/* Decoder layers [layer_begin, layer_end) of the forward (Section 4.2's router backbone / the target's
 * pass) applied to a given residual stream: h_in device fp32 [total_tokens, d_model] is the stream entering
 * layer_begin, h_out (may alias h_in) receives the stream leaving layer_end - 1; no embedding, no final
 * norm.  The step's K/V of those layers are appended as in arb_score_steps.  token_ids is not read.
 * Lets every layer of a deep model be checked at full size without the drift of the layers before it. */
arb_status arb_stage_layers(arb_model *m, const arb_kv *kv, const arb_batch *batch, int32_t layer_begin,
                            int32_t layer_end, const float *h_in, float *h_out, void *ws, size_t ws_bytes,
                            void *stream);

/* Timing hook for measurement harnesses (no paper passage: it computes nothing).
 * While armed, arb_score_steps / arb_prefill record start[i] before and stop[i]
 * after their i-th launch of the given stage on the call's stream, for i < n.
 * start/stop are HOST arrays of n hipEvent_t created by the caller with timing
 * enabled; they must stay valid while armed.  arb_model_trace_count gives the
 * number of launches recorded since arming.  n == 0 disarms. */
typedef enum {
  ARB_STAGE_QKV = 0, ARB_STAGE_ATTENTION = 1, ARB_STAGE_OPROJ = 2, ARB_STAGE_GATE_UP = 3, ARB_STAGE_DOWN = 4,
  ARB_STAGE_NORM = 5, ARB_STAGE_ROPE_APPEND = 6,
  ARB_STAGE_GATE_UP_LARGE = 7 /* the 256x256-tile kernel of the gate/up projection alone (an empty interval
                                 when arb_gemm_large_tile_columns is 0) */
} arb_trace_stage;
arb_status arb_model_trace(arb_model *m, int32_t stage, void *const *start, void *const *stop, int32_t n);
int32_t arb_model_trace_count(const arb_model *m);

const char *arb_last_error(void); /* thread-local; valid until the next call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* ARB_H */
