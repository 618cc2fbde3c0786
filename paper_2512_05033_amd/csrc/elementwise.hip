// Row-wise and per-token kernels of the step-scoring forward: token metadata
// (position, pool slot), rotary table, embedding gather + RMSNorm, RMSNorm,
// rotary embedding + KV append, final RMSNorm + head dot, segmented pooling +
// threshold.  All are HBM-bound and touch T*d elements a handful of times.
#include "common.h"

// ------------------------------------------------------------------ reductions

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Sum over a block of 256 threads; every thread gets the result.
__device__ __forceinline__ float block_sum_256(float v, float *lds4) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds4[w] = v;
  __syncthreads();
  return lds4[0] + lds4[1] + lds4[2] + lds4[3];
}

// ---------------------------------------------------------------- token metadata

// For step token j of sequence b at position pos = p_b + i:
//   slot = block_tables[b][pos / blk] * blk + pos % blk.
__global__ void token_meta_kernel(const int32_t *__restrict__ prefix_lens, const int32_t *__restrict__ cu,
                                  const int32_t *__restrict__ tables, int batch, int T, int max_blocks, int blk,
                                  int32_t *__restrict__ tok_pos, int32_t *__restrict__ tok_slot) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= T) return;
  int lo = 0, hi = batch;                 // largest b with cu[b] <= j
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= j) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int pos = prefix_lens[b] + (j - cu[b]);
  if (tok_pos) tok_pos[j] = pos;
  if (tok_slot) tok_slot[j] = tables[(size_t)b * max_blocks + pos / blk] * blk + pos % blk;
}

arb_status launch_token_meta(const int32_t *prefix_lens, const int32_t *cu_step_lens, const int32_t *block_tables,
                             int batch, int total_tokens, int max_blocks_per_seq, int kv_block, int32_t *tok_pos,
                             int32_t *tok_slot, hipStream_t st) {
  if (total_tokens == 0) return ARB_OK;
  hipLaunchKernelGGL(token_meta_kernel, dim3(ceil_div(total_tokens, 256)), dim3(256), 0, st, prefix_lens,
                     cu_step_lens, block_tables, batch, total_tokens, max_blocks_per_seq, kv_block, tok_pos, tok_slot);
  ARB_CHECK_LAUNCH("token_meta");
  return ARB_OK;
}

// ------------------------------------------------------------- debug: id range check

// err[0]: bit 0 = a token id outside [0, vocab), bit 1 = a referenced block id outside [0, n_blocks);
// err[1] / err[2]: smallest offending index into token_ids / block_tables (INT32_MAX: none).
__global__ void check_ids_init_kernel(int32_t *err) {
  err[0] = 0;
  err[1] = err[2] = INT32_MAX;
  err[3] = 0;
}

// One thread per token id, then one per block-table entry.  Entry j of row b is referenced iff
// j < ceil((p_b + s_b) / blk); the rest of a row may hold anything.
__global__ void check_ids_kernel(const int32_t *__restrict__ token_ids, int T, int vocab,
                                 const int32_t *__restrict__ tables, int batch, int max_blocks,
                                 const int32_t *__restrict__ prefix_lens, const int32_t *__restrict__ cu, int blk,
                                 int n_blocks, int32_t *err) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < T) {
    if (token_ids) {
      const int id = token_ids[i];
      if (id < 0 || id >= vocab) {
        atomicOr(&err[0], 1);
        atomicMin(&err[1], (int)i);
      }
    }
    return;
  }
  const long long e = i - T;
  if (e >= (long long)batch * max_blocks) return;
  const int b = (int)(e / max_blocks), j = (int)(e - (long long)b * max_blocks);
  const int ctx = prefix_lens[b] + cu[b + 1] - cu[b];
  if (j >= (ctx + blk - 1) / blk) return;
  const int id = tables[e];
  if (id < 0 || id >= n_blocks) {
    atomicOr(&err[0], 2);
    atomicMin(&err[2], (int)e);
  }
}

arb_status launch_check_ids(const int32_t *token_ids, int T, int vocab, const int32_t *block_tables, int batch,
                            int max_blocks_per_seq, const int32_t *prefix_lens, const int32_t *cu_step_lens,
                            int kv_block, int n_blocks, int32_t *err, hipStream_t st) {
  hipLaunchKernelGGL(check_ids_init_kernel, dim3(1), dim3(1), 0, st, err);
  ARB_CHECK_LAUNCH("check_ids_init");
  const long long n = (long long)T + (long long)batch * max_blocks_per_seq;
  hipLaunchKernelGGL(check_ids_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, token_ids, T, vocab,
                     block_tables, batch, max_blocks_per_seq, prefix_lens, cu_step_lens, kv_block, n_blocks, err);
  ARB_CHECK_LAUNCH("check_ids");
  return ARB_OK;
}

// -------------------------------------------------------------------- rotary table

// cs[j][t] = (cos, sin) of pos_j * base^(-2t/hd), evaluated in fp64 so that the
// fp32 table is correctly rounded even at positions of tens of thousands.
__global__ void rope_table_kernel(const int32_t *__restrict__ tok_pos, int T, int half, double log2_base,
                                  f32x2 *__restrict__ cs) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= T * half) return;
  const int j = idx / half, t = idx - j * half;
  const double inv_freq = exp2(-(double)t / (double)half * log2_base);
  const double ang = (double)tok_pos[j] * inv_freq;
  double s, c;
  sincos(ang, &s, &c);
  cs[idx] = f32x2{(float)c, (float)s};
}

arb_status launch_rope_table(const int32_t *tok_pos, int total_tokens, int head_dim, float rope_base, f32x2 *cs,
                             hipStream_t st) {
  const int half = head_dim / 2, n = total_tokens * half;
  if (n == 0) return ARB_OK;
  hipLaunchKernelGGL(rope_table_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, st, tok_pos, total_tokens, half,
                     log2((double)rope_base), cs);
  ARB_CHECK_LAUNCH("rope_table");
  return ARB_OK;
}

// ------------------------------------------------------------------------ RMSNorm

// One block of 256 threads per row; a row is held in registers between the
// sum-of-squares pass and the scaling pass (d <= 256*8*ROW_VECS).
#define ROW_VECS 4

// With n_parts > 0 the row is first completed by the split-K partial products of
// the preceding residual projection: h = h_in + sum_s parts[s] (fixed order), and
// written back through h_out when that is not null.
template <bool EMBED, bool HEAD>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *h_in, const float *__restrict__ parts,
                                                      int n_parts, size_t part_stride,
                                                      const bf16 *__restrict__ embed,
                                                      const int32_t *__restrict__ token_ids,
                                                      const float *__restrict__ g, float eps, int d,
                                                      float *h_out, bf16 *__restrict__ x_out,
                                                      const float *__restrict__ w_head,
                                                      const float *__restrict__ w_head1, float *__restrict__ tok_dot) {
  __shared__ float red[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  float v[ROW_VECS][8];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < ROW_VECS; ++it) {
    const int c = (it * 256 + tid) * 8;
    if (c < d) {
      if (EMBED) {
        const bf16x8 e = *(const bf16x8 *)(embed + (size_t)token_ids[row] * d + c);
#pragma unroll
        for (int k = 0; k < 8; ++k) v[it][k] = (float)e[k];
        float *dst = h_out + (size_t)row * d + c;
        *(f32x4 *)dst = f32x4{v[it][0], v[it][1], v[it][2], v[it][3]};
        *(f32x4 *)(dst + 4) = f32x4{v[it][4], v[it][5], v[it][6], v[it][7]};
      } else {
        const float *src = h_in + (size_t)row * d + c;
        f32x4 a = *(const f32x4 *)src, b = *(const f32x4 *)(src + 4);
        if (n_parts > 0) {
          // For the usual split counts the loads of all partial products go out together (a loop over a
          // run-time count waits for each before it asks for the next); the sums keep the fixed order.
          const float *p0 = parts + (size_t)row * d + c;
#define ARB_ADD_PARTS(NP)                                                      \
  {                                                                            \
    f32x4 pa[NP], pb[NP];                                                      \
    _Pragma("unroll") for (int sp = 0; sp < NP; ++sp) {                        \
      pa[sp] = *(const f32x4 *)(p0 + sp * part_stride);                        \
      pb[sp] = *(const f32x4 *)(p0 + sp * part_stride + 4);                    \
    }                                                                          \
    _Pragma("unroll") for (int sp = 0; sp < NP; ++sp) { a += pa[sp]; b += pb[sp]; } \
  }
          switch (n_parts) {
            case 1: ARB_ADD_PARTS(1) break;
            case 2: ARB_ADD_PARTS(2) break;
            case 3: ARB_ADD_PARTS(3) break;
            case 4: ARB_ADD_PARTS(4) break;
            case 5: ARB_ADD_PARTS(5) break;
            case 8: ARB_ADD_PARTS(8) break;
            default:
              for (int sp = 0; sp < n_parts; ++sp) {
                a += *(const f32x4 *)(p0 + sp * part_stride);
                b += *(const f32x4 *)(p0 + sp * part_stride + 4);
              }
          }
#undef ARB_ADD_PARTS
          if (h_out) {                          // the last norm of a pass has no later reader of h
            float *dst = h_out + (size_t)row * d + c;
            *(f32x4 *)dst = a;
            *(f32x4 *)(dst + 4) = b;
          }
        }
        v[it][0] = a[0]; v[it][1] = a[1]; v[it][2] = a[2]; v[it][3] = a[3];
        v[it][4] = b[0]; v[it][5] = b[1]; v[it][6] = b[2]; v[it][7] = b[3];
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) ss += v[it][k] * v[it][k];
    }
  }
  ss = block_sum_256(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  float dot = 0.f;
#pragma unroll
  for (int it = 0; it < ROW_VECS; ++it) {
    const int c = (it * 256 + tid) * 8;
    if (c < d) {
      const f32x4 g0 = *(const f32x4 *)(g + c), g1 = *(const f32x4 *)(g + c + 4);
      float y[8];
#pragma unroll
      for (int k = 0; k < 4; ++k) { y[k] = v[it][k] * r * g0[k]; y[4 + k] = v[it][4 + k] * r * g1[k]; }
      if (HEAD && w_head) {
        f32x4 w0 = *(const f32x4 *)(w_head + c), w1 = *(const f32x4 *)(w_head + c + 4);
        if (w_head1) {           // two-class head: only the difference of the class logits matters (class 1 minus class 0)
          w0 = *(const f32x4 *)(w_head1 + c) - w0;
          w1 = *(const f32x4 *)(w_head1 + c + 4) - w1;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) dot += y[k] * w0[k] + y[4 + k] * w1[k];
      }
      if (x_out) {
        bf16x8 o;
#pragma unroll
        for (int k = 0; k < 8; ++k) o[k] = (bf16)y[k];
        *(bf16x8 *)(x_out + (size_t)row * d + c) = o;
      }
    }
  }
  if (HEAD && tok_dot) {
    dot = block_sum_256(dot, red);
    if (tid == 0) tok_dot[row] = dot;
  }
}

static arb_status check_row_width(int d) {
  if (d <= 0 || d % 8 != 0 || d > 256 * 8 * ROW_VECS)
    return arb_fail(ARB_EUNSUPPORTED, "row width %d: need a multiple of 8 up to %d", d, 256 * 8 * ROW_VECS);
  return ARB_OK;
}

arb_status launch_embed_rmsnorm(const bf16 *embed, const int32_t *token_ids, const float *g, float eps, int T, int d,
                                float *h, bf16 *x, hipStream_t st) {
  if (T == 0) return ARB_OK;
  if (arb_status s = check_row_width(d)) return s;
  hipLaunchKernelGGL((rmsnorm_kernel<true, false>), dim3(T), dim3(256), 0, st, (const float *)nullptr,
                     (const float *)nullptr, 0, (size_t)0, embed, token_ids, g, eps, d, h, x, (const float *)nullptr,
                     (const float *)nullptr, (float *)nullptr);
  ARB_CHECK_LAUNCH("embed_rmsnorm");
  return ARB_OK;
}

arb_status launch_rmsnorm(float *h, const float *parts, int n_parts, const float *g, float eps, int T, int d, bf16 *x,
                          hipStream_t st) {
  if (T == 0) return ARB_OK;
  if (arb_status s = check_row_width(d)) return s;
  hipLaunchKernelGGL((rmsnorm_kernel<false, false>), dim3(T), dim3(256), 0, st, (const float *)h, parts, n_parts,
                     (size_t)T * d, (const bf16 *)nullptr, (const int32_t *)nullptr, g, eps, d, h, x,
                     (const float *)nullptr, (const float *)nullptr, (float *)nullptr);
  ARB_CHECK_LAUNCH("rmsnorm");
  return ARB_OK;
}

arb_status launch_final_norm_head(const float *h, const float *parts, int n_parts, const float *g, float eps, int T,
                                  int d, const float *w_head, const float *w_head1, bf16 *hidden_out, float *tok_dot,
                                  hipStream_t st) {
  if (T == 0) return ARB_OK;
  if (arb_status s = check_row_width(d)) return s;
  // the residual stream is not needed after the last norm, so the completed row is not written back
  hipLaunchKernelGGL((rmsnorm_kernel<false, true>), dim3(T), dim3(256), 0, st, h, parts, n_parts, (size_t)T * d,
                     (const bf16 *)nullptr, (const int32_t *)nullptr, g, eps, d, (float *)nullptr, hidden_out, w_head,
                     w_head1, tok_dot);
  ARB_CHECK_LAUNCH("final_norm_head");
  return ARB_OK;
}

// ------------------------------------------------------- rotary embedding + KV append

// One block per token.  A work unit is (head, two adjacent pair indices t, t+1):
// it reads u[t..t+1] and u[t+half..t+half+1] of that head, rotates q and k heads
// by the token's table row ((a, b) -> (a cos - b sin, b cos + a sin)), writes q
// (bf16) to the qkv row and k, v (bf16) to the token's slot of the pool
// [n_blocks, Hkv, 16, hd].  With PARTS the projection comes as fp32 split-K partial
// products that are added up here (fixed order), so q and k are rounded once.
template <bool PARTS>
__global__ __launch_bounds__(256) void rope_append_kernel(bf16 *__restrict__ qkv, const float *__restrict__ parts,
                                                          int n_parts, size_t part_stride,
                                                          const f32x2 *__restrict__ cs,
                                                          const int32_t *__restrict__ tok_slot,
                                                          bf16 *__restrict__ k_pool, bf16 *__restrict__ v_pool,
                                                          int Hq, int Hkv, int hd, float q_scale) {
  const int j = blockIdx.x;
  const int half = hd / 2, units_per_head = half / 2, n_heads = Hq + 2 * Hkv;
  bf16 *row = qkv + (size_t)j * n_heads * hd;
  const float *prow = PARTS ? parts + (size_t)j * n_heads * hd : nullptr;
  const int slot = tok_slot[j];
  const size_t blk = slot / ARB_KV_BLOCK, off = slot % ARB_KV_BLOCK;
  // one unit per thread: blockIdx.y walks the units of the token in groups of 256, so that a token's row is
  // one round of memory latency whatever its width (a loop over the units took one round per 256 of them,
  // 6 rounds per token on the 8B shape: most of the kernel's time in small batches)
  const int u = blockIdx.y * blockDim.x + threadIdx.x;
  if (u < n_heads * units_per_head) {
    const int head = u / units_per_head, t = (u - head * units_per_head) * 2;
    bf16 *src = row + head * hd;
    float a[2], b[2];
    if (PARTS) {
      a[0] = a[1] = b[0] = b[1] = 0.f;
      for (int p = 0; p < n_parts; ++p) {
        const float *ps = prow + p * part_stride + head * hd;
        const f32x2 pa = *(const f32x2 *)(ps + t), pb = *(const f32x2 *)(ps + t + half);
        a[0] += pa[0]; a[1] += pa[1]; b[0] += pb[0]; b[1] += pb[1];
      }
    } else {
      const bf16x2 va = *(const bf16x2 *)(src + t), vb = *(const bf16x2 *)(src + t + half);
      a[0] = (float)va[0]; a[1] = (float)va[1]; b[0] = (float)vb[0]; b[1] = (float)vb[1];
    }
    bf16x2 oa, ob;
    if (head < Hq + Hkv) {
      const f32x2 cs0 = cs[(size_t)j * half + t], cs1 = cs[(size_t)j * half + t + 1];
      const float f = head < Hq ? q_scale : 1.0f;          // queries may carry a constant factor for the attention kernel
      oa[0] = (bf16)((a[0] * cs0[0] - b[0] * cs0[1]) * f);
      ob[0] = (bf16)((b[0] * cs0[0] + a[0] * cs0[1]) * f);
      oa[1] = (bf16)((a[1] * cs1[0] - b[1] * cs1[1]) * f);
      ob[1] = (bf16)((b[1] * cs1[0] + a[1] * cs1[1]) * f);
    } else {
      oa[0] = (bf16)a[0]; oa[1] = (bf16)a[1]; ob[0] = (bf16)b[0]; ob[1] = (bf16)b[1];
    }
    bf16 *dst;
    if (head < Hq) {
      dst = src;
    } else if (head < Hq + Hkv) {
      dst = k_pool + ((blk * Hkv + (head - Hq)) * ARB_KV_BLOCK + off) * hd;
    } else {
      dst = v_pool + ((blk * Hkv + (head - Hq - Hkv)) * ARB_KV_BLOCK + off) * hd;
    }
    *(bf16x2 *)(dst + t) = oa;
    *(bf16x2 *)(dst + t + half) = ob;
  }
}

arb_status launch_rope_append(bf16 *qkv, const float *parts, int n_parts, const f32x2 *cs, const int32_t *tok_slot,
                              bf16 *k_pool, bf16 *v_pool, int T, int n_q_heads, int n_kv_heads, int head_dim,
                              float q_scale, hipStream_t st) {
  if (T == 0) return ARB_OK;
  const size_t stride = (size_t)T * (n_q_heads + 2 * n_kv_heads) * head_dim;
  const dim3 grid(T, ceil_div((n_q_heads + 2 * n_kv_heads) * (head_dim / 4), 256));
  if (n_parts > 0)
    hipLaunchKernelGGL((rope_append_kernel<true>), grid, dim3(256), 0, st, qkv, parts, n_parts, stride, cs, tok_slot,
                       k_pool, v_pool, n_q_heads, n_kv_heads, head_dim, q_scale);
  else
    hipLaunchKernelGGL((rope_append_kernel<false>), grid, dim3(256), 0, st, qkv, (const float *)nullptr, 0, stride, cs,
                       tok_slot, k_pool, v_pool, n_q_heads, n_kv_heads, head_dim, q_scale);
  ARB_CHECK_LAUNCH("rope_append");
  return ARB_OK;
}

// ------------------------------------------------------- pooling + head + threshold

// One wave per sequence.  tok_dot[j] = w . y_j, so by linearity of the head
// score_b = mean_j tok_dot[j] + c (mean pooling) or tok_dot[last] + c.
// The sum runs in a fixed order, so repeated calls give identical bits.
// With `probability` the pooled value is the difference of two class logits and the score is the
// softmax probability of class 1, 1 / (1 + exp(-z)) (Sec. 4.2: the router's y_hat).
// Decision (Alg. 1): accept iff score <= tau, i.e. escalate = !(score <= tau).
__global__ __launch_bounds__(64) void pool_route_kernel(const float *__restrict__ tok_dot,
                                                        const int32_t *__restrict__ cu, float b_head, int pool,
                                                        int probability, float tau, float *__restrict__ scores,
                                                        uint8_t *__restrict__ escalate) {
  const int b = blockIdx.x, lo = cu[b], hi = cu[b + 1];
  float acc = 0.f;
  if (pool == ARB_POOL_LAST) {
    acc = tok_dot[hi - 1];
  } else {
    for (int j = lo + (int)threadIdx.x; j < hi; j += 64) acc += tok_dot[j];
    acc = wave_sum(acc) / (float)(hi - lo);
  }
  float score = acc + b_head;
  if (probability) score = 1.0f / (1.0f + expf(-score));
  if (threadIdx.x == 0) {
    scores[b] = score;
    if (escalate) escalate[b] = !(score <= tau);
  }
}

arb_status launch_pool_route(const float *tok_dot, const int32_t *cu_step_lens, int batch, float b_head, int pool,
                             int probability, float tau, float *scores, uint8_t *escalate, hipStream_t st) {
  if (batch == 0) return ARB_OK;
  hipLaunchKernelGGL(pool_route_kernel, dim3(batch), dim3(64), 0, st, tok_dot, cu_step_lens, b_head, pool, probability,
                     tau, scores, escalate);
  ARB_CHECK_LAUNCH("pool_route");
  return ARB_OK;
}

__global__ void route_kernel(const float *__restrict__ scores, int n, float tau, int sense,
                             uint8_t *__restrict__ escalate) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float s = scores[i];
  escalate[i] = sense == ARB_ACCEPT_IF_GT ? !(s > tau) : !(s <= tau);
}

arb_status launch_route(const float *scores, int n, float tau, int sense, uint8_t *escalate, hipStream_t st) {
  if (n == 0) return ARB_OK;
  hipLaunchKernelGGL(route_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, st, scores, n, tau, sense, escalate);
  ARB_CHECK_LAUNCH("route");
  return ARB_OK;
}

// ------------------------------------------------------------- advantage routing

// Definitions 4.1 and 4.2, Eq. 4.4: delta = s_t - s_d; escalate iff not (delta <= tau), the same
// comparison as route_kernel; realized score = s_t where escalated, s_d elsewhere.
__global__ void advantage_route_kernel(const float *__restrict__ s_t, const float *__restrict__ s_d, int n, float tau,
                                    const float *__restrict__ tau_device, float *__restrict__ delta,
                                    uint8_t *__restrict__ escalate, float *__restrict__ realized) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float t = tau_device ? *tau_device : tau;
  const float a = s_t[i], b = s_d[i], d = a - b;
  const bool esc = !(d <= t);
  if (delta) delta[i] = d;
  if (escalate) escalate[i] = esc;
  if (realized) realized[i] = esc ? a : b;
}

arb_status launch_advantage_route(const float *s_t, const float *s_d, int n, float tau, const float *tau_device,
                               float *delta, uint8_t *escalate, float *realized, hipStream_t st) {
  if (n == 0) return ARB_OK;
  hipLaunchKernelGGL(advantage_route_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, st, s_t, s_d, n, tau, tau_device, delta,
                     escalate, realized);
  ARB_CHECK_LAUNCH("advantage_route");
  return ARB_OK;
}

// Threshold for a budget of escalations (Theorem B.1): tau = max(0, the (budget+1)-th largest delta),
// found by a most-significant-byte-first radix select in one workgroup (n is a number of reasoning
// steps, not of tokens).  Keys order floats as unsigned integers; NaN, which escalates under any tau,
// ranks above every number, and if the selected entry is a NaN the result is +inf.
__device__ __forceinline__ uint32_t order_key(float x) {
  if (x != x) return 0xFFFFFFFFu;
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(256) void budget_threshold_kernel(const float *__restrict__ delta, int n, int budget,
                                                               float *__restrict__ tau_out) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sel_prefix, sel_rank;
  const int tid = threadIdx.x;
  if (budget >= n) {                        // nothing is cut off: every positive advantage may escalate
    if (tid == 0) *tau_out = 0.f;
    return;
  }
  uint32_t prefix = 0, rank = (uint32_t)budget;        // rank from the top among keys matching the prefix
  for (int shift = 24; shift >= 0; shift -= 8) {
    hist[tid] = 0;
    __syncthreads();
    const uint32_t mask = shift == 24 ? 0u : 0xFFFFFFFFu << (shift + 8);
    for (int i = tid; i < n; i += 256) {
      const uint32_t k = order_key(delta[i]);
      if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t r = rank;
      int b = 255;
      for (; b > 0; --b) {
        if (r < hist[b]) break;
        r -= hist[b];
      }
      sel_prefix = prefix | ((uint32_t)b << shift);
      sel_rank = r;
    }
    __syncthreads();
    prefix = sel_prefix;
    rank = sel_rank;
    __syncthreads();
  }
  if (tid == 0) {
    float t;
    if (prefix == 0xFFFFFFFFu) {
      t = __uint_as_float(0x7F800000u);                 // the NaNs alone exceed the budget
    } else {
      const uint32_t u = (prefix & 0x80000000u) ? (prefix & 0x7FFFFFFFu) : ~prefix;
      t = __uint_as_float(u);
      t = t > 0.f ? t : 0.f;
    }
    *tau_out = t;
  }
}

arb_status launch_budget_threshold(const float *delta, int n, int budget, float *tau_out, hipStream_t st) {
  hipLaunchKernelGGL(budget_threshold_kernel, dim3(1), dim3(256), 0, st, delta, n, budget, tau_out);
  ARB_CHECK_LAUNCH("budget_threshold");
  return ARB_OK;
}

// ------------------------------------------------------- next-token choice (LM head)

// Rows rows[i] of a bf16 [*, d] matrix, copied to a dense [n, d] matrix (the last step token of each
// sequence, as input of the LM head GEMM).
__global__ void gather_rows_kernel(const bf16 *__restrict__ src, const int32_t *__restrict__ rows, int d,
                                   bf16 *__restrict__ dst) {
  const int i = blockIdx.x;
  const bf16 *s = src + (size_t)rows[i] * d;
  for (int c = threadIdx.x * 8; c < d; c += blockDim.x * 8) *(bf16x8 *)(dst + (size_t)i * d + c) = *(const bf16x8 *)(s + c);
}

arb_status launch_gather_rows(const bf16 *src, const int32_t *rows, int n, int d, bf16 *dst, hipStream_t st) {
  if (n == 0) return ARB_OK;
  if (d % 8 != 0) return arb_fail(ARB_EUNSUPPORTED, "gather_rows: width %d is not a multiple of 8", d);
  hipLaunchKernelGGL(gather_rows_kernel, dim3(n), dim3(256), 0, st, src, rows, d, dst);
  ARB_CHECK_LAUNCH("gather_rows");
  return ARB_OK;
}

// One block per row of fp32 logits [n, V].  Greedy (temperature <= 0): the smallest index of the
// maximum.  Otherwise the token is drawn from softmax(logits / temperature) by inversion with the
// caller's uniform u in [0, 1): the smallest k with sum_{i<=k} w_i >= u * sum_i w_i, where
// w_i = exp((l_i - max) / temperature); sums run in index order within a thread's contiguous range
// and in thread order across ranges, so a call is reproducible.
__global__ __launch_bounds__(256) void sample_token_kernel(const float *__restrict__ logits, int V, float temperature,
                                                           const float *__restrict__ uniforms,
                                                           int32_t *__restrict__ token, float *__restrict__ chosen) {
  __shared__ float red_v[256];
  __shared__ int red_i[256];
  const int row = blockIdx.x, tid = threadIdx.x;
  const float *l = logits + (size_t)row * V;
  const int per = (V + 255) / 256, lo = min(tid * per, V), hi = min(lo + per, V);    // contiguous range of this thread
  float best = -INFINITY;
  int arg = V;
  for (int i = lo; i < hi; ++i) {
    const float v = l[i];
    if (v > best) { best = v; arg = i; }
  }
  red_v[tid] = best;
  red_i[tid] = arg;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) {
      const float v = red_v[tid + o];
      const int a = red_i[tid + o];
      if (v > red_v[tid] || (v == red_v[tid] && a < red_i[tid])) { red_v[tid] = v; red_i[tid] = a; }
    }
    __syncthreads();
  }
  const float mx = red_v[0];
  const int amax = red_i[0] < V ? red_i[0] : 0;          // a row of NaNs or -inf picks token 0
  __syncthreads();
  if (!(temperature > 0.f)) {
    if (tid == 0) {
      token[row] = amax;
      if (chosen) chosen[row] = l[amax];
    }
    return;
  }
  const float inv_t = 1.0f / temperature;
  __shared__ float total_s;
  __shared__ int pick_s;
  float part = 0.f;
  for (int i = lo; i < hi; ++i) part += expf((l[i] - mx) * inv_t);
  red_v[tid] = part;
  __syncthreads();
  if (tid == 0) {                                       // exclusive prefix over the 256 ranges, in order
    float run = 0.f;
    for (int t = 0; t < 256; ++t) {
      const float p = red_v[t];
      red_v[t] = run;
      run += p;
    }
    total_s = run;
    pick_s = V;
  }
  __syncthreads();
  const float target = uniforms[row] * total_s;
  const float before = red_v[tid];
  // the range that contains the target: before < target <= before + part (the first range also takes target == 0)
  if (lo < hi && (target > before || tid == 0) && target <= before + part) {
    float run = before;
    int pick = hi - 1;                                  // rounding in the re-summation cannot leave the range
    for (int i = lo; i < hi; ++i) {
      run += expf((l[i] - mx) * inv_t);
      if (run >= target) { pick = i; break; }
    }
    atomicMin(&pick_s, pick);
  }
  __syncthreads();
  if (tid == 0) {
    const int k = pick_s < V ? pick_s : amax;           // no range claimed the target (rounding at the very end): the mode
    token[row] = k;
    if (chosen) chosen[row] = l[k];
  }
}

arb_status launch_sample_token(const float *logits, int n, int V, float temperature, const float *uniforms,
                               int32_t *token, float *chosen, hipStream_t st) {
  if (n == 0) return ARB_OK;
  hipLaunchKernelGGL(sample_token_kernel, dim3(n), dim3(256), 0, st, logits, V, temperature, uniforms, token, chosen);
  ARB_CHECK_LAUNCH("sample_token");
  return ARB_OK;
}

// Length of a generated step (Alg. 1: tokens up to and including the first separator or
// end-of-sequence token) for each row of tokens [n, S]; S if neither occurs.
__global__ void first_stop_kernel(const int32_t *__restrict__ tokens, int n, int S, int sep, int eos,
                                  int32_t *__restrict__ len, uint8_t *__restrict__ ended) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= n) return;
  int L = S;
  uint8_t e = 0;
  for (int i = 0; i < S; ++i) {
    const int t = tokens[(size_t)b * S + i];
    if (t == sep || t == eos) { L = i + 1; e = t == eos; break; }
  }
  len[b] = L;
  if (ended) ended[b] = e;
}

arb_status launch_first_stop(const int32_t *tokens, int n, int S, int sep, int eos, int32_t *len, uint8_t *ended,
                             hipStream_t st) {
  if (n == 0) return ARB_OK;
  hipLaunchKernelGGL(first_stop_kernel, dim3(ceil_div(n, 64)), dim3(64), 0, st, tokens, n, S, sep, eos, len, ended);
  ARB_CHECK_LAUNCH("first_stop");
  return ARB_OK;
}

// One decoding iteration of steps that are generated token by token (Alg. 1: a step ends with its first
// separator or end-of-sequence token, or at S tokens).  Row r = open_rows[j] was fed this iteration and chose
// chosen[j]: the token is appended, len and done are updated, and the rows that stay open are written in
// order to next_rows with their tokens in next_ids (the ids of the next iteration).  One workgroup walks the
// open rows 256 at a time; the order-preserving compaction is a ballot per wave plus a scan over the waves.
__global__ __launch_bounds__(256) void step_advance_kernel(const int32_t *__restrict__ open_rows,
                                                           const int32_t *__restrict__ chosen, int n_open, int S, int sep,
                                                           int eos, int32_t *__restrict__ steps, int32_t *__restrict__ len,
                                                           uint8_t *__restrict__ done, int32_t *__restrict__ next_rows,
                                                           int32_t *__restrict__ next_ids, int32_t *__restrict__ n_next) {
  __shared__ int wave_count[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int base = 0;                                  // rows kept by the chunks before this one
  for (int j0 = 0; j0 < n_open; j0 += 256) {
    const int j = j0 + threadIdx.x;
    bool keep = false;
    int r = 0, t = 0;
    if (j < n_open) {
      r = open_rows[j];
      t = chosen[j];
      const int l = len[r];
      steps[(size_t)r * S + l] = t;
      len[r] = l + 1;
      const bool stop = t == sep || t == eos || l + 1 >= S;
      done[r] = stop ? (t == eos ? 2 : 1) : 0;
      keep = !stop;
    }
    const unsigned long long mask = __builtin_amdgcn_ballot_w64(keep);
    if (lane == 0) wave_count[wave] = __builtin_popcountll(mask);
    __syncthreads();
    int before = base;
    for (int w = 0; w < wave; ++w) before += wave_count[w];
    if (keep) {
      const int pos = before + __builtin_popcountll(mask & ((1ull << lane) - 1ull));
      next_rows[pos] = r;
      next_ids[pos] = t;
    }
    base += wave_count[0] + wave_count[1] + wave_count[2] + wave_count[3];
    __syncthreads();
  }
  if (threadIdx.x == 0) *n_next = base;
}

arb_status launch_step_advance(const int32_t *open_rows, const int32_t *chosen, int n_open, int S, int sep, int eos,
                               int32_t *steps, int32_t *len, uint8_t *done, int32_t *next_rows, int32_t *next_ids,
                               int32_t *n_next, hipStream_t st) {
  hipLaunchKernelGGL(step_advance_kernel, dim3(1), dim3(256), 0, st, open_rows, chosen, n_open, S, sep, eos, steps, len,
                     done, next_rows, next_ids, n_next);
  ARB_CHECK_LAUNCH("step_advance");
  return ARB_OK;
}

// ids[cu[j] + i] = steps[rows[j]][i] for i < cu[j+1] - cu[j]: the steps of the listed rows as one ragged token list
__global__ __launch_bounds__(256) void pack_steps_kernel(const int32_t *__restrict__ steps, int S,
                                                         const int32_t *__restrict__ rows, const int32_t *__restrict__ cu,
                                                         int n_rows, int32_t *__restrict__ ids) {
  const int j = blockIdx.x;
  if (j >= n_rows) return;
  const int r = rows[j], begin = cu[j], n = min(cu[j + 1] - begin, S);
  for (int i = threadIdx.x; i < n; i += blockDim.x) ids[begin + i] = steps[(size_t)r * S + i];
}

arb_status launch_pack_steps(const int32_t *steps, int S, const int32_t *rows, const int32_t *cu, int n_rows, int32_t *ids,
                             hipStream_t st) {
  if (n_rows == 0) return ARB_OK;
  hipLaunchKernelGGL(pack_steps_kernel, dim3(n_rows), dim3(256), 0, st, steps, S, rows, cu, n_rows, ids);
  ARB_CHECK_LAUNCH("pack_steps");
  return ARB_OK;
}

