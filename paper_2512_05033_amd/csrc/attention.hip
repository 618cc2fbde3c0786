// Ragged GQA append-attention over a block-paged bf16 KV cache.
//
// Work decomposition.  For sequence b and kv head hk, the G = Hq/Hkv query heads
// that share hk and the s_b step tokens form s_b*G query rows (row = i*G + g,
// token-major).  A workgroup of 4 waves takes 128 rows (32 per wave) and one
// chunk of the key range ("split"); chunks of a sequence are merged afterwards
// from their online-softmax states (m, l) and normalised partial results (bf16).  Every KV byte is
// streamed from HBM once per 128 rows that need it; rows of different query
// tiles of the same (b, hk) meet in L2.
//
// Per 64-key tile, K and V stream into LDS row-major [key][hd] (XOR-swizzled
// 16-byte chunks) by direct-to-LDS global loads, double-buffered: tile t+1 is in
// flight while tile t is multiplied out.  S^T = K Q^T (keys are MFMA rows, queries are columns), so a
// lane owns one query column: the row max / row sum are in-lane reductions plus
// one cross-half shuffle, and exp2(S^T - m) is already laid out as the B operand
// of O^T = V^T P^T.  The V^T fragments (a lane needs 8 keys of one hd column) come
// from the LDS transpose read ds_read_b64_tr_b16: within 16 lanes, source lane j
// points at 4 consecutive columns of one row and lane i receives element i%4 of
// source lanes i/4, 4+i/4, 8+i/4, 12+i/4; with source lane j addressing key j/4,
// columns 4*(j%4).., lane i gets column i of four consecutive keys.  The pairing of
// MFMA contraction slots with keys follows the 32x32 D layout (lane half h,
// registers 8u..8u+7 of tile t hold keys 32t+16u+4h+{0..3} and
// 32t+16u+8+4h+{0..3}); V^T is read with the same pairing.
#include "common.h"

#include <math.h>

namespace {

constexpr int QROWS = 128;     // query rows per workgroup
constexpr int KT = 64;         // keys per tile
constexpr float kLazyLog2 = 8.0f;   // growth of a row maximum (log2 units) that forces a rescale

typedef short s16x4 __attribute__((ext_vector_type(4)));

#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// Chunk swizzles.  A key row of a stage is HD/8 chunks of 16 bytes; chunk c of key k sits in slot
// c ^ swizzle(k).  The LDS has 64 banks of 4 bytes and serves 256 bytes per clock:
//  - K is read with ds_read_b128, 16 lanes (16 consecutive keys, one chunk) per clock: the slots of
//    16 consecutive keys must cover 256 bytes, so with 256-byte rows the swizzle is k mod 16, with
//    128-byte rows (two keys per 256 bytes) it is (k/2) mod 8;
//  - V is read with ds_read_b64_tr_b16, 32 lanes (4 consecutive keys x 4 consecutive chunks) per
//    clock: the two low key bits must move the slot by multiples of 4, so the key bits are rotated
//    (measured on this access pattern: 171 bytes/clock/CU against 63 with the K swizzle).
template <int HD>
__device__ __forceinline__ int k_swizzle(int key) { return HD == 128 ? (key & 15) : ((key >> 1) & 7); }
template <int HD>
__device__ __forceinline__ int v_swizzle(int key) {
  if (HD == 128) return ((key & 3) << 2) | ((key >> 2) & 3);
  const int x = (key >> 1) & 7;                  // 128-byte rows: the row parity picks the 128-byte half
  return ((x & 1) << 2) | (x >> 1);
}
template <int HD>
__device__ __forceinline__ int k_off(int key, int chunk) { return key * HD + ((chunk ^ k_swizzle<HD>(key)) << 3); }   // elements
template <int HD>
__device__ __forceinline__ int v_off(int key, int chunk) { return key * HD + ((chunk ^ v_swizzle<HD>(key)) << 3); }

// One 64-key tile for one wave: scores, online softmax update, O^T accumulation.
//
// PRESCALED: the queries arrive multiplied by log2(e)/sqrt(hd) (the forward's rotary kernel stores them that
// way, in fp32 before their one rounding), so K Q^T is already the logit in log2 units, and the score MFMAs
// start from the accumulator tuple `negm` (every element = minus the lane's reference maximum): the matrix
// pipe delivers s - m, and the vector ALU, which is the busier pipe of this kernel, is left with one exp2,
// half a max3, half a dot2 (row sum over the rounded probabilities, the ones the PV product uses) and half a
// convert per score.  Otherwise (queries as given, exact) the scale and the reference are applied to the fp32
// scores by one FMA per score; negm[0] then holds minus the reference.
template <int HD, bool PRESCALED>
__device__ __forceinline__ void attend_tile(const bf16 *sk, const bf16 *sv, const bf16x8 (&qf)[HD / 16], f32x16 (&o)[HD / 32],
                                            f32x16 &negm, float &m_run, float &l_run, int ts, int limit, float scale_log2,
                                            int col, int half, int lane) {
  constexpr int KSTEPS = HD / 16, MT = HD / 32;
  f32x16 st[2];
  if (!PRESCALED) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) st[t][r] = 0.f;
  }
  {
    // K fragments are requested two steps ahead of the MFMAs that take them (an LDS read takes longer
    // than the two MFMAs of a step)
    bf16x8 kf[3][2];
#pragma unroll
    for (int pre = 0; pre < 2; ++pre)
#pragma unroll
      for (int t = 0; t < 2; ++t) kf[pre][t] = *(const bf16x8 *)&sk[k_off<HD>(t * 32 + col, pre * 2 + half)];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      if (kk + 2 < KSTEPS) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
          kf[(kk + 2) % 3][t] = *(const bf16x8 *)&sk[k_off<HD>(t * 32 + col, (kk + 2) * 2 + half)];
      }
#pragma unroll
      for (int t = 0; t < 2; ++t)
        st[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk % 3][t], qf[kk], PRESCALED && kk == 0 ? negm : st[t], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // Causal mask (it also hides keys past the context): only tiles that reach some row's limit pay
  // for it.  Register r of tile t holds key ts + 32t + 8(r/4) + 4*half + r%4.
  const int vis = limit - ts - 4 * half;
  if (__builtin_amdgcn_ballot_w64(vis < KT - 1) != 0) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) st[t][r] = (t * 32 + 8 * (r >> 2) + (r & 3)) <= vis ? st[t][r] : -INFINITY;
  }
  // largest logit this lane holds for its query (the positive scale commutes with max), relative to the
  // reference maximum.  A query's keys are split between lanes l and l ^ 32; the two are only combined
  // (a cross-lane exchange) on the rare path below.
  float mx = -INFINITY;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[t][r]);
  if (!PRESCALED) mx = fmaf(mx, scale_log2, negm[0]);
  // The reference maximum m_run is advanced only when some row's maximum has outgrown it by more
  // than kLazyLog2: until then exp2(s - m_run) <= 2^kLazyLog2, far inside the range of bf16 and
  // fp32, and o / l is unchanged because both carry the same factor.  Most tiles then skip the
  // rescaling of the accumulators.  A row without a visible key so far has m_run = -inf and the
  // reference 0; its first visible key always sets the reference.
  if (__builtin_amdgcn_ballot_w64(mx > kLazyLog2 || (m_run == -INFINITY && mx > -INFINITY)) != 0) {
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_use = m_run == -INFINITY ? 0.f : m_run;
    const float m_new = fmaxf(m_run, m_use + mx);                    // -inf only while nothing is visible
    const float m_new_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new_use);   // m_run = -inf -> 0
    l_run *= alpha;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[mt][r] *= alpha;
    if (PRESCALED) {
      const float shift = m_new_use - m_use;                         // the scores were taken against the old reference
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) st[t][r] -= shift;
#pragma unroll
      for (int r = 0; r < 16; ++r) negm[r] = -m_new_use;
    } else {
      negm[0] = -m_new_use;
    }
    m_run = m_new;
  }
  if (!PRESCALED) {
    const float nm = negm[0];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) st[t][r] = fmaf(st[t][r], scale_log2, nm);
  }
  bf16x8 pf[2][2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) pf[t][r >> 3][r & 7] = (bf16)__builtin_amdgcn_exp2f(st[t][r]);   // raw v_exp_f32; -inf -> 0
  // row sum over the probabilities as the PV product sees them (bf16), two per instruction
  {
    bf16x2 ones;
    ones[0] = ones[1] = (bf16)1.0f;
    float l_add = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          bf16x2 pr;
          pr[0] = pf[t][u][e];
          pr[1] = pf[t][u][e + 1];
          l_add = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l_add, false);
        }
    l_run += l_add;
  }
  // O^T += V^T P^T; V^T fragments by transpose reads (see the header comment)
  const int j16 = lane & 15;
  const int vcol = 16 * ((lane >> 4) & 1) + 4 * (j16 & 3);     // within a 32-column tile
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int key0 = t * 32 + u * 16 + 4 * half + (j16 >> 2);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int c = mt * 32 + vcol;
        const bf16 *a0 = &sv[v_off<HD>(key0, c >> 3) + (c & 7)];
        const bf16 *a1 = &sv[v_off<HD>(key0 + 8, c >> 3) + (c & 7)];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)a0);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)a1);
        union { s16x4 s[2]; bf16x8 b; } vf;
        vf.s[0] = lo;
        vf.s[1] = hi;
        o[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.b, pf[t][u], o[mt], 0, 0, 0);
      }
    }
}

template <int HD, bool SPLIT, bool PRESCALED>
__global__ __launch_bounds__(256, 2) void attention_kernel(
    const bf16 *__restrict__ q, int q_row_stride, const bf16 *__restrict__ k_pool, const bf16 *__restrict__ v_pool,
    const int32_t *__restrict__ block_tables, int max_blocks, const int32_t *__restrict__ prefix_lens,
    const int32_t *__restrict__ cu, int T, int Hq, int Hkv, int max_qtiles, int max_splits, int kv_chunk,
    float scale_log2, bf16 *__restrict__ out, bf16 *__restrict__ part_acc, float *__restrict__ part_ml, int n_groups) {
  constexpr int CPK = HD / 8;              // 16-byte chunks per key
  constexpr int LOADS = KT * CPK / 256;    // wave-wide 1 KB loads per wave, operand and tile
  constexpr int KPL = 64 / CPK;            // keys covered by one wave-wide load (4 or 8: inside one block)
  constexpr int KSTEPS = HD / 16;          // MFMA k-steps over the head dimension
  constexpr int MT = HD / 32;              // 32-row tiles of O^T
  // Two stages of K and V; one array per stage so that LDS reads of one stage are not ordered
  // behind the direct-to-LDS loads in flight into the other.
  __shared__ __attribute__((aligned(16))) bf16 K0[KT * HD], K1[KT * HD], V0[KT * HD], V1[KT * HD];

  // Work item of this workgroup.  The hardware deals workgroups round-robin to the 8 XCDs (blockIdx % 8), and
  // an XCD works through its share in order.  The query tiles of one group (sequence, split, kv head) stream the
  // same keys: they stay on one XCD, next to each other in its order, and meet in its L2.  The groups are dealt
  // round-robin with the kv head as the fastest index, then the split: consecutive groups are equally long, so
  // every XCD gets the same share of every sequence.  (With a contiguous range of sequences per XCD the XCD
  // with the longest ones finished last: on 16 contexts of 5 K to 32 K keys only 59 % of the workgroup slots
  // were busy on average, 75 % with this order.)
  const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
  const int qtile = slot % max_qtiles;
  int item = (slot / max_qtiles) * 8 + xcd;                 // group index
  if (item >= n_groups) return;
  const int hk = item % Hkv; item /= Hkv;
  const int split = item % max_splits;
  const int b = item / max_splits;
  const int G = Hq / Hkv;
  const int p = prefix_lens[b], tok0 = cu[b], s = cu[b + 1] - tok0;
  const int rows = s * G, row0 = qtile * QROWS;
  if (row0 >= rows) return;
  const int last_row = min(rows, row0 + QROWS) - 1;
  const int visible = p + last_row / G + 1;            // keys any row of this tile may see
  const int kv_begin = split * kv_chunk;
  if (kv_begin >= visible) return;
  const int kv_end = min(visible, kv_begin + kv_chunk);
  const int ctx = p + s;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const bool wave_active = row0 + wave * 32 < rows;    // waves past the last row only help with the loads

  // this lane's query row
  const int row = row0 + wave * 32 + col;
  const bool row_ok = row < rows;
  const int tok_i = row_ok ? row / G : 0;
  const int head = hk * G + (row_ok ? row - tok_i * G : 0);
  const int limit = p + tok_i;                         // last visible key (inclusive)

  bf16x8 qf[KSTEPS];
  {
    const bf16 *qrow = q + (size_t)(tok0 + tok_i) * q_row_stride + head * HD;
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      if (row_ok) {
        qf[kk] = *(const bf16x8 *)(qrow + kk * 16 + half * 8);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[kk][e] = (bf16)0.f;
      }
    }
  }

  f32x16 o[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[mt][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  f32x16 negm;                               // minus the reference maximum (PRESCALED: in every element, the score MFMAs' C operand)
#pragma unroll
  for (int r = 0; r < 16; ++r) negm[r] = 0.f;

  // Tile loads.  One wave-wide direct-to-LDS load moves KPL whole keys (1 KB) of one 16-key block:
  // the block id is wave-uniform (scalar), lane l lands in chunk slot l % CPK of key l / CPK and
  // fetches the logical chunk that the read-side swizzle expects there.  Keys past the context
  // re-read the last valid key (finite data; they are masked out of the softmax anyway), so every
  // address is in bounds and the loop body needs no branch.
  const int32_t *table = block_tables + (size_t)b * max_blocks;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int last_key = ctx - 1, last_blk = last_key / ARB_KV_BLOCK;
  const int n_tiles = (kv_end - kv_begin + KT - 1) / KT;
  const int lkey = lane / CPK, pchunk = lane % CPK;
  int blk_id[LOADS];                       // pool block of each load of the tile to be issued next
  const unsigned first_blk = (unsigned)kv_begin / ARB_KV_BLOCK + (unsigned)(wave_u * KPL) / ARB_KV_BLOCK;
  auto lookup = [&](int tile) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const unsigned blk = first_blk + (unsigned)(tile * KT + i * 4 * KPL) / ARB_KV_BLOCK;
      blk_id[i] = table[min(blk, (unsigned)last_blk)];
    }
  };
  // Lane-constant part of the addresses: load i of a tile covers keys [wave*KPL, wave*KPL + KPL) of the
  // tile's 16-key block i*KPL/4 + wave*KPL/16, so the key inside its block and the swizzled chunk do not
  // depend on i or on the tile; only the (scalar) pool block does.
  const int kib = (wave_u * KPL + lkey) % ARB_KV_BLOCK;
  const int tkey = wave_u * KPL + lkey;            // tile-local key of load 0 (the others differ by multiples of 16 or 32)
  const unsigned koff = (unsigned)(kib * HD + ((pchunk ^ k_swizzle<HD>(tkey)) << 3)) * 2u;                  // bytes
  const unsigned voff = (unsigned)(kib * HD + ((pchunk ^ v_swizzle<HD>(tkey)) << 3)) * 2u;
  const int kib_tail = min(kib, last_key % ARB_KV_BLOCK);
  const unsigned koff_tail = koff - (unsigned)((kib - kib_tail) * HD) * 2u, voff_tail = voff - (unsigned)((kib - kib_tail) * HD) * 2u;
  const char *k_head = (const char *)(k_pool + (size_t)hk * ARB_KV_BLOCK * HD);
  const char *v_head = (const char *)(v_pool + (size_t)hk * ARB_KV_BLOCK * HD);
  const unsigned blk_bytes = (unsigned)Hkv * ARB_KV_BLOCK * HD * 2u;
  auto dma = [&](bf16 *dk, bf16 *dv, int tile) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int g = i * 4 + wave_u;                                  // 1 KB slot of the tile
      const unsigned blk = first_blk + (unsigned)(tile * KT + i * 4 * KPL) / ARB_KV_BLOCK;
      const bool tail = blk >= (unsigned)last_blk;                    // scalar choice between two lane vectors
      const uint64_t base = (uint64_t)(unsigned)blk_id[i] * blk_bytes;
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(k_head + base + (tail ? koff_tail : koff)), LDS_PTR(dk + g * 512), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(v_head + base + (tail ? voff_tail : voff)), LDS_PTR(dv + g * 512), 16, 0, 0);
    }
  };

  // Tile t is multiplied out of one stage while tile t+1 streams into the other and the block ids
  // of tile t+2 are looked up; the barrier that ends a step also waits for the loads.
  const int last_tile = n_tiles - 1;
  lookup(0);
  dma(K0, V0, 0);
  lookup(min(1, last_tile));
  __syncthreads();
  for (int t = 0; t < n_tiles; t += 2) {
    dma(K1, V1, min(t + 1, last_tile));
    lookup(min(t + 2, last_tile));
    __builtin_amdgcn_sched_barrier(0);
    if (wave_active) attend_tile<HD, PRESCALED>(K0, V0, qf, o, negm, m_run, l_run, kv_begin + t * KT, limit, scale_log2, col, half, lane);
    __syncthreads();
    if (t + 1 < n_tiles) {
      dma(K0, V0, min(t + 2, last_tile));
      lookup(min(t + 3, last_tile));
      __builtin_amdgcn_sched_barrier(0);
      if (wave_active) attend_tile<HD, PRESCALED>(K1, V1, qf, o, negm, m_run, l_run, kv_begin + (t + 1) * KT, limit, scale_log2, col, half, lane);
      __syncthreads();
    }
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (!row_ok) return;
  const size_t orow = (size_t)(tok0 + tok_i) * Hq + head;   // (token, head) index
  if (!SPLIT) {
    const float inv = 1.0f / l_tot;
    bf16 *dst = out + orow * HD;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[mt][r4 * 4 + e] * inv);
        *(bf16x4 *)(dst + mt * 32 + 8 * r4 + 4 * half) = v;
      }
  } else {
    // the split's own normalised result in bf16 (it lies in the hull of the values, like the output)
    // plus its (m, l) in fp32: half the partial traffic of fp32 accumulators
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    bf16 *dst = part_acc + ((size_t)split * T * Hq + orow) * HD;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[mt][r4 * 4 + e] * inv);
        *(bf16x4 *)(dst + mt * 32 + 8 * r4 + 4 * half) = v;
      }
    if (half == 0) {
      float *ml = part_ml + ((size_t)split * T * Hq + orow) * 2;
      ml[0] = m_run;
      ml[1] = l_tot;
    }
  }
}

// Merge of the split partials: out = sum_s w_s l_s o_s / sum_s w_s l_s with
// w_s = exp2(m_s - max_s m_s) and o_s the split's normalised result.  A thread owns eight
// consecutive elements of one (token, head) row, so a workgroup of 256 merges 2048 / HD rows.
template <int HD>
__global__ __launch_bounds__(256) void attention_merge_kernel(const bf16 *__restrict__ part_acc,
                                                              const float *__restrict__ part_ml,
                                                              const int32_t *__restrict__ tok_pos, int T, int Hq,
                                                              int kv_chunk, bf16 *__restrict__ out) {
  constexpr int TPR = HD / 8;                              // threads per row
  const size_t stride = (size_t)T * Hq;
  const size_t idx = (size_t)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;      // token * Hq + head
  if (idx >= stride) return;
  const int piece = threadIdx.x % TPR;
  const int n_splits = tok_pos[idx / Hq] / kv_chunk + 1;   // splits that start at or before this token's position
  float m = -INFINITY, l = 0.f;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  // Splits are taken eight at a time: all their loads go out together (a loop over a run-time count waits for
  // each before it asks for the next), then they are combined under their common maximum; groups of eight are
  // chained by the usual online rescaling.
  for (int s0 = 0; s0 < n_splits; s0 += 8) {
    float2 ml[8];
    bf16x8 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (s0 + j < n_splits) {
        ml[j] = *(const float2 *)(part_ml + ((s0 + j) * stride + idx) * 2);
        v[j] = *(const bf16x8 *)(part_acc + ((s0 + j) * stride + idx) * HD + piece * 8);
      } else {
        ml[j] = float2{-INFINITY, 0.f};
#pragma unroll
        for (int e = 0; e < 8; ++e) v[j][e] = (bf16)0.f;
      }
    }
    float m_new = m;
#pragma unroll
    for (int j = 0; j < 8; ++j) m_new = fmaxf(m_new, ml[j].x);
    if (m_new == -INFINITY) continue;                      // no key of these splits is visible to the row
    const float keep = exp2f(m - m_new);                   // m = -inf: 0
    m = m_new;
    l *= keep;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= keep;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float w = exp2f(ml[j].x - m_new) * ml[j].y;    // a split without visible keys: exp2(-inf) * 0 = 0
      l += w;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += w * (float)v[j][e];
    }
  }
  const float inv = 1.0f / l;
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16)(acc[e] * inv);
  *(bf16x8 *)(out + idx * HD + piece * 8) = r;
}

}  // namespace

static const int kTargetWorkgroups = 512;    // two resident workgroups per CU on 256 CUs
static const int kMinChunk = 256, kMaxChunk = 4096, kMaxChunkDecode = 8192, kMaxSplits = 64;

float attention_q_scale(int head_dim) { return (float)(1.4426950408889634 / sqrt((double)head_dim)); }

int attention_splits_cap(int max_ctx) {
  if (max_ctx <= 0) return 1;
  const int n = ceil_div(max_ctx, kMinChunk);
  return n < kMaxSplits ? n : kMaxSplits;
}

AttnPlan plan_attention(int batch, const int32_t *prefix_host, const int32_t *cu_host, int G, int n_kv_heads) {
  long long keys_streamed = 0;          // sum over (sequence, kv head, query tile) of the context length
  int max_ctx = 0, max_step = 0;
  for (int b = 0; b < batch; ++b) {
    const int s = cu_host[b + 1] - cu_host[b], ctx = prefix_host[b] + s;
    keys_streamed += (long long)ceil_div(s * G, QROWS) * n_kv_heads * ctx;
    max_ctx = ctx > max_ctx ? ctx : max_ctx;
    max_step = s > max_step ? s : max_step;
  }
  // Keys per split: about kTargetWorkgroups workgroups (one resident round) when contexts are short,
  // so that few partial states have to be merged; never more than kMaxChunk keys, so that long
  // ragged contexts become several rounds of similar-sized workgroups instead of one unbalanced round
  // (measured on the ragged workloads: 4096 beats 2048 by 2-3 %, 8192 loses).  A batch whose steps all
  // fit one wave (32 query rows: drafting token by token) only streams the cache: there the longer
  // chunk of kMaxChunkDecode wins (fewer prologues and partial states: 5.3 -> 5.7 TB/s).
  const int cap = max_step * G <= 32 ? kMaxChunkDecode : kMaxChunk;
  long long chunk = (keys_streamed / kTargetWorkgroups + KT - 1) / KT * KT;
  if (chunk > cap) chunk = cap;
  if (chunk < kMinChunk) chunk = kMinChunk;
  while (max_ctx > chunk * kMaxSplits) chunk += KT;
  AttnPlan pl;
  pl.max_qtiles = ceil_div(max_step * G, QROWS);
  pl.kv_chunk = (int)chunk;
  pl.max_splits = max_ctx > 0 ? ceil_div(max_ctx, pl.kv_chunk) : 1;
  return pl;
}

size_t attention_ws_bytes(int max_splits_cap, int total_tokens, int n_q_heads, int head_dim) {
  const size_t rows = (size_t)max_splits_cap * total_tokens * n_q_heads;
  return align_up(rows * head_dim * sizeof(bf16), 256) + align_up(rows * 2 * sizeof(float), 256) +
         align_up((size_t)total_tokens * sizeof(int32_t), 256);
}

arb_status launch_attention(const bf16 *q, int q_row_stride, const bf16 *k_pool, const bf16 *v_pool,
                            const int32_t *block_tables, int max_blocks_per_seq, const int32_t *prefix_lens,
                            const int32_t *cu_step_lens, int batch, int total_tokens, int n_q_heads, int n_kv_heads,
                            int head_dim, const AttnPlan &plan, const int32_t *tok_pos_in, bf16 *out, void *ws, size_t ws_bytes,
                            hipStream_t st, bool q_prescaled) {
  if (batch == 0 || total_tokens == 0) return ARB_OK;
  if (head_dim != 64 && head_dim != 128) return arb_fail(ARB_EUNSUPPORTED, "attention: head_dim %d", head_dim);
  const bool split = plan.max_splits > 1;
  bf16 *part_acc = nullptr;
  float *part_ml = nullptr;
  const int32_t *tok_pos = tok_pos_in;      // position of every step token; computed here when not given
  if (split) {
    const size_t need = attention_ws_bytes(plan.max_splits, total_tokens, n_q_heads, head_dim);
    if (ws == nullptr || ws_bytes < need)
      return arb_fail(ARB_ECAPACITY, "attention: workspace %zu < %zu bytes", ws_bytes, need);
    const size_t rows = (size_t)plan.max_splits * total_tokens * n_q_heads;
    char *pws = (char *)ws;
    part_acc = (bf16 *)pws; pws += align_up(rows * head_dim * sizeof(bf16), 256);
    part_ml = (float *)pws;  pws += align_up(rows * 2 * sizeof(float), 256);
    if (!tok_pos) {
      tok_pos = (int32_t *)pws;
      if (arb_status s = launch_token_meta(prefix_lens, cu_step_lens, block_tables, batch, total_tokens,
                                           max_blocks_per_seq, ARB_KV_BLOCK, (int32_t *)pws, nullptr, st))
        return s;
    }
  }
  const float scale_log2 = attention_q_scale(head_dim);
  const int n_groups = batch * n_kv_heads * plan.max_splits;      // (sequence, split, kv head)
  const dim3 grid(ceil_div(n_groups, 8) * 8 * plan.max_qtiles), block(256);
#define ARB_ATTN_LAUNCH(HD, SPLIT, PRE)                                                                            \
  hipLaunchKernelGGL((attention_kernel<HD, SPLIT, PRE>), grid, block, 0, st, q, q_row_stride, k_pool, v_pool,      \
                     block_tables, max_blocks_per_seq, prefix_lens, cu_step_lens, total_tokens, n_q_heads,         \
                     n_kv_heads, plan.max_qtiles, plan.max_splits, plan.kv_chunk, scale_log2, out, part_acc, part_ml, n_groups)
#define ARB_ATTN_PICK(HD)                                                                                          \
  if (split) { if (q_prescaled) ARB_ATTN_LAUNCH(HD, true, true); else ARB_ATTN_LAUNCH(HD, true, false); }          \
  else       { if (q_prescaled) ARB_ATTN_LAUNCH(HD, false, true); else ARB_ATTN_LAUNCH(HD, false, false); }
  if (head_dim == 128) { ARB_ATTN_PICK(128) } else { ARB_ATTN_PICK(64) }
#undef ARB_ATTN_PICK
#undef ARB_ATTN_LAUNCH
  ARB_CHECK_LAUNCH("attention");
  if (split) {
    const dim3 mgrid(ceil_div(total_tokens * n_q_heads, 2048 / head_dim)), mblock(256);
    if (head_dim == 128)
      hipLaunchKernelGGL((attention_merge_kernel<128>), mgrid, mblock, 0, st, part_acc, part_ml, tok_pos, total_tokens,
                         n_q_heads, plan.kv_chunk, out);
    else
      hipLaunchKernelGGL((attention_merge_kernel<64>), mgrid, mblock, 0, st, part_acc, part_ml, tok_pos, total_tokens,
                         n_q_heads, plan.kv_chunk, out);
    ARB_CHECK_LAUNCH("attention_merge");
  }
  return ARB_OK;
}
