// Projection GEMM with 4-bit weights and bf16 activations (the weight-quantized draft of the
// self-draft regime, Section 5.1): C[M,N] = A[M,K] * W'[N,K]^T with
// W'[n,k] = q[n,k] * scale[n, k/128], q in [-8, 7] stored as offset-binary nibbles, eight
// consecutive k per uint32, scale bf16.
//
// Structure of the 128x128x64 bf16 kernel (4 waves of 64x64, double-buffered LDS, A by direct-to-LDS
// loads), except for the weight operand: each thread fetches 16 bytes of packed weights (32 nibbles of
// one row) one step ahead into registers, expands them to the bf16 integers -8..7 (exact) and stores
// them into the LDS stage.  The MFMAs therefore accumulate sum_k a[m,k] q[n,k] per group of 128 k
// (two steps) into a temporary accumulator; at the end of a group it is folded into the result with
// one fp32 multiply by the group's scale.  No product q*scale is ever rounded to bf16, so the result
// differs from the definition only by fp32 accumulation.  Weight traffic is a quarter of the bf16
// kernel's, which is what the small-M (decode) case is bound by.
#include "common.h"

namespace {

constexpr int BM = 128, BN = 128, BK = 64, GROUP = 128;
constexpr int LDS_TILE = BM * BK;
constexpr int kSkinnyRows = 32;     // up to this many activation rows the weight-streaming kernel runs
constexpr int kSkinnyAhead = 3;     // groups of packed weights a wave of that kernel has in flight

#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ int lds_off(int row, int chunk) {   // element offset of a 16-byte chunk, 128-byte rows
  return row * BK + ((chunk ^ ((row >> 1) & 7)) << 3);
}

// eight nibbles (k ascending from the least significant) -> the bf16 integers nibble - 8
__device__ __forceinline__ bf16x8 expand_nibbles(uint32_t w) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    // 2^23 + nibble as a float, minus (2^23 + 8): exact
    const float f = __uint_as_float(0x4B000000u | ((w >> (4 * e)) & 15u)) - 8388616.0f;
    o[e] = (bf16)f;
  }
  return o;
}

// Eight nibbles as the bf16 values 16 + nibble = 24 + q, without a conversion instruction (those run at a quarter
// of the rate of plain integer instructions here, and sixteen of them per word bound the kernel): in the binade
// [16, 32) a bf16 is 16 (1 + m / 128), so a nibble placed in the four top bits of the mantissa adds exactly its
// value.  Two nibbles four apart are placed by one shift and one and-or, so the elements come out in the order
// 0, 4, 1, 5, 2, 6, 3, 7 (the caller orders the other operand alike).  The constant 24 is taken out again in
// fp32: sum_k a_k (24 + q_k) - 24 sum_k a_k, with the second sum from an MFMA against ones; the terms are about
// five times the size of the result, so fp32 loses two or three more bits than without the detour, far below
// what the rounding of the output, or an fp32 test bar of 1e-5, sees.
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t bits) {      // (x & mask) | bits, one instruction
  uint32_t d;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(x), "s"(mask), "v"(bits));
  return d;
}
__device__ __forceinline__ bf16x8 expand_nibbles_plus24(uint32_t w) {
  const uint32_t mask = 0x00780078u, bits = 0x41804180u;
  u32x4 d;
  d[0] = and_or(w << 3, mask, bits);
  d[1] = and_or(w >> 1, mask, bits);
  d[2] = and_or(w >> 5, mask, bits);
  d[3] = and_or(w >> 9, mask, bits);
  return __builtin_bit_cast(bf16x8, d);
}
// elements 0..7 -> 0, 4, 1, 5, 2, 6, 3, 7
__device__ __forceinline__ bf16x8 interleave_halves(bf16x8 a) {
  const u32x4 r = __builtin_bit_cast(u32x4, a);
  u32x4 d;
  d[0] = __builtin_amdgcn_perm(r[2], r[0], 0x05040100u);
  d[1] = __builtin_amdgcn_perm(r[2], r[0], 0x07060302u);
  d[2] = __builtin_amdgcn_perm(r[3], r[1], 0x05040100u);
  d[3] = __builtin_amdgcn_perm(r[3], r[1], 0x07060302u);
  return __builtin_bit_cast(bf16x8, d);
}

// QMAX = 7: 4-bit integers -8..7; QMAX = 3: 3-bit integers -4..3 (same nibble storage)
template <int QMAX>
__global__ __launch_bounds__(256) void w4_quantize_kernel(const bf16 *__restrict__ W, int N, int K,
                                                          uint32_t *__restrict__ packed, bf16 *__restrict__ scales) {
  // 16 threads per group of 128 weights, 8 weights (one word) each
  const int groups_per_row = K / GROUP;
  const long long gid = (long long)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int l16 = threadIdx.x & 15;
  if (gid >= (long long)N * groups_per_row) return;
  const int n = (int)(gid / groups_per_row), g = (int)(gid - (long long)n * groups_per_row);
  const bf16x8 w = *(const bf16x8 *)(W + (size_t)n * K + g * GROUP + l16 * 8);
  float m = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf((float)w[e]));
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 16));
  const bf16 scale = (bf16)(m / (float)QMAX);
  const float sf = (float)scale;
  uint32_t word = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float q = sf == 0.f ? 0.f : rintf((float)w[e] / sf);
    q = fminf(fmaxf(q, -(float)(QMAX + 1)), (float)QMAX);
    word |= (uint32_t)((int)q + 8) << (4 * e);
  }
  packed[(size_t)n * (K / 8) + g * 16 + l16] = word;
  if (l16 == 0) scales[gid] = scale;
}

constexpr int EPI_PARTIAL_F32 = ARB_EPI_STORE_F32;   // in a split-K launch split s stores to C + s*M*N

template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_w4_kernel(const bf16 *__restrict__ A, const uint32_t *__restrict__ Bq,
                                                      const bf16 *__restrict__ Bscale, void *__restrict__ Cv, int M,
                                                      int N, int K, int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(16))) bf16 As0[LDS_TILE], As1[LDS_TILE], Bs0[LDS_TILE], Bs1[LDS_TILE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  constexpr int TILE_GROUP = 4;
  tile_of<TILE_GROUP>(xcd_remap(blockIdx.x, tiles_m * tiles_n), tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM;
  const int frag_row = lane & 31, frag_half = lane >> 5;

  // weight row of tile-local B row r.  SwiGLU: wave column r/64, MFMA tile (r%64)/32 (0 = gate, 1 = up),
  // feature offset r%32; N = F there and the up rows follow the F gate rows.
  auto weight_row = [&](int r) {
    if (EPI == ARB_EPI_SWIGLU_BF16) {
      const int f = tile_n * 64 + (r >> 6) * 32 + (r & 31);
      return ((r >> 5) & 1) ? N + f : f;
    }
    return tile_n * BN + r;
  };

  // A: four 16-byte chunks per thread and step, by direct-to-LDS loads (swizzle on the global side)
  const bf16 *a_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + 256 * i, row = c >> 3, chunk = (c & 7) ^ ((row >> 1) & 7);
    int am = m0 + row;
    am = am < M ? am : M - 1;                       // tail rows re-read the last row; never stored
    a_src[i] = A + (size_t)am * K + chunk * 8;
  }
  // B: 32 nibbles (16 bytes) of tile row tid/2 per thread and step
  const int b_row = tid >> 1, b_half = tid & 1;
  const uint32_t *bq_src = Bq + (size_t)weight_row(b_row) * (K / 8) + b_half * 4;
  // scales of this lane's two output column tiles
  const bf16 *sc_src[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) sc_src[j] = Bscale + (size_t)weight_row(wn * 64 + j * 32 + frag_row) * (K / GROUP);

  f32x16 acc[2][2], tmp[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = tmp[i][j][r] = 0.f;

  // K range of this workgroup in whole groups (two steps each)
  const int ng_all = K / GROUP;
  const int g_begin = (int)((long long)ng_all * blockIdx.y / gridDim.y);
  const int ng = (int)((long long)ng_all * (blockIdx.y + 1) / gridDim.y) - g_begin;
  const int nk = 2 * ng, last = nk - 1;
#pragma unroll
  for (int i = 0; i < 4; ++i) a_src[i] += (size_t)g_begin * GROUP;
  bq_src += (size_t)g_begin * (GROUP / 8);

  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto dma_a = [&](int buf, int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(a_src[i] + (size_t)kt * BK), LDS_PTR((buf ? As1 : As0) + (i * 4 + wave_u) * 512), 16, 0, 0);
  };
  auto load_b = [&](int kt) { return *(const u32x4 *)(bq_src + (size_t)kt * (BK / 8)); };
  auto store_b = [&](int buf, u32x4 w) {
#pragma unroll
    for (int c = 0; c < 4; ++c) *(bf16x8 *)&(buf ? Bs1 : Bs0)[lds_off(b_row, b_half * 4 + c)] = expand_nibbles(w[c]);
  };
  auto compute = [&](int buf) {
    bf16x8 fa[2][2], fb[2][2];
    auto frags = [&](int slot, int kk) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[slot][i] = *(const bf16x8 *)&(buf ? As1 : As0)[lds_off(wm * 64 + i * 32 + frag_row, kk * 2 + frag_half)];
        fb[slot][i] = *(const bf16x8 *)&(buf ? Bs1 : Bs0)[lds_off(wn * 64 + i * 32 + frag_row, kk * 2 + frag_half)];
      }
    };
    frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) frags((kk + 1) & 1, kk + 1);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          tmp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i], fb[kk & 1][j], tmp[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Step kt is multiplied out of stage kt%2 while the A tile of step kt+1 streams into the other stage
  // and the packed weights of step kt+2 are on their way to registers; the weights of step kt+1 are
  // expanded into the other stage after the MFMAs of step kt.  Steps come in pairs (one group).
  dma_a(0, 0);
  u32x4 bw = load_b(0);
  store_b(0, bw);
  bw = load_b(min(1, last));
  __syncthreads();
  for (int kt = 0; kt < nk; kt += 2) {
    const int g = g_begin + (kt >> 1);
    const float sc0 = (float)sc_src[0][g], sc1 = (float)sc_src[1][g];
    dma_a(1, kt + 1);
    __builtin_amdgcn_sched_barrier(0);
    compute(0);
    store_b(1, bw);
    bw = load_b(min(kt + 2, last));
    __syncthreads();
    dma_a(0, min(kt + 2, last));
    __builtin_amdgcn_sched_barrier(0);
    compute(1);
    store_b(0, bw);
    bw = load_b(min(kt + 3, last));
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc[i][0][r] = fmaf(tmp[i][0][r], sc0, acc[i][0][r]);
        acc[i][1][r] = fmaf(tmp[i][1][r], sc1, acc[i][1][r]);
        tmp[i][0][r] = 0.f;
        tmp[i][1][r] = 0.f;
      }
    __syncthreads();
  }

  // D layout of the 32x32 MFMA: lane holds column lane%32 and rows 8*(r/4) + 4*(lane/32) + r%4.
  if (EPI == ARB_EPI_SWIGLU_BF16) {
    bf16 *C = (bf16 *)Cv;
    const int col = tile_n * 64 + wn * 32 + frag_row;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
        if (m < M) {
          const float gte = acc[i][0][r], up = acc[i][1][r];
          C[(size_t)m * N + col] = (bf16)(gte * __builtin_amdgcn_rcpf(1.0f + __expf(-gte)) * up);
        }
      }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = tile_n * BN + wn * 64 + j * 32 + frag_row;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
          if (m < M) {
            if (EPI == ARB_EPI_STORE_BF16) {
              ((bf16 *)Cv)[(size_t)m * N + col] = (bf16)acc[i][j][r];
            } else if (EPI == EPI_PARTIAL_F32) {
              ((float *)Cv)[((size_t)blockIdx.y * M + m) * N + col] = acc[i][j][r];
            } else {
              float *dst = (float *)Cv + (size_t)m * N + col;
              *dst += acc[i][j][r];
            }
          }
        }
      }
  }
}


// Few tokens (M <= 32: drafting token by token): the product is bound by streaming the packed weights once,
// so there is no tile of A to share.  A workgroup owns 64 weight rows (SwiGLU: 32 gate rows and the 32 up
// rows of the same features) and a K range; its four waves take the 128-wide groups of that range in turn and
// each multiplies whole groups: a lane fetches the 32 + 32 bytes of its two weight rows (one per 32-row
// block) and of a group half straight from memory, kSkinnyAhead groups ahead, expands them in registers and
// feeds them to the MFMAs as the column operand, against activation fragments from a tile of the wave's own in
// LDS (MR rows x 128, direct-to-LDS loads NS - 1 groups ahead; fetched straight into registers, 16 bytes per
// lane from up to 32 rows, the time grew with the number of rows).  What bounds a wave is the chain of round
// trips to memory, one per group it cannot request early enough: with the activations one group ahead the 8B
// gate/up shape took 30 us whatever the expansion cost (three versions of it) and even with all weights
// resident in L2; hence the deeper ring where the tile is small (16 rows: four stages).  Within a group lane
// half h owns k = 64 h .. 64 h + 63, eight per MFMA step: the contraction order is free as long as both operands
// agree.  The four partial results meet in LDS for the epilogue.  Arithmetic as in the tile kernel: integer
// weights in the MFMAs (here 24 + q, see expand_nibbles_plus24), one fp32 multiply by the group's scale per group.
template <int EPI, int MR, int NS>
__global__ __launch_bounds__(256, 2) void gemm_w4_skinny_kernel(const bf16 *__restrict__ A, const uint32_t *__restrict__ Bq,
                                                                const bf16 *__restrict__ Bscale, void *__restrict__ Cv,
                                                                int M, int N, int K) {
  static_assert((MR == 16 && NS == 4) || (MR == 32 && NS == 2), "64 KB of stages");
  constexpr int NW = kSkinnyAhead + 1;                 // register sets of packed weights
  static_assert(NW % NS == 0 && NW >= NS, "one unrolled ring for both");
  constexpr int WAVE_TILE = MR * GROUP;                // elements of a wave's activation tile
  // One array per stage, so that reads of one are not ordered behind the loads in flight into another.  After the
  // loop the first arrays hold the partial results: per wave [row block][accumulator register][lane] floats (8 KB).
  __shared__ __attribute__((aligned(16))) bf16 St0[4 * WAVE_TILE], St1[4 * WAVE_TILE], St2[NS > 2 ? 4 * WAVE_TILE : 8],
      St3[NS > 2 ? 4 * WAVE_TILE : 8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int tile = blockIdx.x;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int ng_all = K / GROUP;
  const int g_begin = (int)((long long)ng_all * blockIdx.y / gridDim.y);
  const int g_end = (int)((long long)ng_all * (blockIdx.y + 1) / gridDim.y);
  const uint32_t *bq[2];
  const bf16 *sc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = EPI == ARB_EPI_SWIGLU_BF16 ? (j ? N : 0) + tile * 32 + col : tile * 64 + j * 32 + col;
    bq[j] = Bq + (size_t)row * (K / 8) + half * 8;
    sc[j] = Bscale + (size_t)row * (K / GROUP);
  }
  auto stage = [&](int st) -> bf16 * {
    return (st == 0 ? St0 : st == 1 ? St1 : st == 2 ? St2 : St3) + wave_u * WAVE_TILE;
  };
  // A direct-to-LDS load moves four activation rows of the group (4 x 256 bytes, 16 lanes each); a row's sixteen
  // 16-byte chunks land XORed with the row number so that the fragment reads (16 rows, one chunk) are free of
  // bank conflicts.  Rows past M re-read the last row: they only feed output rows that are never stored.
  const int dma_row = lane >> 4, dma_slot = lane & 15;
  auto dma_a = [&](int g, int st) {
    g = g < g_end ? g : g_end - 1;                       // past the range: a valid group, not used
    bf16 *dst = stage(st);
#pragma unroll
    for (int j = 0; j < MR / 4; ++j) {
      const int r = 4 * j + dma_row;
      const bf16 *src = A + (size_t)(r < M ? r : M - 1) * K + (size_t)g * GROUP + ((dma_slot ^ (r & 15)) << 3);
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src), LDS_PTR(dst + j * 512), 16, 0, 0);
    }
  };
  // Fragments of the eight MFMA steps of a group: this lane's row (rows past the tile repeat it), chunks 8 half + i.
  // They are read by inline assembly with its own wait: for LDS reads that it can see, the compiler makes the wave
  // wait for every load in flight whenever it cannot tell their stage from the one a direct-to-LDS load is filling
  // (here: in two of four groups), which puts a round trip to memory into each of those groups.
  const int frag_row = col & (MR - 1);
  unsigned frag_off[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) frag_off[i] = (unsigned)(frag_row * GROUP + (((half * 8 + i) ^ (frag_row & 15)) << 3)) * 2u;
  auto read_frags = [&](int st, bf16x8 (&fa)[8]) {
    const unsigned base = (unsigned)(uintptr_t)LDS_PTR(stage(st));
    asm volatile(
        "ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %10\n\tds_read_b128 %3, %11\n\t"
        "ds_read_b128 %4, %12\n\tds_read_b128 %5, %13\n\tds_read_b128 %6, %14\n\tds_read_b128 %7, %15\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(fa[0]), "=&v"(fa[1]), "=&v"(fa[2]), "=&v"(fa[3]), "=&v"(fa[4]), "=&v"(fa[5]), "=&v"(fa[6]), "=&v"(fa[7])
        : "v"(base + frag_off[0]), "v"(base + frag_off[1]), "v"(base + frag_off[2]), "v"(base + frag_off[3]),
          "v"(base + frag_off[4]), "v"(base + frag_off[5]), "v"(base + frag_off[6]), "v"(base + frag_off[7])
        : "memory");
  };

  f32x16 acc[2], tmp[2], asum;                         // asum: the activations' own sum over the group, per output row
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[0][r] = acc[1][r] = tmp[0][r] = tmp[1][r] = asum[r] = 0.f;

  // The packed weights of a group and, with them, their scales (loads complete in order, so a scale fetched when
  // it is needed would make the wave wait for everything requested before it).  Requested by inline assembly: the
  // compiler then keeps no account of them, and the one counted wait in front of a group is the only wait there
  // is; for loads that it issues itself it falls back to waiting for all of them wherever it loses count (across
  // the loop's back edge: once per turn).  A set is read only behind the counted wait that covers it.
  struct Fetched { u32x4 w[2][2]; unsigned s[2]; };
  auto load_w = [&](int g, Fetched &f) {
    g = g < g_end ? g : g_end - 1;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t *src = bq[j] + (size_t)g * 16;
      asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(f.w[j][0]) : "v"(src) : "memory");
      asm volatile("global_load_dwordx4 %0, %1, off offset:16" : "=&v"(f.w[j][1]) : "v"(src) : "memory");
      asm volatile("global_load_ushort %0, %1, off" : "=&v"(f.s[j]) : "v"(sc[j] + g) : "memory");
    }
  };

  // The n-th group of a wave uses weight set n % NW and stage n % NS; the loop is unrolled over NW groups so that
  // both are fixed per position.  In front of group n the wave requests the tile of group n + NS - 1 and then the
  // weights of group n + NW - 1 (6 loads); the prologue issues the same requests in the same order.
  const int g_first = g_begin + wave_u;
  if (g_first < g_end) {
    Fetched f[NW];
#pragma unroll
    for (int d = 0; d < NW - NS; ++d) load_w(g_first + 4 * d, f[d]);
#pragma unroll
    for (int k = 0; k < NS - 1; ++k) {
      asm volatile("" ::: "memory");       // the compiler keeps the order of the requests: the counted wait relies on it
      dma_a(g_first + 4 * k, k);
      asm volatile("" ::: "memory");
      load_w(g_first + 4 * (NW - NS + k), f[NW - NS + k]);
    }
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (bf16)1.0f;
    for (int base = g_first; base < g_end; base += 4 * NW) {
#pragma unroll
      for (int u = 0; u < NW; ++u) {
        const int gg = base + 4 * u;
        if (gg >= g_end) break;
        // What this group reads must have landed: its tile, requested NS - 1 groups ago, and its weights, requested
        // NW - 1 groups ago, i.e. earlier than the tile (NW > NS) or right behind it (NW == NS).  Every group since
        // has requested MR / 4 + 6 loads, and loads complete in order, so: at most 6 outstanding (the weights that
        // followed the tile, NW > NS = 2), or at most (NS - 2) (MR / 4 + 6) = 20 (NW == NS = 4).  The wave reads
        // only its own tile, so no barrier is needed.
        static_assert((NS == 2 && NW > NS) || (NS == 4 && NW == NS && (NS - 2) * (MR / 4 + 6) == 20), "the counted waits below");
        if (NS == 2) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(20)" ::: "memory");
        dma_a(gg + 4 * (NS - 1), (u + NS - 1) % NS);
        asm volatile("" ::: "memory");
        load_w(gg + 4 * (NW - 1), f[(u + NW - 1) % NW]);
        asm volatile("" ::: "memory");
        const Fetched &cur = f[u];
        const float s0 = __uint_as_float(cur.s[0] << 16), s1 = __uint_as_float(cur.s[1] << 16);     // bf16 -> fp32
        bf16x8 frags[8];
        read_frags(u % NS, frags);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const bf16x8 fa = interleave_halves(frags[i]);
          tmp[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, expand_nibbles_plus24(cur.w[0][i >> 2][i & 3]), tmp[0], 0, 0, 0);
          tmp[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, expand_nibbles_plus24(cur.w[1][i >> 2][i & 3]), tmp[1], 0, 0, 0);
          asum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, ones, asum, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          acc[0][r] = fmaf(fmaf(-24.f, asum[r], tmp[0][r]), s0, acc[0][r]);
          acc[1][r] = fmaf(fmaf(-24.f, asum[r], tmp[1][r]), s1, acc[1][r]);
          tmp[0][r] = 0.f;
          tmp[1][r] = 0.f;
          asum[r] = 0.f;
        }
      }
    }
  }

  __syncthreads();                                       // every wave is done with its stage reads (and loads)
  // partial results of wave w: 8 KB each, four of them in the first array (32-row tiles) or two per array
  auto part = [&](int w) -> float * {
    return MR == 32 ? (float *)St0 + w * 2048 : (float *)(w < 2 ? St0 : St1) + (w & 1) * 2048;
  };
  {
    float *mine = part(wave_u);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) mine[(j * 16 + r) * 64 + lane] = acc[j][r];
  }
  __syncthreads();
  // D layout of the 32x32 MFMA: lane holds column lane%32 (a weight row) and rows (tokens) 8*(r/4) + 4*(lane/32) + r%4.
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int idx = tid + 256 * p, r = idx >> 6, L = idx & 63;
    const int m = 8 * (r >> 2) + 4 * (L >> 5) + (r & 3), c = L & 31;
    float v[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int at = (j * 16 + r) * 64 + L;
      v[j] = (part(0)[at] + part(1)[at]) + (part(2)[at] + part(3)[at]);
    }
    if (m >= M) continue;
    if (EPI == ARB_EPI_SWIGLU_BF16) {
      ((bf16 *)Cv)[(size_t)m * N + tile * 32 + c] = (bf16)(v[0] * __builtin_amdgcn_rcpf(1.0f + __expf(-v[0])) * v[1]);
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const size_t at = (size_t)m * N + tile * 64 + j * 32 + c;
        if (EPI == ARB_EPI_STORE_BF16) ((bf16 *)Cv)[at] = (bf16)v[j];
        else if (EPI == EPI_PARTIAL_F32) ((float *)Cv)[(size_t)blockIdx.y * M * N + at] = v[j];
        else ((float *)Cv)[at] += v[j];
      }
    }
  }
}

}  // namespace

arb_status launch_w4_quantize(const bf16 *W, int N, int K, uint32_t *packed, bf16 *scales, int bits, hipStream_t st) {
  if (N == 0) return ARB_OK;
  if (bits != 3 && bits != 4) return arb_fail(ARB_EUNSUPPORTED, "weight quantization to %d bits (3 or 4)", bits);
  if (N < 0 || K <= 0 || K % GROUP != 0) return arb_fail(ARB_EUNSUPPORTED, "w4_quantize: N=%d, K=%d (K must be a multiple of %d)", N, K, GROUP);
  const long long groups = (long long)N * (K / GROUP);
  const dim3 grid((unsigned)((groups + 15) / 16)), block(256);
  if (bits == 4) hipLaunchKernelGGL(w4_quantize_kernel<7>, grid, block, 0, st, W, N, K, packed, scales);
  else hipLaunchKernelGGL(w4_quantize_kernel<3>, grid, block, 0, st, W, N, K, packed, scales);
  ARB_CHECK_LAUNCH("w4_quantize");
  return ARB_OK;
}

arb_status launch_gemm_w4(const bf16 *A, const uint32_t *Bq, const bf16 *Bscale, void *C, int M, int N, int K,
                          int epilogue, hipStream_t st, int splits) {
  if (M == 0) return ARB_OK;
  if (M < 0 || N <= 0 || K <= 0) return arb_fail(ARB_EINVAL, "gemm_w4: M=%d N=%d K=%d", M, N, K);
  if (K % GROUP != 0) return arb_fail(ARB_EUNSUPPORTED, "gemm_w4: K=%d is not a multiple of %d", K, GROUP);
  const int tiles_m = ceil_div(M, BM);
  int tiles_n;
  if (epilogue == ARB_EPI_SWIGLU_BF16) {
    if (N % 64 != 0) return arb_fail(ARB_EUNSUPPORTED, "gemm_w4: SwiGLU width %d is not a multiple of 64", N);
    tiles_n = N / 64;
  } else {
    if (N % BN != 0) return arb_fail(ARB_EUNSUPPORTED, "gemm_w4: N=%d is not a multiple of %d", N, BN);
    tiles_n = N / BN;
  }
  if (splits > 1 && epilogue != ARB_EPI_RESIDUAL_F32 && epilogue != ARB_EPI_STORE_F32)
    return arb_fail(ARB_EINVAL, "gemm_w4: split-K needs an fp32 epilogue (partial products)");
  if (splits < 1 || splits > K / GROUP) return arb_fail(ARB_EINVAL, "gemm_w4: %d splits of %d groups", splits, K / GROUP);
  const bool skinny = M <= kSkinnyRows;                // few tokens: the weight-streaming kernel, 64 weight rows per workgroup
  const dim3 grid(skinny ? (epilogue == ARB_EPI_SWIGLU_BF16 ? N / 32 : N / 64) : tiles_m * tiles_n, splits), block(256);
#define ARB_W4(E)                                                                                                    \
  do {                                                                                                               \
    if (skinny && M <= 16)                                                                                           \
      hipLaunchKernelGGL((gemm_w4_skinny_kernel<E, 16, 4>), grid, block, 0, st, A, Bq, Bscale, C, M, N, K);          \
    else if (skinny)                                                                                                 \
      hipLaunchKernelGGL((gemm_w4_skinny_kernel<E, 32, 2>), grid, block, 0, st, A, Bq, Bscale, C, M, N, K);          \
    else hipLaunchKernelGGL((gemm_w4_kernel<E>), grid, block, 0, st, A, Bq, Bscale, C, M, N, K, tiles_m, tiles_n);   \
  } while (0)
  switch (epilogue) {
    case ARB_EPI_STORE_BF16: ARB_W4(ARB_EPI_STORE_BF16); break;
    case ARB_EPI_RESIDUAL_F32:
      if (splits > 1) ARB_W4(EPI_PARTIAL_F32); else ARB_W4(ARB_EPI_RESIDUAL_F32);
      break;
    case ARB_EPI_SWIGLU_BF16: ARB_W4(ARB_EPI_SWIGLU_BF16); break;
    case ARB_EPI_STORE_F32: ARB_W4(ARB_EPI_STORE_F32); break;
    default: return arb_fail(ARB_EINVAL, "gemm_w4: unknown epilogue %d", epilogue);
  }
#undef ARB_W4
  ARB_CHECK_LAUNCH("gemm_w4");
  return ARB_OK;
}
