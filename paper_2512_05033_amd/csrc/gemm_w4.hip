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

// The same eight nibbles as the bf16 integers 16 * (nibble - 8), with half the instructions: nibble ^ 8 is the
// two's-complement form of nibble - 8, and in the high half of a byte it is the signed byte 16 * (nibble - 8),
// which one conversion with a sign-extending byte select turns into a float.  The factor 16 goes into the
// group's scale.
template <int BYTE>
__device__ __forceinline__ float signed_byte_to_float(uint32_t x) {
  float f;
  if (BYTE == 0) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0" : "=v"(f) : "v"(x));
  if (BYTE == 1) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1" : "=v"(f) : "v"(x));
  if (BYTE == 2) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2" : "=v"(f) : "v"(x));
  if (BYTE == 3) asm("v_cvt_f32_i32_sdwa %0, sext(%1) dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3" : "=v"(f) : "v"(x));
  return f;
}
__device__ __forceinline__ bf16x8 expand_nibbles_x16(uint32_t w) {
  const uint32_t t = w ^ 0x88888888u;
  const uint32_t even = (t << 4) & 0xF0F0F0F0u, odd = t & 0xF0F0F0F0u;      // nibbles 0,2,4,6 / 1,3,5,7 as signed bytes
  bf16x8 o;
  o[0] = (bf16)signed_byte_to_float<0>(even); o[1] = (bf16)signed_byte_to_float<0>(odd);
  o[2] = (bf16)signed_byte_to_float<1>(even); o[3] = (bf16)signed_byte_to_float<1>(odd);
  o[4] = (bf16)signed_byte_to_float<2>(even); o[5] = (bf16)signed_byte_to_float<2>(odd);
  o[6] = (bf16)signed_byte_to_float<3>(even); o[7] = (bf16)signed_byte_to_float<3>(odd);
  return o;
}

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
  const bf16 scale = (bf16)(m / 7.0f);
  const float sf = (float)scale;
  uint32_t word = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float q = sf == 0.f ? 0.f : rintf((float)w[e] / sf);
    q = fminf(fmaxf(q, -8.f), 7.f);
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
// so there is no tile of A to share and no LDS stage.  A workgroup owns 64 weight rows (SwiGLU: 32 gate rows
// and the 32 up rows of the same features) and a K range; its four waves take the 128-wide groups of that range
// in turn and each multiplies whole groups: a lane fetches the 32 + 32 bytes of its two weight rows (one per
// 32-row block) and of a group half straight from memory, several groups ahead, expands them in registers and
// feeds them to the MFMAs as the column operand, against activation fragments from a tile of its own in LDS,
// loaded one group ahead (fetched straight into registers, 16 bytes per lane from up to 32 rows, the time grew
// with the number of rows: 30 us at one row, 38 us at 32 on the 8B gate/up shape; staged, 30-33 us at any).  Within a group lane half h owns k = 64 h .. 64 h + 63, eight per MFMA step: the
// contraction order is free as long as both operands agree.  The four partial results meet in LDS for the
// epilogue.  Same arithmetic as the tile kernel: integer weights in the MFMAs (here 16 q, exact in bf16), one
// fp32 multiply by the group's scale (here scale / 16, exact) per group.
template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_w4_skinny_kernel(const bf16 *__restrict__ A, const uint32_t *__restrict__ Bq,
                                                                const bf16 *__restrict__ Bscale, void *__restrict__ Cv,
                                                                int M, int N, int K) {
  // Activations: every wave stages the 32 x 128 tile of its group in a region of its own (8 KB per stage, two
  // stages; one array per stage so that reads of one are not ordered behind the loads in flight into the other).
  // After the loop the first stage array holds the partial results: [wave][row block][accumulator register][lane].
  __shared__ __attribute__((aligned(16))) bf16 St0[4 * 32 * GROUP], St1[4 * 32 * GROUP];
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
  // A direct-to-LDS load moves four activation rows of the group (4 x 256 bytes, 16 lanes each); a row's sixteen
  // 16-byte chunks land XORed with the row number so that the fragment reads (16 rows, one chunk) are free of
  // bank conflicts.  Only the rows that exist are loaded: the others only feed output rows that are never stored.
  const int n_dma = (M + 3) / 4;
  const int dma_row = lane >> 4, dma_slot = lane & 15;
  auto dma_a = [&](int g, int stage) {
    g = g < g_end ? g : g_end - 1;
    bf16 *dst = (stage ? St1 : St0) + wave_u * (32 * GROUP);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (j < n_dma) {
        const int r = 4 * j + dma_row;
        const bf16 *src = A + (size_t)(r < M ? r : M - 1) * K + (size_t)g * GROUP + ((dma_slot ^ (r & 15)) << 3);
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src), LDS_PTR(dst + j * 512), 16, 0, 0);
      }
    }
  };
  // fragment of MFMA step i: this lane's row, chunk 8 half + i
  const int frag_off = col * GROUP;
  auto frag_a = [&](int stage, int i) {
    const bf16 *reg = (stage ? St1 : St0) + wave_u * (32 * GROUP);
    return *(const bf16x8 *)&reg[frag_off + (((half * 8 + i) ^ (col & 15)) << 3)];
  };

  f32x16 acc[2], tmp[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = tmp[j][r] = 0.f;

  // the packed weights of a group and, with them, their scales: loads complete in order, so a scale fetched when it
  // is needed would make the wave wait for everything requested before it
  struct Fetched { u32x4 w[2][2]; bf16 s[2]; };
  auto load_w = [&](int g, Fetched &f) {
    g = g < g_end ? g : g_end - 1;                       // past the range: a valid group, not used
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      f.w[j][0] = *(const u32x4 *)(bq[j] + (size_t)g * 16);
      f.w[j][1] = *(const u32x4 *)(bq[j] + (size_t)g * 16 + 4);
      f.s[j] = sc[j][g];
    }
  };
  // The weights of kAhead groups are in flight while one is multiplied (a ring of kAhead + 1 register sets, the
  // loop unrolled over it so that every set has a fixed place); activations one group ahead.
  constexpr int NW = kSkinnyAhead + 1;
  static_assert(NW % 2 == 0, "the activation sets alternate inside the unrolled ring");
  const int g_first = g_begin + wave;
  if (g_first < g_end) {
    Fetched f[NW];
    dma_a(g_first, 0);
#pragma unroll
    for (int d = 0; d < NW - 1; ++d) load_w(g_first + 4 * d, f[d]);
    for (int base = g_first; base < g_end; base += 4 * NW) {
#pragma unroll
      for (int u = 0; u < NW; ++u) {
        const int gg = base + 4 * u;
        if (gg >= g_end) break;
        // The activation tile of this group was requested before the latest set of weights (4 + 2 loads): once
        // at most those are outstanding it has landed (loads complete in order; the wave reads only its own tile,
        // so no barrier is needed).
        asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        dma_a(gg + 4, (u + 1) & 1);          // first: needed earlier than the weights requested below
        load_w(gg + 4 * (NW - 1), f[(u + NW - 1) % NW]);
        const Fetched &cur = f[u];
        const float s0 = (float)cur.s[0] * 0.0625f, s1 = (float)cur.s[1] * 0.0625f;     // the weights come as 16 q
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const bf16x8 fa = frag_a(u & 1, i);
          tmp[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, expand_nibbles_x16(cur.w[0][i >> 2][i & 3]), tmp[0], 0, 0, 0);
          tmp[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, expand_nibbles_x16(cur.w[1][i >> 2][i & 3]), tmp[1], 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          acc[0][r] = fmaf(tmp[0][r], s0, acc[0][r]);
          acc[1][r] = fmaf(tmp[1][r], s1, acc[1][r]);
          tmp[0][r] = 0.f;
          tmp[1][r] = 0.f;
        }
      }
    }
  }

  __syncthreads();                                       // every wave is done with its stage reads
  float (*part)[2][16][64] = (float (*)[2][16][64])St0;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) part[wave][j][r][lane] = acc[j][r];
  __syncthreads();
  // D layout of the 32x32 MFMA: lane holds column lane%32 (a weight row) and rows (tokens) 8*(r/4) + 4*(lane/32) + r%4.
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int idx = tid + 256 * p, r = idx >> 6, L = idx & 63;
    const int m = 8 * (r >> 2) + 4 * (L >> 5) + (r & 3), c = L & 31;
    float v[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) v[j] = (part[0][j][r][L] + part[1][j][r][L]) + (part[2][j][r][L] + part[3][j][r][L]);
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

arb_status launch_w4_quantize(const bf16 *W, int N, int K, uint32_t *packed, bf16 *scales, hipStream_t st) {
  if (N == 0) return ARB_OK;
  if (N < 0 || K <= 0 || K % GROUP != 0) return arb_fail(ARB_EUNSUPPORTED, "w4_quantize: N=%d, K=%d (K must be a multiple of %d)", N, K, GROUP);
  const long long groups = (long long)N * (K / GROUP);
  hipLaunchKernelGGL(w4_quantize_kernel, dim3((unsigned)((groups + 15) / 16)), dim3(256), 0, st, W, N, K, packed, scales);
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
    if (skinny) hipLaunchKernelGGL((gemm_w4_skinny_kernel<E>), grid, block, 0, st, A, Bq, Bscale, C, M, N, K);       \
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
