// Projection GEMM with 4-bit weights and bf16 activations (the weight-quantized draft of the
// self-draft regime, Section 5.1): C[M,N] = A[M,K] * W'[N,K]^T with
// W'[n,k] = q[n,k] * scale[n, k/128], q in [-8, 7] stored as offset-binary nibbles, eight
// consecutive k per uint32, scale bf16.
//
// The tile kernel (more than 32 activation rows) has the geometry of the 128x128x64 bf16 kernel (4 waves of 64x64,
// A by direct-to-LDS loads), except for the weight operand: each thread fetches 16 bytes of packed weights (32 nibbles
// of one row) into registers, expands them to the bf16 integers -8..7 (exact) and stores them into an LDS stage.  The
// MFMAs therefore accumulate sum_k a[m,k] q[n,k] per group of 128 k (two steps) into a temporary accumulator; at the
// end of a group it is folded into the result with one fp32 multiply by the group's scale.  No product q*scale is ever
// rounded to bf16, so the result differs from the definition only by fp32 accumulation.  Weight traffic is a quarter
// of the bf16 kernel's.  Up to 32 rows a weight-streaming kernel runs instead (below).
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

// nibble of a word that holds input e of its eight: the even inputs in nibbles 0..3, the odd ones in nibbles 4..7
__host__ __device__ constexpr int nibble_of(int e) { return e / 2 + 4 * (e % 2); }

// a packed word -> its eight inputs as the bf16 integers nibble - 8, k ascending
__device__ __forceinline__ bf16x8 expand_nibbles(uint32_t w) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    // 2^23 + nibble as a float, minus (2^23 + 8): exact
    const float f = __uint_as_float(0x4B000000u | ((w >> (4 * nibble_of(e))) & 15u)) - 8388616.0f;
    o[e] = (bf16)f;
  }
  return o;
}

// A packed word as the bf16 values 16 + nibble = 24 + q, k ascending, without a conversion instruction (those run at
// a quarter of the rate of plain integer instructions here, and sixteen of them per word bound the kernel): in the
// binade [16, 32) a bf16 is 16 (1 + m / 128), so a nibble placed in the four top bits of the mantissa adds exactly
// its value.  The storage format puts two neighbours 16 bits apart, so one shift and one and-or place a pair.  The
// constant 24 is taken out again in fp32: sum_k a_k (24 + q_k) - 24 sum_k a_k, with the second sum from an MFMA
// against ones; the terms are about five times the size of the result, so fp32 loses two or three more bits than
// without the detour, far below what the rounding of the output, or an fp32 test bar of 1e-5, sees.
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
    word |= (uint32_t)((int)q + 8) << (4 * nibble_of(e));
  }
  packed[(size_t)n * (K / 8) + g * 16 + l16] = word;
  if (l16 == 0) scales[gid] = scale;
}

constexpr int EPI_PARTIAL_F32 = ARB_EPI_STORE_F32;   // in a split-K launch split s stores to C + s*M*N

// Epilogue of a 128x128 tile held as 4 waves x (2 x 2) MFMA results (wave (wm, wn) owns rows 64 wm.., columns 64 wn..).
template <int EPI>
__device__ __forceinline__ void w4_tile_epilogue(const f32x16 (&acc)[2][2], void *__restrict__ Cv, int M, int N, int m0,
                                                 int tile_n, int wm, int wn, int frag_row, int frag_half) {
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

// The tile kernel.  Every wait is counted by hand: left to the compiler, a turn of this loop held three round trips to
// memory (it waits for all loads in flight before an LDS read that it cannot tell apart from a direct-to-LDS load in
// flight, and a workgroup fence does so in front of each barrier), and a launch of one tile row (up to 128 tokens, one
// workgroup per CU) has nothing else to run meanwhile: 75 us on the 8B gate/up shape whatever the row count.  Here the
// packed weights go to registers six steps ahead and the scales two groups ahead, by inline assembly (the compiler
// keeps no account of them); the activation tile streams two steps ahead into a ring of three LDS stages; the
// fragments are read by inline assembly one MFMA step ahead (the compiler sees neither an LDS read that could meet a
// load in flight nor a load it would have to wait for), and the one wait of a step, in front of its barrier, lets the
// eight requests made since the tile of the next step stay in flight: loads complete in order, so everything older
// has landed.  A register that a load in flight will write is named by the wait that covers it (and by a last wait
// behind the loop): the compiler then neither reads it earlier nor gives it to another value.
// What bounds it now is the expansion (exact: two integer instructions, a subtraction and half a conversion per
// weight; without it the 8B gate/up shape at 128 rows takes 41 instead of 59 us, without the MFMAs 56).  The
// conversion-free expansion of the few-token kernel was tried here too (with the row sums from a third MFMA per
// row block and, in a second version, two accumulator sets so that the fold of a group runs between the MFMAs of
// the next): its longer fold (two fused multiply-adds per element and the reads of accumulator registers) costs what
// the expansion saves, 63-67 us.
template <int AOFF, int BOFF>
__device__ __forceinline__ void w4_request_frags(unsigned a_addr, unsigned b_addr, bf16x8 &fa0, bf16x8 &fa1, bf16x8 &fb0,
                                                 bf16x8 &fb1) {
  asm volatile("ds_read_b128 %0, %4 offset:%6\n\tds_read_b128 %1, %4 offset:%7\n\t"
               "ds_read_b128 %2, %5 offset:%8\n\tds_read_b128 %3, %5 offset:%9"
               : "=&v"(fa0), "=&v"(fa1), "=&v"(fb0), "=&v"(fb1)
               : "v"(a_addr), "v"(b_addr), "n"(AOFF), "n"(AOFF + 32 * BK * 2), "n"(BOFF), "n"(BOFF + 32 * BK * 2)
               : "memory");
}
// the requested fragments have landed (and every LDS write of this wave is done); naming them keeps their readers behind
__device__ __forceinline__ void w4_await_frags(bf16x8 &fa0, bf16x8 &fa1, bf16x8 &fb0, bf16x8 &fb1) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fa0), "+v"(fa1), "+v"(fb0), "+v"(fb1) : : "memory");
}

template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_w4_kernel(const bf16 *__restrict__ A, const uint32_t *__restrict__ Bq,
                                                      const bf16 *__restrict__ Bscale, void *__restrict__ Cv, int M,
                                                      int N, int K, int tiles_m, int tiles_n) {
  constexpr int NA = 3, AHEAD_W = 6;                    // activation stages; steps the packed weights are ahead
  // Two objects: the activation ring only ever sees direct-to-LDS loads and the assembly's reads, so the stores of
  // expanded weights into the other one are not ordered behind loads in flight.
  __shared__ __attribute__((aligned(16))) bf16 Ring[NA * LDS_TILE], Bs[2 * LDS_TILE];

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

  const int ng_all = K / GROUP;
  const int g_begin = (int)((long long)ng_all * blockIdx.y / gridDim.y);
  const int ng = (int)((long long)ng_all * (blockIdx.y + 1) / gridDim.y) - g_begin;
  const int nk = 2 * ng, last = nk - 1;

  const bf16 *a_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + 256 * i, row = c >> 3, chunk = (c & 7) ^ ((row >> 1) & 7);
    int am = m0 + row;
    am = am < M ? am : M - 1;                            // tail rows re-read the last row; never stored
    a_src[i] = A + (size_t)am * K + (size_t)g_begin * GROUP + chunk * 8;
  }
  const int b_row = tid >> 1, b_half = tid & 1;
  const uint32_t *bq_src = Bq + (size_t)weight_row(b_row) * (K / 8) + (size_t)g_begin * (GROUP / 8) + b_half * 4;
  const bf16 *sc_src[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) sc_src[j] = Bscale + (size_t)weight_row(wn * 64 + j * 32 + frag_row) * (K / GROUP) + g_begin;

  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto dma_a = [&](int stage, int kt) {                  // four wave-wide direct-to-LDS loads
    kt = kt < last ? kt : last;                          // past the range: a valid step, never read
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(a_src[i] + (size_t)kt * BK), LDS_PTR(Ring + stage * LDS_TILE + (i * 4 + wave_u) * 512), 16, 0, 0);
  };
  u32x4 wq[AHEAD_W];                                     // packed weights of steps kt+1 .. kt+6, slot = step % 6
  unsigned sc[3][2];                                     // scales (bf16 bits) of three groups, slot = group % 3
  auto load_w = [&](int slot, int kt) {
    kt = kt < last ? kt : last;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(wq[slot]) : "v"(bq_src + (size_t)kt * (BK / 8)) : "memory");
  };
  auto load_sc = [&](int slot, int g) {
    g = g < ng ? g : ng - 1;
    asm volatile("global_load_ushort %0, %1, off" : "=&v"(sc[slot][0]) : "v"(sc_src[0] + g) : "memory");
    asm volatile("global_load_ushort %0, %1, off" : "=&v"(sc[slot][1]) : "v"(sc_src[1] + g) : "memory");
  };
  auto store_b = [&](int buf, const u32x4 &w) {
#pragma unroll
    for (int c = 0; c < 4; ++c) *(bf16x8 *)&Bs[buf * LDS_TILE + lds_off(b_row, b_half * 4 + c)] = expand_nibbles(w[c]);
  };

  // byte addresses of this lane's fragments of MFMA step kk in stage 0: the row block's first row; the second row
  // block, the stage and the operand's array are constant displacements
  unsigned a_addr[4], b_addr[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    a_addr[kk] = (unsigned)(uintptr_t)LDS_PTR(Ring) + 2u * lds_off(wm * 64 + frag_row, kk * 2 + frag_half);
    b_addr[kk] = (unsigned)(uintptr_t)LDS_PTR(Bs) + 2u * lds_off(wn * 64 + frag_row, kk * 2 + frag_half);
  }

  f32x16 acc[2][2], tmp[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = tmp[i][j][r] = 0.f;

  // Request order of the prologue = that of the loop: (tile, weights[, scales]) per step, the scales on even steps.
#pragma unroll
  for (int d = 0; d < AHEAD_W - 1; ++d) load_w(d, d);
  load_sc(0, 0);
  load_sc(1, 1);
  asm volatile("" ::: "memory");
  dma_a(0, 0);
  asm volatile("" ::: "memory");
  dma_a(1, 1);
  asm volatile("" ::: "memory");
  load_w(AHEAD_W - 1, AHEAD_W - 1);
  // all but the second tile and the last weights have landed; a wait names the registers whose loads it covers and
  // that are read before the next wait does so, or the compiler could move their readers above it
  asm volatile("s_waitcnt vmcnt(5)" : "+v"(wq[0]), "+v"(wq[1]), "+v"(sc[0][0]), "+v"(sc[0][1]) : : "memory");
  store_b(0, wq[0]);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();

  bf16x8 fa[2][2], fb[2][2];
  // One step (64 k): u = its position in a turn of six (three groups), so that stage (u % 3), weight stage (u % 2),
  // register set (u % 6) and scale set are fixed per position.
  auto step = [&](auto u_, int kt) {
    constexpr int U = decltype(u_)::value;
    constexpr int SA = (U % NA) * LDS_TILE * 2, SB = (U % 2) * LDS_TILE * 2;
    dma_a((U + 2) % NA, kt + 2);                         // into the stage step kt-1 was read from
    asm volatile("" ::: "memory");
    load_w(U % AHEAD_W, kt + AHEAD_W);                   // that set went into LDS during step kt-1
    if (U % 2 == 0) load_sc((U / 2 + 2) % 3, (kt >> 1) + 2);
    asm volatile("" ::: "memory");
    w4_request_frags<SA, SB>(a_addr[0], b_addr[0], fa[0][0], fa[0][1], fb[0][0], fb[0][1]);
    const u32x4 &next_w = wq[(U + 1) % AHEAD_W];
    bf16 *next_b = Bs + ((U + 1) % 2) * LDS_TILE;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      w4_await_frags(fa[kk & 1][0], fa[kk & 1][1], fb[kk & 1][0], fb[kk & 1][1]);
      if (kk == 0) w4_request_frags<SA, SB>(a_addr[1], b_addr[1], fa[1][0], fa[1][1], fb[1][0], fb[1][1]);
      if (kk == 1) w4_request_frags<SA, SB>(a_addr[2], b_addr[2], fa[0][0], fa[0][1], fb[0][0], fb[0][1]);
      if (kk == 2) w4_request_frags<SA, SB>(a_addr[3], b_addr[3], fa[1][0], fa[1][1], fb[1][0], fb[1][1]);
      // the MFMAs stay behind the request (left alone, the scheduler moves them up and the wave then waits out the
      // LDS latency of every request with nothing to do)
      __builtin_amdgcn_sched_barrier(0);
      // a quarter of the next step's weights per MFMA step: expanded and stored while the matrix pipe runs
      *(bf16x8 *)&next_b[lds_off(b_row, b_half * 4 + kk)] = expand_nibbles(next_w[kk]);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          tmp[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i], fb[kk & 1][j], tmp[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (U % 2 == 1) {                                    // end of a group
      const float s0 = __uint_as_float(sc[U / 2][0] << 16), s1 = __uint_as_float(sc[U / 2][1] << 16);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          acc[i][0][r] = fmaf(tmp[i][0][r], s0, acc[i][0][r]);
          acc[i][1][r] = fmaf(tmp[i][1][r], s1, acc[i][1][r]);
          tmp[i][0][r] = 0.f;
          tmp[i][1][r] = 0.f;
        }
    }
    // The tile of step kt+1 was requested at the top of step kt-1; since then: that step's weights, this step's
    // tile and weights, and the scales of whichever of the two steps is even: 1 + 4 + 1 + 2 = 8 requests.
    // Everything older has landed, among it the weights the next step expands and the scales the next step folds in.
    if (U % 2 == 0)
      asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" : "+v"(wq[(U + 2) % AHEAD_W]), "+v"(sc[U / 2][0]), "+v"(sc[U / 2][1]) : : "memory");
    else
      asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" : "+v"(wq[(U + 2) % AHEAD_W]) : : "memory");
    __builtin_amdgcn_s_barrier();
  };
  for (int kt = 0; kt < nk; kt += 6) {
    step(std::integral_constant<int, 0>{}, kt);
    step(std::integral_constant<int, 1>{}, kt + 1);
    if (kt + 2 >= nk) break;
    step(std::integral_constant<int, 2>{}, kt + 2);
    step(std::integral_constant<int, 3>{}, kt + 3);
    if (kt + 4 >= nk) break;
    step(std::integral_constant<int, 4>{}, kt + 4);
    step(std::integral_constant<int, 5>{}, kt + 5);
  }
  // The clamped requests past the end: their registers stay named until they have landed (a register the compiler
  // takes for dead it hands to something else, and a load that lands in it afterwards overwrites that).
  asm volatile("s_waitcnt vmcnt(0)"
               : "+v"(wq[0]), "+v"(wq[1]), "+v"(wq[2]), "+v"(wq[3]), "+v"(wq[4]), "+v"(wq[5]), "+v"(sc[0][0]), "+v"(sc[0][1]),
                 "+v"(sc[1][0]), "+v"(sc[1][1]), "+v"(sc[2][0]), "+v"(sc[2][1])
               : : "memory");
  w4_tile_epilogue<EPI>(acc, Cv, M, N, m0, tile_n, wm, wn, frag_row, frag_half);
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
        // (the wait names the registers of the set it covers, so that the compiler keeps their readers behind it)
        Fetched &got = f[u];
#define ARB_W4_COVERED "+v"(got.w[0][0]), "+v"(got.w[0][1]), "+v"(got.w[1][0]), "+v"(got.w[1][1]), "+v"(got.s[0]), "+v"(got.s[1])
        if (NS == 2) asm volatile("s_waitcnt vmcnt(6)" : ARB_W4_COVERED : : "memory");
        else asm volatile("s_waitcnt vmcnt(20)" : ARB_W4_COVERED : : "memory");
#undef ARB_W4_COVERED
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
          const bf16x8 fa = frags[i];
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
    // The clamped requests past the range: their registers stay named until they have landed (a register the compiler
    // takes for dead it hands to something else, and a load that lands in it afterwards overwrites that).
#pragma unroll
    for (int d = 0; d < NW; ++d)
      asm volatile("s_waitcnt vmcnt(0)"
                   : "+v"(f[d].w[0][0]), "+v"(f[d].w[0][1]), "+v"(f[d].w[1][0]), "+v"(f[d].w[1][1]), "+v"(f[d].s[0]), "+v"(f[d].s[1])
                   : : "memory");
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
