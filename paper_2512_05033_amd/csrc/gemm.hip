// Projection GEMM C[M,N] = A[M,K] * B[N,K]^T on the gfx950 matrix cores:
// bf16 operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16), LDS-staged tiles.
//
// Both operands are K-contiguous, so a lane's MFMA fragment (8 consecutive k of
// one row) is one 16-byte LDS read.  A workgroup of 4 waves owns a 128x128 tile
// of C; each wave owns 64x64 of it as 2x2 MFMA tiles.  K is walked in steps of
// 64 through a double-buffered LDS stage filled by direct-to-LDS global loads
// (global_load_lds_dwordx4), one step ahead of the MFMAs.  16-byte LDS chunks are XOR-swizzled by row/2: a 16-byte
// LDS read is served 16 lanes (256 bytes, all 64 banks) at a time, rows are 128
// bytes, so 16 consecutive rows must spread over (row parity, 8 chunk slots).
//
// Epilogues: store bf16; accumulate into an fp32 residual stream; SwiGLU, where
// the B tile is 64 gate rows and the 64 matching up rows arranged so that one
// lane ends up holding gate and up of the same (row, feature).
#include "common.h"

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_TILE = BM * BK;   // elements per operand tile

#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ int lds_off(int row, int chunk) {   // element offset of a 16-byte chunk
  return row * BK + ((chunk ^ ((row >> 1) & 7)) << 3);
}

// fp32 store; in a split-K launch split s stores its partial product to C + s*M*N.
constexpr int EPI_PARTIAL_F32 = ARB_EPI_STORE_F32;

template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ B,
                                                   void *__restrict__ Cv, int M, int N, int K, int tiles_m,
                                                   int tiles_n, int tile_n0) {
  // One array per operand and stage: the compiler orders LDS reads against in-flight direct-to-LDS
  // loads by object, so separate objects let the reads of one stage overlap the loads into the other.
  __shared__ __attribute__((aligned(16))) bf16 As0[LDS_TILE], As1[LDS_TILE], Bs0[LDS_TILE], Bs1[LDS_TILE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  constexpr int TILE_GROUP = 4;
  tile_of<TILE_GROUP>(xcd_remap(blockIdx.x, tiles_m * tiles_n), tiles_m, tiles_n, tile_m, tile_n);
  tile_n += tile_n0;                 // this launch covers n-tiles [tile_n0, tile_n0 + tiles_n)
  const int m0 = tile_m * BM;

  // Global source of this thread's four 16-byte chunks per operand.  Tiles are brought in by
  // direct-to-LDS loads: one wave-wide load fills 1 KB of LDS in lane order (8 tile rows of 8
  // chunk slots), so the XOR swizzle is applied on the global side: the lane that owns slot
  // (row, p) fetches logical chunk p ^ swz(row).
  const bf16 *a_src[4], *b_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + 256 * i, row = c >> 3, chunk = (c & 7) ^ ((row >> 1) & 7);
    int am = m0 + row;
    am = am < M ? am : M - 1;                       // tail rows re-read the last row; never stored
    a_src[i] = A + (size_t)am * K + chunk * 8;
    int bn;
    if (EPI == ARB_EPI_SWIGLU_BF16) {
      // tile-local row r: wave column r/64, MFMA tile (r%64)/32 (0 = gate, 1 = up), feature offset r%32
      const int f = tile_n * 64 + (row >> 6) * 32 + (row & 31);
      bn = ((row >> 5) & 1) ? N + f : f;            // N = F here
    } else {
      bn = tile_n * BN + row;
    }
    b_src[i] = B + (size_t)bn * K + chunk * 8;
  }

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // K range of this workgroup (the whole of K unless the launch is split along K)
  const int nk_all = K / BK;
  const int kt_begin = (int)((long long)nk_all * blockIdx.y / gridDim.y);
  const int nk = (int)((long long)nk_all * (blockIdx.y + 1) / gridDim.y) - kt_begin;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a_src[i] += (size_t)kt_begin * BK;
    b_src[i] += (size_t)kt_begin * BK;
  }

  // While step kt is multiplied out of LDS buffer kt%2, the loads of step kt+1 stream from global
  // memory straight into the other buffer (no register staging, no LDS-write phase); the barrier
  // that ends the step also waits for them.
  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto dma = [&](int buf, int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int slot = (i * 4 + wave_u) * 512;      // 1 KB (8 rows) per wave-wide load
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(a_src[i] + (size_t)kt * BK), LDS_PTR((buf ? As1 : As0) + slot), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(b_src[i] + (size_t)kt * BK), LDS_PTR((buf ? Bs1 : Bs0) + slot), 16, 0, 0);
    }
  };
  // MFMAs of one K-step; the LDS reads of sub-step kk+1 are issued before the MFMAs of kk.
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
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i], fb[kk & 1][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // The loop body is branch-free (loads past the end are clamped to the last step; their copy is
  // never read).
  const int last = nk - 1;
  dma(0, 0);
  __syncthreads();
  int kt = 0;
  for (; kt + 2 <= nk; kt += 2) {
    dma(1, kt + 1);
    __builtin_amdgcn_sched_barrier(0);      // keep the loads ahead of the MFMAs they overlap with
    compute(0);
    __syncthreads();
    dma(0, min(kt + 2, last));
    __builtin_amdgcn_sched_barrier(0);
    compute(1);
    __syncthreads();
  }
  if (kt < nk) compute(0);     // odd number of steps: the last one sits in buffer 0

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

// ---------------------------------------------------------------------------------------------
// Deep-ring kernel for launches of at most one workgroup per CU (narrow projections, remainders,
// split-K launches sized to one round).  Such a launch is bound by what a CU can pull in: it only has
// the loads of its one workgroup in flight, and its one address unit handles a half-used cache line
// like a whole one.  So K is walked in steps of 64 (every row piece is a whole 128-byte line) through
// a ring of LDS stages that fills the CU's LDS: all stages but one are loading or loaded ahead of the
// one being multiplied out.  (Steps of 32 with twice the stages keep the same bytes in flight but
// move half lines: QKV 17.5 -> 14.5 us on the 1.5B shape with steps of 64.)
// MI = 32-row MFMA tiles per wave along M: 2 gives the 128x128 tile (4 stages), 1 a 64x128 tile
// (6 stages) for launches that would otherwise leave more than half of the CUs without a workgroup,
// 4 a 256x128 tile (3 stages) for launches that are one well-filled round of such tiles.
#ifndef ARB_RING_K
#define ARB_RING_K 64
#endif
constexpr int RK = ARB_RING_K;                      // K per stage: 64 makes every row piece a whole 128-byte line
constexpr int ring_stages(int mi) { return RK == 32 ? 8 : (mi == 1 ? 6 : mi == 2 ? 4 : 3); }   // 144, 128, 144 KB for K 64

__device__ __forceinline__ int lds_off32(int row, int chunk) {   // element offset of a 16-byte chunk, 64-byte rows
  return row * 32 + ((chunk ^ ((row >> 2) & 3)) << 3);
}

__device__ __forceinline__ int lds_off_ring(int row, int chunk) {   // element offset of a 16-byte chunk in a stage row
  // 16 lanes read 16 consecutive rows of one chunk: 64-byte rows put 4 rows into 256 bytes (swizzle by row/4),
  // 128-byte rows 2 (swizzle by row/2)
  return RK == 32 ? row * 32 + ((chunk ^ ((row >> 2) & 3)) << 3) : row * 64 + ((chunk ^ ((row >> 1) & 7)) << 3);
}

// s_waitcnt immediates (vmcnt in bits 3:0 and 15:14, lgkmcnt in 11:8, expcnt 6:4 left at "no wait")
constexpr int waitcnt_vm_lgkm0(int vm) { return (vm & 15) | ((vm >> 4) << 14) | 0x70; }

template <int EPI, int MI>
__global__ __launch_bounds__(256, 1) void gemm_ring_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ B,
                                                   void *__restrict__ Cv, int M, int N, int K, int tiles_m,
                                                   int tiles_n, int tile_n0) {
  constexpr int RBM = 64 * MI;                              // rows of the tile
  constexpr int RING_STAGES = ring_stages(MI);
  constexpr int RING_STAGE_ELEMS = (RBM + BN) * RK;         // A rows then B rows
  constexpr int CPR = RK / 8, RPL = 64 / CPR;               // 16-byte chunks per stage row; rows per wave-wide load
  constexpr int A_LOADS = RBM / (4 * RPL), B_LOADS = BN / (4 * RPL);   // wave-wide loads per wave and step
  constexpr int LOADS = A_LOADS + B_LOADS;
  constexpr int NS = RK / 16;                               // MFMA sub-steps per stage
  constexpr int UNUSED = 8;
  // one array per stage (the compiler orders LDS reads against in-flight loads by object)
  __shared__ __attribute__((aligned(16))) bf16 St0[RING_STAGE_ELEMS], St1[RING_STAGE_ELEMS], St2[RING_STAGE_ELEMS],
      St3[RING_STAGES > 3 ? RING_STAGE_ELEMS : UNUSED], St4[RING_STAGES > 4 ? RING_STAGE_ELEMS : UNUSED], St5[RING_STAGES > 5 ? RING_STAGE_ELEMS : UNUSED],
      St6[RING_STAGES > 6 ? RING_STAGE_ELEMS : UNUSED], St7[RING_STAGES > 7 ? RING_STAGE_ELEMS : UNUSED];
  static_assert(RING_STAGES >= 3 && RING_STAGES <= 8, "stage arrays");
#define ARB_ST(s) ((s) == 0 ? St0 : (s) == 1 ? St1 : (s) == 2 ? St2 : (s) == 3 ? St3 : (s) == 4 ? St4 : (s) == 5 ? St5 : (s) == 6 ? St6 : St7)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  constexpr int TILE_GROUP = 512 / RBM;            // 512 rows
  tile_of<TILE_GROUP>(xcd_remap(blockIdx.x, tiles_m * tiles_n), tiles_m, tiles_n, tile_m, tile_n);
  tile_n += tile_n0;                 // this launch covers n-tiles [tile_n0, tile_n0 + tiles_n)
  const int m0 = tile_m * RBM;

  // This thread's 16-byte chunks per step: tile rows row0 + 4 RPL i of A (i < A_LOADS) and of B (i < B_LOADS),
  // the same chunk for all (the swizzle term of a row does not change when 4 RPL is added to it).
  const int row0 = tid / CPR;
  const int chunk = (tid % CPR) ^ (RK == 32 ? ((row0 >> 2) & 3) : ((row0 >> 1) & 7));
  const bf16 *a_src[A_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    int am = m0 + row0 + 4 * RPL * i;
    am = am < M ? am : M - 1;                       // tail rows re-read the last row; never stored
    a_src[i] = A + (size_t)am * K + chunk * 8;
  }
  // B rows.  For SwiGLU the tile-local row r maps to wave column r/64, MFMA tile (r%64)/32 (0 = gate, 1 = up) and
  // feature offset r%32, i.e. feature tile_n*64 + (r/64)*32 + r%32 of the gate or up half; N = F there.
  const bf16 *b_src[B_LOADS];
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) {
    const int r = row0 + 4 * RPL * i;
    const int brow = EPI == ARB_EPI_SWIGLU_BF16 ? tile_n * 64 + (r >> 6) * 32 + (r & 31) + ((r >> 5) & 1) * N : tile_n * BN + r;
    b_src[i] = B + (size_t)brow * K + chunk * 8;
  }

  f32x16 acc[MI][2];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // K range of this workgroup (the whole of K unless the launch is split along K)
  const int nk_all = K / RK;
  const int kt_begin = (int)((long long)nk_all * blockIdx.y / gridDim.y);
  const int nk = (int)((long long)nk_all * (blockIdx.y + 1) / gridDim.y) - kt_begin, last = nk - 1;
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) a_src[i] += (size_t)kt_begin * RK;
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) b_src[i] += (size_t)kt_begin * RK;

  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto dma_a = [&](int s, int kt) {
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i)
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(a_src[i] + (size_t)kt * RK), LDS_PTR(ARB_ST(s) + (i * 4 + wave_u) * 512), 16, 0, 0);
  };
  auto dma_b = [&](int s, int kt) {
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i)
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(b_src[i] + (size_t)kt * RK), LDS_PTR(ARB_ST(s) + RBM * RK + (i * 4 + wave_u) * 512), 16, 0, 0);
  };
  // The swizzle term of a fragment row depends on frag_row only, so each operand needs one LDS offset
  // per sub-step; MFMA tile and stage are constant displacements from it.
  int a_off[NS], b_off[NS];
#pragma unroll
  for (int kk = 0; kk < NS; ++kk) {
    a_off[kk] = lds_off_ring(wm * 32 * MI + frag_row, 2 * kk + frag_half);
    b_off[kk] = RBM * RK + lds_off_ring(wn * 64 + frag_row, 2 * kk + frag_half);
  }
  bf16x8 fa[2][MI], fb[2][2];
  auto frags = [&](int slot, int s, int kk) {
#pragma unroll
    for (int i = 0; i < MI; ++i) fa[slot][i] = *(const bf16x8 *)&ARB_ST(s)[a_off[kk] + i * 32 * RK];
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[slot][j] = *(const bf16x8 *)&ARB_ST(s)[b_off[kk] + j * 32 * RK];
  };
  auto mfmas = [&](int slot) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
  };
  // Step out of stage s (NS sub-steps of 2 MI MFMAs); on entry fragment slot 0 holds its first sub-step.
  // `refill` is the step loaded into the stage before s, which every wave left at the previous barrier
  // (clamped to the last step past the end; those copies are never read).  Before the barrier this
  // wave's reads of stage s have returned and its loads of the next step have landed: they are the
  // oldest of its loads in flight, the LOADS * (RING_STAGES - 3) + A_LOADS issued since may stay in flight.  (A full
  // workgroup fence would wait for all of them.)
  auto step = [&](int s, int refill) {
    const int prev = (s + RING_STAGES - 1) % RING_STAGES, next = (s + 1) % RING_STAGES;
#pragma unroll
    for (int kk = 0; kk + 1 < NS; ++kk) {
      frags((kk + 1) & 1, s, kk + 1);
      if (kk == 0) dma_a(prev, refill);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(kk & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(LOADS * (RING_STAGES - 3) + A_LOADS));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    frags(0, next, 0);
    dma_b(prev, refill);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(1);
    __builtin_amdgcn_sched_barrier(0);
  };
  // The same without a refill, for the steps after the last whole turn of the ring: nothing is loaded
  // any more, so the wait is for everything still in flight.
  auto drain_step = [&](int s) {
#pragma unroll
    for (int kk = 0; kk + 1 < NS; ++kk) {
      frags((kk + 1) & 1, s, kk + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(kk & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    frags(0, (s + 1) % RING_STAGES, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(1);
    __builtin_amdgcn_sched_barrier(0);
  };

#pragma unroll
  for (int s = 0; s < RING_STAGES - 1; ++s) {
    dma_a(s, min(s, last));
    dma_b(s, min(s, last));
  }
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(LOADS * (RING_STAGES - 2)));   // step 0 has landed
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  frags(0, 0, 0);
  // Whole turns of the ring in a branch-free body, then the 0..RING_STAGES-1 steps that are left.
  int kt = 0;
  for (; kt + RING_STAGES <= nk; kt += RING_STAGES) {
#pragma unroll
    for (int s = 0; s < RING_STAGES; ++s) step(s, min(kt + s + RING_STAGES - 1, last));
  }
  const int rem = nk - kt;
#pragma unroll
  for (int s = 0; s < RING_STAGES - 1; ++s)
    if (s < rem) drain_step(s);
#undef ARB_ST

  // D layout of the 32x32 MFMA: lane holds column lane%32 and rows 8*(r/4) + 4*(lane/32) + r%4.
  if (EPI == ARB_EPI_SWIGLU_BF16) {
    bf16 *C = (bf16 *)Cv;
    const int col = tile_n * 64 + wn * 32 + frag_row;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 32 * MI + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
        if (m < M) {
          const float gte = acc[i][0][r], up = acc[i][1][r];
          C[(size_t)m * N + col] = (bf16)(gte * __builtin_amdgcn_rcpf(1.0f + __expf(-gte)) * up);
        }
      }
  } else {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = tile_n * BN + wn * 64 + j * 32 + frag_row;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + wm * 32 * MI + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
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

// ---------------------------------------------------------------------------------------------
// Large-tile variant for launches that fill the chip with 256x256 tiles.  Global->LDS traffic
// per flop halves against the 128x128 tile (a CU's vector-memory path moves ~50-60 bytes/clock,
// which caps the small tile at about half the MFMA rate), and a fragment read (1 KB per wave)
// serves more MFMAs: 4 waves, one per SIMD, each own 128x128 of the tile as 4x4 MFMA tiles (8
// fragment reads per 16 MFMAs), the 256 accumulator registers in the AGPR half of the wave's 512.
//
// With one wave per SIMD nothing else covers a stall, so every kind of instruction is spread
// evenly through the MFMA stream.  K is walked in steps of 32 through four LDS stages (128 KB):
// while step k is multiplied out of stage k%4, the loads of step k+3 stream into the stage that
// step k-1 has just left, one load per four MFMAs, so the vector-memory path never sees a burst
// and a load has three steps to land.  Per step there are two sub-steps of 16 MFMAs; the fragments
// of the next sub-step are read between the MFMAs of the current one.  The barrier of a step sits
// before its second sub-step: past it every wave is done reading the previous stage and the next
// stage has landed.  LDS rows are 64 bytes here, so the 16-byte chunks are swizzled by row/4.
constexpr int LM = 256, LN = 256, LK = 32;
constexpr int L_TILE = LM * LK;          // elements per operand and stage


// BLOCKED: B is the K-blocked copy of the weights, [K/32][rows][32] (arb_pack_k_blocked): the 16 rows of a
// wave-wide load of one K step are then 1 KB of consecutive memory, whole cache lines, instead of 16 half lines.
template <int EPI, bool BLOCKED>
__global__ __launch_bounds__(256, 1) void gemm256_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ B,
                                                         void *__restrict__ Cv, int M, int N, int K, int tiles_m,
                                                         int tiles_n) {
  // one array per operand and stage (the compiler orders LDS reads against in-flight loads by object)
  __shared__ __attribute__((aligned(16))) bf16 As0[L_TILE], As1[L_TILE], As2[L_TILE], As3[L_TILE];
  __shared__ __attribute__((aligned(16))) bf16 Bs0[L_TILE], Bs1[L_TILE], Bs2[L_TILE], Bs3[L_TILE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  constexpr int TILE_GROUP = 4;
  tile_of<TILE_GROUP>(xcd_remap(blockIdx.x, tiles_m * tiles_n), tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * LM;

  // This thread's four 16-byte chunks per operand and step: tile rows tid/4 + 64 i, and the same
  // chunk for every i (the swizzle term (row/4)%4 does not depend on i).  One wave-wide load fills
  // 1 KB of LDS in lane order, i.e. 16 rows of 4 chunk slots.
  const int row0 = tid >> 2, chunk = (tid & 3) ^ ((row0 >> 2) & 3);
  const bf16 *a_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int am = m0 + row0 + 64 * i;
    am = am < M ? am : M - 1;                       // tail rows re-read the last row; never stored
    a_src[i] = A + (size_t)am * K + chunk * 8;
  }
  // B rows of chunk i are b_row0 + i * b_rows_per_i.  For SwiGLU the tile-local row r maps to wave column
  // r/128, MFMA tile (r%128)/32 (even = gate, odd = up) and feature offset r%32, i.e. feature
  // tile_n*128 + (r/64)*32 + r%32 of the gate (r/32 even) or up (odd) half; N = F there.
  const int b_row0 = EPI == ARB_EPI_SWIGLU_BF16 ? tile_n * 128 + (row0 & 31) + ((row0 >> 5) & 1) * N : tile_n * LN + row0;
  const size_t b_rows = EPI == ARB_EPI_SWIGLU_BF16 ? 2 * (size_t)N : (size_t)N;      // rows of the weight matrix
  const size_t b_row_pitch = BLOCKED ? 32 : (size_t)K;                                  // elements between rows
  const size_t b_k_pitch = BLOCKED ? b_rows * 32 : (size_t)LK;                          // elements between K steps
  const size_t b_step = (size_t)(EPI == ARB_EPI_SWIGLU_BF16 ? 32 : 64) * b_row_pitch;
  const bf16 *b_src = B + (size_t)b_row0 * b_row_pitch + chunk * 8;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // K range of this workgroup (the whole of K unless the launch is split along K), in pairs of steps
  const int pairs_all = K / (2 * LK);
  const int kt_begin = 2 * (int)((long long)pairs_all * blockIdx.y / gridDim.y);
  const int nk = 2 * (int)((long long)pairs_all * (blockIdx.y + 1) / gridDim.y) - kt_begin, last = nk - 1;
#pragma unroll
  for (int i = 0; i < 4; ++i) a_src[i] += (size_t)kt_begin * LK;
  b_src += (size_t)kt_begin * b_k_pitch;
  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#define ARB_STAGE(base, s) ((s) == 0 ? base##0 : (s) == 1 ? base##1 : (s) == 2 ? base##2 : base##3)
  auto dma_a = [&](int s, int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(a_src[i] + (size_t)kt * LK), LDS_PTR(ARB_STAGE(As, s) + (i * 4 + wave_u) * 512), 16, 0, 0);
  };
  auto dma_b = [&](int s, int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(b_src + i * b_step + (size_t)kt * b_k_pitch), LDS_PTR(ARB_STAGE(Bs, s) + (i * 4 + wave_u) * 512), 16, 0, 0);
  };
  bf16x8 fa[2][4], fb[2][4];
  // Fragment reads in the order the MFMAs (row-major over the 4x4 tiles) first need them.
  // The swizzle term of a fragment row depends on frag_row only, so each operand needs one LDS
  // offset per sub-step; MFMA tile and stage are constant displacements from it.
  const int a_off[2] = {lds_off32(wm * 128 + frag_row, frag_half), lds_off32(wm * 128 + frag_row, 2 + frag_half)};
  const int b_off[2] = {lds_off32(wn * 128 + frag_row, frag_half), lds_off32(wn * 128 + frag_row, 2 + frag_half)};
  auto frags = [&](int slot, int s, int kk) {
    auto rd_a = [&](int i) { fa[slot][i] = *(const bf16x8 *)&ARB_STAGE(As, s)[a_off[kk] + i * 32 * LK]; };
    auto rd_b = [&](int j) { fb[slot][j] = *(const bf16x8 *)&ARB_STAGE(Bs, s)[b_off[kk] + j * 32 * LK]; };
    rd_a(0); rd_b(0); rd_b(1); rd_b(2); rd_b(3); rd_a(1); rd_a(2); rd_a(3);
  };
  auto mfmas = [&](int slot) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
  };
  // 16 MFMAs with at most one other memory instruction between two of them: 8 fragment reads and 4
  // global->LDS loads behind the first twelve, so the reads have returned by the end of the sub-step
  auto spread = [&]() {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // 1 global->LDS load
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    __builtin_amdgcn_sched_barrier(0);
  };
  // Step out of stage s; on entry fragment slot 0 holds its first sub-step.  `refill` is the step
  // loaded into the stage before s (clamped to the last step past the end; those copies are never read).
  auto step = [&](int s, int refill) {
    const int prev = (s + 3) & 3, next = (s + 1) & 3;
    frags(1, s, 1);
    dma_a(prev, refill);
    mfmas(0);
    spread();
    // Hand-over of the stages.  Before the barrier this wave's reads of stage s have returned
    // (lgkmcnt 0) and its loads of the next step have landed: those are the oldest 8 of its loads in
    // flight, the 12 issued since may stay in flight (vmcnt 12).  A full workgroup fence would wait
    // for all of them.
    __builtin_amdgcn_s_waitcnt(0x007C);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    frags(0, next, 0);
    dma_b(prev, refill);
    mfmas(1);
    spread();
  };

  dma_a(0, 0); dma_b(0, 0);
  dma_a(1, min(1, last)); dma_b(1, min(1, last));
  dma_a(2, min(2, last)); dma_b(2, min(2, last));
  __builtin_amdgcn_s_waitcnt(0x4070);       // vmcnt(16) lgkmcnt(0): step 0 has landed, steps 1 and 2 may be in flight
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  frags(0, 0, 0);
  int kt = 0;
  for (; kt + 4 <= nk; kt += 4) {
    step(0, min(kt + 3, last));
    step(1, min(kt + 4, last));
    step(2, min(kt + 5, last));
    step(3, min(kt + 6, last));
  }
  if (kt < nk) {                              // K is a multiple of 64, so two steps are left
    step(0, last);
    step(1, last);
  }
#undef ARB_STAGE

  if (EPI == ARB_EPI_SWIGLU_BF16) {
    // A lane holds single elements of 128 rows: stored from registers they would leave in 2-byte
    // pieces (128 stores per lane through the address unit).  The wave's 128 x 64 block goes through
    // the LDS instead (the stages are free now, 16 KB per wave) and leaves in 16-byte pieces of whole
    // 128-byte rows.  The 16-byte chunks of a row are swizzled by bit 2 of the row so that the two
    // lane halves, four rows apart, write different banks.
    bf16 *C = (bf16 *)Cv;
    __syncthreads();                      // every wave is done reading the last stage
    bf16 *stage = wave_u == 0 ? As0 : wave_u == 1 ? As1 : wave_u == 2 ? As2 : As3;
#pragma unroll
    for (int jp = 0; jp < 2; ++jp)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3), f = jp * 32 + frag_row;
          const float gte = acc[i][2 * jp][r], up = acc[i][2 * jp + 1][r];
          stage[row * 64 + ((((f >> 3) ^ (((row >> 2) & 1) << 2))) << 3) + (f & 7)] =
              (bf16)(gte * __builtin_amdgcn_rcpf(1.0f + __expf(-gte)) * up);
        }
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int row = it * 8 + (lane >> 3), chunk = lane & 7;
      const bf16x8 v = *(const bf16x8 *)&stage[row * 64 + ((chunk ^ (((row >> 2) & 1) << 2)) << 3)];
      const int m = m0 + wm * 128 + row;
      if (m < M) *(bf16x8 *)(C + (size_t)m * N + tile_n * 128 + wn * 64 + chunk * 8) = v;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = tile_n * LN + wn * 128 + j * 32 + frag_row;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
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

}  // namespace

// K splits of a projection with fp32 partial products that runs in 256x256 tiles: few token rows
// (M a little above a multiple of 128 wastes most of a 128-row tile row) and a long K, where 128x128 tiles would
// be a single under-filled round (more than 256 of them, so no deep-ring kernel either).  0: not such a launch.
static int gemm_large_splits(int M, int N, int K) {
  if (M <= 0 || N <= 0 || N % LN != 0 || K < 2048) return 0;
  const int tiles_small = ceil_div(M, BM) * (N / BN), tm256 = ceil_div(M, 256);
  if (tiles_small <= 256 || 512 / tiles_small > 1) return 0;                     // ring kernels / split small tiles
  if (tm256 * (N / BN) >= 192 && tm256 * (N / BN) <= 256) return 0;              // one round of 256x128 ring tiles
  const int tiles = ceil_div(M, LM) * (N / LN);
  int s = 256 / tiles;
  if (s > K / (16 * LK)) s = K / (16 * LK);                                       // at least 16 steps per split
  if (s > 8) s = 8;
  return s >= 2 && tiles * s >= 205 ? s : 0;
}

int gemm_residual_splits(int M, int N, int K) {
  if (const int s = gemm_large_splits(M, N, K)) return s;
  // as many workgroups as are resident at once (two per CU on 256 CUs) without starting a second
  // round, each keeping at least 4 K-steps; the partials cost 8 bytes of traffic per element and
  // split, so no more splits than that (measured on the 1.5B shape: 5 beats 4 and 6 for K = 8960).
  // With a short K (at most 32 steps) the launch is kept to one workgroup per CU instead, which the
  // deep-ring kernel serves better and which halves the partial traffic (measured: 2 beats 5 for K = 1536).
  const int tiles = ceil_div(M, BM) * (N / BN), nk = K / BK;
  int s = (nk <= 32 ? 256 : 512) / tiles;
  if (s > nk / 4) s = nk / 4;
  if (s > 8) s = 8;
  return s < 1 ? 1 : s;
}

int gemm_large_cols(int M, int N, int K, int epilogue, int splits) {
  // Large tiles run one per CU, so they go in whole rounds of 256: as many n-tile columns as fill whole
  // rounds (all of them when the last round would be at least 80 % full), the remaining columns in
  // 128x128 tiles.  With less than one round of large tiles everything runs in small ones.
  const int big_n = epilogue == ARB_EPI_SWIGLU_BF16 ? 128 : LN;       // a large n-tile is two small ones
  if (splits > 1 && (epilogue == ARB_EPI_RESIDUAL_F32 || epilogue == ARB_EPI_STORE_F32) &&
      splits == gemm_large_splits(M, N, K))
    return N / LN;                                                     // split-K partial products in large tiles
  if (splits != 1 || M <= 0 || N <= 0 || N % big_n != 0) return 0;
  const int tm = ceil_div(M, LM), tn = N / big_n, total = tm * tn, tail = total % 256;
  if (total < 205) return 0;
  return 5 * tail >= 4 * 256 || tail == 0 ? tn : (total - tail) / tm;
}

arb_status launch_gemm(const bf16 *A, const bf16 *B, void *C, int M, int N, int K, int epilogue, hipStream_t st,
                       int splits, int part, const bf16 *B_blocked) {
  if (M == 0) return ARB_OK;
  if (M < 0 || N <= 0 || K <= 0) return arb_fail(ARB_EINVAL, "gemm: M=%d N=%d K=%d", M, N, K);
  if (K % BK != 0) return arb_fail(ARB_EUNSUPPORTED, "gemm: K=%d is not a multiple of %d", K, BK);
  const int tiles_m = ceil_div(M, BM);
  int tiles_n;
  if (epilogue == ARB_EPI_SWIGLU_BF16) {
    if (N % 64 != 0) return arb_fail(ARB_EUNSUPPORTED, "gemm: SwiGLU width %d is not a multiple of 64", N);
    tiles_n = N / 64;
  } else {
    if (N % BN != 0) return arb_fail(ARB_EUNSUPPORTED, "gemm: N=%d is not a multiple of %d", N, BN);
    tiles_n = N / BN;
  }
  if (splits > 1 && epilogue != ARB_EPI_RESIDUAL_F32 && epilogue != ARB_EPI_STORE_F32)
    return arb_fail(ARB_EINVAL, "gemm: split-K needs an fp32 epilogue (partial products)");
  if (splits < 1 || splits > K / BK) return arb_fail(ARB_EINVAL, "gemm: %d splits of %d K-steps", splits, K / BK);
  const int big_cols = gemm_large_cols(M, N, K, epilogue, splits);   // n-tile columns given to the large-tile kernel
  if (big_cols > 0 && part != GEMM_PART_SMALL) {
    const int tm = ceil_div(M, LM);
    const dim3 bgrid(tm * big_cols, splits), bblock(256);
#define ARB_BIG(E)                                                                                                     \
  do {                                                                                                                 \
    if (B_blocked)                                                                                                     \
      hipLaunchKernelGGL((gemm256_kernel<E, true>), bgrid, bblock, 0, st, A, B_blocked, C, M, N, K, tm, big_cols);     \
    else                                                                                                               \
      hipLaunchKernelGGL((gemm256_kernel<E, false>), bgrid, bblock, 0, st, A, B, C, M, N, K, tm, big_cols);            \
  } while (0)
    switch (epilogue) {
      case ARB_EPI_STORE_BF16: ARB_BIG(ARB_EPI_STORE_BF16); break;
      case ARB_EPI_RESIDUAL_F32:
        if (splits > 1) ARB_BIG(EPI_PARTIAL_F32); else ARB_BIG(ARB_EPI_RESIDUAL_F32);
        break;
      case ARB_EPI_STORE_F32: ARB_BIG(ARB_EPI_STORE_F32); break;
      case ARB_EPI_SWIGLU_BF16: ARB_BIG(ARB_EPI_SWIGLU_BF16); break;
      default: return arb_fail(ARB_EINVAL, "gemm: unknown epilogue %d", epilogue);
    }
#undef ARB_BIG
    ARB_CHECK_LAUNCH("gemm256");
  }
  const int tile_n0 = big_cols * 2;                   // small n-tiles covered by the large-tile launch
  tiles_n -= tile_n0;
  if (tiles_n == 0 || part == GEMM_PART_LARGE) return ARB_OK;
  const dim3 block(256);
  const bool ring = tiles_m * tiles_n * splits <= 256;      // at most one workgroup per CU: latency-bound
  const bool half = tiles_m * tiles_n * splits <= 128;      // not even half of the CUs: 64-row tiles
  // More than one round of 128-row tiles that is one well-filled round of 256-row tiles (the split-K down
  // projection): the taller tile reads 0.75 KB of LDS per MFMA instead of 1 KB, needs a third less ingest
  // per flop and runs on the deep-ring kernel.
  const int tm256 = ceil_div(M, 256);
  const bool tall = !ring && tm256 * tiles_n * splits <= 256 && tm256 * tiles_n * splits >= 192;
  const int tm64 = ceil_div(M, 64);
  const dim3 grid(tiles_m * tiles_n, splits), grid64(tm64 * tiles_n, splits), grid256(tm256 * tiles_n, splits);
#define ARB_SMALL(E)                                                                                                  \
  do {                                                                                                                \
    if (tall)                                                                                                         \
      hipLaunchKernelGGL((gemm_ring_kernel<E, 4>), grid256, block, 0, st, A, B, C, M, N, K, tm256, tiles_n, tile_n0); \
    else if (half)                                                                                                    \
      hipLaunchKernelGGL((gemm_ring_kernel<E, 1>), grid64, block, 0, st, A, B, C, M, N, K, tm64, tiles_n, tile_n0);   \
    else if (ring)                                                                                                    \
      hipLaunchKernelGGL((gemm_ring_kernel<E, 2>), grid, block, 0, st, A, B, C, M, N, K, tiles_m, tiles_n, tile_n0);  \
    else                                                                                                              \
      hipLaunchKernelGGL((gemm_kernel<E>), grid, block, 0, st, A, B, C, M, N, K, tiles_m, tiles_n, tile_n0);          \
  } while (0)
  switch (epilogue) {
    case ARB_EPI_STORE_BF16: ARB_SMALL(ARB_EPI_STORE_BF16); break;
    case ARB_EPI_RESIDUAL_F32:
      if (splits > 1) ARB_SMALL(EPI_PARTIAL_F32); else ARB_SMALL(ARB_EPI_RESIDUAL_F32);
      break;
    case ARB_EPI_SWIGLU_BF16: ARB_SMALL(ARB_EPI_SWIGLU_BF16); break;
    case ARB_EPI_STORE_F32: ARB_SMALL(ARB_EPI_STORE_F32); break;
    default: return arb_fail(ARB_EINVAL, "gemm: unknown epilogue %d", epilogue);
  }
#undef ARB_SMALL
  ARB_CHECK_LAUNCH("gemm");
  return ARB_OK;
}

// packed[(kb * rows + r) * 32 + j] = W[r][kb * 32 + j]: one thread per 16-byte chunk
__global__ __launch_bounds__(256) void pack_k_blocked_kernel(const bf16 *__restrict__ W, size_t rows, int K,
                                                             bf16 *__restrict__ packed) {
  const size_t chunks_per_row = K / 8, total = rows * chunks_per_row;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t r = i / chunks_per_row, c = i - r * chunks_per_row;      // source row and 16-byte chunk
    const size_t kb = c / 4;
    *(bf16x8 *)(packed + (kb * rows + r) * 32 + (c % 4) * 8) = *(const bf16x8 *)(W + r * (size_t)K + c * 8);
  }
}

arb_status launch_pack_k_blocked(const bf16 *W, size_t rows, int K, bf16 *packed, hipStream_t st) {
  if (rows == 0) return ARB_OK;
  if (K <= 0 || K % 32 != 0) return arb_fail(ARB_EUNSUPPORTED, "pack_k_blocked: K=%d is not a multiple of 32", K);
  const size_t chunks = rows * (size_t)(K / 8);
  const int blocks = (int)((chunks + 255) / 256 < 8192 ? (chunks + 255) / 256 : 8192);
  hipLaunchKernelGGL(pack_k_blocked_kernel, dim3(blocks), dim3(256), 0, st, W, rows, K, packed);
  ARB_CHECK_LAUNCH("pack_k_blocked");
  return ARB_OK;
}
