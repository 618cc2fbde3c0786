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

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Give
// every XCD a contiguous range of logical tiles so that the m-tiles that share a
// weight tile run on the same L2.
__device__ __forceinline__ int xcd_remap(int bid, int total) {
  const int per = total / 8, rem = total % 8;
  const int xcd = bid % 8, j = bid / 8;
  // XCDs [0, rem) hold per+1 tiles, the rest hold per
  const int base = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
  return base + j;
}

__device__ __forceinline__ int lds_off(int row, int chunk) {   // element offset of a 16-byte chunk
  return row * BK + ((chunk ^ ((row >> 1) & 7)) << 3);
}

// Internal epilogue: split s of a split-K launch stores its fp32 partial product to C + s*M*N.
constexpr int EPI_PARTIAL_F32 = 3;

template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ B,
                                                   void *__restrict__ Cv, int M, int N, int K, int tiles_m,
                                                   int tiles_n) {
  // One array per operand and stage: the compiler orders LDS reads against in-flight direct-to-LDS
  // loads by object, so separate objects let the reads of one stage overlap the loads into the other.
  __shared__ __attribute__((aligned(16))) bf16 As0[LDS_TILE], As1[LDS_TILE], Bs0[LDS_TILE], Bs1[LDS_TILE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int logical = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tile_n = logical / tiles_m, tile_m = logical - tile_n * tiles_m;
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
          C[(size_t)m * N + col] = (bf16)(gte / (1.0f + __expf(-gte)) * up);
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
// Large-tile variant for launches that fill the chip with 256x256 tiles.  Global->LDS traffic
// per flop halves against the 128x128 tile (a CU's vector-memory path moves ~50-60 bytes/clock,
// which caps the small tile at about half the MFMA rate), and each LDS fragment read feeds more
// MFMAs: 8 waves, wave tile 128x64 (4x2 MFMA tiles: 6 fragment reads per 8 MFMAs).  128 KB of
// LDS (two stages of A and B), one workgroup per CU, two waves per SIMD.
constexpr int LM = 256, LN = 256;
constexpr int L_TILE = LM * BK;          // elements per operand tile

template <int EPI>
__global__ __launch_bounds__(512, 1) void gemm256_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ B,
                                                         void *__restrict__ Cv, int M, int N, int K, int tiles_m,
                                                         int tiles_n) {
  __shared__ __attribute__((aligned(16))) bf16 As0[L_TILE], As1[L_TILE], Bs0[L_TILE], Bs1[L_TILE];   // 128 KB

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int logical = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tile_n = logical / tiles_m, tile_m = logical - tile_n * tiles_m;
  const int m0 = tile_m * LM;

  const bf16 *a_src[4], *b_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + 512 * i, row = c >> 3, chunk = (c & 7) ^ ((row >> 1) & 7);   // swizzle on the global side
    int am = m0 + row;
    am = am < M ? am : M - 1;
    a_src[i] = A + (size_t)am * K + chunk * 8;
    int bn;
    if (EPI == ARB_EPI_SWIGLU_BF16) {
      // tile-local row r: wave column r/64, MFMA tile (r%64)/32 (0 = gate, 1 = up), feature offset r%32
      const int f = tile_n * 128 + (row >> 6) * 32 + (row & 31);
      bn = ((row >> 5) & 1) ? N + f : f;            // N = F here
    } else {
      bn = tile_n * LN + row;
    }
    b_src[i] = B + (size_t)bn * K + chunk * 8;
  }

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = K / BK, last = nk - 1;
  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto dma = [&](int buf, int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int slot = (i * 8 + wave_u) * 512;
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(a_src[i] + (size_t)kt * BK), LDS_PTR((buf ? As1 : As0) + slot), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(b_src[i] + (size_t)kt * BK), LDS_PTR((buf ? Bs1 : Bs0) + slot), 16, 0, 0);
    }
  };
  auto compute = [&](int buf) {
    bf16x8 fa[2][4], fb[2][2];
    auto frags = [&](int slot, int kk) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        fa[slot][i] = *(const bf16x8 *)&(buf ? As1 : As0)[lds_off(wm * 128 + i * 32 + frag_row, kk * 2 + frag_half)];
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[slot][j] = *(const bf16x8 *)&(buf ? Bs1 : Bs0)[lds_off(wn * 64 + j * 32 + frag_row, kk * 2 + frag_half)];
    };
    frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) frags((kk + 1) & 1, kk + 1);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i], fb[kk & 1][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // The loads of step kt+1 stream into the other LDS stage while step kt is multiplied out
  // (branch-free body, see the small-tile kernel).
  dma(0, 0);
  __syncthreads();
  int kt = 0;
  for (; kt + 2 <= nk; kt += 2) {
    dma(1, kt + 1);
    __builtin_amdgcn_sched_barrier(0);
    compute(0);
    __syncthreads();
    dma(0, min(kt + 2, last));
    __builtin_amdgcn_sched_barrier(0);
    compute(1);
    __syncthreads();
  }
  if (kt < nk) compute(0);

  if (EPI == ARB_EPI_SWIGLU_BF16) {
    bf16 *C = (bf16 *)Cv;
    const int col = tile_n * 128 + wn * 32 + frag_row;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
        if (m < M) {
          const float gte = acc[i][0][r], up = acc[i][1][r];
          C[(size_t)m * N + col] = (bf16)(gte / (1.0f + __expf(-gte)) * up);
        }
      }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = tile_n * LN + wn * 64 + j * 32 + frag_row;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
          if (m < M) {
            if (EPI == ARB_EPI_STORE_BF16) {
              ((bf16 *)Cv)[(size_t)m * N + col] = (bf16)acc[i][j][r];
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

static const int kBigTileMinTiles = 200;

int gemm_residual_splits(int M, int N, int K) {
  // enough workgroups to fill 256 CUs, each keeping at least 4 K-steps; the partials cost
  // 8 bytes of traffic per element and split, so no more splits than that needs
  const int tiles = ceil_div(M, BM) * (N / BN), nk = K / BK;
  int s = ceil_div(384, tiles);
  if (s > nk / 4) s = nk / 4;
  if (s > 8) s = 8;
  return s < 1 ? 1 : s;
}

arb_status launch_gemm(const bf16 *A, const bf16 *B, void *C, int M, int N, int K, int epilogue, hipStream_t st,
                       int splits) {
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
  if (splits > 1 && epilogue != ARB_EPI_RESIDUAL_F32) return arb_fail(ARB_EINVAL, "gemm: split-K needs the residual epilogue");
  if (splits < 1 || splits > K / BK) return arb_fail(ARB_EINVAL, "gemm: %d splits of %d K-steps", splits, K / BK);
  // Large tiles (one per CU at a time) when whole rounds of 256 of them are at least 80 % full
  const int big_n = epilogue == ARB_EPI_SWIGLU_BF16 ? 128 : LN;
  const int big_tiles = N % big_n == 0 ? ceil_div(M, LM) * (N / big_n) : 0;
  if (splits == 1 && big_tiles >= kBigTileMinTiles && 5 * big_tiles >= 4 * 256 * ceil_div(big_tiles, 256)) {
    const int tm = ceil_div(M, LM), tn = N / big_n;
    const dim3 bgrid(tm * tn), bblock(512);
#define ARB_BIG(E) hipLaunchKernelGGL((gemm256_kernel<E>), bgrid, bblock, 0, st, A, B, C, M, N, K, tm, tn)
    switch (epilogue) {
      case ARB_EPI_STORE_BF16: ARB_BIG(ARB_EPI_STORE_BF16); break;
      case ARB_EPI_RESIDUAL_F32: ARB_BIG(ARB_EPI_RESIDUAL_F32); break;
      case ARB_EPI_SWIGLU_BF16: ARB_BIG(ARB_EPI_SWIGLU_BF16); break;
      default: return arb_fail(ARB_EINVAL, "gemm: unknown epilogue %d", epilogue);
    }
#undef ARB_BIG
    ARB_CHECK_LAUNCH("gemm256");
    return ARB_OK;
  }
  const dim3 grid(tiles_m * tiles_n, splits), block(256);
  switch (epilogue) {
    case ARB_EPI_STORE_BF16:
      hipLaunchKernelGGL((gemm_kernel<ARB_EPI_STORE_BF16>), grid, block, 0, st, A, B, C, M, N, K, tiles_m, tiles_n);
      break;
    case ARB_EPI_RESIDUAL_F32:
      if (splits > 1)
        hipLaunchKernelGGL((gemm_kernel<EPI_PARTIAL_F32>), grid, block, 0, st, A, B, C, M, N, K, tiles_m, tiles_n);
      else
        hipLaunchKernelGGL((gemm_kernel<ARB_EPI_RESIDUAL_F32>), grid, block, 0, st, A, B, C, M, N, K, tiles_m, tiles_n);
      break;
    case ARB_EPI_SWIGLU_BF16:
      hipLaunchKernelGGL((gemm_kernel<ARB_EPI_SWIGLU_BF16>), grid, block, 0, st, A, B, C, M, N, K, tiles_m, tiles_n);
      break;
    default:
      return arb_fail(ARB_EINVAL, "gemm: unknown epilogue %d", epilogue);
  }
  ARB_CHECK_LAUNCH("gemm");
  return ARB_OK;
}
