// Projection GEMM C[M,N] = A[M,K] * B[N,K]^T on the gfx950 matrix cores:
// bf16 operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16), LDS-staged tiles.
//
// Both operands are K-contiguous, so a lane's MFMA fragment (8 consecutive k of
// one row) is one 16-byte LDS read.  A workgroup of 4 waves owns a 128x128 tile
// of C; each wave owns 64x64 of it as 2x2 MFMA tiles.  K is walked in steps of
// 64 through a double-buffered LDS stage fed from registers, with the global
// loads running two steps ahead of the MFMAs (HBM/L2 latency is several times
// one step's MFMA time).  16-byte LDS chunks are XOR-swizzled by row/2: a 16-byte
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
  __shared__ __attribute__((aligned(16))) bf16 As[2][LDS_TILE];
  __shared__ __attribute__((aligned(16))) bf16 Bs[2][LDS_TILE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int logical = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tile_n = logical / tiles_m, tile_m = logical - tile_n * tiles_m;
  const int m0 = tile_m * BM;

  // global source rows of this thread's four 16-byte chunks per operand
  const bf16 *a_src[4], *b_src[4];
  int st_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + 256 * i, row = c >> 3, chunk = c & 7;
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
    st_off[i] = lds_off(row, chunk);
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

  // Software pipeline, two K-steps deep: while step kt is multiplied out of LDS buffer kt%2, the
  // global loads of step kt+2 are in flight into one register set and the loads of step kt+1
  // (issued one step earlier, into the other set) are written to the other LDS buffer.
  u32x4 ra[2][4], rb[2][4];
  const int frag_row = lane & 31, frag_half = lane >> 5;
  auto gload = [&](int set, int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ra[set][i] = *(const u32x4 *)(a_src[i] + (size_t)kt * BK);
      rb[set][i] = *(const u32x4 *)(b_src[i] + (size_t)kt * BK);
    }
  };
  auto lstore = [&](int buf, int set) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *(u32x4 *)&As[buf][st_off[i]] = ra[set][i];
      *(u32x4 *)&Bs[buf][st_off[i]] = rb[set][i];
    }
  };
  // MFMAs of one K-step; the LDS reads of sub-step kk+1 are issued before the MFMAs of kk.
  auto compute = [&](int buf) {
    bf16x8 fa[2][2], fb[2][2];
    auto frags = [&](int slot, int kk) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[slot][i] = *(const bf16x8 *)&As[buf][lds_off(wm * 64 + i * 32 + frag_row, kk * 2 + frag_half)];
        fb[slot][i] = *(const bf16x8 *)&Bs[buf][lds_off(wn * 64 + i * 32 + frag_row, kk * 2 + frag_half)];
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

  // The loop body is kept free of branches (loads past the end are clamped to the last step and
  // their LDS copy is never read): the compiler's wait-count tracking is exact only in
  // straight-line code, and a conservative wait here would drain the loads just issued.
  const int last = nk - 1;
  gload(0, 0);
  gload(1, min(1, last));
  lstore(0, 0);
  __syncthreads();
  int kt = 0;
  for (; kt + 2 <= nk; kt += 2) {
    gload(0, min(kt + 2, last));
    __builtin_amdgcn_sched_barrier(0);      // keep the loads ahead of the MFMAs they overlap with
    compute(0);
    lstore(1, 1);
    __syncthreads();
    gload(1, min(kt + 3, last));
    __builtin_amdgcn_sched_barrier(0);
    compute(1);
    lstore(0, 0);
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
  extern __shared__ __attribute__((aligned(16))) bf16 smem[];
  bf16 *As = smem, *Bs = smem + 2 * L_TILE;       // [2][L_TILE] each

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int logical = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tile_n = logical / tiles_m, tile_m = logical - tile_n * tiles_m;
  const int m0 = tile_m * LM;

  const bf16 *a_src[4], *b_src[4];
  int st_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + 512 * i, row = c >> 3, chunk = c & 7;
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
    st_off[i] = lds_off(row, chunk);
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
  u32x4 ra[4], rb[4];
  auto gload = [&](int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ra[i] = *(const u32x4 *)(a_src[i] + (size_t)kt * BK);
      rb[i] = *(const u32x4 *)(b_src[i] + (size_t)kt * BK);
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *(u32x4 *)&As[buf * L_TILE + st_off[i]] = ra[i];
      *(u32x4 *)&Bs[buf * L_TILE + st_off[i]] = rb[i];
    }
  };
  auto compute = [&](int buf) {
    bf16x8 fa[2][4], fb[2][2];
    auto frags = [&](int slot, int kk) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        fa[slot][i] = *(const bf16x8 *)&As[buf * L_TILE + lds_off(wm * 128 + i * 32 + frag_row, kk * 2 + frag_half)];
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[slot][j] = *(const bf16x8 *)&Bs[buf * L_TILE + lds_off(wn * 64 + j * 32 + frag_row, kk * 2 + frag_half)];
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

  // One K-step ahead in registers: the loads of step kt+1 are issued before the MFMAs of step kt and
  // written to the other LDS stage after them (branch-free body, see the small-tile kernel).
  gload(0);
  lstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    gload(min(kt + 1, last));
    __builtin_amdgcn_sched_barrier(0);
    compute(kt & 1);
    lstore((kt + 1) & 1);
    __syncthreads();
  }

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
    const size_t lds = 4 * L_TILE * sizeof(bf16);
    static bool attr_set[3] = {false, false, false};
#define ARB_BIG(E)                                                                                             \
  do {                                                                                                         \
    if (!attr_set[E]) {                                                                                        \
      ARB_CHECK_HIP(hipFuncSetAttribute((const void *)gemm256_kernel<E>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                        (int)lds));                                                            \
      attr_set[E] = true;                                                                                      \
    }                                                                                                          \
    hipLaunchKernelGGL((gemm256_kernel<E>), bgrid, bblock, lds, st, A, B, C, M, N, K, tm, tn);                 \
  } while (0)
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
