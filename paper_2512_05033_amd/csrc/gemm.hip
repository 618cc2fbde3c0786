// Projection GEMM C[M,N] = A[M,K] * B[N,K]^T on the gfx950 matrix cores:
// bf16 operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16), LDS-staged tiles.
//
// Both operands are K-contiguous, so a lane's MFMA fragment (8 consecutive k of
// one row) is one 16-byte LDS read.  A workgroup of 4 waves owns a 128x128 tile
// of C; each wave owns 64x64 of it as 2x2 MFMA tiles.  K is walked in steps of
// 64 through a double-buffered LDS stage: the next step's global loads are
// issued into registers before the MFMAs of the current step and written to the
// other LDS buffer after them.  16-byte LDS chunks are XOR-swizzled by row so
// that the 8 lanes served together hit 8 different bank groups.
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
  return row * BK + ((chunk ^ (row & 7)) << 3);
}

// Internal epilogue: split s of a split-K launch stores its fp32 partial product to C + s*M*N.
constexpr int EPI_PARTIAL_F32 = 3;

template <int EPI>
__global__ __launch_bounds__(256) void gemm_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ B,
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

  u32x4 ra[4], rb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ra[i] = *(const u32x4 *)a_src[i];
    rb[i] = *(const u32x4 *)b_src[i];
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    *(u32x4 *)&As[0][st_off[i]] = ra[i];
    *(u32x4 *)&Bs[0][st_off[i]] = rb[i];
  }
  __syncthreads();

  const int frag_row = lane & 31, frag_half = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ra[i] = *(const u32x4 *)(a_src[i] + (size_t)(kt + 1) * BK);
        rb[i] = *(const u32x4 *)(b_src[i] + (size_t)(kt + 1) * BK);
      }
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *(const bf16x8 *)&As[cur][lds_off(wm * 64 + i * 32 + frag_row, kk * 2 + frag_half)];
        fb[i] = *(const bf16x8 *)&Bs[cur][lds_off(wn * 64 + i * 32 + frag_row, kk * 2 + frag_half)];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *(u32x4 *)&As[cur ^ 1][st_off[i]] = ra[i];
        *(u32x4 *)&Bs[cur ^ 1][st_off[i]] = rb[i];
      }
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

}  // namespace

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
