// RMSNorm fused with a linear layer: the "sum + sum" cascade (paper Appendix
// A.2) in single-loop form.
//   stage 1: ss_i   = sum_k x[i,k]^2
//   stage 2: y[i,n] = sum_k (x[i,k] g[k]) w[k,n] * H(ss_i),  H(ss) = (ss/K + eps)^(-1/2)
// H does not depend on k, so the running state carries the H-free accumulator
// (Eq. (8)): one GEMM pass over K accumulates acc[i,n] = sum_k x g w with bf16
// MFMA (fp32 accumulate) while a side accumulator collects ss_i from the very
// same X tile on its way to LDS; the epilogue applies H(ss_i) once per row.
//
// The product is computed transposed, Y^T = W^T (X g)^T, so that each lane of
// the accumulator owns one output row i (one H(ss_i) per lane) and four
// consecutive output columns per register group (8-byte stores).
//   A operand = W^T tile: W rows are transposed in registers while staging.
//   B operand = (X g) tile: x*g rounded to bf16 once, while staging.
#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

namespace {

constexpr int kGWaves = 4;
constexpr int kGThreads = kGWaves * kWave;
constexpr int kBM = 128, kBN = 128, kBKK = 64;

__device__ __forceinline__ uint32_t pair_lo(uint32_t x, uint32_t y) {
  return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ uint32_t pair_hi(uint32_t x, uint32_t y) {
  return __builtin_amdgcn_perm(y, x, 0x07060302u);
}
// Tiles in LDS: 64 contraction slots (128 bytes) per row, 16-byte pieces
// XOR-swizzled by row so that 16 consecutive rows hit all banks.
__device__ __forceinline__ int tile_off(int row, int piece) {
  return row * (kBKK * 2) + ((piece ^ ((row >> 1) & 7)) << 4);
}

}  // namespace

__global__ __launch_bounds__(kGThreads) void rmsnorm_gemm_bf16_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ g, const bf16_t* __restrict__ w,
    bf16_t* __restrict__ y, int M, int K, int N, int64_t ldx, int64_t ldw, int64_t ldy,
    float inv_k, float eps, int n_mtiles) {
  __shared__ __attribute__((aligned(16))) unsigned char xs[kBM * kBKK * 2];   // (x g)[m][k]
  __shared__ __attribute__((aligned(16))) unsigned char wts[kBN * kBKK * 2];  // w^T[n][k]
  __shared__ float s_rstd[kBM];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int i32 = lane & 31;
  const int hh = lane >> 5;
  const int wm = wave & 1;   // wavefront's 64-row half of the M tile
  const int wn = wave >> 1;  // wavefront's 64-column half of the N tile

  const int mt = blockIdx.x % n_mtiles;
  const int nt = blockIdx.x / n_mtiles;
  const int m0 = mt * kBM, n0 = nt * kBN;

  // staging roles
  const int xpiece = tid & 7;    // 8 k-values of an X row
  const int xrow = tid >> 3;     // + 32e, e = 0..3
  const int wpiece = tid & 15;   // 8 n-values of a W row
  const int wkg = tid >> 4;      // group of 4 consecutive k rows, 0..15
  const int wn_src = min(n0 + 8 * wpiece, N - 8);

  f32x16 acc[2][2];  // [ni][mi]: Y^T tile (rows n, columns m)
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;
  float ss[4] = {0.f, 0.f, 0.f, 0.f};

  u32x4 xreg[4], wreg[4], greg;
  auto load_tiles = [&](int k0) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int row = min(m0 + xrow + 32 * e, M - 1);
      xreg[e] = *reinterpret_cast<const u32x4*>(x + (int64_t)row * ldx + k0 + 8 * xpiece);
    }
    greg = *reinterpret_cast<const u32x4*>(g + k0 + 8 * xpiece);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr)
      wreg[rr] = *reinterpret_cast<const u32x4*>(w + (int64_t)(k0 + 4 * wkg + rr) * ldw + wn_src);
  };
  auto store_tiles = [&]() {
    float gf[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) { gf[2 * j] = bf16_lo(greg[j]); gf[2 * j + 1] = bf16_hi(greg[j]); }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      u32x4 r;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a = bf16_lo(xreg[e][j]), bq = bf16_hi(xreg[e][j]);
        ss[e] = fmaf(a, a, ss[e]);   // stage 1 side accumulator
        ss[e] = fmaf(bq, bq, ss[e]);
        r[j] = pack_bf16(a * gf[2 * j], bq * gf[2 * j + 1]);
      }
      *reinterpret_cast<u32x4*>(xs + tile_off(xrow + 32 * e, xpiece)) = r;
    }
    // W: 4 k-rows x 8 n-columns -> 8 rows of w^T, 4 k-values (8 bytes) each
#pragma unroll
    for (int tp = 0; tp < 4; ++tp) {
      u32x2 lo2, hi2;
      lo2[0] = pair_lo(wreg[0][tp], wreg[1][tp]);
      lo2[1] = pair_lo(wreg[2][tp], wreg[3][tp]);
      hi2[0] = pair_hi(wreg[0][tp], wreg[1][tp]);
      hi2[1] = pair_hi(wreg[2][tp], wreg[3][tp]);
      const int nrow = 8 * wpiece + 2 * tp;
      *reinterpret_cast<u32x2*>(wts + tile_off(nrow, wkg >> 1) + 8 * (wkg & 1)) = lo2;
      *reinterpret_cast<u32x2*>(wts + tile_off(nrow + 1, wkg >> 1) + 8 * (wkg & 1)) = hi2;
    }
  };

  load_tiles(0);
  for (int k0 = 0; k0 < K; k0 += kBKK) {
    __syncthreads();
    store_tiles();
    __syncthreads();
    if (k0 + kBKK < K) load_tiles(k0 + kBKK);
#pragma unroll
    for (int kk = 0; kk < kBKK / 16; ++kk) {
      u32x4 af[2], bfr[2];
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
        af[ni] = *reinterpret_cast<const u32x4*>(wts + tile_off(64 * wn + 32 * ni + i32, 2 * kk + hh));
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
        bfr[mi] = *reinterpret_cast<const u32x4*>(xs + tile_off(64 * wm + 32 * mi + i32, 2 * kk + hh));
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
          acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, af[ni]), __builtin_bit_cast(bf16x8, bfr[mi]), acc[ni][mi],
              0, 0, 0);
    }
  }

  // stage 1 result: the 8 lanes that share an X row add their partial sums
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float s = ss[e];
    s += dpp_f32<kDppQuadXor1>(s);
    s += dpp_f32<kDppQuadXor2>(s);
    s += dpp_f32<kDppRowHalfMirror>(s);
    if (xpiece == 0) s_rstd[xrow + 32 * e] = 1.0f / sqrtf(s * inv_k + eps);
  }
  __syncthreads();

  // epilogue: y = acc * H(ss)
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
    const int mloc = 64 * wm + 32 * mi + i32;
    const int m = m0 + mloc;
    const float rs = s_rstd[mloc];
    if (m >= M) continue;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int n = n0 + 64 * wn + 32 * ni + 8 * r4 + 4 * hh;
        if (n < N) {
          u32x2 o2;
          o2[0] = pack_bf16(acc[ni][mi][4 * r4] * rs, acc[ni][mi][4 * r4 + 1] * rs);
          o2[1] = pack_bf16(acc[ni][mi][4 * r4 + 2] * rs, acc[ni][mi][4 * r4 + 3] * rs);
          *reinterpret_cast<u32x2*>(y + (int64_t)m * ldy + n) = o2;
        }
      }
    }
  }
}

hipError_t launch_rmsnorm_gemm_bf16(const void* x, const void* g, const void* w, void* y, int M,
                                    int K, int N, int64_t ldx, int64_t ldw, int64_t ldy, float eps,
                                    hipStream_t s) {
  const int n_mtiles = (M + kBM - 1) / kBM;
  const int n_ntiles = (N + kBN - 1) / kBN;
  const int64_t grid = (int64_t)n_mtiles * n_ntiles;
  if (grid > INT32_MAX) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rmsnorm_gemm_bf16_kernel, dim3((unsigned)grid), dim3(kGThreads), 0, s,
                     (const bf16_t*)x, (const bf16_t*)g, (const bf16_t*)w, (bf16_t*)y, M, K, N, ldx,
                     ldw, ldy, 1.0f / (float)K, eps, n_mtiles);
  return hipGetLastError();
}

}  // namespace rf
