// RMSNorm fused with a linear layer: the "sum + sum" cascade (paper Appendix
// A.2) in single-loop form.
//   stage 1: ss_i   = sum_k x[i,k]^2
//   stage 2: y[i,n] = sum_k (x[i,k] g[k]) w[k,n] * H(ss_i),  H(ss) = (ss/K + eps)^(-1/2)
// H does not depend on k, so the running state carries the H-free accumulator
// (Eq. (8)): one GEMM pass over K accumulates acc[i,n] = sum_k x g w with bf16
// MFMA (fp32 accumulate) while a side accumulator collects ss_i from the very
// same X tile on its way to LDS; the epilogue applies H(ss_i) once per row.
//
// Tiling.  One workgroup of 8 wavefronts owns a 256 x 256 output tile and walks
// K in steps of 64 through double-buffered LDS (one barrier per step).  The
// product is computed transposed, Y^T = W^T (X g)^T, so that each accumulator
// lane owns one output row i (one H(ss_i) per lane) and four consecutive output
// columns per register group.
//   A operand = W^T: the W tile goes HBM -> LDS with direct-to-LDS 128-bit loads
//               and is read back with 64-bit LDS transpose reads.
//   B operand = (X g): x*g is rounded to bf16 once, in registers, on the way
//               from HBM to LDS; x^2 is accumulated there too.
// Each wavefront owns a 64 (n) x 128 (m) sub-tile: 8 MFMAs per 4 + 4 LDS
// fragment reads, register double-buffered over the four 16-wide contraction
// steps of a K step.
#include <type_traits>

#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

namespace {

constexpr int kGWaves = 8;
constexpr int kGThreads = kGWaves * kWave;
constexpr int kBM = 256, kBN = 256, kBKK = 64;
constexpr int kXTileB = kBM * kBKK * 2;   // 32 KB, [m][k], 128-byte rows
constexpr int kWTileB = kBKK * kBN * 2;   // 32 KB, [k][n], 512-byte rows
constexpr int kStageB = kXTileB + kWTileB;

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_cvoid;

// 16-byte slot swizzles (slot = piece ^ f(row)).
__device__ __forceinline__ int fX(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int fW(int krow) { return (krow & 3) << 2; }

}  // namespace

__global__ __launch_bounds__(kGThreads, 1) void rmsnorm_gemm_bf16_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ g, const bf16_t* __restrict__ w,
    bf16_t* __restrict__ y, int M, int K, int N, int64_t ldx, int64_t ldw, int64_t ldy,
    float inv_k, float eps, int n_mtiles, int n_ntiles) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * kStageB];
  __shared__ float s_rstd[kBM];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int i32 = lane & 31;
  const int hh = lane >> 5;
  const int wn = wave & 3;   // 64-column block of the N tile
  const int wm = wave >> 2;  // 128-row block of the M tile

  // XCD-aware numbering: workgroups are dealt round-robin to the 8 XCDs, each with its
  // own L2.
  int mt, nt;
  {
    const int n_mtiles = gridDim.x / n_ntiles;
    if ((n_mtiles & 3) == 0 && (n_ntiles & 1) == 0) {
      // XCD x owns the block of (n_mtiles/4) x (n_ntiles/2) output tiles at block row x/2,
      // block column x%2: the squarest split into 8, so its L2 fetches the fewest
      // X row panels plus W column panels.
      const int bm = n_mtiles >> 2, bn = n_ntiles >> 1;
      const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
      mt = (xcd >> 1) * bm + jj / bn;
      nt = (xcd & 1) * bn + jj % bn;
    } else {
      mt = blockIdx.x / n_ntiles;
      nt = blockIdx.x % n_ntiles;
    }
  }
  const int m0 = mt * kBM, n0 = nt * kBN;

  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;

  // ---- X staging role: one half row (32 k-values) per thread ----
  const int xrow = tid >> 1;
  const int xhalf = tid & 1;
  const bf16_t* xsrc = x + (int64_t)min(m0 + xrow, M - 1) * ldx + 32 * xhalf;
  const bf16_t* gsrc = g + 32 * xhalf;
  int xdst[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) xdst[c] = xrow * 128 + (((4 * xhalf + c) ^ fX(xrow)) << 4);

  // ---- W direct-to-LDS role: 4 loads per wavefront per K step, 2 k-rows each ----
  uint32_t wsrc_off[4];  // byte offset from w + k0*ldw (the tile's first row)
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int krow = 8 * wave + 2 * e + (lane >> 5);
    const int piece = (lane & 31) ^ fW(krow);
    const int ncol = min(n0 + 8 * piece, N - 8);
    wsrc_off[e] = (uint32_t)(((int64_t)krow * ldw + ncol) * 2);
  }
  auto issue_w = [&](int k0, int buf) {
    const char* wt = reinterpret_cast<const char*>(w) + (int64_t)k0 * ldw * 2;
    unsigned char* dst = lds + buf * kStageB + kXTileB + wave * 4096;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      __builtin_amdgcn_global_load_lds((global_cvoid*)(wt + wsrc_off[e]), (lds_void*)(dst + e * 1024),
                                       16, 0, 0);
  };

  // ---- fragment read addresses (LDS byte addresses, stage 0; + stage/step immediates) ----
  // B operand (X g): lane (i32, hh) of column tile mi reads row 128wm + 32mi + i32, slot 2kk + hh
  uint32_t xaddr[2][4];  // [stage][kk]; + mi * 32 * 128
  {
    const int row = 128 * wm + i32;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      xaddr[0][kk] = lds_base + row * 128 + (((2 * kk + hh) ^ fX(row)) << 4);
      xaddr[1][kk] = xaddr[0][kk] + kStageB;
    }
  }
  // A operand (W^T) by transpose reads: lane = 32hh + 16g2 + 4j + a reads 8 bytes of k-row
  // 16kk + 8hh + 4w2 + j at column 64wn + 32ni + 16g2 + 4a
  uint32_t waddr[2][2][2];  // [stage][ni][w2]; + kk * 16 * 512
  {
    const int i16 = lane & 15, g2 = (lane >> 4) & 1;
    const int j = i16 >> 2, a = i16 & 3;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int w2 = 0; w2 < 2; ++w2) {
        const int krow = 8 * hh + 4 * w2 + j;
        const int piece = (64 * wn + 32 * ni + 16 * g2 + 4 * a) >> 3;
        waddr[0][ni][w2] =
            lds_base + kXTileB + krow * 512 + ((piece ^ fW(krow)) << 4) + 8 * (a & 1);
        waddr[1][ni][w2] = waddr[0][ni][w2] + kStageB;
      }
  }

  f32x16 acc[2][4];  // [ni][mi]: Y^T tile (rows n, columns m)
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;
  float ss = 0.f;

  // X and g tiles travel through registers.  Their loads are raw instructions with
  // hand-placed waits: all vector-memory traffic of the main loop is ordered by hand
  // so that the prefetches stay in flight across barriers.
  u32x4 xreg[4], greg[4];
  auto load_x = [&](int k0) {
    const bf16_t* xp = xsrc + k0;
    const bf16_t* gp = gsrc + k0;
#define RF_LD(DST, PTR, OFF) \
  asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(DST) : "v"(PTR), "n"(OFF));
    RF_LD(xreg[0], xp, 0) RF_LD(xreg[1], xp, 16) RF_LD(xreg[2], xp, 32) RF_LD(xreg[3], xp, 48)
    RF_LD(greg[0], gp, 0) RF_LD(greg[1], gp, 16) RF_LD(greg[2], gp, 32) RF_LD(greg[3], gp, 48)
#undef RF_LD
  };
  // wait until at most PENDING younger vector-memory operations are in flight
#define RF_WAIT_X(PENDING)                                                                   \
  asm volatile("s_waitcnt vmcnt(%8)"                                                         \
               : "+v"(xreg[0]), "+v"(xreg[1]), "+v"(xreg[2]), "+v"(xreg[3]), "+v"(greg[0]),  \
                 "+v"(greg[1]), "+v"(greg[2]), "+v"(greg[3])                                 \
               : "n"(PENDING));
  // x*g -> bf16 -> LDS stage BUF (raw LDS writes: the compiler would order ordinary
  // ones behind the direct-to-LDS loads still in flight)
  uint32_t xdst_addr[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) xdst_addr[c] = lds_base + xdst[c];
  auto store_x = [&](auto buf_tag, auto pending_tag) {
    constexpr int BUF = decltype(buf_tag)::value;
    constexpr int PENDING = decltype(pending_tag)::value;
    RF_WAIT_X(PENDING)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      u32x4 r;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a = bf16_lo(xreg[c][j]), b = bf16_hi(xreg[c][j]);
        ss = fmaf(a, a, ss);  // stage 1 side accumulator
        ss = fmaf(b, b, ss);
        r[j] = pack_bf16(a * bf16_lo(greg[c][j]), b * bf16_hi(greg[c][j]));
      }
      const uint32_t addr = xdst_addr[c] + BUF * kStageB;  // (stage offset exceeds the 16-bit field)
      asm volatile("ds_write_b128 %0, %1" : : "v"(addr), "v"(r) : "memory");
    }
  };

  // One K step out of LDS stage BUF.  Fragment reads are raw instructions with
  // hand-placed waits (the compiler would otherwise wait for the in-flight
  // direct-to-LDS loads of the next stage before every transpose read).
  auto compute = [&](auto buf_tag) {
    constexpr int BUF = decltype(buf_tag)::value;
    u32x2 af[2][2][2];  // [stage][ni][w2]
    u32x4 bfr[2][4];    // [stage][mi]
#define RF_ISSUE(STAGE, KK)                                                                  \
  _Pragma("unroll") for (int ni = 0; ni < 2; ++ni) {                                         \
    _Pragma("unroll") for (int w2 = 0; w2 < 2; ++w2) asm volatile(                           \
        "ds_read_b64_tr_b16 %0, %1 offset:%2"                                                \
        : "=v"(af[STAGE][ni][w2])                                                            \
        : "v"(waddr[BUF][ni][w2]), "n"((KK) * 16 * 512));                                    \
  }                                                                                          \
  _Pragma("unroll") for (int mi = 0; mi < 4; ++mi) asm volatile(                             \
      "ds_read_b128 %0, %1 offset:%2"                                                        \
      : "=v"(bfr[STAGE][mi])                                                                 \
      : "v"(xaddr[BUF][KK]), "n"(mi * 32 * 128));
#define RF_WAIT(STAGE, PENDING)                                                              \
  asm volatile("s_waitcnt lgkmcnt(%8)"                                                       \
               : "+v"(af[STAGE][0][0]), "+v"(af[STAGE][0][1]), "+v"(af[STAGE][1][0]),        \
                 "+v"(af[STAGE][1][1]), "+v"(bfr[STAGE][0]), "+v"(bfr[STAGE][1]),            \
                 "+v"(bfr[STAGE][2]), "+v"(bfr[STAGE][3])                                    \
               : "n"(PENDING));
#define RF_MFMA(STAGE)                                                                       \
  _Pragma("unroll") for (int ni = 0; ni < 2; ++ni) {                                         \
    u32x4 a;                                                                                 \
    a[0] = af[STAGE][ni][0][0]; a[1] = af[STAGE][ni][0][1];                                  \
    a[2] = af[STAGE][ni][1][0]; a[3] = af[STAGE][ni][1][1];                                  \
    _Pragma("unroll") for (int mi = 0; mi < 4; ++mi) acc[ni][mi] =                           \
        __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),               \
                                                __builtin_bit_cast(bf16x8, bfr[STAGE][mi]),  \
                                                acc[ni][mi], 0, 0, 0);                       \
  }
    RF_ISSUE(0, 0)
    RF_ISSUE(1, 1)
    RF_WAIT(0, 8)
    RF_MFMA(0)
    RF_ISSUE(0, 2)
    RF_WAIT(1, 8)
    RF_MFMA(1)
    RF_ISSUE(1, 3)
    RF_WAIT(0, 8)
    RF_MFMA(0)
    RF_WAIT(1, 0)
    RF_MFMA(1)
#undef RF_ISSUE
#undef RF_WAIT
#undef RF_MFMA
  };

  // K step k0 computes out of stage BUF while tile k0+64 is converted into stage
  // BUF^1 (its X registers were loaded one step earlier) and tile k0+128 is fetched.
  // The two wavefronts that share a SIMD (w and w+4) take the two phases in opposite
  // order, so one's MFMA phase overlaps the other's VALU phase.
  // Vector-memory issue order per step: 4 W loads (top), 8 X/g loads (end); loads
  // retire in order, which fixes the counts in the waits below.
  using std::integral_constant;
  auto k_step = [&](int k0, auto buf_tag) {
    constexpr int BUF = decltype(buf_tag)::value;
    using other = integral_constant<int, BUF ^ 1>;
    const bool more = k0 + kBKK < K;
    // this stage's W loads have landed (the 8 younger X/g loads may still fly) and our
    // LDS writes are done
    if (more)
      asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
    else
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();  // the whole stage is in LDS; the other stage is free
    if (more) issue_w(k0 + kBKK, BUF ^ 1);
    const bool more2 = k0 + 2 * kBKK < K;
    // (one program point for the asynchronous X loads: their registers must not be
    // copied by the compiler while the loads are in flight)
    if (wave < 4) compute(buf_tag);
    if (more) store_x(other{}, integral_constant<int, 4>{});
    if (more2) load_x(k0 + 2 * kBKK);  // a whole step ahead of its use
    if (wave >= 4) compute(buf_tag);
  };

  issue_w(0, 0);
  load_x(0);
  store_x(integral_constant<int, 0>{}, integral_constant<int, 0>{});
  if (kBKK < K) load_x(kBKK);
  for (int k0 = 0; k0 < K; k0 += 2 * kBKK) {
    k_step(k0, integral_constant<int, 0>{});
    if (k0 + kBKK < K) k_step(k0 + kBKK, integral_constant<int, 1>{});
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#undef RF_WAIT_X

  // stage 1 result: the two lanes that share an X row add their partial sums
  ss += dpp_f32<kDppQuadXor1>(ss);
  if (xhalf == 0) s_rstd[xrow] = 1.0f / sqrtf(ss * inv_k + eps);
  __syncthreads();

  // epilogue: y = acc * H(ss)
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int mloc = 128 * wm + 32 * mi + i32;
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
  if (ldw >= (1 << 24)) return hipErrorInvalidValue;  // 32-bit byte offsets inside a 64-row tile
  hipLaunchKernelGGL(rmsnorm_gemm_bf16_kernel, dim3((unsigned)grid), dim3(kGThreads), 0, s,
                     (const bf16_t*)x, (const bf16_t*)g, (const bf16_t*)w, (bf16_t*)y, M, K, N, ldx,
                     ldw, ldy, 1.0f / (float)K, eps, n_mtiles, n_ntiles);
  return hipGetLastError();
}

}  // namespace rf
