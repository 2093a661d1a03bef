// Measurement aids (not part of the cascaded-reduction path): the two ceilings the
// roofline fractions are put next to.
//   - a plain streaming copy kernel of known size (HBM ceiling; also the reference
//     dispatch that scales the FETCH_SIZE / WRITE_SIZE hardware counters),
//   - a read-only streaming kernel (what a kernel that only reads HBM can reach),
//   - an MFMA-only loop (dense bf16 32x32x16) with constant or pseudo-random operands:
//     the matrix-pipe ceiling depends strongly on the operand values (clock / power).
#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

__global__ __launch_bounds__(256) void diag_copy_kernel(const u32x4* __restrict__ src,
                                                        u32x4* __restrict__ dst, int64_t n_vec) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Reads n_vec 128-bit vectors once (non-temporal), every workgroup a contiguous share with
// eight loads in flight per lane, folds them, and writes one word per wavefront (the XOR of what it
// read) so that the loads cannot be dropped.
__global__ __launch_bounds__(256) void diag_read_kernel(const u32x4* __restrict__ src, int64_t n_vec,
                                                        uint32_t* __restrict__ sink) {
  const int64_t per_wg = (n_vec + gridDim.x - 1) / gridDim.x;
  const int64_t lo = (int64_t)blockIdx.x * per_wg;
  const int64_t hi = min(n_vec, lo + per_wg);
  u32x4 acc = u32x4{0u, 0u, 0u, 0u};
  int64_t i = lo + threadIdx.x;
  for (; i + 7 * 256 < hi; i += 8 * 256) {
    u32x4 r[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) r[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= r[u];
  }
  for (; i < hi; i += 256) acc ^= __builtin_nontemporal_load(src + i);
  uint32_t w = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) w ^= __shfl_xor(w, off, 64);
  if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = w;
}

__device__ __forceinline__ uint32_t diag_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// Every wavefront issues 32 * iters MFMAs on 8 independent accumulators.
__global__ __launch_bounds__(256) void diag_mfma_kernel(float* __restrict__ sink, int iters,
                                                        int random_operands) {
  f32x16 c[8];
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) c[t][r] = 0.f;
  u32x4 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t h1 = diag_hash(threadIdx.x * 131u + blockIdx.x * 7u + i * 17u + j);
      const uint32_t h2 = diag_hash(h1 + 99u);
      // bf16 pairs with random sign and mantissa, magnitude in [0.5, 2)
      a[i][j] = random_operands ? ((h1 & 0x80ff80ffu) | 0x3f003f00u) : 0x3f803f80u;
      b[i][j] = random_operands ? ((h2 & 0x80ff80ffu) | 0x3f003f00u) : 0x3f803f80u;
    }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 32; ++j)
      c[j & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[j & 7]),
                                                         __builtin_bit_cast(bf16x8, b[(j >> 2) & 7]),
                                                         c[j & 7], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c[t][r];
  sink[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

hipError_t launch_diag_copy(const void* src, void* dst, int64_t bytes, hipStream_t s) {
  const int64_t n_vec = bytes / 16;
  const int64_t want = (n_vec + 255) / 256;
  const unsigned grid = (unsigned)(want < 1 ? 1 : (want > 65536 ? 65536 : want));
  hipLaunchKernelGGL(diag_copy_kernel, dim3(grid), dim3(256), 0, s, (const u32x4*)src, (u32x4*)dst,
                     n_vec);
  return hipGetLastError();
}

hipError_t launch_diag_read(const void* src, int64_t bytes, void* sink, hipStream_t s) {
  hipLaunchKernelGGL(diag_read_kernel, dim3(kDiagReadWorkgroups), dim3(256), 0, s, (const u32x4*)src,
                     bytes / 16, (uint32_t*)sink);
  return hipGetLastError();
}

hipError_t launch_diag_mfma(float* sink, int workgroups, int iters, int random_operands,
                            hipStream_t s) {
  hipLaunchKernelGGL(diag_mfma_kernel, dim3((unsigned)workgroups), dim3(256), 0, s, sink, iters,
                     random_operands);
  return hipGetLastError();
}

}  // namespace rf
