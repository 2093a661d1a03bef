// Safe softmax over the last axis: the max -> sum-exp cascade (paper
// Section 2.2; Appendix A.2, first two reductions) fused at wavefront level.
//
// Kernel 1 (rows that fit in registers): one 64-lane wavefront owns one row.
// The row is read once with 128-bit loads and stays in registers; the row max
// and the row sum are reduced lane-locally, then across the wavefront with
// DPP; the normalised row is written once with 128-bit stores.  HBM traffic is
// the algorithmic minimum (one read + one write).
//
// Kernel 2 (any row length / alignment): one workgroup streams a row, every
// lane carrying the level-1 incremental state (m, l) (Appendix A.2,
// incremental form), corrected once per 128-bit vector; lane states are merged
// with the level-k fused expression (Section 3.2 Eq. (11)) across the wavefront
// and then across wavefronts through LDS; a second sweep over the row writes
// the result.
#include <type_traits>

#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

constexpr int kSoftmaxWavesPerWg = 4;

// One wavefront per row; NCH 128-bit chunks per lane; n % kPerVec == 0.
// LANE_LEVEL = false (the shipped path): the two reductions are fused at wavefront level,
// the row max is known before the sum starts, nothing is ever corrected.
// LANE_LEVEL = true (fusion-level study only, Section 5.3): every lane runs the level-1
// incremental form over its own elements, one correction per element, and the 64 lane
// states are merged with the level-k fused expression.
// Wavefronts per SIMD the register allocator has to leave room for, by the number of fp32 values
// a lane holds: without the bound the scheduler spends registers on instruction-level
// parallelism this HBM-bound kernel has no use for, and occupancy (bytes in flight) drops.
constexpr int softmax_waves_per_simd(int floats_per_lane) {
  return floats_per_lane <= 32 ? 8 : floats_per_lane <= 64 ? 4 : 2;
}

template <typename T, int NCH, bool LANE_LEVEL = false>
__global__ __launch_bounds__(kSoftmaxWavesPerWg * kWave,
                             softmax_waves_per_simd(NCH * Elem<T>::kPerVec) * 4 / kSoftmaxWavesPerWg)
void softmax_row_in_regs_kernel(
    const T* __restrict__ x, T* __restrict__ y, int64_t rows, int n, int64_t x_pitch,
    int64_t y_pitch) {
  constexpr int V = Elem<T>::kPerVec;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t row = (int64_t)blockIdx.x * kSoftmaxWavesPerWg + (threadIdx.x >> 6);
  if (row >= rows) return;
  const u32x4* xr = reinterpret_cast<const u32x4*>(x + row * x_pitch);
  u32x4* yr = reinterpret_cast<u32x4*>(y + row * y_pitch);
  const int nvec = n / V;

  // Straight-line code: vectors past the end of the row are loaded from the last valid
  // vector and replaced by -inf (the identity of the max stage; exp gives 0 for the sum
  // stage), so no stage below needs a branch.  Only the stores are predicated.
  // The row lives in registers as fp32 from here on: e[][] holds x, then exp(x - m).
  constexpr uint32_t kNegInf = std::is_same<T, float>::value ? 0xFF800000u : 0xFF80FF80u;
  // Full vectors sit at one lane address plus a constant; the vector that holds the end of the
  // row (and any vector past it) is read at a clamped address of its own.
  const u32x4* xl = xr + lane;
  const u32x4* xt = xr + min((nvec - 1) / kWave * kWave + lane, nvec - 1);
  float e[NCH][V];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int idx = c * kWave + lane;
    const bool full = (c + 1) * kWave <= nvec;  // wave-uniform
    u32x4 r = __builtin_nontemporal_load(full ? xl + c * kWave : xt);
    const bool ok = idx < nvec;
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = ok ? r[j] : kNegInf;
    Elem<T>::unpack(r, e[c]);
  }
  float m = -INFINITY;
  float l = 0.f;
  if constexpr (LANE_LEVEL) {
    // per-lane incremental state, then the merge; exponentials are taken again afterwards
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      if (c * kWave + lane < nvec) {
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const float mn = fmaxf(m, e[c][i]);
          l = l * fast_exp2((m - mn) * kLog2e) + fast_exp2((e[c][i] - mn) * kLog2e);
          m = mn;
        }
      }
    }
    const float mw = wave_max(m);
    l = wave_sum((m == -INFINITY) ? 0.f : l * fast_exp2((m - mw) * kLog2e));
    m = mw;
    const float mb = -m * kLog2e;
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
      for (int i = 0; i < V; ++i) e[c][i] = fast_exp2(fmaf(e[c][i], kLog2e, mb));
  } else {
    // cascade stage 1: row max
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
      for (int i = 0; i < V; ++i) m = fmaxf(m, e[c][i]);
    m = wave_max(m);
    // cascade stage 2: sum of exp(x - m), exponentials kept for the epilogue
    const float mb = -m * kLog2e;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
#pragma unroll
      for (int i = 0; i < V; ++i) {
        e[c][i] = fast_exp2(fmaf(e[c][i], kLog2e, mb));
        l += e[c][i];
      }
      __builtin_amdgcn_sched_barrier(0);  // one vector at a time: no extra live temporaries
    }
    l = wave_sum(l);
  }
  const float inv = 1.0f / l;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int idx = c * kWave + lane;
    if (idx < nvec) {
      float f[V];
#pragma unroll
      for (int i = 0; i < V; ++i) f[i] = e[c][i] * inv;
      __builtin_nontemporal_store(Elem<T>::pack(f), yr + idx);
    }
  }
}

// Short rows (at most LPR vectors of 16 bytes): 64 / LPR rows per wavefront, one vector per
// lane, the two reductions over the LPR lanes of a row by butterfly shuffles.  A wavefront per
// row would leave most lanes (and most of every 128-byte line fetched) idle.
template <typename T, int LPR>
__global__ __launch_bounds__(kSoftmaxWavesPerWg * kWave) void softmax_short_rows_kernel(
    const T* __restrict__ x, T* __restrict__ y, int64_t rows, int n, int64_t x_pitch,
    int64_t y_pitch) {
  constexpr int V = Elem<T>::kPerVec;
  constexpr int RPW = kWave / LPR;  // rows per wavefront
  constexpr uint32_t kNegInf = std::is_same<T, float>::value ? 0xFF800000u : 0xFF80FF80u;
  const int lane = threadIdx.x & (kWave - 1);
  const int sub = lane % LPR;       // vector index inside the row
  const int64_t row = ((int64_t)blockIdx.x * kSoftmaxWavesPerWg + (threadIdx.x >> 6)) * RPW + lane / LPR;
  const int nvec = n / V;
  const bool ok = row < rows && sub < nvec;
  // lanes without a vector read a valid address (their own row's first vector, or row 0's)
  const u32x4* src = reinterpret_cast<const u32x4*>(x + (row < rows ? row : 0) * x_pitch) + (sub < nvec ? sub : 0);
  u32x4 r = __builtin_nontemporal_load(src);
#pragma unroll
  for (int j = 0; j < 4; ++j) r[j] = ok ? r[j] : kNegInf;
  float e[V];
  Elem<T>::unpack(r, e);
  float m = e[0];
#pragma unroll
  for (int i = 1; i < V; ++i) m = fmaxf(m, e[i]);
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
  const float mb = -m * kLog2e;
  float l = 0.f;
#pragma unroll
  for (int i = 0; i < V; ++i) {
    e[i] = fast_exp2(fmaf(e[i], kLog2e, mb));
    l += e[i];
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) l += __shfl_xor(l, off, kWave);
  const float inv = 1.0f / l;
#pragma unroll
  for (int i = 0; i < V; ++i) e[i] *= inv;
  if (ok) __builtin_nontemporal_store(Elem<T>::pack(e), reinterpret_cast<u32x4*>(y + row * y_pitch) + sub);
}

// Long rows that still fit the registers of one workgroup (up to WAVES * 64 lanes * 64 values):
// one workgroup per row, the row read once and kept as fp32; the two reductions go through
// the wavefronts' DPP reductions and one LDS exchange each.
template <typename T, int NCH, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void softmax_row_in_regs_wg_kernel(
    const T* __restrict__ x, T* __restrict__ y, int64_t rows, int n, int64_t x_pitch,
    int64_t y_pitch) {
  constexpr int V = Elem<T>::kPerVec;
  constexpr int TH = WAVES * kWave;
  constexpr uint32_t kNegInf = std::is_same<T, float>::value ? 0xFF800000u : 0xFF80FF80u;
  __shared__ float s_max[WAVES], s_sum[WAVES];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const u32x4* xr = reinterpret_cast<const u32x4*>(x + row * x_pitch);
  u32x4* yr = reinterpret_cast<u32x4*>(y + row * y_pitch);
  const int nvec = n / V;
  float e[NCH][V];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int idx = c * TH + tid;
    u32x4 r = __builtin_nontemporal_load(xr + min(idx, nvec - 1));
    const bool ok = idx < nvec;
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = ok ? r[j] : kNegInf;
    Elem<T>::unpack(r, e[c]);
  }
  // cascade stage 1: row max
  float m = -INFINITY;
#pragma unroll
  for (int c = 0; c < NCH; ++c)
#pragma unroll
    for (int i = 0; i < V; ++i) m = fmaxf(m, e[c][i]);
  m = wave_max(m);
  if ((tid & (kWave - 1)) == 0) s_max[tid >> 6] = m;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < WAVES; ++w) m = fmaxf(m, s_max[w]);
  // cascade stage 2: sum of exp(x - m), exponentials kept for the epilogue
  const float mb = -m * kLog2e;
  float l = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
#pragma unroll
    for (int i = 0; i < V; ++i) {
      e[c][i] = fast_exp2(fmaf(e[c][i], kLog2e, mb));
      l += e[c][i];
    }
  }
  l = wave_sum(l);
  if ((tid & (kWave - 1)) == 0) s_sum[tid >> 6] = l;
  __syncthreads();
  l = 0.f;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) l += s_sum[w];   // same order in every lane
  const float inv = 1.0f / l;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int idx = c * TH + tid;
    if (idx < nvec) {
      float f[V];
#pragma unroll
      for (int i = 0; i < V; ++i) f[i] = e[c][i] * inv;
      __builtin_nontemporal_store(Elem<T>::pack(f), yr + idx);
    }
  }
}

// One workgroup per row, any n; two sweeps over the row (the second one is served by the
// L2 for rows of a few hundred KB).  VEC: rows are 16-byte aligned, so both sweeps use
// 128-bit accesses and the incremental state is corrected once per vector; otherwise
// scalar accesses, one correction per element.
constexpr int kStreamThreads = 256;
template <typename T, bool VEC>
__global__ __launch_bounds__(kStreamThreads) void softmax_row_streaming_kernel(
    const T* __restrict__ x, T* __restrict__ y, int64_t rows, int64_t n, int64_t x_pitch,
    int64_t y_pitch) {
  constexpr int V = Elem<T>::kPerVec;
  __shared__ float sm[kStreamThreads / kWave];
  __shared__ float sl[kStreamThreads / kWave];
  const int64_t row = blockIdx.x;
  if (row >= rows) return;
  const T* xr = x + row * x_pitch;
  T* yr = y + row * y_pitch;
  const int64_t nvec = VEC ? n / V : 0;   // full vectors; the rest is handled element-wise
  // level-1 incremental state per lane
  float m = -INFINITY, l = 0.f;
  if constexpr (VEC) {
    const u32x4* xv = reinterpret_cast<const u32x4*>(xr);
    for (int64_t j = threadIdx.x; j < nvec; j += kStreamThreads) {
      float f[V];
      Elem<T>::unpack(xv[j], f);
      float vm = f[0];
#pragma unroll
      for (int i = 1; i < V; ++i) vm = fmaxf(vm, f[i]);
      const float mn = fmaxf(m, vm);
      const float mb = -mn * kLog2e;
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < V; ++i) sum += fast_exp2(fmaf(f[i], kLog2e, mb));
      l = l * fast_exp2((m - mn) * kLog2e) + sum;  // exp(m - mn) with m = -inf and l = 0 adds nothing
      m = mn;
    }
  }
  for (int64_t j = nvec * V + threadIdx.x; j < n; j += kStreamThreads) {
    const float v = Elem<T>::load(xr + j);
    const float mn = fmaxf(m, v);
    l = l * fast_exp2((m - mn) * kLog2e) + fast_exp2((v - mn) * kLog2e);
    m = mn;
  }
  // merge lane states across the wavefront: l_c * exp(m_c - m)
  const float mw = wave_max(m);
  float lw = (m == -INFINITY) ? 0.f : l * fast_exp2((m - mw) * kLog2e);
  lw = wave_sum(lw);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sm[wave] = mw; sl[wave] = lw; }
  __syncthreads();
  float mg = -INFINITY;
#pragma unroll
  for (int w = 0; w < kStreamThreads / kWave; ++w) mg = fmaxf(mg, sm[w]);
  float lg = 0.f;
#pragma unroll
  for (int w = 0; w < kStreamThreads / kWave; ++w)
    lg += (sm[w] == -INFINITY) ? 0.f : sl[w] * fast_exp2((sm[w] - mg) * kLog2e);
  const float inv = 1.0f / lg;
  const float mb = -mg * kLog2e;
  if constexpr (VEC) {
    const u32x4* xv = reinterpret_cast<const u32x4*>(xr);
    u32x4* yv = reinterpret_cast<u32x4*>(yr);
    for (int64_t j = threadIdx.x; j < nvec; j += kStreamThreads) {
      float f[V];
      Elem<T>::unpack(xv[j], f);
#pragma unroll
      for (int i = 0; i < V; ++i) f[i] = fast_exp2(fmaf(f[i], kLog2e, mb)) * inv;
      __builtin_nontemporal_store(Elem<T>::pack(f), yv + j);
    }
  }
  for (int64_t j = nvec * V + threadIdx.x; j < n; j += kStreamThreads) {
    const float v = Elem<T>::load(xr + j);
    Elem<T>::store(yr + j, fast_exp2(fmaf(v, kLog2e, mb)) * inv);
  }
}

template <typename T>
static hipError_t launch_softmax_t(const T* x, T* y, int64_t rows, int64_t n, int64_t x_pitch,
                                   int64_t y_pitch, bool vec_ok, hipStream_t s) {
  constexpr int V = Elem<T>::kPerVec;
  const int64_t per_chunk = (int64_t)V * kWave;
  if (vec_ok && n % V == 0 && n > 0 && n <= 32 * V) {
    // short rows: 2, 4, 8 or 16 rows per wavefront
    const int nvec = (int)(n / V);
    const int lpr = nvec <= 4 ? 4 : nvec <= 8 ? 8 : nvec <= 16 ? 16 : 32;
    const int64_t rows_per_wg = (int64_t)kSoftmaxWavesPerWg * (kWave / lpr);
    const unsigned grid = (unsigned)((rows + rows_per_wg - 1) / rows_per_wg);
    const dim3 block(kSoftmaxWavesPerWg * kWave);
#define RF_SOFTMAX_SHORT(L)                                                               \
  hipLaunchKernelGGL((softmax_short_rows_kernel<T, L>), dim3(grid), block, 0, s, x, y, rows, \
                     (int)n, x_pitch, y_pitch)
    if (lpr == 4) RF_SOFTMAX_SHORT(4);
    else if (lpr == 8) RF_SOFTMAX_SHORT(8);
    else if (lpr == 16) RF_SOFTMAX_SHORT(16);
    else RF_SOFTMAX_SHORT(32);
#undef RF_SOFTMAX_SHORT
  } else if (vec_ok && n % V == 0 && n <= (64 / V) * per_chunk) {
    // one wavefront per row, at most 64 values per lane
    const int nch = (int)((n + per_chunk - 1) / per_chunk);
    const unsigned grid = (unsigned)((rows + kSoftmaxWavesPerWg - 1) / kSoftmaxWavesPerWg);
    const dim3 block(kSoftmaxWavesPerWg * kWave);
#define RF_SOFTMAX_CASE(N)                                                              \
  hipLaunchKernelGGL((softmax_row_in_regs_kernel<T, N>), dim3(grid), block, 0, s, x, y, \
                     rows, (int)n, x_pitch, y_pitch)
    if (nch <= 1) RF_SOFTMAX_CASE(1);
    else if (nch <= 2) RF_SOFTMAX_CASE(2);
    else if (nch <= 4) RF_SOFTMAX_CASE(4);
    else if (nch <= 8) RF_SOFTMAX_CASE(8);
    else RF_SOFTMAX_CASE(16);
#undef RF_SOFTMAX_CASE
  } else if (vec_ok && n % V == 0 && n <= 16 * 64 * (int64_t)kWave) {
    // up to 64 values per lane, 2 / 4 / 8 / 16 wavefronts: rows of 8K, 16K, 32K, 64K values
    constexpr int NCHW = 64 / V;
    const int64_t per_wave = (int64_t)NCHW * V * kWave;   // 4096 values
#define RF_SOFTMAX_WG(W)                                                                       \
  hipLaunchKernelGGL((softmax_row_in_regs_wg_kernel<T, NCHW, W>), dim3((unsigned)rows),        \
                     dim3(W * kWave), 0, s, x, y, rows, (int)n, x_pitch, y_pitch)
    if (n <= 2 * per_wave) RF_SOFTMAX_WG(2);
    else if (n <= 4 * per_wave) RF_SOFTMAX_WG(4);
    else if (n <= 8 * per_wave) RF_SOFTMAX_WG(8);
    else RF_SOFTMAX_WG(16);
#undef RF_SOFTMAX_WG
  } else if (vec_ok) {
    hipLaunchKernelGGL((softmax_row_streaming_kernel<T, true>), dim3((unsigned)rows),
                       dim3(kStreamThreads), 0, s, x, y, rows, n, x_pitch, y_pitch);
  } else {
    hipLaunchKernelGGL((softmax_row_streaming_kernel<T, false>), dim3((unsigned)rows),
                       dim3(kStreamThreads), 0, s, x, y, rows, n, x_pitch, y_pitch);
  }
  return hipGetLastError();
}

// ---- fusion-level study (Section 5.3): the unfused chain as three kernels ----
// One wavefront per row, 128-bit loads; m and l pass through memory between the kernels.
// PASS 0: m = max x;  PASS 1: l = sum exp(x - m);  PASS 2: y = exp(x - m) / l.
template <typename T, int PASS>
__global__ __launch_bounds__(kSoftmaxWavesPerWg * kWave) void softmax_unfused_pass_kernel(
    const T* __restrict__ x, T* __restrict__ y, float* __restrict__ m_buf, float* __restrict__ l_buf,
    int64_t rows, int n, int64_t x_pitch, int64_t y_pitch) {
  constexpr int V = Elem<T>::kPerVec;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t row = (int64_t)blockIdx.x * kSoftmaxWavesPerWg + (threadIdx.x >> 6);
  if (row >= rows) return;
  const u32x4* xr = reinterpret_cast<const u32x4*>(x + row * x_pitch);
  u32x4* yr = reinterpret_cast<u32x4*>(y + row * y_pitch);
  const int nvec = n / V;
  float acc = PASS == 0 ? -INFINITY : 0.f;
  const float mb = PASS == 0 ? 0.f : -m_buf[row] * kLog2e;
  const float inv = PASS == 2 ? 1.0f / l_buf[row] : 0.f;
  for (int idx = lane; idx < nvec; idx += kWave) {
    float f[V];
    Elem<T>::unpack(xr[idx], f);
    if constexpr (PASS == 0) {
#pragma unroll
      for (int i = 0; i < V; ++i) acc = fmaxf(acc, f[i]);
    } else if constexpr (PASS == 1) {
#pragma unroll
      for (int i = 0; i < V; ++i) acc += fast_exp2(fmaf(f[i], kLog2e, mb));
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i) f[i] = fast_exp2(fmaf(f[i], kLog2e, mb)) * inv;
      yr[idx] = Elem<T>::pack(f);
    }
  }
  if constexpr (PASS == 0) { acc = wave_max(acc); if (lane == 0) m_buf[row] = acc; }
  if constexpr (PASS == 1) { acc = wave_sum(acc); if (lane == 0) l_buf[row] = acc; }
}

// ---- fusion-level study: fused across workgroups (the paper's inter-block level) ----
// A row is cut into kInterBlockSegs segments, one wavefront (of different workgroups) each.
// Kernel 1 reads its segment once and stores the segment's fused state (m_s, l_s); kernel 2
// merges the row's states with the level-k expression (Eq. (11)), reads its segment again and
// writes y.  Two reads of x and a round trip of the states through memory: the cost the paper
// attributes to this level.  m_buf, l_buf: rows * kInterBlockSegs floats each.
constexpr int kInterBlockSegs = 4;
template <typename T, int PASS>
__global__ __launch_bounds__(kSoftmaxWavesPerWg * kWave) void softmax_interblock_kernel(
    const T* __restrict__ x, T* __restrict__ y, float* __restrict__ m_buf, float* __restrict__ l_buf,
    int64_t rows, int n, int64_t x_pitch, int64_t y_pitch) {
  constexpr int V = Elem<T>::kPerVec;
  const int lane = threadIdx.x & (kWave - 1);
  // consecutive wavefronts of a workgroup take different rows: the segments of one row run in
  // different workgroups
  const int64_t unit = (int64_t)blockIdx.x * kSoftmaxWavesPerWg + (threadIdx.x >> 6);
  const int seg = (int)(unit / rows);
  const int64_t row = unit % rows;
  if (seg >= kInterBlockSegs) return;
  const int nvec = n / V;
  const int per_seg = (nvec + kInterBlockSegs - 1) / kInterBlockSegs;
  const int v0 = seg * per_seg, v1 = min(nvec, v0 + per_seg);
  const u32x4* xr = reinterpret_cast<const u32x4*>(x + row * x_pitch);
  if constexpr (PASS == 0) {
    // the segment's state, level-1 incremental form per lane, lanes merged with Eq. (11)
    float m = -INFINITY, l = 0.f;
    for (int idx = v0 + lane; idx < v1; idx += kWave) {
      float f[V];
      Elem<T>::unpack(xr[idx], f);
      float vm = f[0];
#pragma unroll
      for (int i = 1; i < V; ++i) vm = fmaxf(vm, f[i]);
      const float m_new = fmaxf(m, vm);
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < V; ++i) part += fast_exp2((f[i] - m_new) * kLog2e);
      l = l * ((m == -INFINITY) ? 0.f : fast_exp2((m - m_new) * kLog2e)) + part;
      m = m_new;
    }
    const float mw = wave_max(m);
    const float lw = wave_sum((m == -INFINITY) ? 0.f : l * fast_exp2((m - mw) * kLog2e));
    if (lane == 0) { m_buf[row * kInterBlockSegs + seg] = mw; l_buf[row * kInterBlockSegs + seg] = lw; }
  } else {
    float ms[kInterBlockSegs], ls[kInterBlockSegs];
    float m = -INFINITY;
#pragma unroll
    for (int c = 0; c < kInterBlockSegs; ++c) {
      ms[c] = m_buf[row * kInterBlockSegs + c];
      ls[c] = l_buf[row * kInterBlockSegs + c];
      m = fmaxf(m, ms[c]);
    }
    float l = 0.f;
#pragma unroll
    for (int c = 0; c < kInterBlockSegs; ++c) l += (ms[c] == -INFINITY) ? 0.f : ls[c] * fast_exp2((ms[c] - m) * kLog2e);
    const float inv = 1.0f / l, mb = -m * kLog2e;
    u32x4* yr = reinterpret_cast<u32x4*>(y + row * y_pitch);
    for (int idx = v0 + lane; idx < v1; idx += kWave) {
      float f[V];
      Elem<T>::unpack(xr[idx], f);
#pragma unroll
      for (int i = 0; i < V; ++i) f[i] = fast_exp2(fmaf(f[i], kLog2e, mb)) * inv;
      yr[idx] = Elem<T>::pack(f);
    }
  }
}

// level 0: unfused (three kernels, needs ml_buf = 2 * rows floats); 1: fused per lane;
// 2: fused per wavefront (the shipped kernel for rows of up to 4096 values); 3: fused per workgroup (the streaming kernel);
// 4: fused across workgroups (two kernels, needs ml_buf = 8 * rows floats).
// bf16 only, n a multiple of 8 and at most 8192, 16-byte aligned rows.
hipError_t launch_softmax_level(const void* x, void* y, int64_t rows, int64_t n, int64_t x_pitch,
                                int64_t y_pitch, int level, float* ml_buf, hipStream_t s) {
  typedef bf16_t T;
  const T* xp = (const T*)x;
  T* yp = (T*)y;
  const int64_t per_chunk = (int64_t)Elem<T>::kPerVec * kWave;
  if (n % Elem<T>::kPerVec != 0 || n > 16 * per_chunk || level < 0 || level > 4) return hipErrorInvalidValue;
  const unsigned grid = (unsigned)((rows + kSoftmaxWavesPerWg - 1) / kSoftmaxWavesPerWg);
  const dim3 block(kSoftmaxWavesPerWg * kWave);
  if (level == 0) {
    if (ml_buf == nullptr) return hipErrorInvalidValue;
    hipLaunchKernelGGL((softmax_unfused_pass_kernel<T, 0>), dim3(grid), block, 0, s, xp, yp, ml_buf, ml_buf + rows, rows, (int)n, x_pitch, y_pitch);
    hipLaunchKernelGGL((softmax_unfused_pass_kernel<T, 1>), dim3(grid), block, 0, s, xp, yp, ml_buf, ml_buf + rows, rows, (int)n, x_pitch, y_pitch);
    hipLaunchKernelGGL((softmax_unfused_pass_kernel<T, 2>), dim3(grid), block, 0, s, xp, yp, ml_buf, ml_buf + rows, rows, (int)n, x_pitch, y_pitch);
  } else if (level == 1 || level == 2) {
    const int nch = (int)((n + per_chunk - 1) / per_chunk);
#define RF_SOFTMAX_LEVEL_CASE(N)                                                                    \
  if (level == 1)                                                                                   \
    hipLaunchKernelGGL((softmax_row_in_regs_kernel<T, N, true>), dim3(grid), block, 0, s, xp, yp,   \
                       rows, (int)n, x_pitch, y_pitch);                                             \
  else                                                                                              \
    hipLaunchKernelGGL((softmax_row_in_regs_kernel<T, N, false>), dim3(grid), block, 0, s, xp, yp,  \
                       rows, (int)n, x_pitch, y_pitch)
    if (nch <= 1) { RF_SOFTMAX_LEVEL_CASE(1); }
    else if (nch <= 2) { RF_SOFTMAX_LEVEL_CASE(2); }
    else if (nch <= 4) { RF_SOFTMAX_LEVEL_CASE(4); }
    else if (nch <= 8) { RF_SOFTMAX_LEVEL_CASE(8); }
    else { RF_SOFTMAX_LEVEL_CASE(16); }
#undef RF_SOFTMAX_LEVEL_CASE
  } else if (level == 3) {
    hipLaunchKernelGGL((softmax_row_streaming_kernel<T, true>), dim3((unsigned)rows), dim3(kStreamThreads), 0, s,
                       xp, yp, rows, n, x_pitch, y_pitch);
  } else {
    if (ml_buf == nullptr) return hipErrorInvalidValue;
    const int64_t units = rows * kInterBlockSegs;
    const int64_t g4 = (units + kSoftmaxWavesPerWg - 1) / kSoftmaxWavesPerWg;
    if (g4 > INT32_MAX) return hipErrorInvalidValue;
    float* lb = ml_buf + rows * kInterBlockSegs;
    hipLaunchKernelGGL((softmax_interblock_kernel<T, 0>), dim3((unsigned)g4), block, 0, s, xp, yp, ml_buf, lb, rows, (int)n, x_pitch, y_pitch);
    hipLaunchKernelGGL((softmax_interblock_kernel<T, 1>), dim3((unsigned)g4), block, 0, s, xp, yp, ml_buf, lb, rows, (int)n, x_pitch, y_pitch);
  }
  return hipGetLastError();
}

hipError_t launch_softmax(const void* x, void* y, bool is_bf16, int64_t rows, int64_t n,
                          int64_t x_pitch, int64_t y_pitch, bool vec_ok, hipStream_t s) {
  if (is_bf16)
    return launch_softmax_t<bf16_t>((const bf16_t*)x, (bf16_t*)y, rows, n, x_pitch, y_pitch,
                                    vec_ok, s);
  return launch_softmax_t<float>((const float*)x, (float*)y, rows, n, x_pitch, y_pitch, vec_ok, s);
}

}  // namespace rf
