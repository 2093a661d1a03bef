// Mean and population variance over the last axis: the cascade
//   m = (1/L) sum_l x[l];   var = (1/L) sum_l (x[l] - m)^2
// (paper Appendix, evaluation on non-ML workloads) in single-pass form.
//
// The second map (x - m)^2 is not G(x) (x) H(m) for one pair of operators;
// expanding the square gives decomposable terms, and carrying them as
// (count, mean, M2 = sum (x - mean)^2) gives a running state whose merge is
//   n = n_a + n_b;  d = mean_b - mean_a;  mean = mean_a + d n_b / n;
//   M2 = M2_a + M2_b + d^2 n_a n_b / n
// (the level-k fused expression of Section 3.2 for this cascade; the cross term
// of the expanded square vanishes).  It is associative and commutative, so the
// same operator merges vectors, lanes, wavefronts.
//
// One workgroup (4 wavefronts, or 16 when rows are few and long) streams one row once.  Every lane turns each
// 128-bit vector into an exact state (two passes over 4 or 8 registers), merges
// the eight vectors of a chunk pairwise (equal counts: no division), and folds
// the result into its running state (what is left of a row after the full chunks
// goes through chunks of 4, 2 and 1 vectors per lane); lanes merge through DPP / shuffles,
// wavefronts through LDS.  HBM traffic is one read of x.
#include <type_traits>

#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

namespace {

struct VarState {
  float n, mean, m2;
};

__device__ __forceinline__ VarState var_merge(const VarState& a, const VarState& b) {
  VarState r;
  r.n = a.n + b.n;
  const float inv = r.n > 0.f ? fast_rcp(r.n) : 0.f;  // empty + empty stays empty
  const float d = b.mean - a.mean;
  const float wb = b.n * inv;
  r.mean = fmaf(d, wb, a.mean);
  r.m2 = a.m2 + b.m2 + d * d * a.n * wb;
  return r;
}
// both sides hold the same, non-zero count
__device__ __forceinline__ VarState var_merge_equal(const VarState& a, const VarState& b) {
  VarState r;
  const float d = b.mean - a.mean;
  r.n = a.n + a.n;
  r.mean = fmaf(d, 0.5f, a.mean);
  r.m2 = a.m2 + b.m2 + d * d * (0.5f * a.n);
  return r;
}
// exact state of the first `cnt` of V values held in registers
template <int V>
__device__ __forceinline__ VarState var_of_vector(const float* f, int cnt) {
  VarState r;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < V; ++i) s += (i < cnt) ? f[i] : 0.f;
  r.n = (float)cnt;
  r.mean = cnt > 0 ? s / (float)cnt : 0.f;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const float d = f[i] - r.mean;
    q += (i < cnt) ? d * d : 0.f;
  }
  r.m2 = q;
  return r;
}
template <int V>
__device__ __forceinline__ VarState var_of_full_vector(const float* f) {
  VarState r;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < V; ++i) s += f[i];
  r.n = (float)V;
  r.mean = s * (1.0f / V);
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const float d = f[i] - r.mean;
    q = fmaf(d, d, q);
  }
  r.m2 = q;
  return r;
}

__device__ __forceinline__ VarState var_shfl_xor(const VarState& a, int mask) {
  VarState b;
  b.n = __shfl_xor(a.n, mask, 64);
  b.mean = __shfl_xor(a.mean, mask, 64);
  b.m2 = __shfl_xor(a.m2, mask, 64);
  return b;
}

constexpr int kVarUnroll = 8;  // 128-bit loads in flight per lane in a full chunk

}  // namespace

// VEC: the row base and pitch allow 128-bit loads.  kVarWaves wavefronts share a row: 4 when
// there are enough rows to fill the GPU, 16 when there are few (each row then needs more loads
// in flight to be read at speed).
template <typename T, bool VEC, int kVarWaves>
__global__ __launch_bounds__(kVarWaves * kWave) void variance_kernel(const T* __restrict__ x,
                                                                     float* __restrict__ mean_out,
                                                                     float* __restrict__ var_out,
                                                                     int64_t n, int64_t x_pitch) {
  constexpr int kVarThreads = kVarWaves * kWave;
  constexpr int V = Elem<T>::kPerVec;
  __shared__ float s_n[kVarWaves], s_mean[kVarWaves], s_m2[kVarWaves];
  const int tid = threadIdx.x;
  const int64_t row = blockIdx.x;
  const T* xr = x + row * x_pitch;

  VarState st{0.f, 0.f, 0.f};
  if constexpr (VEC) {
    const u32x4* xv = reinterpret_cast<const u32x4*>(xr);
    const int64_t nvec = n / V;  // full vectors
    int64_t base = 0;
    // a chunk: every lane owns U full vectors, all U loads in flight together
    auto chunk = [&](auto utag) {
      constexpr int U = decltype(utag)::value;
      u32x4 raw[U];
#pragma unroll
      for (int u = 0; u < U; ++u) raw[u] = __builtin_nontemporal_load(xv + base + u * kVarThreads + tid);
      VarState c[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float f[V];
        Elem<T>::unpack(raw[u], f);
        c[u] = var_of_full_vector<V>(f);
      }
      // pairwise tree over the equal-count states
#pragma unroll
      for (int w = 1; w < U; w <<= 1) {
#pragma unroll
        for (int u = 0; u < U; u += 2 * w) c[u] = var_merge_equal(c[u], c[u + w]);
      }
      st = var_merge(st, c[0]);
      base += (int64_t)U * kVarThreads;
    };
    while (base + (int64_t)kVarUnroll * kVarThreads <= nvec) chunk(std::integral_constant<int, kVarUnroll>{});
    if (base + 4 * (int64_t)kVarThreads <= nvec) chunk(std::integral_constant<int, 4>{});
    if (base + 2 * (int64_t)kVarThreads <= nvec) chunk(std::integral_constant<int, 2>{});
    if (base + (int64_t)kVarThreads <= nvec) chunk(std::integral_constant<int, 1>{});
    // fewer than one vector per lane left, then the ragged tail (fewer than V elements)
    if (base + tid < nvec) {
      float f[V];
      Elem<T>::unpack(__builtin_nontemporal_load(xv + base + tid), f);
      st = var_merge(st, var_of_full_vector<V>(f));
    }
    const int64_t tail0 = nvec * V;
    if (tid == 0 && tail0 < n) {
      float f[V];
#pragma unroll
      for (int i = 0; i < V; ++i) f[i] = (tail0 + i < n) ? Elem<T>::load(xr + tail0 + i) : 0.f;
      st = var_merge(st, var_of_vector<V>(f, (int)(n - tail0)));
    }
  } else {
    // level-1 incremental form, one element at a time
    for (int64_t i = tid; i < n; i += kVarThreads) {
      const float v = Elem<T>::load(xr + i);
      st = var_merge(st, VarState{1.f, v, 0.f});
    }
  }

  // merge the 64 lane states, then the wavefront states
#pragma unroll
  for (int mask = 1; mask < 64; mask <<= 1) st = var_merge(st, var_shfl_xor(st, mask));
  const int wave = tid >> 6;
  if ((tid & 63) == 0) { s_n[wave] = st.n; s_mean[wave] = st.mean; s_m2[wave] = st.m2; }
  __syncthreads();
  if (tid == 0) {
    VarState r{s_n[0], s_mean[0], s_m2[0]};
#pragma unroll
    for (int w = 1; w < kVarWaves; ++w) r = var_merge(r, VarState{s_n[w], s_mean[w], s_m2[w]});
    mean_out[row] = r.mean;
    var_out[row] = r.m2 / (float)n;
  }
}

hipError_t launch_variance(const void* x, bool is_bf16, float* mean, float* var, int64_t rows,
                           int64_t n, int64_t x_pitch, bool vec_ok, hipStream_t s) {
  if (rows > INT32_MAX) return hipErrorInvalidValue;
  // Few long rows: 16 wavefronts per row instead of 4.  Measured per call under graph replay:
  // 128 rows of 32768 go from 8.5 to 6.0 us, one such row from 4.2 to 3.8; rows of 8192 are
  // faster with 4 wavefronts (2.7 against 3.2 us), and so are 512 rows or more of any length.
  const bool wide = rows <= 256 && n >= 16384;
  const dim3 grid((unsigned)rows), block((wide ? 16 : 4) * kWave);
#define RF_LAUNCH_VAR(T, VEC)                                                                    \
  if (wide) hipLaunchKernelGGL((variance_kernel<T, VEC, 16>), grid, block, 0, s, (const T*)x, mean, var, n, x_pitch); \
  else hipLaunchKernelGGL((variance_kernel<T, VEC, 4>), grid, block, 0, s, (const T*)x, mean, var, n, x_pitch);
  if (is_bf16) {
    if (vec_ok) { RF_LAUNCH_VAR(bf16_t, true) } else { RF_LAUNCH_VAR(bf16_t, false) }
  } else {
    if (vec_ok) { RF_LAUNCH_VAR(float, true) } else { RF_LAUNCH_VAR(float, false) }
  }
#undef RF_LAUNCH_VAR
  return hipGetLastError();
}

}  // namespace rf
