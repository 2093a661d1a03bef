// Merge of partial (m, l, acc) states: the level-k fused expression of the
// attention cascade (paper Section 3.2 Eq. (11); Appendix A.2 level-k form)
//   m = max_c m_c;  l = sum_c l_c exp(m_c - m);  O = sum_c acc_c exp(m_c - m) / l
// One workgroup per output row.  Thread (sg, c) accumulates a float4 column c
// of acc over the chunks s = sg, sg + G, ...; the G partial sums are added
// through LDS.  Every partial-state byte is read once, with 128-bit loads.
#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

constexpr int kMergeThreads = 256;

constexpr int kPre = 8;  // acc loads a thread can issue before it knows the weights

template <bool OUT_BF16, bool PREFETCHED>
__global__ __launch_bounds__(kMergeThreads) void merge_states_kernel(
    const float* __restrict__ part_m, const float* __restrict__ part_l,
    const float* __restrict__ part_acc, void* __restrict__ o, int Hq, int Lq, int S, int d,
    int ncol_p2, Strides4 so) {
  __shared__ float s_red[kMergeThreads / kWave];
  __shared__ float s_red2[kMergeThreads / kWave];
  __shared__ f32x4 s_part[kMergeThreads];

  const int64_t row = blockIdx.x;
  const int i = (int)(row % Lq);
  const int h = (int)((row / Lq) % Hq);
  const int b = (int)(row / ((int64_t)Lq * Hq));
  const float* pm = part_m + row * S;
  const float* pl = part_l + row * S;
  const float* pa = part_acc + row * (int64_t)S * d;
  const int tid = threadIdx.x;

  // The acc loads do not depend on the weights: when a thread has at most kPre
  // chunks, issue them all now so that the whole kernel pays one memory latency.
  f32x4 pre[kPre];
  if (PREFETCHED) {
    const int G0 = kMergeThreads / ncol_p2;
    const int c0 = tid % ncol_p2, sg0 = tid / ncol_p2;
    if (c0 < d / 4) {
#pragma unroll
      for (int i = 0; i < kPre; ++i) {
        const int s = sg0 + i * G0;
        pre[i] = (s < S) ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(pa + (int64_t)s * d + 4 * c0))
                         : f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
  }

  // m = max over chunks
  float m = -INFINITY;
  for (int s = tid; s < S; s += kMergeThreads) m = fmaxf(m, pm[s]);
  m = wave_max(m);
  if ((tid & 63) == 0) s_red[tid >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  const float m_use = (m == -INFINITY) ? 0.f : m;
  // l = sum over chunks of l_c exp(m_c - m)
  float l = 0.f;
  for (int s = tid; s < S; s += kMergeThreads) {
    const float mc = pm[s];
    if (mc != -INFINITY) l += pl[s] * fast_exp2((mc - m_use) * kLog2e);
  }
  l = wave_sum(l);
  if ((tid & 63) == 0) s_red2[tid >> 6] = l;
  __syncthreads();
  l = (s_red2[0] + s_red2[1]) + (s_red2[2] + s_red2[3]);
  const float inv = l > 0.f ? 1.0f / l : 0.f;

  // O = sum over chunks of acc_c exp(m_c - m) / l
  const int ncol = d / 4;
  const int G = kMergeThreads / ncol_p2;  // chunk groups
  const int c = tid % ncol_p2;
  const int sg = tid / ncol_p2;
  f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
  if (c < ncol) {
    if (PREFETCHED) {
      // (the kPre loads of this thread were issued at kernel entry)
#pragma unroll
      for (int i = 0; i < kPre; ++i) {
        const int s = sg + i * G;
        if (s < S) {
          const float mc = pm[s];
          const float w = (mc == -INFINITY) ? 0.f : fast_exp2((mc - m_use) * kLog2e);
          sum += ((mc == -INFINITY) ? f32x4{0.f, 0.f, 0.f, 0.f} : pre[i]) * w;
        }
      }
    } else {
      for (int s = sg; s < S; s += G) {
        const float mc = pm[s];
        if (mc == -INFINITY) continue;
        const float w = fast_exp2((mc - m_use) * kLog2e);
        const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(pa + (int64_t)s * d + 4 * c));
        sum += a * w;
      }
    }
  }
  s_part[tid] = sum;
  __syncthreads();
  if (sg == 0 && c < ncol) {
    for (int gq = 1; gq < G; ++gq) sum += s_part[gq * ncol_p2 + c];
    sum *= inv;
    const int64_t off = (int64_t)b * so.b + (int64_t)h * so.h + (int64_t)i * so.l + 4 * c;
    if (OUT_BF16) {
      u32x2 r;
      r[0] = pack_bf16(sum[0], sum[1]);
      r[1] = pack_bf16(sum[2], sum[3]);
      *reinterpret_cast<u32x2*>(reinterpret_cast<bf16_t*>(o) + off) = r;
    } else {
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(o) + off) = sum;
    }
  }
}

hipError_t launch_merge_states(const float* part_m, const float* part_l, const float* part_acc,
                               void* o, bool o_is_bf16, int B, int Hq, int Lq, int S, int d,
                               Strides4 so, hipStream_t s) {
  const int64_t rows = (int64_t)B * Hq * Lq;
  if (rows > INT32_MAX) return hipErrorInvalidValue;
  const int ncol = d / 4;
  int p2 = 1;
  while (p2 < ncol) p2 <<= 1;
  if (p2 > kMergeThreads) return hipErrorInvalidValue;
  const bool pre = S <= kPre * (kMergeThreads / p2);
#define RF_MERGE_LAUNCH(B16, PRE)                                                                  \
  hipLaunchKernelGGL((merge_states_kernel<B16, PRE>), dim3((unsigned)rows), dim3(kMergeThreads), 0, \
                     s, part_m, part_l, part_acc, o, Hq, Lq, S, d, p2, so)
  if (o_is_bf16) { if (pre) RF_MERGE_LAUNCH(true, true); else RF_MERGE_LAUNCH(true, false); }
  else { if (pre) RF_MERGE_LAUNCH(false, true); else RF_MERGE_LAUNCH(false, false); }
#undef RF_MERGE_LAUNCH
  return hipGetLastError();
}

}  // namespace rf
