// fp32 fused attention, single-segment strategy (paper Section 4.3; Appendix
// A.2 incremental forms), full-precision fp32 MFMA (16x16x4).
//
// One workgroup owns 16 query rows of one (batch, head).  Its NW wavefronts
// split the key axis by interleaved 16-key tiles; each wavefront streams its
// tiles carrying the running state (m, l, acc) of the max -> sum-exp ->
// weighted-sum cascade and rescales it as each tile arrives.  The NW states
// are then merged through LDS with the level-k fused expression (Section 3.2
// Eq. (11)); acc is divided by l once, in that merge.
//
// The score tile is computed transposed, S^T = K Q^T, so that the MFMA
// accumulator layout (lane = query column, registers = key rows) is already
// the B-operand layout of the second product O^T = V^T P^T: the probabilities
// never leave their registers.
#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

template <int D, int NW>
__global__ __launch_bounds__(NW * kWave) void attention_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v,
    float* __restrict__ o, Strides4 sq, Strides4 sk, Strides4 sv, Strides4 so, int Hq, int Hkv,
    int Lq, int Lk, float scale_log2e, int causal, int n_qtiles) {
  constexpr int DJ = D / 16;  // 16-wide slices of the head dim
  __shared__ float s_m[NW][16];
  __shared__ float s_l[NW][16];
  __shared__ float s_acc[NW][16][D + 4];

  // (every argument is named here so that the compiler fetches the whole argument block with its
  // first scalar loads and waits for it once: fetched where first used, the block came in three
  // round trips, each behind the wait for the previous one)
  // (n_qtiles passes through the statement: the index arithmetic below depends on it and so
  // cannot be scheduled ahead of it)
  asm volatile("" : "+s"(n_qtiles) : "s"(q), "s"(k), "s"(v), "s"(o), "s"(sq.b), "s"(sq.h), "s"(sq.l), "s"(sk.b),
               "s"(sk.h), "s"(sk.l), "s"(sv.b), "s"(sv.h), "s"(sv.l), "s"(so.b), "s"(so.h), "s"(so.l),
               "s"(Hq), "s"(Hkv), "s"(Lq), "s"(Lk), "s"(scale_log2e), "s"(causal));
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int i16 = lane & 15;  // query column / key row / head-dim row inside a tile
  const int g = lane >> 4;    // lane group 0..3

  // (integer division runs on the vector unit even for wave-uniform operands: the results are
  // handed back to the scalar unit, so that the base pointers below are scalar)
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Numbered so that XCD x
  // takes a run of consecutive (head, query tile) pairs, the query tiles of one head read its K
  // and V through one L2 instead of eight (batched fp32 launch, 512 heads of 128 x 512 x 64:
  // 1.09 GB fetched from the fabric before, against 0.15 GB of inputs).
  int wg = blockIdx.x;
  if ((gridDim.x & 7) == 0) wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  const int qt = __builtin_amdgcn_readfirstlane(wg % n_qtiles);
  const int bh = __builtin_amdgcn_readfirstlane(wg / n_qtiles);
  const int h = __builtin_amdgcn_readfirstlane(bh % Hq);
  const int b = __builtin_amdgcn_readfirstlane(bh / Hq);
  const int hk = __builtin_amdgcn_readfirstlane(h / (Hq / Hkv));
  const int q0 = qt * 16;

  const float* qb = q + (int64_t)b * sq.b + (int64_t)h * sq.h;
  const float* kb = k + (int64_t)b * sk.b + (int64_t)hk * sk.h;
  const float* vb = v + (int64_t)b * sv.b + (int64_t)hk * sv.h;
  // At the sizes this kernel serves, the run time is a chain of memory latencies.  All kernel
  // arguments are therefore fetched in one go (the K/V base pointers are formed here, ahead of
  // the first load, instead of behind the wait for Q), and Q is read without branches, so
  // that its loads are only waited for at the first product, with the first K/V group already
  // on its way.
  asm volatile("" : : "s"(kb), "s"(vb));

  // Q^T fragments.  Contraction slot (g, e) of step j stands for head-dim index
  // 16j + 4g + e on both operands.
  f32x4 qf[DJ];
  {
    // (rows past the end repeat the last query: their results are computed and never stored)
    const int qi = min(q0 + i16, Lq - 1);
#pragma unroll
    for (int j = 0; j < DJ; ++j)
      qf[j] = *reinterpret_cast<const f32x4*>(qb + (int64_t)qi * sq.l + 16 * j + 4 * g);
  }

  // last visible key of this lane's query, and of the whole query tile
  const int shift = Lk - Lq;
  const int my_q = q0 + i16;
  const int my_last = causal ? min(Lk - 1, my_q + shift) : Lk - 1;
  const int tile_last = causal ? min(Lk - 1, min(Lq - 1, q0 + 15) + shift) : Lk - 1;
  const int n_ktiles = tile_last >= 0 ? tile_last / 16 + 1 : 0;

  float m2 = -INFINITY;  // running max, in log2 units (score * scale * log2 e)
  float l = 0.f;         // running sum, this lane's keys only
  // Row i of the t-th O^T tile stands for head-dim index DJ * i + t (not 16 t + i): the DJ
  // A-operand values a lane needs for one key are then DJ consecutive floats of the V row,
  // fetched with 128-bit loads, and one load instruction reads whole 64 DJ-byte row pieces.
  f32x4 acc[DJ];         // acc[t][r] = O^T[head-dim DJ * (4g + r) + t][query i16]
#pragma unroll
  for (int t = 0; t < DJ; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // A wavefront's tiles are taken TG at a time: all K and V fragments of the group are
  // requested before the first product, so memory latency is paid once per group, not twice
  // per tile (at the small sizes this kernel serves, that latency is most of the run time).
  constexpr int TG = (D == 64 && NW <= 8) ? 4 : 2;
  const bool small_pitch = sk.l < (1 << 26) && sv.l < (1 << 26);  // 32-bit byte offsets inside a 16-key tile
  const uint32_t k_lane = (uint32_t)(((int64_t)i16 * sk.l + 4 * g) * 4);
  const uint32_t v_lane = (uint32_t)(((int64_t)(4 * g) * sv.l + DJ * i16) * 4);
  for (int kt0 = wave; kt0 < n_ktiles; kt0 += NW * TG) {
    f32x4 kf[TG][DJ];
    f32x4 vf[TG][4][DJ / 4];  // vf[.][u][c][e] = V[key of step u][DJ * i16 + 4c + e]
#pragma unroll
    for (int jj = 0; jj < TG; ++jj) {
      const int key0 = min(kt0 + NW * jj, n_ktiles - 1) * 16;  // (a surplus slot re-reads the last tile)
      if (key0 + 16 <= Lk && small_pitch) {
        // whole tile: a wavefront-uniform base (scalar unit) plus loop-invariant 32-bit lane
        // offsets, no per-lane 64-bit address arithmetic (which is most of this kernel's set-up)
        const char* kbase = reinterpret_cast<const char*>(kb) + (int64_t)key0 * sk.l * 4;
#pragma unroll
        for (int j = 0; j < DJ; ++j)
          kf[jj][j] = *reinterpret_cast<const f32x4*>(kbase + k_lane + 64 * j);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          // contraction slot g of step u stands for key key0 + 4g + u
          const char* vbase = reinterpret_cast<const char*>(vb) + (int64_t)(key0 + u) * sv.l * 4;
#pragma unroll
          for (int c = 0; c < DJ / 4; ++c)
            vf[jj][u][c] = *reinterpret_cast<const f32x4*>(vbase + v_lane + 16 * c);
        }
      } else {
        const float* kp = kb + (int64_t)min(key0 + i16, Lk - 1) * sk.l + 4 * g;
#pragma unroll
        for (int j = 0; j < DJ; ++j) kf[jj][j] = *reinterpret_cast<const f32x4*>(kp + 16 * j);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float* vp = vb + (int64_t)min(key0 + 4 * g + u, Lk - 1) * sv.l + DJ * i16;
#pragma unroll
          for (int c = 0; c < DJ / 4; ++c) vf[jj][u][c] = *reinterpret_cast<const f32x4*>(vp + 4 * c);
        }
      }
    }
#pragma unroll
    for (int jj = 0; jj < TG; ++jj) {
      const int kt = kt0 + NW * jj;
      if (kt >= n_ktiles) break;  // uniform per wavefront
      const int key0 = kt * 16;
      // ---- S^T tile = K_tile Q^T (fp32 MFMA), as two independent accumulation chains ----
      f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f}, s_b = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < DJ; j += 2) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          s = __builtin_amdgcn_mfma_f32_16x16x4f32(kf[jj][j][e], qf[j][e], s, 0, 0, 0);
          s_b = __builtin_amdgcn_mfma_f32_16x16x4f32(kf[jj][j + 1][e], qf[j + 1][e], s_b, 0, 0, 0);
        }
      }
      s += s_b;
      // s[r] = score(key key0 + 4g + r, query i16); mask, then stage 1: running max
      float tmax = -INFINITY;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int key = key0 + 4 * g + r;
        s[r] = (key <= my_last) ? s[r] * scale_log2e : -INFINITY;
        tmax = fmaxf(tmax, s[r]);
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m2, tmax);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;  // identity repair
      const float corr = fast_exp2(m2 - m_use);                // 0 when m2 == -inf
      m2 = m_new;
      // stage 2: running sum of exponentials
      float p[4];
      float psum = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        p[r] = fast_exp2(s[r] - m_use);
        psum += p[r];
      }
      l = l * corr + psum;
      // stage 3: rescale acc, then acc += V^T P^T
#pragma unroll
      for (int t = 0; t < DJ; ++t) {
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] *= corr;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int t = 0; t < DJ; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(vf[jj][u][t / 4][t % 4], p[u], acc[t], 0, 0, 0);
      }
    }
  }

  // ---- merge the NW wavefront states (level-k fused expression) ----
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);
  if (g == 0) { s_m[wave][i16] = m2; s_l[wave][i16] = l; }
#pragma unroll
  for (int t = 0; t < DJ; ++t) {
#pragma unroll
    for (int r = 0; r < 4; ++r) s_acc[wave][i16][DJ * (4 * g + r) + t] = acc[t][r];
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 16 * (D / 4); idx += NW * kWave) {
    const int qi = idx / (D / 4);
    const int c4 = idx % (D / 4);
    float mg = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mg = fmaxf(mg, s_m[w][qi]);
    float lg = 0.f;
    f32x4 og = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float mw = s_m[w][qi];
      const float wgt = (mw == -INFINITY) ? 0.f : fast_exp2(mw - mg);
      lg += s_l[w][qi] * wgt;
      const f32x4 a = *reinterpret_cast<const f32x4*>(&s_acc[w][qi][4 * c4]);
      og += a * wgt;
    }
    const float inv = lg > 0.f ? 1.0f / lg : 0.f;
    if (q0 + qi < Lq) {
      float* op = o + (int64_t)b * so.b + (int64_t)h * so.h + (int64_t)(q0 + qi) * so.l + 4 * c4;
      *reinterpret_cast<f32x4*>(op) = og * inv;
    }
  }
}

hipError_t launch_attention_f32(const float* q, const float* k, const float* v, float* o,
                                Strides4 sq, Strides4 sk, Strides4 sv, Strides4 so,
                                const AttnShape& a, hipStream_t s) {
  const int n_qtiles = (a.Lq + 15) / 16;
  const int64_t grid = (int64_t)n_qtiles * a.B * a.Hq;
  if (grid > INT32_MAX) return hipErrorInvalidValue;
  const float sl2 = a.scale * kLog2e;
  if (a.d == 64 && grid < 256 && a.Lk > 128) {
    // few workgroups and many keys: 16 wavefronts share the key axis of a query tile
    hipLaunchKernelGGL((attention_f32_kernel<64, 16>), dim3((unsigned)grid), dim3(16 * kWave), 0, s,
                       q, k, v, o, sq, sk, sv, so, a.Hq, a.Hkv, a.Lq, a.Lk, sl2, a.causal,
                       n_qtiles);
  } else if (a.d == 64) {
    hipLaunchKernelGGL((attention_f32_kernel<64, 8>), dim3((unsigned)grid), dim3(8 * kWave), 0, s,
                       q, k, v, o, sq, sk, sv, so, a.Hq, a.Hkv, a.Lq, a.Lk, sl2, a.causal,
                       n_qtiles);
  } else {
    hipLaunchKernelGGL((attention_f32_kernel<128, 4>), dim3((unsigned)grid), dim3(4 * kWave), 0, s,
                       q, k, v, o, sq, sk, sv, so, a.Hq, a.Hkv, a.Lq, a.Lk, sl2, a.causal,
                       n_qtiles);
  }
  return hipGetLastError();
}

}  // namespace rf
