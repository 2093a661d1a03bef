// Multi-segment strategy for long-context decode (paper Section 4.3; partial
// kernel of Appendix A.4): the key axis is cut into S chunks, one workgroup
// per (batch, KV head, chunk).  All query rows that share the KV head (the
// Hq/Hkv grouped heads times Lq) ride in one 16-column MFMA tile, so every
// K/V byte is fetched from HBM once for the whole group.
//
// Inside a workgroup the chunk is split again over 4 wavefronts by
// interleaved 32-key tiles; each wavefront carries the running (m, l, acc) of
// the max -> sum-exp -> weighted-sum cascade (Appendix A.2 incremental form),
// the four states are merged through LDS with the level-k fused expression
// (Section 3.2 Eq. (11)) and the chunk's UNNORMALISED state is written out.
//
// Data movement (K and V are read once: non-temporal loads, which stream measurably
// faster than cached ones).  K: coalesced 128-bit global loads -> wavefront-private,
// XOR-swizzled LDS tile -> 128-bit LDS reads in MFMA A-operand layout.
// V: 128-bit global loads of whole rows straight into registers, followed by
// an 8x8 16-bit register transpose that yields the A operand of
// O^T = V^T P^T.  Scores are computed transposed (S^T = K Q^T) so that the
// probabilities are already in B-operand layout.
#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

namespace {

constexpr int kSplitWaves = 4;
constexpr int kD = 128;                  // head dim of this kernel
constexpr int kTileKeys = 32;            // keys per wavefront step
constexpr int kRowBytes = kD * 2;        // one K/V row
constexpr int kKTileBytes = kTileKeys * kRowBytes;  // 8 KB per wavefront

// low halves / high halves of two packed bf16 pairs
__device__ __forceinline__ uint32_t pair_lo(uint32_t x, uint32_t y) {
  return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ uint32_t pair_hi(uint32_t x, uint32_t y) {
  return __builtin_amdgcn_perm(y, x, 0x07060302u);
}

}  // namespace

// Two workgroups per compute unit: bounding the registers for three was measured 1.4 % slower
// (back-to-back launches, same process) although it hides a workgroup's prologue and epilogue.
__global__ __launch_bounds__(kSplitWaves * kWave, 2) void attention_splitk_bf16_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    Strides4 sq, Strides4 sk, Strides4 sv, float* __restrict__ part_m,
    float* __restrict__ part_l, float* __restrict__ part_acc, int Hq, int Hkv, int Lq, int Lk,
    int S, int chunk, float scale_log2e, int causal) {
  // K staging (4 x 8 KB) and the cross-wavefront merge buffers share this space.
  constexpr int kAccPitch = kD + 4;
  constexpr int kMergeFloats = kSplitWaves * 16 * kAccPitch + 2 * kSplitWaves * 16;
  constexpr int kSmemBytes =
      (kMergeFloats * 4 > kSplitWaves * kKTileBytes) ? kMergeFloats * 4 : kSplitWaves * kKTileBytes;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kSmemBytes];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int i16 = lane & 15;
  const int g = lane >> 4;

  const int c = blockIdx.x % S;
  const int hk = (blockIdx.x / S) % Hkv;
  const int b = blockIdx.x / (S * Hkv);
  const int grp = Hq / Hkv;
  const int R = grp * Lq;  // query rows sharing this KV head

  const int lo = min(Lk, c * chunk);
  const int hi = min(Lk, lo + chunk);
  const int shift = Lk - Lq;

  const bf16_t* kb = k + (int64_t)b * sk.b + (int64_t)hk * sk.h;
  const bf16_t* vb = v + (int64_t)b * sv.b + (int64_t)hk * sv.h;
  unsigned char* ktile = smem + wave * kKTileBytes;

  for (int r0 = 0; r0 < R; r0 += 16) {
    // this lane's query row (column of the transposed score tile)
    const int r = r0 + i16;
    const bool row_ok = r < R;
    const int h = hk * grp + (row_ok ? r / Lq : 0);
    const int iq = row_ok ? r % Lq : 0;
    const int my_last = row_ok ? (causal ? min(hi - 1, iq + shift) : hi - 1) : -1;

    // Q^T fragments: contraction slot (g, e) of step kb stands for d = 32kb + 8g + e
    u32x4 qf[4];
    {
      const bf16_t* qp = q + (int64_t)b * sq.b + (int64_t)h * sq.h + (int64_t)iq * sq.l + 8 * g;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        qf[kk] = row_ok ? *reinterpret_cast<const u32x4*>(qp + 32 * kk) : u32x4{0u, 0u, 0u, 0u};
    }

    float m2 = -INFINITY, l = 0.f;
    f32x4 acc[8];  // acc[t][rr] = O[row i16][d = 32g + 8rr + t]
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // K of a step is fetched one step ahead (two register sets) and V at the start of its
    // step: K is needed first (it goes through LDS before the first MFMA), V only after the
    // scores and the softmax, which cover its latency.  Two full sets do not fit the registers.
    // slot e of kreg: key row 4e + g; slot e of vreg: key 4g + e (e < 4), 16 + 4g + (e - 4).
    // Full tiles: wave-uniform tile base (scalar registers) + loop-invariant 32-bit lane offsets.
    uint32_t koff[8], voff[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      koff[e] = (uint32_t)(((int64_t)(4 * e + g) * sk.l + 8 * i16) * 2);
      voff[e] = (uint32_t)(((int64_t)((e < 4) ? (4 * g + e) : (16 + 4 * g + (e - 4))) * sv.l + 8 * i16) * 2);
    }
    const bool small_stride = sk.l < (1 << 24) && sv.l < (1 << 24);  // offsets fit 32 bits
    auto issue_k = [&](int key0_, u32x4 (&kreg)[8]) {
      const int key0 = __builtin_amdgcn_readfirstlane(key0_);
      if (key0 + kTileKeys <= Lk && small_stride) {
        const char* kt = reinterpret_cast<const char*>(kb) + (int64_t)key0 * sk.l * 2;
#pragma unroll
        for (int e = 0; e < 8; ++e)
          kreg[e] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kt + koff[e]));
      } else {  // ragged last tile: rows past the end re-read the last key (masked later)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int key = min(key0 + 4 * e + g, Lk - 1);
          kreg[e] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + (int64_t)key * sk.l + 8 * i16));
        }
      }
    };
    auto issue_v = [&](int key0_, u32x4 (&vreg)[8]) {
      const int key0 = __builtin_amdgcn_readfirstlane(key0_);
      if (key0 + kTileKeys <= Lk && small_stride) {
        const char* vt = reinterpret_cast<const char*>(vb) + (int64_t)key0 * sv.l * 2;
#pragma unroll
        for (int e = 0; e < 8; ++e)
          vreg[e] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vt + voff[e]));
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int key = min(key0 + ((e < 4) ? (4 * g + e) : (16 + 4 * g + (e - 4))), Lk - 1);
          vreg[e] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vb + (int64_t)key * sv.l + 8 * i16));
        }
      }
    };
    auto tile_step = [&](int key0, u32x4 (&kreg)[8], u32x4 (&vreg)[8]) {
      // ---- K tile: registers -> LDS (swizzled) ----
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = 4 * e + g;
        *reinterpret_cast<u32x4*>(ktile + row * kRowBytes + ((i16 ^ (row & 15)) << 4)) = kreg[e];
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

      // ---- S^T = K Q^T for the two 16-key halves ----
      f32x4 sA = f32x4{0.f, 0.f, 0.f, 0.f}, sB = sA;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int piece = 4 * kk + g;
        const u32x4 ka =
            *reinterpret_cast<const u32x4*>(ktile + i16 * kRowBytes + ((piece ^ i16) << 4));
        const u32x4 kbv = *reinterpret_cast<const u32x4*>(ktile + (16 + i16) * kRowBytes +
                                                          ((piece ^ i16) << 4));
        sA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka),
                                                     __builtin_bit_cast(bf16x8, qf[kk]), sA, 0, 0, 0);
        sB = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kbv),
                                                     __builtin_bit_cast(bf16x8, qf[kk]), sB, 0, 0, 0);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();

      // ---- stage 1: running max ----
      float sc[8];
      float tmax = -INFINITY;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int key = key0 + ((e < 4) ? (4 * g + e) : (16 + 4 * g + (e - 4)));
        const float sv_ = (e < 4) ? sA[e] : sB[e - 4];
        sc[e] = (key <= my_last) ? sv_ * scale_log2e : -INFINITY;
        tmax = fmaxf(tmax, sc[e]);
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m2, tmax);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float corr = fast_exp2(m2 - m_use);
      m2 = m_new;
      // ---- stage 2: running sum of exponentials ----
      float p[8];
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = fast_exp2(sc[e] - m_use);
        psum += p[e];
      }
      l = l * corr + psum;
      u32x4 pb;
#pragma unroll
      for (int e = 0; e < 4; ++e) pb[e] = pack_bf16(p[2 * e], p[2 * e + 1]);

      // ---- stage 3: acc = acc * corr + V^T P^T ----
#pragma unroll
      for (int t = 0; t < 8; ++t) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) acc[t][rr] *= corr;
      }
      // 8x8 transpose of 16-bit elements: vt[t] holds, for d = 8*i16 + t, the 8 slots e
#pragma unroll
      for (int tp = 0; tp < 4; ++tp) {
        u32x4 lo4, hi4;
#pragma unroll
        for (int ep = 0; ep < 4; ++ep) {
          lo4[ep] = pair_lo(vreg[2 * ep][tp], vreg[2 * ep + 1][tp]);
          hi4[ep] = pair_hi(vreg[2 * ep][tp], vreg[2 * ep + 1][tp]);
        }
        acc[2 * tp] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, lo4), __builtin_bit_cast(bf16x8, pb), acc[2 * tp], 0, 0, 0);
        acc[2 * tp + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, hi4), __builtin_bit_cast(bf16x8, pb), acc[2 * tp + 1], 0, 0,
            0);
      }
    };

    constexpr int kStride = kSplitWaves * kTileKeys;
    u32x4 kA[8], kB[8], vv[8];
    int key0 = lo + wave * kTileKeys;
    if (key0 < hi) issue_k(key0, kA);
    while (key0 < hi) {
      const int key1 = key0 + kStride;
      issue_v(key0, vv);
      if (key1 < hi) issue_k(key1, kB);
      tile_step(key0, kA, vv);
      if (key1 >= hi) break;
      const int key2 = key1 + kStride;
      issue_v(key1, vv);
      if (key2 < hi) issue_k(key2, kA);
      tile_step(key1, kB, vv);
      key0 = key2;
    }

    // ---- merge the four wavefront states, write the chunk state ----
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    __syncthreads();  // K staging is dead from here on
    float* s_acc = reinterpret_cast<float*>(smem);
    float* s_m = s_acc + kSplitWaves * 16 * kAccPitch;
    float* s_l = s_m + kSplitWaves * 16;
    if (g == 0) { s_m[wave * 16 + i16] = m2; s_l[wave * 16 + i16] = l; }
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      float* dst = s_acc + (wave * 16 + i16) * kAccPitch + 32 * g + 8 * rr;
      *reinterpret_cast<f32x4*>(dst) = f32x4{acc[0][rr], acc[1][rr], acc[2][rr], acc[3][rr]};
      *reinterpret_cast<f32x4*>(dst + 4) = f32x4{acc[4][rr], acc[5][rr], acc[6][rr], acc[7][rr]};
    }
    __syncthreads();
    const int rows_here = min(16, R - r0);
    for (int idx = threadIdx.x; idx < rows_here * (kD / 4); idx += kSplitWaves * kWave) {
      const int rr = idx / (kD / 4);
      const int c4 = idx % (kD / 4);
      float mg = -INFINITY;
#pragma unroll
      for (int w = 0; w < kSplitWaves; ++w) mg = fmaxf(mg, s_m[w * 16 + rr]);
      const float mg_use = (mg == -INFINITY) ? 0.f : mg;
      float lg = 0.f;
      f32x4 og = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < kSplitWaves; ++w) {
        const float mw = s_m[w * 16 + rr];
        const float wgt = (mw == -INFINITY) ? 0.f : fast_exp2(mw - mg_use);
        lg += s_l[w * 16 + rr] * wgt;
        og += *reinterpret_cast<const f32x4*>(s_acc + (w * 16 + rr) * kAccPitch + 4 * c4) * wgt;
      }
      const int rq = r0 + rr;
      const int hh = hk * grp + rq / Lq;
      const int ii = rq % Lq;
      const int64_t prow = (((int64_t)b * Hq + hh) * Lq + ii) * S + c;
      // Non-temporal stores: ordinary ones, left in L2 among the streaming K/V reads, cost the
      // launch 6 % (342 against 323 us on B16 Hkv8 Lk32768 S64; without any store of the state it
      // runs in 311 us).
      __builtin_nontemporal_store(og, reinterpret_cast<f32x4*>(part_acc + prow * kD + 4 * c4));
      if (c4 == 0) {
        part_m[prow] = mg * 0.6931471805599453f;  // back to natural-log units
        part_l[prow] = lg;
      }
    }
    __syncthreads();  // merge buffers are reused as K staging by the next row tile
  }
}

hipError_t launch_attention_splitk_bf16(const void* q, const void* k, const void* v, Strides4 sq,
                                        Strides4 sk, Strides4 sv, int num_splits, float* part_m,
                                        float* part_l, float* part_acc, const AttnShape& a,
                                        hipStream_t s) {
  if (a.d != kD) return hipErrorInvalidValue;
  const int64_t grid = (int64_t)a.B * a.Hkv * num_splits;
  if (grid > INT32_MAX) return hipErrorInvalidValue;
  const int chunk = (a.Lk + num_splits - 1) / num_splits;
  hipLaunchKernelGGL(attention_splitk_bf16_kernel, dim3((unsigned)grid),
                     dim3(kSplitWaves * kWave), 0, s, (const bf16_t*)q, (const bf16_t*)k,
                     (const bf16_t*)v, sq, sk, sv, part_m, part_l, part_acc, a.Hq, a.Hkv, a.Lq,
                     a.Lk, num_splits, chunk, a.scale * kLog2e, a.causal);
  return hipGetLastError();
}

}  // namespace rf
