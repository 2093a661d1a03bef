// bf16 fused attention, single-segment strategy (paper Section 4.3; Appendix
// A.2 incremental forms; Appendix A.4 tile-level structure), bf16 MFMA
// 32x32x16 with fp32 accumulation.
//
// One workgroup (4 wavefronts) owns 128 query rows of one (batch, head); each
// wavefront owns 32 of them as the N dimension of its MFMA tiles and streams
// the keys in tiles of 64, carrying the running state (m, l, acc) of the
// max -> sum-exp -> weighted-sum cascade.  acc stays unnormalised (Eq. (8))
// and is divided by l once in the epilogue.
//
//   S^T = K Q^T        A = K tile (LDS, XOR-swizzled rows), B = Q^T (registers)
//   O^T += V^T P^T     A = V^T tile (LDS, transposed while staging), B = P^T
//
// Computing the scores transposed makes the accumulator layout of S^T (lane =
// query column, registers = key rows) coincide with the B-operand layout of
// the second product, so probabilities go from fp32 accumulators to bf16
// operands without leaving their lane.  The key order inside each 16-key group
// is permuted identically on both operands of the second product (a sum over
// keys does not care), which lets each lane fetch its eight keys of V^T with a
// single 128-bit LDS read.
#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * kWave;
constexpr int kBQ = 128;  // query rows per workgroup
constexpr int kBK = 64;   // keys per tile

__device__ __forceinline__ uint32_t pair_lo(uint32_t x, uint32_t y) {
  return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ uint32_t pair_hi(uint32_t x, uint32_t y) {
  return __builtin_amdgcn_perm(y, x, 0x07060302u);
}

// K tile in LDS: row = key (D bf16), 16-byte pieces XOR-swizzled by row.
template <int D>
__device__ __forceinline__ int k_lds_off(int row, int piece) {
  constexpr int P = D / 8;  // pieces per row
  const int f = (P == 16) ? (row & 15) : ((row >> 1) & 7);
  return row * (D * 2) + (((piece ^ f) & (P - 1)) << 4);
}
// V^T tile in LDS: row = head-dim index (64 key slots, 128 bytes), 16-byte
// granules XOR-swizzled by row.  Slot order inside a 16-key group: bits 2 and 3
// of the key index are swapped.
__device__ __forceinline__ int vt_lds_off(int d, int granule) {
  const int f = ((d >> 1) ^ (d >> 4)) & 7;
  return d * (kBK * 2) + ((granule ^ f) << 4);
}

}  // namespace

template <int D>
__global__ __launch_bounds__(kThreads) void attention_bf16_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    bf16_t* __restrict__ o, Strides4 sq, Strides4 sk, Strides4 sv, Strides4 so, int Hq, int Hkv,
    int Lq, int Lk, float scale_log2e, int causal, int n_qtiles) {
  constexpr int KS = D / 16;   // contraction steps of S^T = K Q^T
  constexpr int DT = D / 32;   // 32-row tiles of O^T
  constexpr int P = D / 8;     // 16-byte pieces per K/V row
  constexpr int KLD = kBK * P / kThreads;       // K loads per thread per tile
  constexpr int VROWS = 4;                      // keys per thread in the V transpose
  constexpr int NVB = (kBK / VROWS) * P;        // 4-key x 8-column V blocks per tile
  constexpr int VBLK = (NVB + kThreads - 1) / kThreads;  // V blocks per thread per tile

  __shared__ __attribute__((aligned(16))) unsigned char k_lds[kBK * D * 2];
  __shared__ __attribute__((aligned(16))) unsigned char vt_lds[D * kBK * 2];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int i32 = lane & 31;
  const int hh = lane >> 5;

  // heavy (late) query tiles first: under a causal mask they have the most keys
  const int qt = n_qtiles - 1 - (int)(blockIdx.x % n_qtiles);
  const int bh = blockIdx.x / n_qtiles;
  const int h = bh % Hq;
  const int b = bh / Hq;
  const int hk = h / (Hq / Hkv);
  const int q0 = qt * kBQ;

  const bf16_t* qb = q + (int64_t)b * sq.b + (int64_t)h * sq.h;
  const bf16_t* kb = k + (int64_t)b * sk.b + (int64_t)hk * sk.h;
  const bf16_t* vb = v + (int64_t)b * sv.b + (int64_t)hk * sv.h;

  // Q^T fragments: slot (hh, e) of step kk stands for d = 16kk + 8hh + e
  const int my_q = q0 + wave * 32 + i32;
  u32x4 qf[KS];
  {
    const bf16_t* qp = qb + (int64_t)min(my_q, Lq - 1) * sq.l + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = *reinterpret_cast<const u32x4*>(qp + 16 * kk);
  }

  const int shift = Lk - Lq;
  const int my_last = causal ? min(Lk - 1, my_q + shift) : Lk - 1;
  const int wave_min_last = causal ? min(Lk - 1, q0 + wave * 32 + shift) : Lk - 1;
  const int wave_last = causal ? min(Lk - 1, min(Lq - 1, q0 + wave * 32 + 31) + shift) : Lk - 1;
  const int wg_last = causal ? min(Lk - 1, min(Lq - 1, q0 + kBQ - 1) + shift) : Lk - 1;
  const int n_ktiles = wg_last >= 0 ? wg_last / kBK + 1 : 0;

  float m2 = -INFINITY, l = 0.f;
  f32x16 acc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  // staging registers
  u32x4 kreg[KLD];
  u32x4 vreg[VBLK][VROWS];

  auto load_tile = [&](int key0) {
#pragma unroll
    for (int e = 0; e < KLD; ++e) {
      const int idx = e * kThreads + tid;
      const int row = idx / P, piece = idx % P;
      const int key = min(key0 + row, Lk - 1);
      kreg[e] = *reinterpret_cast<const u32x4*>(kb + (int64_t)key * sk.l + 8 * piece);
    }
#pragma unroll
    for (int e = 0; e < VBLK; ++e) {
      const int idx = e * kThreads + tid;
      if (idx >= NVB) break;
      const int jg = idx / P, piece = idx % P;  // jg: group of 4 consecutive keys
#pragma unroll
      for (int rr = 0; rr < VROWS; ++rr) {
        const int key = min(key0 + 4 * jg + rr, Lk - 1);
        vreg[e][rr] = *reinterpret_cast<const u32x4*>(vb + (int64_t)key * sv.l + 8 * piece);
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int e = 0; e < KLD; ++e) {
      const int idx = e * kThreads + tid;
      const int row = idx / P, piece = idx % P;
      *reinterpret_cast<u32x4*>(k_lds + k_lds_off<D>(row, piece)) = kreg[e];
    }
#pragma unroll
    for (int e = 0; e < VBLK; ++e) {
      const int idx = e * kThreads + tid;
      if (idx >= NVB) break;
      const int jg = idx / P, piece = idx % P;
      // slot of key 4jg + rr inside its 16-key group: swap bits 2 and 3
      const int slot0 = 16 * (jg >> 2) + 8 * (jg & 1) + 4 * ((jg >> 1) & 1);
      const int granule = slot0 >> 3;
      const int half = (slot0 >> 2) & 1;
#pragma unroll
      for (int tp = 0; tp < 4; ++tp) {
        // 4 keys x 2 head-dim columns -> two 8-byte rows of V^T
        u32x2 lo2, hi2;
        lo2[0] = pair_lo(vreg[e][0][tp], vreg[e][1][tp]);
        lo2[1] = pair_lo(vreg[e][2][tp], vreg[e][3][tp]);
        hi2[0] = pair_hi(vreg[e][0][tp], vreg[e][1][tp]);
        hi2[1] = pair_hi(vreg[e][2][tp], vreg[e][3][tp]);
        const int d0 = 8 * piece + 2 * tp;
        *reinterpret_cast<u32x2*>(vt_lds + vt_lds_off(d0, granule) + 8 * half) = lo2;
        *reinterpret_cast<u32x2*>(vt_lds + vt_lds_off(d0 + 1, granule) + 8 * half) = hi2;
      }
    }
  };

  if (n_ktiles > 0) load_tile(0);
  for (int kt = 0; kt < n_ktiles; ++kt) {
    const int key0 = kt * kBK;
    __syncthreads();  // previous tile's LDS reads are done
    store_tile();
    __syncthreads();
    if (kt + 1 < n_ktiles) load_tile(key0 + kBK);
    if (key0 > wave_last) continue;  // nothing visible for this wavefront (uniform)

    // ---- S^T = K Q^T : two 32-key row tiles ----
    f32x16 s[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[rt][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        const u32x4 a =
            *reinterpret_cast<const u32x4*>(k_lds + k_lds_off<D>(32 * rt + i32, 2 * kk + hh));
        s[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                        __builtin_bit_cast(bf16x8, qf[kk]), s[rt],
                                                        0, 0, 0);
      }
    }
    // s[rt][r] = score(key key0 + 32rt + 8(r/4) + 4hh + r%4, query my_q)
    const bool need_mask = key0 + kBK - 1 > wave_min_last;  // uniform per wavefront
    float tmax = -INFINITY;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float x = s[rt][r] * scale_log2e;
        if (need_mask) {
          const int key = key0 + 32 * rt + 8 * (r >> 2) + 4 * hh + (r & 3);
          x = (key <= my_last) ? x : -INFINITY;
        }
        s[rt][r] = x;
        tmax = fmaxf(tmax, x);
      }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    // ---- stage 1: running max; stage 2: running sum of exponentials ----
    const float m_new = fmaxf(m2, tmax);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float corr = fast_exp2(m2 - m_use);
    m2 = m_new;
    float psum = 0.f;
    u32x4 pb[4];  // B operands of the 4 contraction steps (16 keys each)
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r2 = 0; r2 < 8; ++r2) {
        const float p0 = fast_exp2(s[rt][2 * r2] - m_use);
        const float p1 = fast_exp2(s[rt][2 * r2 + 1] - m_use);
        psum += p0 + p1;
        pb[2 * rt + (r2 >> 2)][r2 & 3] = pack_bf16(p0, p1);
      }
    l = l * corr + psum;
    // ---- stage 3: acc = acc * corr + V^T P^T ----
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][r] *= corr;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
      for (int t = 0; t < DT; ++t) {
        const u32x4 a =
            *reinterpret_cast<const u32x4*>(vt_lds + vt_lds_off(32 * t + i32, 2 * u + hh));
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                         __builtin_bit_cast(bf16x8, pb[u]), acc[t],
                                                         0, 0, 0);
      }
    }
  }

  // ---- epilogue: O = acc / l ----
  l += __shfl_xor(l, 32, 64);
  const float inv = l > 0.f ? 1.0f / l : 0.f;
  if (my_q < Lq) {
    bf16_t* op = o + (int64_t)b * so.b + (int64_t)h * so.h + (int64_t)my_q * so.l;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        // acc[t][4r4 + j] = O[my_q][32t + 8r4 + 4hh + j]
        u32x2 w;
        w[0] = pack_bf16(acc[t][4 * r4] * inv, acc[t][4 * r4 + 1] * inv);
        w[1] = pack_bf16(acc[t][4 * r4 + 2] * inv, acc[t][4 * r4 + 3] * inv);
        *reinterpret_cast<u32x2*>(op + 32 * t + 8 * r4 + 4 * hh) = w;
      }
  }
}

hipError_t launch_attention_bf16(const void* q, const void* k, const void* v, void* o, Strides4 sq,
                                 Strides4 sk, Strides4 sv, Strides4 so, const AttnShape& a,
                                 hipStream_t s) {
  const int n_qtiles = (a.Lq + kBQ - 1) / kBQ;
  const int64_t grid = (int64_t)n_qtiles * a.B * a.Hq;
  if (grid > INT32_MAX) return hipErrorInvalidValue;
  const float sl2 = a.scale * kLog2e;
  if (a.d == 128) {
    hipLaunchKernelGGL((attention_bf16_kernel<128>), dim3((unsigned)grid), dim3(kThreads), 0, s,
                       (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, sq, sk, sv,
                       so, a.Hq, a.Hkv, a.Lq, a.Lk, sl2, a.causal, n_qtiles);
  } else if (a.d == 64) {
    hipLaunchKernelGGL((attention_bf16_kernel<64>), dim3((unsigned)grid), dim3(kThreads), 0, s,
                       (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, sq, sk, sv,
                       so, a.Hq, a.Hkv, a.Lq, a.Lk, sl2, a.causal, n_qtiles);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rf
