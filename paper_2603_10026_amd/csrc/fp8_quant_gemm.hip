// FP8 per-token quantisation fused with a GEMM (paper Section 3.4, case study):
//   stage 1: m_i   = max_k |a[i,k]|
//   stage 2: c[i,n] = sum_k q(MAX a[i,k] / m_i) w[n,k],   q = rounding to FP8 (OCP E4M3, MAX = 448)
// in the tile-wise incremental form: for every 128-wide tile of k
//   m_new = max(m_old, max_tile |a|);   acc = acc * (m_old / m_new) + q(MAX a_tile / m_new) w_tile
// Each tile is quantised with the running maximum that includes it; earlier tiles keep
// their codes and are only rescaled.  The result returned is acc * m / MAX, which
// approximates a @ w^T.  The weights arrive in FP8, as w[N,K] (row n = output channel n).
//
// Tiling.  One workgroup of 8 wavefronts owns a 128 (m) x 512 (n) output tile (128 x 256 when
// that tiling still fits the chip in one round of workgroups: shapes with few output tiles
// then occupy up to twice as many compute units) and walks K in steps of 128 (one barrier per
// step).  The product is computed transposed,
// C^T = W A_q^T, with v_mfma_f32_32x32x64_f8f6f4 (FP8 x FP8, fp32 accumulate), so each
// accumulator lane owns one token (one rescale factor per lane).
//   A operand = W rows: every wavefront streams ITS OWN 64 (or 32) output channels HBM -> LDS with
//               direct-to-LDS 128-bit loads into a private ring of three 64-k slots; no
//               other wavefront reads them, so no barrier guards them.
//   B operand = quantised tokens: a tile of `a` is loaded into registers, its maximum is
//               merged into the running maximum (4 lanes share a token), it is scaled,
//               rounded to FP8 with v_cvt_pk_fp8_f32 and written to LDS two steps before it
//               is multiplied (three stages); the rescale factor m_old / m_new travels with
//               the stage.
// With three token stages the one barrier of a step does not have to sit in front of the
// step's first LDS reads: it sits behind the first four MFMAs, and the fragments of a step's
// first weight tile are requested at the end of the step before, so no wavefront waits for
// LDS data right behind a barrier.
// The vector-ALU work of the quantisation is cut into half pieces placed behind the MFMAs.
// All waits are hand-placed; loads retire in order, which fixes the counts.
#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

namespace {

constexpr int kQWaves = 8;
constexpr int kQThreads = kQWaves * kWave;
constexpr int kQM = 128, kQK = 128;              // K step in elements = bytes of FP8
constexpr int kQXStageB = kQM * kQK;             // 16 KB: [m][k] bytes, 128-byte rows
constexpr int kQXStages = 3;                     // token tiles s, s+1 (being read) and s+2 (being written)
// A wavefront owns NI blocks of 32 output channels: the N tile of a workgroup is 256 NI wide.
template <int NI>
struct QLayout {
  static constexpr int kN = 256 * NI;
  static constexpr int kWaveN = 32 * NI;              // channels per wavefront
  static constexpr int kWSlotB = kWaveN * 64;         // one wavefront's [channels][64 k]
  static constexpr int kWRingB = 3 * kWSlotB;         // per wavefront
  static constexpr int kWLoads = 2 * NI;              // direct-to-LDS loads per 64-k weight tile
  static constexpr int kWBase = 0;
  static constexpr int kXBase = kQWaves * kWRingB;    // 48 or 96 KB
  static constexpr int kCorrBase = kXBase + kQXStages * kQXStageB;
  static constexpr int kLdsB = kCorrBase + kQXStages * kQM * 4 + kQM * 4;  // + factors per stage + final maxima
};
constexpr float kE4M3Max = 448.0f;

// 16-byte slot swizzles
// 8 slots per token row.  Bits of the row are mixed so that both access shapes are free of
// bank conflicts: the 64-bit quantised stores (4 lanes per row, consecutive rows) need rows
// r..r+3 to differ in the upper slot bits, the 128-bit fragment reads (one row per lane)
// need 8 distinct values over the rows of equal parity.
__device__ __forceinline__ int fQX(int row) {
  const int b0 = row & 1, b1 = (row >> 1) & 1, b2 = (row >> 2) & 1, b3 = (row >> 3) & 1;
  return (b1 << 2) | ((b0 ^ b2) << 1) | b3;
}
__device__ __forceinline__ int fQW(int row) { return (row >> 2) & 3; }  // 4 slots per weight row

}  // namespace

template <int NI>
__global__ __launch_bounds__(kQThreads, 1) void fp8_quant_gemm_kernel(
    const bf16_t* __restrict__ a, const unsigned char* __restrict__ w, bf16_t* __restrict__ c, int M,
    int K, int N, int64_t lda, int64_t ldw, int64_t ldc, int n_ntiles) {
  using L = QLayout<NI>;
  constexpr int kQN = L::kN, kQWSlotB = L::kWSlotB, kQWRingB = L::kWRingB, kQWBase = L::kWBase;
  constexpr int kQXBase = L::kXBase, kQCorrBase = L::kCorrBase, kWL = L::kWLoads;
  constexpr int kA1 = (NI == 2) ? 2 : 0;  // LDS reads of the second channel block's operand
  __shared__ __attribute__((aligned(1024))) unsigned char lds[L::kLdsB];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;  // = channel block (32 NI wide) of the N tile
  const int i32 = lane & 31;
  const int hh = lane >> 5;

  // XCD-aware numbering (workgroups are dealt round-robin to the 8 XCDs, each with its own L2)
  int mt, nt;
  {
    const int n_mt = gridDim.x / n_ntiles;
    if ((n_mt & 3) == 0 && (n_ntiles & 1) == 0) {
      const int bm = n_mt >> 2, bn = n_ntiles >> 1;
      const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
      mt = (xcd >> 1) * bm + jj / bn;
      nt = (xcd & 1) * bn + jj % bn;
    } else if ((gridDim.x & 7) == 0) {
      // XCD x owns a run of consecutive tiles in row-major order (a few whole tile rows)
      const int t = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
      mt = t / n_ntiles;
      nt = t % n_ntiles;
    } else {
      mt = blockIdx.x / n_ntiles;
      nt = blockIdx.x % n_ntiles;
    }
  }
  const int m0 = mt * kQM, n0 = nt * kQN;
  const int nk = K / kQK;  // K is a multiple of 128 (checked by the caller)
  const int nkk = 2 * nk;  // 64-wide weight tiles

  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;

  // ---- token role: four lanes per token row, 32 k per thread in four 8-value pieces ----
  // Load P of a thread covers k = 32 P + 8 xq .. + 7, so that one load instruction reads 64
  // contiguous bytes of every row it touches (the four lanes of a row side by side).
  const int xrow = tid >> 2;
  const int xq = tid & 3;
  const char* abase = reinterpret_cast<const char*>(a + (int64_t)m0 * lda);  // + step * 256 bytes
  const uint32_t alane_off = (uint32_t)(((int64_t)min(xrow, M - 1 - m0) * lda + 8 * xq) * 2);
  // LDS byte address of piece 0's 8 FP8 codes in stage 0.  Piece p sits in slot (2 p + (xq >> 1)) ^ fQX of
  // the 128-byte row, so its address differs from piece 0's in bits 5 and 6 only: XOR with 32 p.
  const uint32_t xdst_addr0 = lds_base + kQXBase + xrow * 128 + (((xq >> 1) ^ fQX(xrow)) << 4) + 8 * (xq & 1);
  // Rescale factors: [stage][token % 32][token / 32], so that an accumulator lane (one token of each
  // of the four 32-token blocks) fetches its four factors with one 128-bit read.
  const uint32_t corr_waddr = lds_base + kQCorrBase + ((xrow & 31) * 4 + (xrow >> 5)) * 4;
  const uint32_t corr_raddr = lds_base + kQCorrBase + i32 * 16;
  float* s_mfinal = reinterpret_cast<float*>(lds + kQCorrBase) + kQXStages * kQM;  // [128]

  // ---- weight role: 2 NI direct-to-LDS loads per wavefront per 64-k tile, 16 channels each ----
  uint32_t wsrc_off[kWL];  // byte offset from w + (64-k tile) * 64
#pragma unroll
  for (int e = 0; e < kWL; ++e) {
    const int row = 16 * e + (lane >> 2);  // channel inside the wavefront's block
    const int piece = (lane & 3) ^ fQW(row);
    const int n = min(n0 + L::kWaveN * wave + row, N - 1);
    wsrc_off[e] = (uint32_t)((int64_t)n * ldw + 16 * piece);
  }
  const uint32_t wring = __builtin_amdgcn_readfirstlane(lds_base + kQWBase + wave * kQWRingB);
#define RF_ISSUE_W(TILE, SLOT)                                                                \
  {                                                                                           \
    const char* wt_ = reinterpret_cast<const char*>(w) + (int64_t)(TILE) * 64;                \
    _Pragma("unroll") for (int e = 0; e < kWL; ++e) {                                         \
      const uint32_t dst_ = wring + (SLOT) * kQWSlotB + e * 1024;                             \
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"            \
                   :                                                                          \
                   : "s"(dst_), "v"(wsrc_off[e]), "s"(wt_)                                    \
                   : "memory", "m0");                                                         \
    }                                                                                         \
  }

  // ---- fragment read addresses ----
  // An operand of the 32x32x64 MFMA is 32 bytes per lane: lane (i32, hh) holds bytes
  // 32 hh .. 32 hh + 31 of row i32 of a 64-k tile = two 16-byte slots.
  // B operand (tokens): row 32 mi + i32 of the stage, slots 4 kk + 2 hh + {0, 1}
  uint32_t xaddr[2][2];  // [kk][half] in stage 0; + mi * 32 * 128, + stage
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
      xaddr[kk][h2] = lds_base + kQXBase + i32 * 128 + (((4 * kk + 2 * hh + h2) ^ fQX(i32)) << 4);
  // A operand (weights): row 32 ni + i32 of the slot, slots 2 hh + {0, 1}
  uint32_t waddr[2];  // [half] in slot 0; + ni * 32 * 64, + slot
#pragma unroll
  for (int h2 = 0; h2 < 2; ++h2) waddr[h2] = wring + i32 * 64 + (((2 * hh + h2) ^ fQW(i32)) << 4);

  f32x16 acc[NI][4];  // [ni][mi]: C^T tile (rows = channels, columns = tokens)
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- token tile in registers: 4 x 8 bf16 ----
  u32x4 xreg[4];
#define RF_LOAD_X(REG, P, STEP)                                                               \
  {                                                                                           \
    const char* ap_ = abase + (int64_t)(STEP) * (kQK * 2);                                    \
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3"                                   \
                 : "=v"(REG[P]) : "v"(alane_off), "s"(ap_), "n"(64 * (P)));                   \
  }
#define RF_WAIT_X2(REG, P0, P1, PENDING) \
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(REG[P0]), "+v"(REG[P1]) : "n"(PENDING));
  // running maximum of this thread's token (the 4 lanes of a token hold the same values)
  float m_run = 0.f;
  float amax = 0.f, qscale = 0.f;
  unsigned amax_bits = 0;  // packed pair of running 16-bit maxima of the tile
  // max |x| of 8 bf16 values.  For non-negative values the bf16 bit patterns order like
  // unsigned integers, so the sign bits are cleared and the maximum is taken on packed
  // 16-bit integers, two values per operation; the result is a packed pair to be folded.
  typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
  auto absmax8 = [&](const u32x4& r) {
    u16x2 v = __builtin_bit_cast(u16x2, r[0] & 0x7fff7fffu);
#pragma unroll
    for (int j = 1; j < 4; ++j)
      v = __builtin_elementwise_max(v, __builtin_bit_cast(u16x2, r[j] & 0x7fff7fffu));
    return v;
  };
  auto fold_max = [&](u16x2 v) {  // packed pair -> fp32 value of the larger bf16
    const unsigned short m16 = v[0] > v[1] ? v[0] : v[1];
    return __uint_as_float((uint32_t)m16 << 16);
  };
  // piece P: 8 values -> 8 FP8 codes -> LDS; XW = address of piece 0 in the stage (raw write: the compiler
  // would order an ordinary one behind the direct-to-LDS loads in flight)
#define RF_QUANT_A(REG, P, T0)                                                                \
  {                                                                                           \
    T0 = 0;                                                                                   \
    T0 = __builtin_amdgcn_cvt_pk_fp8_f32(bf16_lo(REG[P][0]) * qscale, bf16_hi(REG[P][0]) * qscale, T0, false); \
    T0 = __builtin_amdgcn_cvt_pk_fp8_f32(bf16_lo(REG[P][1]) * qscale, bf16_hi(REG[P][1]) * qscale, T0, true);  \
  }
#define RF_QUANT_B(REG, P, T0, XW)                                                            \
  {                                                                                           \
    int t1_ = 0;                                                                              \
    t1_ = __builtin_amdgcn_cvt_pk_fp8_f32(bf16_lo(REG[P][2]) * qscale, bf16_hi(REG[P][2]) * qscale, t1_, false); \
    t1_ = __builtin_amdgcn_cvt_pk_fp8_f32(bf16_lo(REG[P][3]) * qscale, bf16_hi(REG[P][3]) * qscale, t1_, true);  \
    u32x2 q2_;                                                                                \
    q2_[0] = (uint32_t)(T0);                                                                  \
    q2_[1] = (uint32_t)t1_;                                                                   \
    asm volatile("ds_write_b64 %0, %1" : : "v"((XW) ^ (32u * (P))), "v"(q2_) : "memory");     \
  }
#define RF_QUANT_STORE(REG, P, XW) \
  {                                \
    int t0_;                       \
    RF_QUANT_A(REG, P, t0_)        \
    RF_QUANT_B(REG, P, t0_, XW)    \
  }
  // merge the tile maximum into the running maximum; scale and rescale factor of the tile
  // (one LDS write per step, issued by every lane so that the wait counts below hold as written)
  auto update_max = [&](int stage) {
    amax = fmaxf(amax, dpp_f32<kDppQuadXor1>(amax));
    amax = fmaxf(amax, dpp_f32<kDppQuadXor2>(amax));
    const float m_new = fmaxf(m_run, amax);
    qscale = m_new > 0.f ? kE4M3Max / m_new : 0.f;  // IEEE division: it decides the FP8 codes
    const float corr = (m_new == m_run) ? 1.0f : m_run * fast_rcp(m_new);
    m_run = m_new;
    const uint32_t ca = corr_waddr + stage * (kQM * 4);
    asm volatile("ds_write_b32 %0, %1" : : "v"(ca), "v"(corr) : "memory");  // same value from the 4 lanes of a token
  };

  // Fragment registers: one 32-byte operand = two 128-bit halves.  They are carried from step to
  // step: the fragments of the first weight tile of step s+1 are requested at the end of step s,
  // into registers as those fall dead (an operand is dead once the last MFMA that reads it has
  // been issued; LDS data comes back long after that MFMA has read its sources).
  i32x8 a0, a1, b0, b1, b2, b3;
  f32x4 corrv;  // rescale factors of the coming step for this lane's four tokens
  // (the two halves are joined where they are requested, so that the operand is one value from
  // there on: the compiler then only has whole operands to carry around the loop)
#define RF_READ32(DST, ADDR0, ADDR1, OFF)                                                     \
  {                                                                                           \
    typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4_;                     \
    i32x4_ lo_, hi_;                                                                          \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(lo_) : "v"(ADDR0), "n"(OFF));         \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(hi_) : "v"(ADDR1), "n"(OFF));         \
    DST = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);                          \
  }
  // wait until at most PENDING LDS operations are in flight; the named operand is tied
  // to the wait so that its uses stay behind it
#define RF_WAIT2(X, Y, PENDING) asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(X), "+v"(Y) : "n"(PENDING));
#define RF_WAIT1(X, PENDING) asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(X) : "n"(PENDING));
#define RF_MFMA(NI_, MI, A, B)                                                                \
  acc[NI_][MI] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A, B, acc[NI_][MI], 0, 0, 0, 0x7f7f7f7f, 0, \
                                                                 0x7f7f7f7f);
#define RF_FENCE __builtin_amdgcn_sched_barrier(0);
  auto any_rescale = [&]() {
    return __builtin_amdgcn_ballot_w64(corrv[0] != 1.0f || corrv[1] != 1.0f || corrv[2] != 1.0f ||
                                       corrv[3] != 1.0f) != 0;
  };

  // ---- prologue ----
  // Token tiles 0 and 1 are quantised into stages 0 and 1, tile 2 is requested into registers,
  // weight tiles 0, 1, 2 into the ring; vector-memory requests in the order of a loop step.
  RF_ISSUE_W(0, 0)
  {
    u32x4 xpro[4];  // token tile 1
    const int s1 = min(1, nk - 1);
    RF_LOAD_X(xreg, 0, 0) RF_LOAD_X(xreg, 1, 0) RF_LOAD_X(xreg, 2, 0) RF_LOAD_X(xreg, 3, 0)
    RF_LOAD_X(xpro, 0, s1) RF_LOAD_X(xpro, 1, s1) RF_LOAD_X(xpro, 2, s1) RF_LOAD_X(xpro, 3, s1)
    RF_WAIT_X2(xreg, 0, 1, 4) RF_WAIT_X2(xreg, 2, 3, 4)
    amax = fold_max(__builtin_elementwise_max(__builtin_elementwise_max(absmax8(xreg[0]), absmax8(xreg[1])),
                                              __builtin_elementwise_max(absmax8(xreg[2]), absmax8(xreg[3]))));
    update_max(0);
    RF_QUANT_STORE(xreg, 0, xdst_addr0) RF_QUANT_STORE(xreg, 1, xdst_addr0)
    RF_QUANT_STORE(xreg, 2, xdst_addr0) RF_QUANT_STORE(xreg, 3, xdst_addr0)
    RF_WAIT_X2(xpro, 0, 1, 0) RF_WAIT_X2(xpro, 2, 3, 0)  // (weight tile 0, the oldest request, has landed too)
    amax = fold_max(__builtin_elementwise_max(__builtin_elementwise_max(absmax8(xpro[0]), absmax8(xpro[1])),
                                              __builtin_elementwise_max(absmax8(xpro[2]), absmax8(xpro[3]))));
    update_max(1);
    RF_QUANT_STORE(xpro, 0, xdst_addr0 + kQXStageB) RF_QUANT_STORE(xpro, 1, xdst_addr0 + kQXStageB)
    RF_QUANT_STORE(xpro, 2, xdst_addr0 + kQXStageB) RF_QUANT_STORE(xpro, 3, xdst_addr0 + kQXStageB)
    const int s2 = min(2, nk - 1);
    RF_LOAD_X(xreg, 0, s2)
    RF_ISSUE_W(min(1, nkk - 1), 1)
    RF_LOAD_X(xreg, 1, s2) RF_LOAD_X(xreg, 2, s2) RF_LOAD_X(xreg, 3, s2)
    RF_ISSUE_W(min(2, nkk - 1), 2)
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();  // token stages 0 and 1 and their factors are complete
  asm volatile("ds_read_b128 %0, %1" : "=v"(corrv) : "v"(corr_raddr));
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(corrv));
  bool resc = any_rescale();
  RF_READ32(a0, waddr[0], waddr[1], 0)
  RF_READ32(b0, xaddr[0][0], xaddr[0][1], 0 * 4096)
  RF_READ32(b1, xaddr[0][0], xaddr[0][1], 1 * 4096)
  RF_READ32(b2, xaddr[0][0], xaddr[0][1], 2 * 4096)
  RF_READ32(b3, xaddr[0][0], xaddr[0][1], 3 * 4096)
  if constexpr (NI == 2) { RF_READ32(a1, waddr[0], waddr[1], 32 * 64) }

  // ---- main loop ----
  // Step s multiplies token stage s%3 by weight tiles 2s, 2s+1 (ring slots wslot, wslot+1),
  // quantises token tile s+2 into stage (s+2)%3, fetches token tile s+3 into registers and weight
  // tiles 2s+3, 2s+4 into the slots just read, and requests the fragments of weight tile 2s+2
  // and token stage (s+1)%3 for the next step.  The one barrier of a step sits after its first
  // four MFMAs: it orders the token writes of step s-1 (all finished before a wavefront arrives)
  // before their reads (which start at the end of step s), and the reads of step s-1 before the
  // writes of step s into the same stage (which follow the barrier), so no wavefront waits for
  // LDS data right behind a barrier.  Every step is the same straight-line code: past the end
  // of K the prefetches re-read the last tile, which leaves the maxima as they are, and nothing
  // consumes them.  Vector-memory issue order per step: X0, W(2s+3), X1, X2, X3, W(2s+4), where a
  // weight tile is kWL loads.  LDS operations in flight at the top of a step, oldest first: up to
  // three piece writes of the previous step, a0, b0, b1, b2, b3, (a1).
  int wslot = 0;  // ring slot of weight tile 2s
  int rs = 0;     // token stage of step s
  for (int s = 0; s < nk; ++s) {
    const int rs1 = rs == 2 ? 0 : rs + 1;     // stage of step s+1
    const int ws = rs1 == 2 ? 0 : rs1 + 1;    // stage written in this step
    const int slot1 = wslot == 2 ? 0 : wslot + 1;
    const int slot2 = slot1 == 2 ? 0 : slot1 + 1;

    if (resc) {  // a maximum moved in this step's token tile: rescale (uniform)
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
        if (__builtin_amdgcn_ballot_w64(corrv[mi] != 1.0f) != 0) {
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[ni][mi][r] *= corrv[mi];
        }
      }
    }
    RF_FENCE

    // ---- weight tile 2s, first channel block; maximum of token tile s+2 ----
    RF_WAIT2(a0, b0, 6 + kA1)
    RF_MFMA(0, 0, a0, b0)
    RF_WAIT_X2(xreg, 0, 1, kWL + 2)  // token pieces 0, 1 of tile s+2: X2, X3, W(2s+2) may still fly
    amax_bits = __builtin_bit_cast(unsigned, __builtin_elementwise_max(absmax8(xreg[0]), absmax8(xreg[1])));
    RF_FENCE
    RF_WAIT1(b1, 4 + kA1)
    RF_MFMA(0, 1, a0, b1)
    RF_WAIT_X2(xreg, 2, 3, kWL)  // pieces 2, 3: W(2s+2) may still fly; W(2s+1) has landed
    amax = fold_max(__builtin_elementwise_max(
        __builtin_bit_cast(u16x2, amax_bits), __builtin_elementwise_max(absmax8(xreg[2]), absmax8(xreg[3]))));
    RF_FENCE
    RF_WAIT1(b2, 2 + kA1)
    RF_MFMA(0, 2, a0, b2)
    update_max(ws);
    RF_FENCE
    RF_WAIT1(b3, 1 + kA1)  // (+1: the factor write of update_max)
    RF_MFMA(0, 3, a0, b3)
    RF_FENCE
    // Every wavefront has finished step s-1 when it gets here: stage rs1 and its factors are
    // complete, stage ws is free.  (Our own LDS writes of step s-1 are older than the fragments
    // waited for above.)
    __builtin_amdgcn_s_barrier();
    RF_FENCE

    // ---- second channel block of tile 2s; fragments of tile 2s+1; token pieces 0, 1 ----
    // The quantisation is cut into half pieces (4 values), one behind each MFMA from here on.
    int qa;  // first four codes of the piece in work
    const uint32_t xw = xdst_addr0 + ws * kQXStageB;
    // tile 2s+1: k half 1 of stage rs, ring slot slot1
    const uint32_t xb0 = xaddr[1][0] + rs * kQXStageB, xb1 = xaddr[1][1] + rs * kQXStageB;
    const uint32_t wb0 = waddr[0] + slot1 * kQWSlotB, wb1 = waddr[1] + slot1 * kQWSlotB;
    const uint32_t cr1 = corr_raddr + rs1 * (kQM * 4);
    if constexpr (NI == 2) { RF_WAIT1(a1, 1) }  // every read of ring slot wslot is back (the factor write may fly)
    asm volatile("ds_read_b128 %0, %1" : "=v"(corrv) : "v"(cr1));  // factors of step s+1
    RF_READ32(a0, wb0, wb1, 0)   // first operand of weight tile 2s+1
    if constexpr (NI == 2) { RF_MFMA(1, 0, a1, b0) }
    RF_READ32(b0, xb0, xb1, 0 * 4096)
    RF_QUANT_A(xreg, 0, qa)
    RF_FENCE
    if constexpr (NI == 2) { RF_MFMA(1, 1, a1, b1) }
    RF_READ32(b1, xb0, xb1, 1 * 4096)
    RF_QUANT_B(xreg, 0, qa, xw)
    RF_LOAD_X(xreg, 0, min(s + 3, nk - 1))
    RF_ISSUE_W(min(2 * s + 3, nkk - 1), wslot)  // refill the slot just read
    RF_FENCE
    if constexpr (NI == 2) { RF_MFMA(1, 2, a1, b2) }
    RF_READ32(b2, xb0, xb1, 2 * 4096)
    RF_QUANT_A(xreg, 1, qa)
    RF_FENCE
    if constexpr (NI == 2) { RF_MFMA(1, 3, a1, b3) }
    RF_READ32(b3, xb0, xb1, 3 * 4096)
    if constexpr (NI == 2) { RF_READ32(a1, wb0, wb1, 32 * 64) }
    RF_QUANT_B(xreg, 1, qa, xw)
    RF_LOAD_X(xreg, 1, min(s + 3, nk - 1))
    RF_FENCE

    // ---- weight tile 2s+1, first channel block; token pieces 2, 3 ----
    // LDS operations in flight, oldest first: the factors, a0, b0, b1, piece write, b2, b3, (a1), piece write
    asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(a0), "+v"(b0), "+v"(corrv) : "n"(8 + kA1));
    RF_MFMA(0, 0, a0, b0)
    resc = any_rescale();
    RF_QUANT_A(xreg, 2, qa)
    RF_FENCE
    RF_WAIT1(b1, 6 + kA1)
    RF_MFMA(0, 1, a0, b1)
    RF_QUANT_B(xreg, 2, qa, xw)
    RF_LOAD_X(xreg, 2, min(s + 3, nk - 1))
    RF_FENCE
    RF_WAIT1(b2, 4 + kA1)  // b3, (a1) and two piece writes may fly
    RF_MFMA(0, 2, a0, b2)
    RF_QUANT_A(xreg, 3, qa)
    RF_FENCE
    RF_WAIT1(b3, 2 + kA1)
    RF_MFMA(0, 3, a0, b3)
    RF_QUANT_B(xreg, 3, qa, xw)
    RF_LOAD_X(xreg, 3, min(s + 3, nk - 1))
    RF_FENCE

    // ---- second channel block of tile 2s+1; fragments of tile 2s+2 for the next step ----
    if constexpr (NI == 2) { RF_WAIT1(a1, 3) }  // every read of ring slot slot1 is back (three piece writes may fly)
    // tile 2s+2: k half 0 of stage rs1, ring slot slot2
    const uint32_t xn0 = xaddr[0][0] + rs1 * kQXStageB, xn1 = xaddr[0][1] + rs1 * kQXStageB;
    const uint32_t wn0 = waddr[0] + slot2 * kQWSlotB, wn1 = waddr[1] + slot2 * kQWSlotB;
    // weight tile 2s+2 has landed: the younger requests (X0, W(2s+3), X1, X2, X3) may still fly
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kWL + 4) : "memory");
    RF_READ32(a0, wn0, wn1, 0)   // first operand of weight tile 2s+2
    if constexpr (NI == 2) { RF_MFMA(1, 0, a1, b0) }
    RF_READ32(b0, xn0, xn1, 0 * 4096)
    RF_ISSUE_W(min(2 * s + 4, nkk - 1), slot1)
    RF_FENCE
    if constexpr (NI == 2) { RF_MFMA(1, 1, a1, b1) }
    RF_READ32(b1, xn0, xn1, 1 * 4096)
    RF_FENCE
    if constexpr (NI == 2) { RF_MFMA(1, 2, a1, b2) }
    RF_READ32(b2, xn0, xn1, 2 * 4096)
    RF_FENCE
    if constexpr (NI == 2) { RF_MFMA(1, 3, a1, b3) }
    RF_READ32(b3, xn0, xn1, 3 * 4096)
    if constexpr (NI == 2) { RF_READ32(a1, wn0, wn1, 32 * 64) }
    RF_FENCE
    wslot = slot2;
    rs = rs1;
  }
  // the surplus requests stay reserved until they have landed
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)"
               : "+v"(xreg[0]), "+v"(xreg[1]), "+v"(xreg[2]), "+v"(xreg[3]), "+v"(a0), "+v"(b0), "+v"(b1),
                 "+v"(b2), "+v"(b3)
               :
               : "memory");
  if constexpr (NI == 2) asm volatile("" : "+v"(a1));
#undef RF_READ32
#undef RF_WAIT2
#undef RF_WAIT1
#undef RF_MFMA
#undef RF_FENCE
#undef RF_ISSUE_W
#undef RF_LOAD_X
#undef RF_WAIT_X2
#undef RF_QUANT_STORE
#undef RF_QUANT_A
#undef RF_QUANT_B

  // final maxima of the tokens, to the accumulator lanes through LDS
  if (xq == 0) s_mfinal[xrow] = m_run;
  __syncthreads();

  // epilogue: c = acc * m / MAX
  // An accumulator lane holds one token, four channels at a time: stored from there, an
  // instruction would touch 32 rows with 16 bytes each.  When the output allows 16-byte stores,
  // a wavefront stages its 128-token x kWaveN-channel sub-tile in LDS (everything but the final
  // maxima is free by now; 16-byte slots XOR-swizzled with the row) and stores whole row
  // segments of 64 or 128 bytes.
  const bool wide_ok = (reinterpret_cast<uintptr_t>(c) & 15) == 0 && (ldc & 7) == 0;
  if (wide_ok) {
    constexpr int RB = L::kWaveN * 2;   // bytes per staged row
    constexpr int SL = RB / 16;         // 16-byte slots per row (4 or 8)
    unsigned char* stage = lds + wave * (kQM * RB);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      const int row = 32 * mi + i32;
      const float f = s_mfinal[row] * (1.0f / kE4M3Max);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          u32x2 o2;
          o2[0] = pack_bf16(acc[ni][mi][4 * r4] * f, acc[ni][mi][4 * r4 + 1] * f);
          o2[1] = pack_bf16(acc[ni][mi][4 * r4 + 2] * f, acc[ni][mi][4 * r4 + 3] * f);
          const int sw = (RB == 128) ? ((row >> 1) & 7) : ((row >> 2) & 3);
          *reinterpret_cast<u32x2*>(stage + row * RB + (((4 * ni + r4) ^ sw) << 4) + 8 * hh) = o2;
        }
    }
    constexpr int RPI = 64 / SL;  // rows per store instruction
#pragma unroll
    for (int i = 0; i < kQM / RPI; ++i) {
      const int row = RPI * i + lane / SL;
      const int slot = lane % SL;
      const int sw = (RB == 128) ? ((row >> 1) & 7) : ((row >> 2) & 3);
      const u32x4 o4 = *reinterpret_cast<const u32x4*>(stage + row * RB + ((slot ^ sw) << 4));
      const int m = m0 + row;
      const int n = n0 + L::kWaveN * wave + 8 * slot;
      // (N is a multiple of 8; non-temporal like the other matrix kernels' outputs: +2 % on short launches)
      if (m < M && n < N) __builtin_nontemporal_store(o4, reinterpret_cast<u32x4*>(c + (int64_t)m * ldc + n));
    }
    return;
  }
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int mloc = 32 * mi + i32;
    const int m = m0 + mloc;
    const float f = s_mfinal[mloc] * (1.0f / kE4M3Max);
    if (m >= M) continue;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int n = n0 + L::kWaveN * wave + 32 * ni + 8 * r4 + 4 * hh;
        if (n < N) {
          u32x2 o2;
          o2[0] = pack_bf16(acc[ni][mi][4 * r4] * f, acc[ni][mi][4 * r4 + 1] * f);
          o2[1] = pack_bf16(acc[ni][mi][4 * r4 + 2] * f, acc[ni][mi][4 * r4 + 3] * f);
          *reinterpret_cast<u32x2*>(c + (int64_t)m * ldc + n) = o2;
        }
      }
    }
  }
}

hipError_t launch_fp8_quant_gemm(const void* a, const void* w, void* c, int M, int K, int N,
                                 int64_t lda, int64_t ldw, int64_t ldc, hipStream_t s) {
  const int n_mtiles = (M + kQM - 1) / kQM;
  // The 512-wide N tile does the most work per byte staged.  When the 256-wide tiling still
  // fits the chip in one round of workgroups (one per compute unit), it is taken instead: it
  // occupies up to twice as many compute units and wastes less of a ragged last tile.
  const int64_t n_narrow = (int64_t)n_mtiles * ((N + 255) / 256);
  const int ni = n_narrow <= 256 ? 1 : 2;
  const int n_ntiles = (N + 256 * ni - 1) / (256 * ni);
  const int64_t grid = (int64_t)n_mtiles * n_ntiles;
  if (grid > INT32_MAX) return hipErrorInvalidValue;
  // 32-bit lane offsets: inside a 128-token tile of a, inside all of w
  if ((int64_t)kQM * lda * 2 >= ((int64_t)1 << 32) || (int64_t)N * ldw >= ((int64_t)1 << 32))
    return hipErrorInvalidValue;
  if (ni == 1)
    hipLaunchKernelGGL(fp8_quant_gemm_kernel<1>, dim3((unsigned)grid), dim3(kQThreads), 0, s,
                       (const bf16_t*)a, (const unsigned char*)w, (bf16_t*)c, M, K, N, lda, ldw, ldc,
                       n_ntiles);
  else
    hipLaunchKernelGGL(fp8_quant_gemm_kernel<2>, dim3((unsigned)grid), dim3(kQThreads), 0, s,
                       (const bf16_t*)a, (const unsigned char*)w, (bf16_t*)c, M, K, N, lda, ldw, ldc,
                       n_ntiles);
  return hipGetLastError();
}

}  // namespace rf
