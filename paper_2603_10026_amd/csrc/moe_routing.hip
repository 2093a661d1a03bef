// MoE routing: scores GEMM -> softmax -> top-k (paper Appendix A.2, "MoE
// routing"), as a multi-segment cascade (Section 4.3):
//   p[e] = sum_c x[c] w[c,e];  m = max_e p[e];  t = sum_e exp(p[e]-m);
//   s = TopK_e p[e];  output exp(s-m)/t with the experts' indices.
// TopK acts on the raw scores (softmax keeps their order); equal scores are
// ordered by expert index, lowest first.
//
// The router GEMM is skinny (a few thousand tokens x 32..128 experts) and its
// cost is reading x once, so the contraction axis is split over workgroups:
//
// Kernel 1 (scores): workgroup (row block of 64 tokens, k slice).  x and w tiles
//   of 128 k go HBM -> LDS with direct-to-LDS 128-bit loads two tiles ahead of their
//   use (three LDS stages), one barrier per tile.  The product is computed
//   transposed, P^T = W^T X^T, with 32x32x16 bf16 MFMAs: W^T fragments come from 64-bit LDS transpose reads, X
//   fragments from 128-bit reads.  The four wavefronts split the eight 16-wide
//   contraction steps of a tile, so every LDS byte is read exactly once; their
//   accumulators are summed through LDS in a fixed order and the fp32 partial
//   scores of the slice are written to the caller's workspace.
// Kernel 2 (cascade): 16 lanes per token add the slices' partial scores in slice
//   order, then run the cascade: each lane reduces its experts, lanes merge
//   (max; sum with the exp rescale; TopK of the union) with DPP lane exchanges.
#include <atomic>

#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

// Scratch memory of the entry point that must not allocate: fp32 partial scores of one call.
// A file-scope device array: every GPU the library runs on holds its own copy, at its own
// address, until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels are always handed the address that call returned.
static __device__ __align__(256) unsigned char scratch[kMoeStaticScratchBytes];

namespace {

constexpr int kMoeThreads = 256;
constexpr int kMoeRows = 64;    // tokens per workgroup
constexpr int kMoeKB = 128;     // k per LDS tile
constexpr int kMoeXTileB = kMoeRows * kMoeKB * 2;  // 16 KB, [row][k], 256-byte rows

typedef __attribute__((address_space(3))) void lds_void_m;
typedef __attribute__((address_space(1))) const void global_cvoid_m;

// 16-byte slot swizzles (slot = piece ^ f(row))
__device__ __forceinline__ int fXm(int row) { return row & 15; }
template <int PPR>
__device__ __forceinline__ int fWm(int krow) { return ((krow & 3) << 2) & (PPR - 1); }

}  // namespace

template <int EPL>
__device__ __forceinline__ void moe_cascade_token(const float (&p)[EPL], int q, int row, bool live,
                                                  int topk, float* __restrict__ prob,
                                                  int32_t* __restrict__ idx, int64_t ldp, int64_t ldi);

// NT = E / 32.  part[ks][row][e] = sum over the k slice of x[row,k] w[k,e].
// FUSED (single-segment strategy, Section 4.3: the whole contraction axis in one workgroup, grid
// y = 1): the scores never leave the chip; the workgroup runs the cascade on them itself and
// writes prob / idx.  Chosen when the contraction axis is short enough that splitting it only
// buys a second launch.
template <int NT, bool FUSED>
__global__ __launch_bounds__(kMoeThreads) void moe_scores_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ w, float* __restrict__ part, int S,
    int n_kblocks, int64_t ldx, int64_t ldw, int topk, float* __restrict__ prob,
    int32_t* __restrict__ idx, int64_t ldp, int64_t ldi) {
  constexpr int E = 32 * NT;
  constexpr int PPR = E / 8;               // 16-byte pieces per W row
  constexpr int kWTileB = kMoeKB * E * 2;  // [k][e]
  constexpr int kStageB = kMoeXTileB + kWTileB;
  constexpr int kWLoads = kWTileB / 1024 / 4;  // direct-to-LDS loads per wavefront per tile
  constexpr int kAccB = 2 * NT * 16 * 64 * 4;  // one wavefront's accumulators
  constexpr int kStages = 3;
  constexpr int kLdsB = (kStages * kStageB > 4 * kAccB) ? kStages * kStageB : 4 * kAccB;
  constexpr int kLoadsPerTile = 4 + kWLoads;  // per wavefront
  __shared__ __attribute__((aligned(1024))) unsigned char lds[kLdsB];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int i32 = lane & 31;
  const int hh = lane >> 5;
  const int row0 = blockIdx.x * kMoeRows;
  const int KS = gridDim.y;
  const int ks = blockIdx.y;
  // this slice's tiles: [b0, b1)
  const int b0 = (int)((int64_t)n_kblocks * ks / KS);
  const int b1 = (int)((int64_t)n_kblocks * (ks + 1) / KS);

  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;

  // ---- direct-to-LDS roles ----
  // X: 4 loads per wavefront per tile; load e covers rows 16 wave + 4e .. +3, lane -> (row, slot)
  uint32_t xsrc_off[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int row = 16 * wave + 4 * e + (lane >> 4);
    const int piece = (lane & 15) ^ fXm(row);
    xsrc_off[e] = (uint32_t)(((int64_t)min(row0 + row, S - 1) * ldx + 8 * piece) * 2);
  }
  // W: pieces numbered row-major over the tile; load e of wavefront `wave` covers pieces
  // 64 (kWLoads wave + e) .. +63
  uint32_t wsrc_off[kWLoads];
#pragma unroll
  for (int e = 0; e < kWLoads; ++e) {
    const int p = 64 * (kWLoads * wave + e) + lane;
    const int krow = p / PPR;
    const int piece = (p % PPR) ^ fWm<PPR>(krow);
    wsrc_off[e] = (uint32_t)(((int64_t)krow * ldw + 8 * piece) * 2);
  }
  auto issue_tile = [&](int blk, int stage) {
    const char* xt = reinterpret_cast<const char*>(x) + (int64_t)blk * kMoeKB * 2;
    const char* wt = reinterpret_cast<const char*>(w) + (int64_t)blk * kMoeKB * ldw * 2;
    unsigned char* xdst = lds + stage * kStageB + wave * 4096;
    unsigned char* wdst = lds + stage * kStageB + kMoeXTileB + wave * (kWLoads * 1024);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      __builtin_amdgcn_global_load_lds((global_cvoid_m*)(xt + xsrc_off[e]),
                                       (lds_void_m*)(xdst + e * 1024), 16, 0, 0);
#pragma unroll
    for (int e = 0; e < kWLoads; ++e)
      __builtin_amdgcn_global_load_lds((global_cvoid_m*)(wt + wsrc_off[e]),
                                       (lds_void_m*)(wdst + e * 1024), 16, 0, 0);
  };

  // ---- fragment read addresses (stage 0, this wavefront's two contraction steps) ----
  // B operand (X): lane (i32, hh) of token tile mi reads row 32mi + i32, slot 2kk + hh
  uint32_t xaddr[2][2];  // [step][mi]
#pragma unroll
  for (int st = 0; st < 2; ++st)
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
      const int row = 32 * mi + i32;
      const int kk = 2 * wave + st;
      xaddr[st][mi] = lds_base + row * 256 + (((2 * kk + hh) ^ fXm(row)) << 4);
    }
  // A operand (W^T) by transpose reads: lane = 32hh + 16g2 + 4j + a reads 8 bytes of k-row
  // 16kk + 8hh + 4w2 + j at expert column 32ni + 16g2 + 4a
  uint32_t waddr[2][NT][2];  // [step][ni][w2]
  {
    const int i16 = lane & 15, g2 = (lane >> 4) & 1;
    const int j = i16 >> 2, a = i16 & 3;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int ni = 0; ni < NT; ++ni)
#pragma unroll
        for (int w2 = 0; w2 < 2; ++w2) {
          const int krow = 16 * (2 * wave + st) + 8 * hh + 4 * w2 + j;
          const int piece = (32 * ni + 16 * g2 + 4 * a) >> 3;
          waddr[st][ni][w2] = lds_base + kMoeXTileB + krow * (E * 2) +
                              ((piece ^ fWm<PPR>(krow)) << 4) + 8 * (a & 1);
        }
  }

  f32x16 acc[NT][2];  // [ni][mi]: P^T tile (rows = experts, columns = tokens)
#pragma unroll
  for (int a = 0; a < NT; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;

  if (b0 < b1) issue_tile(b0, 0);
  if (b0 + 1 < b1) issue_tile(b0 + 1, 1);
  int stage = 0;
  for (int blk = b0; blk < b1; ++blk) {
    // This wavefront's loads of the tile have landed (loads retire in order; only the
    // next tile's may still be in flight); then everyone's have, and everyone is done
    // reading the stage that the tile after next goes to.
    if (blk + 1 < b1)
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(kLoadsPerTile) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (blk + 2 < b1) issue_tile(blk + 2, stage == 0 ? 2 : stage - 1);
    const uint32_t soff = stage * kStageB;
    stage = stage == 2 ? 0 : stage + 1;
    // Fragment reads are raw instructions with a hand-placed wait: through the compiler's
    // intrinsics every LDS read would first wait for the direct-to-LDS loads of the next
    // tile, just issued.
    u32x2 af[2][NT][2];
    u32x4 bfr[2][2];
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      const uint32_t xa0 = xaddr[st][0] + soff, xa1 = xaddr[st][1] + soff;
#pragma unroll
      for (int ni = 0; ni < NT; ++ni)
#pragma unroll
        for (int w2 = 0; w2 < 2; ++w2) {
          const uint32_t wa = waddr[st][ni][w2] + soff;
          asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(af[st][ni][w2]) : "v"(wa));
        }
      asm volatile("ds_read_b128 %0, %1" : "=v"(bfr[st][0]) : "v"(xa0));
      asm volatile("ds_read_b128 %0, %1" : "=v"(bfr[st][1]) : "v"(xa1));
    }
    // all reads of this step are back (the fragment registers are tied to the wait)
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
      for (int ni = 0; ni < NT; ++ni)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(af[st][ni][0]), "+v"(af[st][ni][1]));
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bfr[st][0]), "+v"(bfr[st][1]));
    }
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) {
        u32x4 a;
        a[0] = af[st][ni][0][0]; a[1] = af[st][ni][0][1];
        a[2] = af[st][ni][1][0]; a[3] = af[st][ni][1][1];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
          acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, bfr[st][mi]), acc[ni][mi],
              0, 0, 0);
      }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __syncthreads();  // every wavefront has left the loop: LDS is free

  // ---- sum the four wavefronts' accumulators (fixed order 0, 1, 2, 3) ----
  // Every wavefront parks its accumulators in LDS as 128-bit chunks [chunk][lane]; chunk
  // c = (ni * 2 + mi) * 4 + r4 holds P[token 32 mi + i32][experts 32 ni + 8 r4 + 4 hh .. +3].
  // Wavefront v then sums chunks [v CPW, (v+1) CPW) over the four copies and stores them.
  constexpr int kChunks = 2 * NT * 4;
  constexpr int CPW = kChunks / 4;
  f32x4* red = reinterpret_cast<f32x4*>(lds);
  {
    f32x4* dst = red + wave * (kChunks * 64) + lane;
#pragma unroll
    for (int ni = 0; ni < NT; ++ni)
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 v;
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = acc[ni][mi][4 * r4 + j];
          dst[((ni * 2 + mi) * 4 + r4) * 64] = v;
        }
  }
  __syncthreads();
  if constexpr (!FUSED) {
    float* prow = part + ((int64_t)ks * S) * E;
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
      const int c = wave * CPW + cc;
      f32x4 v = red[c * 64 + lane];
#pragma unroll
      for (int r = 1; r < 4; ++r) v += red[r * (kChunks * 64) + c * 64 + lane];
      const int ni = c >> 3, mi = (c >> 2) & 1, r4 = c & 3;
      const int m = row0 + 32 * mi + i32;
      if (m < S) *reinterpret_cast<f32x4*>(prow + (int64_t)m * E + 32 * ni + 8 * r4 + 4 * hh) = v;
    }
  } else {
    // sums in the same fixed order, kept in registers until every wavefront has read the four
    // copies, then laid out [token][expert] at the start of LDS
    f32x4 sum[CPW];
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
      const int c = wave * CPW + cc;
      sum[cc] = red[c * 64 + lane];
#pragma unroll
      for (int r = 1; r < 4; ++r) sum[cc] += red[r * (kChunks * 64) + c * 64 + lane];
    }
    __syncthreads();
    float* sc = reinterpret_cast<float*>(lds);  // [kMoeRows][E + 4] (padded rows)
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
      const int c = wave * CPW + cc;
      const int ni = c >> 3, mi = (c >> 2) & 1, r4 = c & 3;
      *reinterpret_cast<f32x4*>(sc + (32 * mi + i32) * (E + 4) + 32 * ni + 8 * r4 + 4 * hh) = sum[cc];
    }
    __syncthreads();
    // the cascade: 16 lanes per token, 16 tokens per pass
    constexpr int EPL = E / 16;
    const int q = tid & 15;
#pragma unroll 1
    for (int pass = 0; pass < kMoeRows / 16; ++pass) {
      const int tl = 16 * pass + (tid >> 4);
      const int row = row0 + tl;
      float p[EPL];
#pragma unroll
      for (int i = 0; i < EPL; i += 2) {
        const float2 v2 = *reinterpret_cast<const float2*>(sc + tl * (E + 4) + q * EPL + i);
        p[i] = v2.x;
        p[i + 1] = v2.y;
      }
      moe_cascade_token<EPL>(p, q, row, row < S, topk, prob, idx, ldp, ldi);
    }
  }
}

// 16 lanes per token; lane q owns experts [q EPL, (q+1) EPL).
constexpr int kCascadeThreads = 64;  // one wavefront = 4 tokens per workgroup

// The cascade of one token on the scores p[EPL] its 16 lanes hold (lane q: experts q EPL ..).
template <int EPL>
__device__ __forceinline__ void moe_cascade_token(const float (&p)[EPL], int q, int row, bool live,
                                                  int topk, float* __restrict__ prob,
                                                  int32_t* __restrict__ idx, int64_t ldp, int64_t ldi) {
  constexpr int E = 16 * EPL;
  // stage 1: max;  stage 2: sum of exponentials (lane-level fused form, merged across
  // the 16 lanes with the level-k expression)
  float m = p[0];
#pragma unroll
  for (int i = 1; i < EPL; ++i) m = fmaxf(m, p[i]);
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < EPL; ++i) t += fast_exp2((p[i] - m) * kLog2e);
  // (four DPP exchange patterns whose composition reaches all 16 lanes of a row)
#define RF_MERGE_MT(CTRL)                                                          \
  {                                                                                \
    const float m_o = dpp_f32<CTRL>(m), t_o = dpp_f32<CTRL>(t);                    \
    const float m_n = fmaxf(m, m_o);                                               \
    t = t * fast_exp2((m - m_n) * kLog2e) + t_o * fast_exp2((m_o - m_n) * kLog2e); \
    m = m_n;                                                                       \
  }
  RF_MERGE_MT(kDppQuadXor1) RF_MERGE_MT(kDppQuadXor2) RF_MERGE_MT(kDppRowHalfMirror) RF_MERGE_MT(kDppRowMirror)
#undef RF_MERGE_MT
  const float inv_t = 1.0f / t;
  // stage 3: TopK.  Each round takes the largest remaining score of the token (ties: the
  // lowest expert index): lane-local best, then a 16-lane merge of (score, index) pairs.
  uint32_t taken = 0;
  float my_prob = 0.f;
  int my_idx = 0;
  for (int j = 0; j < topk; ++j) {
    float bv = -INFINITY;
    int bi = E;  // no candidate
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const bool ok = !((taken >> i) & 1u) && (p[i] > bv);  // strict: keeps the lowest index
      bv = ok ? p[i] : bv;
      bi = ok ? q * EPL + i : bi;
    }
#define RF_MERGE_TOP(CTRL)                                         \
  {                                                                \
    const float ov = dpp_f32<CTRL>(bv);                            \
    const int oi = dpp_i32<CTRL>(bi);                              \
    const bool take = (ov > bv) || (ov == bv && oi < bi);          \
    bv = take ? ov : bv;                                           \
    bi = take ? oi : bi;                                           \
  }
    RF_MERGE_TOP(kDppQuadXor1) RF_MERGE_TOP(kDppQuadXor2) RF_MERGE_TOP(kDppRowHalfMirror) RF_MERGE_TOP(kDppRowMirror)
#undef RF_MERGE_TOP
    if (bi / EPL == q && bi < E) taken |= 1u << (bi % EPL);
    if ((j & 15) == q) {
      my_prob = fast_exp2((bv - m) * kLog2e) * inv_t;
      my_idx = bi;
    }
  }
  if (live && q < topk) {
    prob[(int64_t)row * ldp + q] = my_prob;
    idx[(int64_t)row * ldi + q] = my_idx;
  }
}

template <int EPL>
__global__ __launch_bounds__(kCascadeThreads) void moe_cascade_kernel(
    const float* __restrict__ part, int KS, int S, int topk, float* __restrict__ prob,
    int32_t* __restrict__ idx, int64_t ldp, int64_t ldi) {
  constexpr int E = 16 * EPL;
  const int tid = threadIdx.x;
  const int q = tid & 15;
  const int row = blockIdx.x * (kCascadeThreads / 16) + (tid >> 4);
  const bool live = row < S;
  const int rrow = live ? row : S - 1;  // dead groups repeat the last token, store nothing

  // scores: slices added in slice order
  float p[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) p[i] = 0.f;
#pragma unroll 8
  for (int s = 0; s < KS; ++s) {
    const float* src = part + ((int64_t)s * S + rrow) * E + q * EPL;
#pragma unroll
    for (int i = 0; i < EPL; i += 2) {
      const float2 v = *reinterpret_cast<const float2*>(src + i);
      p[i] += v.x;
      p[i + 1] += v.y;
    }
  }
  moe_cascade_token<EPL>(p, q, row, live, topk, prob, idx, ldp, ldi);
}

// Device address of `scratch` on the current device, resolved once per device (with that
// device current) and kept.  Returns nullptr if the runtime cannot resolve the symbol.
static float* moe_static_scratch() {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> cache[kMaxDevices];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* ptr = cache[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return nullptr;
    cache[dev].store(ptr, std::memory_order_release);  // (two threads racing here store the same address)
  }
  return static_cast<float*>(ptr);
}

hipError_t launch_moe_routing_static(const void* x, const void* w, int S, int hd, int E, int topk,
                                     int64_t ldx, int64_t ldw, float* prob, int32_t* idx,
                                     int64_t ldp, int64_t ldi, hipStream_t s) {
  if ((size_t)moe_num_slices(S, hd) * (size_t)S * (size_t)E * sizeof(float) > kMoeStaticScratchBytes)
    return hipErrorInvalidValue;  // (the C-ABI layer has already refused this size)
  float* part = moe_static_scratch();
  if (part == nullptr) return hipErrorInvalidSymbol;
  // Nothing in the scratch array has to start at zero: the scores kernel writes every partial
  // score the cascade kernel reads, and what an earlier, larger call left behind is never read.
  return launch_moe_routing(x, w, S, hd, E, topk, ldx, ldw, prob, idx, ldp, ldi, part, s);
}

// Contraction axes of at most this length are not split: one launch, scores stay on chip.
// Measured on 2048 tokens: with only S/64 workgroups, each streaming all of w, the single
// segment wins at hd = 768 and 1024 (by half a microsecond per call under graph replay) and
// loses from hd = 2048 on (18 us against 11 us for 64 experts, 29 against 17.5 for 128).
constexpr int kMoeSingleSegmentMaxHd = 1024;

int moe_num_slices(int S, int hd) {
  if (hd <= kMoeSingleSegmentMaxHd) return 1;  // (one slice is still what the workspace query promises room for)
  const int n_rb = (S + kMoeRows - 1) / kMoeRows;
  const int n_kblocks = hd / kMoeKB;
  int ks = (256 + n_rb - 1) / n_rb;  // aim at one workgroup per CU
  if (ks > n_kblocks) ks = n_kblocks;
  if (ks > 64) ks = 64;
  if (ks < 1) ks = 1;
  return ks;
}

hipError_t launch_moe_routing(const void* x, const void* w, int S, int hd, int E, int topk,
                              int64_t ldx, int64_t ldw, float* prob, int32_t* idx, int64_t ldp,
                              int64_t ldi, float* part, hipStream_t s) {
  const int n_rb = (S + kMoeRows - 1) / kMoeRows;
  const int n_kblocks = hd / kMoeKB;
  const int KS = moe_num_slices(S, hd);
  // 32-bit lane offsets inside x and inside one 128-row tile of w
  if ((int64_t)S * ldx * 2 >= ((int64_t)1 << 32) || (int64_t)kMoeKB * ldw * 2 >= ((int64_t)1 << 32))
    return hipErrorInvalidValue;
  const dim3 grid1((unsigned)n_rb, (unsigned)KS), block(kMoeThreads);
  const bf16_t* xb = (const bf16_t*)x;
  const bf16_t* wb = (const bf16_t*)w;
  if (hd <= kMoeSingleSegmentMaxHd) {
    // single-segment strategy: scores GEMM and cascade in one kernel
    switch (E) {
      case 32: hipLaunchKernelGGL((moe_scores_kernel<1, true>), grid1, block, 0, s, xb, wb, part, S, n_kblocks, ldx, ldw, topk, prob, idx, ldp, ldi); break;
      case 64: hipLaunchKernelGGL((moe_scores_kernel<2, true>), grid1, block, 0, s, xb, wb, part, S, n_kblocks, ldx, ldw, topk, prob, idx, ldp, ldi); break;
      case 128: hipLaunchKernelGGL((moe_scores_kernel<4, true>), grid1, block, 0, s, xb, wb, part, S, n_kblocks, ldx, ldw, topk, prob, idx, ldp, ldi); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  switch (E) {
    case 32: hipLaunchKernelGGL((moe_scores_kernel<1, false>), grid1, block, 0, s, xb, wb, part, S, n_kblocks, ldx, ldw, topk, prob, idx, ldp, ldi); break;
    case 64: hipLaunchKernelGGL((moe_scores_kernel<2, false>), grid1, block, 0, s, xb, wb, part, S, n_kblocks, ldx, ldw, topk, prob, idx, ldp, ldi); break;
    case 128: hipLaunchKernelGGL((moe_scores_kernel<4, false>), grid1, block, 0, s, xb, wb, part, S, n_kblocks, ldx, ldw, topk, prob, idx, ldp, ldi); break;
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid2((unsigned)((S + kCascadeThreads / 16 - 1) / (kCascadeThreads / 16))), block2(kCascadeThreads);
  switch (E) {
    case 32: hipLaunchKernelGGL((moe_cascade_kernel<2>), grid2, block2, 0, s, part, KS, S, topk, prob, idx, ldp, ldi); break;
    case 64: hipLaunchKernelGGL((moe_cascade_kernel<4>), grid2, block2, 0, s, part, KS, S, topk, prob, idx, ldp, ldi); break;
    case 128: hipLaunchKernelGGL((moe_cascade_kernel<8>), grid2, block2, 0, s, part, KS, S, topk, prob, idx, ldp, ldi); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rf
