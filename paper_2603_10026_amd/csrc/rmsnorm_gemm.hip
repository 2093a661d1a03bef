// RMSNorm fused with a linear layer: the "sum + sum" cascade (paper Appendix
// A.2) in single-loop form.
//   stage 1: ss_i   = sum_k x[i,k]^2
//   stage 2: y[i,n] = sum_k (x[i,k] g[k]) w[k,n] * H(ss_i),  H(ss) = (ss/K + eps)^(-1/2)
// H does not depend on k, so the running state carries the H-free accumulator
// (Eq. (8)): one GEMM pass over K accumulates acc[i,n] = sum_k x g w with bf16
// MFMA (fp32 accumulate) while a side accumulator collects ss_i from the very
// same X tile on its way to LDS; the epilogue applies H(ss_i) once per row.
//
// Tiling.  One workgroup of 8 wavefronts owns a 128 (m) x 512 (n) output tile and
// walks K in steps of 64 through double-buffered LDS (one barrier per step).  The
// tile is wide in n because the X conversion below is vector-ALU work that every
// workgroup repeats for its rows: its cost per MFMA falls with the tile width.
// The product is computed transposed, Y^T = W^T (X g)^T, so that each accumulator
// lane owns one output row i (one H(ss_i) per lane) and four consecutive output
// columns per register group.
//   A operand = W^T: the W tile goes HBM -> LDS with direct-to-LDS 128-bit loads
//               and is read back with 64-bit LDS transpose reads.
//   B operand = (X g): x*g is rounded to bf16 once, in registers, on the way
//               from HBM to LDS; x^2 is accumulated there too.
// Each wavefront owns a 64 (n) x 128 (m) sub-tile: 32 MFMAs per K step.  The
// vector-ALU work of the X conversion for the NEXT step is cut into 8 pieces that
// are placed between those MFMAs, so the matrix pipe and the vector ALU run side
// by side inside every wavefront.
#include <type_traits>

#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

namespace {

constexpr int kGWaves = 8;
constexpr int kGThreads = kGWaves * kWave;
constexpr int kBM = 128, kBN = 512, kBKK = 64;
constexpr int kXTileB = kBM * kBKK * 2;   // 16 KB, [m][k], 128-byte rows
constexpr int kWRowB = kBN * 2;           // 1024-byte rows
constexpr int kWTileB = kBKK * kWRowB;    // 64 KB, [k][n]
constexpr int kXBase = 2 * kWTileB;              // W stages first, then the X stages
constexpr int kLdsB = 2 * kWTileB + 2 * kXTileB;  // 160 KB

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_cvoid;

// 16-byte slot swizzles (slot = piece ^ f(row)).
// X rows are 128 bytes = 8 slots.  The row bits are mixed so that both access shapes of the X
// stage are free of bank conflicts: the 128-bit stores of the staging role (four lanes per
// row, consecutive rows) and the 128-bit fragment reads (one row per lane).  Found by timing
// every XOR-linear 3-bit function of the low five row bits on the GPU; (row >> 1) & 7, the
// obvious choice, makes the stores 2-way conflicted.
__device__ __forceinline__ int fX(int row) {
  return ((row ^ (row >> 2)) & 1) | (((row ^ (row >> 3)) & 1) << 1) | (((row >> 1) & 1) << 2);
}
__device__ __forceinline__ int fW(int krow) { return (krow & 3) << 2; }

}  // namespace

__global__ __launch_bounds__(kGThreads, 1) void rmsnorm_gemm_bf16_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ g, const bf16_t* __restrict__ w,
    bf16_t* __restrict__ y, int M, int K, int N, int64_t ldx, int64_t ldw, int64_t ldy,
    float inv_k, float eps, int n_mtiles, int n_ntiles) {
  // [0, 128K): two W stages; [128K, 160K): two X stages
  __shared__ __attribute__((aligned(1024))) unsigned char lds[kLdsB];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;  // = 64-column block of the N tile
  const int i32 = lane & 31;
  const int hh = lane >> 5;

  // XCD-aware numbering: workgroups are dealt round-robin to the 8 XCDs, each with its
  // own L2.
  int mt, nt;
  {
    const int n_mt = gridDim.x / n_ntiles;
    if ((n_mt & 3) == 0 && (n_ntiles & 1) == 0) {
      // XCD x owns the block of (n_mt/4) x (n_ntiles/2) output tiles at block row x/2,
      // block column x%2, so that its L2 fetches few X row panels and W column panels.
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
  const int m0 = mt * kBM, n0 = nt * kBN;
  const int nk = K / kBKK;  // K is a multiple of 64 (checked by the caller)

  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;

  // ---- X staging role: a quarter row (16 k-values) per thread, in two 8-value pieces ----
  // Loads use a wave-uniform 64-bit base (advanced once per step on the scalar unit)
  // plus a loop-invariant 32-bit lane offset, so they cost no vector-ALU address math.
  const int xrow = tid >> 2;
  const int xq = tid & 3;
  const char* xbase = reinterpret_cast<const char*>(x + (int64_t)m0 * ldx);  // + step * 128 bytes
  const char* gbase = reinterpret_cast<const char*>(g);
  const uint32_t xlane_off = (uint32_t)(((int64_t)min(xrow, M - 1 - m0) * ldx + 16 * xq) * 2);
  const uint32_t glane_off = 32 * xq;
  uint32_t xdst_addr[2][2];  // [stage][piece]: LDS byte address
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    xdst_addr[0][c] = lds_base + kXBase + xrow * 128 + (((2 * xq + c) ^ fX(xrow)) << 4);
    xdst_addr[1][c] = xdst_addr[0][c] + kXTileB;
  }

  // ---- W direct-to-LDS role: 8 loads per wavefront per K step, one k-row each ----
  // Raw instructions: scalar base (w + step * 64 rows), 32-bit lane offset, LDS
  // destination of the wavefront's row in M0.
  uint32_t wsrc_off[8];  // byte offset from the tile's first row
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int krow = 8 * wave + e;
    const int piece = lane ^ fW(krow);
    const int ncol = min(n0 + 8 * piece, N - 8);
    wsrc_off[e] = (uint32_t)(((int64_t)krow * ldw + ncol) * 2);
  }
  const uint32_t wdst0 = __builtin_amdgcn_readfirstlane(lds_base + wave * 8 * kWRowB);
  const int64_t wstep_b = (int64_t)kBKK * ldw * 2;
#define RF_ISSUE_W(STEP, STAGE)                                                              \
  {                                                                                          \
    const char* wt_ = reinterpret_cast<const char*>(w) + (int64_t)(STEP) * wstep_b;          \
    _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                          \
      const uint32_t dst_ = wdst0 + (STAGE) * kWTileB + e * kWRowB;                          \
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"          \
                   :                                                                         \
                   : "s"(dst_), "v"(wsrc_off[e]), "s"(wt_)                                   \
                   : "memory", "m0");                                                        \
    }                                                                                        \
  }

  // ---- fragment read addresses (LDS byte addresses in stage 0) ----
  // B operand (X g): lane (i32, hh) of column tile mi reads row 32mi + i32, slot 2kk + hh
  uint32_t xaddr[2][4];  // [stage][kk]; + mi * 32 * 128
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    xaddr[0][kk] = lds_base + kXBase + i32 * 128 + (((2 * kk + hh) ^ fX(i32)) << 4);
    xaddr[1][kk] = xaddr[0][kk] + kXTileB;
  }
  // A operand (W^T) by transpose reads: lane = 32hh + 16g2 + 4j + a reads 8 bytes of k-row
  // 16kk + 8hh + 4w2 + j at column 64wave + 32ni + 16g2 + 4a
  uint32_t waddr[2][2][2];  // [stage][ni][w2]; + kk * 16 * kWRowB
  {
    const int i16 = lane & 15, g2 = (lane >> 4) & 1;
    const int j = i16 >> 2, a = i16 & 3;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int w2 = 0; w2 < 2; ++w2) {
        const int krow = 8 * hh + 4 * w2 + j;
        const int piece = (64 * wave + 32 * ni + 16 * g2 + 4 * a) >> 3;
        waddr[0][ni][w2] = lds_base + krow * kWRowB + ((piece ^ fW(krow)) << 4) + 8 * (a & 1);
        waddr[1][ni][w2] = waddr[0][ni][w2] + kWTileB;
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

  // X and g pieces travel through registers.  Their loads are raw instructions with
  // hand-placed waits: all vector-memory traffic of the main loop is ordered by hand so
  // that the prefetches stay in flight across barriers.  Piece c of a step is fetched
  // right after piece c of the previous step has been converted (same registers).
  u32x4 xreg[2], greg[2];
#define RF_LOAD_PIECE(C, STEP)                                                               \
  {                                                                                          \
    const char* xp_ = xbase + (int64_t)(STEP) * (kBKK * 2);                                  \
    const char* gp_ = gbase + (int64_t)(STEP) * (kBKK * 2);                                  \
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3"                                  \
                 : "=v"(xreg[C]) : "v"(xlane_off), "s"(xp_), "n"(16 * (C)));                 \
    asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3"                                  \
                 : "=v"(greg[C]) : "v"(glane_off), "s"(gp_), "n"(16 * (C)));                 \
  }
  // wait until at most PENDING younger vector-memory operations are in flight
#define RF_WAIT_PIECE(C, PENDING) \
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(xreg[C]), "+v"(greg[C]) : "n"(PENDING));
  // one bf16 pair of piece C: stage-1 side sum and the g scaling
#define RF_CONVERT_PAIR(C, J)                                                                \
  {                                                                                          \
    /* ss += x_lo^2 + x_hi^2 in one instruction (written out: the builtin applied to an   */ \
    /* element of a 4-vector was seen to read element 0 every time)                       */ \
    asm("v_dot2c_f32_bf16 %0, %1, %1" : "+v"(ss) : "v"(xreg[C][J]));                         \
    conv[J] = pack_bf16(bf16_lo(xreg[C][J]) * bf16_lo(greg[C][J]),                           \
                        bf16_hi(xreg[C][J]) * bf16_hi(greg[C][J]));                          \
  }
  // raw LDS write (the compiler would order an ordinary one behind the direct-to-LDS
  // loads still in flight)
#define RF_STORE_PIECE(C, STAGE) \
  asm volatile("ds_write_b128 %0, %1" : : "v"(xdst_addr[STAGE][C]), "v"(conv) : "memory");

  // ---- prologue: W tile 0 in flight, X tile 0 converted, X tile 1 in flight ----
  RF_ISSUE_W(0, 0)
  {
    u32x4 conv;
    RF_LOAD_PIECE(0, 0) RF_LOAD_PIECE(1, 0)
    RF_WAIT_PIECE(0, 0) RF_WAIT_PIECE(1, 0)
    RF_CONVERT_PAIR(0, 0) RF_CONVERT_PAIR(0, 1) RF_CONVERT_PAIR(0, 2) RF_CONVERT_PAIR(0, 3)
    RF_STORE_PIECE(0, 0)
    RF_CONVERT_PAIR(1, 0) RF_CONVERT_PAIR(1, 1) RF_CONVERT_PAIR(1, 2) RF_CONVERT_PAIR(1, 3)
    RF_STORE_PIECE(1, 0)
    RF_LOAD_PIECE(0, min(1, nk - 1)) RF_LOAD_PIECE(1, min(1, nk - 1))
  }

  // ---- main loop ----
  // Step s multiplies out of stage s%2, converts X tile s+1 into X stage (s+1)%2, fetches
  // X tile s+2 into registers and W tile s+1 into W stage (s+1)%2.  Every step runs the
  // same straight-line code: past the end of K the prefetches re-read the last tile
  // (harmless: nothing consumes it), and the side sum is taken from a snapshot made
  // before the last step's surplus conversion.
  // Vector-memory issue order per step: 8 W loads, then (x, g) of piece 0 and of piece
  // 1; loads retire in order, which fixes the counts in the waits: the loads of piece c
  // were issued one step earlier and 10 younger operations follow them; at the top of a
  // step the 8 W loads of its tile are followed by the 4 piece loads of the previous
  // step.  Fragment reads and piece writes are raw LDS instructions with hand-placed
  // waits (the compiler would otherwise wait for the in-flight direct-to-LDS loads
  // before every LDS access).
  float ss_done = 0.f;
  // Fragment registers, two buffers.  They outlive a step: the 8 MFMAs of a step's last
  // contraction step are issued only after the NEXT step's barrier, while that step's first
  // fragment reads are on their way (their operands sit in buffer 1 across the barrier).
  // Without this the matrix pipe idles from the barrier until the first fragments arrive,
  // with both wavefronts of every SIMD waiting for the same thing.
  u32x2 af[2][2][2];  // [buffer][ni][w2]
  u32x4 bfr[2][4];    // [buffer][mi]
#pragma unroll
  for (int ni = 0; ni < 2; ++ni)
#pragma unroll
    for (int w2 = 0; w2 < 2; ++w2) af[1][ni][w2] = u32x2{0u, 0u};  // (the first step has nothing deferred:
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) bfr[1][mi] = u32x4{0u, 0u, 0u, 0u};  //  zero operands add nothing)
  auto k_step = [&](int s, auto stage_tag) {
    constexpr int ST = decltype(stage_tag)::value;  // LDS stage of this step (= s % 2)
    ss_done = ss;  // complete once s is the last step
    // W tile s has landed; our own LDS writes of the previous step are done, and so are its
    // fragment reads (buffer 1 is complete)
    asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();  // stages of step s complete; stages of step s-1 free

    u32x4 conv;
#define RF_ISSUE(BUFR, KK)                                                                   \
  _Pragma("unroll") for (int ni = 0; ni < 2; ++ni) {                                         \
    _Pragma("unroll") for (int w2 = 0; w2 < 2; ++w2) asm volatile(                           \
        "ds_read_b64_tr_b16 %0, %1 offset:%2"                                                \
        : "=v"(af[BUFR][ni][w2])                                                             \
        : "v"(waddr[ST][ni][w2]), "n"((KK) * 16 * kWRowB));                                  \
  }                                                                                          \
  _Pragma("unroll") for (int mi = 0; mi < 4; ++mi) asm volatile(                             \
      "ds_read_b128 %0, %1 offset:%2"                                                        \
      : "=v"(bfr[BUFR][mi])                                                                  \
      : "v"(xaddr[ST][KK]), "n"(mi * 32 * 128));
#define RF_WAIT(BUFR, PENDING)                                                               \
  asm volatile("s_waitcnt lgkmcnt(%8)"                                                       \
               : "+v"(af[BUFR][0][0]), "+v"(af[BUFR][0][1]), "+v"(af[BUFR][1][0]),           \
                 "+v"(af[BUFR][1][1]), "+v"(bfr[BUFR][0]), "+v"(bfr[BUFR][1]),               \
                 "+v"(bfr[BUFR][2]), "+v"(bfr[BUFR][3])                                      \
               : "n"(PENDING));
#define RF_MFMA4(BUFR, NI)                                                                   \
  {                                                                                          \
    u32x4 a_;                                                                                \
    a_[0] = af[BUFR][NI][0][0]; a_[1] = af[BUFR][NI][0][1];                                  \
    a_[2] = af[BUFR][NI][1][0]; a_[3] = af[BUFR][NI][1][1];                                  \
    _Pragma("unroll") for (int mi = 0; mi < 4; ++mi) acc[NI][mi] =                           \
        __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_),              \
                                                __builtin_bit_cast(bf16x8, bfr[BUFR][mi]),   \
                                                acc[NI][mi], 0, 0, 0);                       \
  }
    // the 8 MFMAs of one contraction step out of fragment buffer BUFR, with pairs J0 and
    // J0+1 of piece C converted between them
#define RF_GROUP(BUFR, C, J0)                                                                \
  if constexpr ((J0) == 0) { RF_WAIT_PIECE(C, 10) }                                          \
  RF_MFMA4(BUFR, 0)                                                                          \
  RF_CONVERT_PAIR(C, J0)                                                                     \
  __builtin_amdgcn_sched_barrier(0);                                                         \
  RF_MFMA4(BUFR, 1)                                                                          \
  RF_CONVERT_PAIR(C, (J0) + 1)                                                               \
  if constexpr ((J0) == 2) {                                                                 \
    RF_STORE_PIECE(C, ST ^ 1)                                                                \
    RF_LOAD_PIECE(C, min(s + 2, nk - 1))                                                     \
  }                                                                                          \
  __builtin_amdgcn_sched_barrier(0);

    RF_ISSUE(0, 0)
    // (issued while the first fragments are on their way)
    RF_ISSUE_W(min(s + 1, nk - 1), ST ^ 1)
    // the previous step's last contraction step, out of buffer 1
    RF_MFMA4(1, 0)
    RF_MFMA4(1, 1)
    __builtin_amdgcn_sched_barrier(0);
    RF_ISSUE(1, 1)
    RF_WAIT(0, 8)
    RF_GROUP(0, 0, 0)
    RF_ISSUE(0, 2)
    RF_WAIT(1, 8)
    RF_GROUP(1, 0, 2)
    RF_ISSUE(1, 3)
    RF_WAIT(0, 8)
    RF_GROUP(0, 1, 0)
    // the last contraction step: its fragments must be back before the next barrier (the stage
    // is overwritten after it); its conversion work is done here, its MFMAs after that barrier
    RF_WAIT(1, 0)
    RF_CONVERT_PAIR(1, 2)
    RF_CONVERT_PAIR(1, 3)
    RF_STORE_PIECE(1, ST ^ 1)
    RF_LOAD_PIECE(1, min(s + 2, nk - 1))
    __builtin_amdgcn_sched_barrier(0);
#undef RF_ISSUE
#undef RF_WAIT
#undef RF_MFMA4
#undef RF_GROUP
  };
  for (int s = 0; s < nk; s += 2) {
    k_step(s, std::integral_constant<int, 0>{});
    if (s + 1 < nk) k_step(s + 1, std::integral_constant<int, 1>{});
  }
  // the last step's deferred contraction step
#define RF_MFMA4(BUFR, NI)                                                                   \
  {                                                                                          \
    u32x4 a_;                                                                                \
    a_[0] = af[BUFR][NI][0][0]; a_[1] = af[BUFR][NI][0][1];                                  \
    a_[2] = af[BUFR][NI][1][0]; a_[3] = af[BUFR][NI][1][1];                                  \
    _Pragma("unroll") for (int mi = 0; mi < 4; ++mi) acc[NI][mi] =                           \
        __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_),              \
                                                __builtin_bit_cast(bf16x8, bfr[BUFR][mi]),   \
                                                acc[NI][mi], 0, 0, 0);                       \
  }
  RF_MFMA4(1, 0)
  RF_MFMA4(1, 1)
#undef RF_MFMA4
  ss = ss_done;
  // (the registers of the surplus prefetch stay reserved until it has landed)
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)"
               : "+v"(xreg[0]), "+v"(xreg[1]), "+v"(greg[0]), "+v"(greg[1])
               :
               : "memory");
#undef RF_LOAD_PIECE
#undef RF_ISSUE_W
#undef RF_WAIT_PIECE
#undef RF_CONVERT_PAIR
#undef RF_STORE_PIECE

  // stage 1 result: the four lanes that share an X row add their partial sums.  The
  // per-row factors go through LDS (W stage 0 is free once every wavefront has left the
  // loop).
  float* s_rstd = reinterpret_cast<float*>(lds);
  ss += dpp_f32<kDppQuadXor1>(ss);
  ss += dpp_f32<kDppQuadXor2>(ss);
  __syncthreads();
  if (xq == 0) s_rstd[xrow] = 1.0f / sqrtf(ss * inv_k + eps);
  __syncthreads();

  // epilogue: y = acc * H(ss)
  // An accumulator lane holds one output row, four columns at a time: stored from there, an
  // instruction would touch 32 rows with 16 bytes each.  When the output allows 16-byte stores,
  // a wavefront stages its 128 x 64 sub-tile in LDS (all stages are free by now; rows of 128
  // bytes, 16-byte slots XOR-swizzled with the row) and stores whole 128-byte row segments.
  const bool wide_ok = (reinterpret_cast<uintptr_t>(y) & 15) == 0 && (ldy & 7) == 0;
  if (wide_ok) {
    unsigned char* stage = lds + 1024 + wave * (kBM * 128);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      const int row = 32 * mi + i32;
      const float rs = s_rstd[row];
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          u32x2 o2;
          o2[0] = pack_bf16(acc[ni][mi][4 * r4] * rs, acc[ni][mi][4 * r4 + 1] * rs);
          o2[1] = pack_bf16(acc[ni][mi][4 * r4 + 2] * rs, acc[ni][mi][4 * r4 + 3] * rs);
          *reinterpret_cast<u32x2*>(stage + row * 128 + (((4 * ni + r4) ^ ((row >> 1) & 7)) << 4) + 8 * hh) = o2;
        }
    }
#pragma unroll
    for (int i = 0; i < kBM / 8; ++i) {
      const int row = 8 * i + (lane >> 3);
      const int slot = lane & 7;
      const u32x4 o4 = *reinterpret_cast<const u32x4*>(stage + row * 128 + ((slot ^ ((row >> 1) & 7)) << 4));
      const int m = m0 + row;
      const int n = n0 + 64 * wave + 8 * slot;
      if (m < M) {
        bf16_t* dst = y + (int64_t)m * ldy + n;
        if (n + 8 <= N) {
          // (non-temporal: the output is not read again here, and leaving it in L2 costs the
          // X and W panels their place: measured 1 % on 4096^3)
          __builtin_nontemporal_store(o4, reinterpret_cast<u32x4*>(dst));
        } else if (n + 4 <= N) {
          u32x2 o2;
          o2[0] = o4[0];
          o2[1] = o4[1];
          *reinterpret_cast<u32x2*>(dst) = o2;
        }
      }
    }
    return;
  }
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int mloc = 32 * mi + i32;
    const int m = m0 + mloc;
    const float rs = s_rstd[mloc];
    if (m >= M) continue;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int n = n0 + 64 * wave + 32 * ni + 8 * r4 + 4 * hh;
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
  // 32-bit byte offsets: inside a 64-row tile of w, inside a 128-row tile of x (the C-ABI
  // layer rejects such pitches as unsupported before it gets here)
  if (ldw >= (1 << 24) || ldx >= (1 << 24)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rmsnorm_gemm_bf16_kernel, dim3((unsigned)grid), dim3(kGThreads), 0, s,
                     (const bf16_t*)x, (const bf16_t*)g, (const bf16_t*)w, (bf16_t*)y, M, K, N, ldx,
                     ldw, ldy, 1.0f / (float)K, eps, n_mtiles, n_ntiles);
  return hipGetLastError();
}

}  // namespace rf
