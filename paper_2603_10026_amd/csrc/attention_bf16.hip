// bf16 fused attention, single-segment strategy (paper Section 4.3; Appendix
// A.2 incremental forms; Appendix A.4 tile-level structure), bf16 MFMA
// 32x32x16 with fp32 accumulation.
//
// One workgroup (4 or 8 wavefronts) owns 128 or 256 query rows of one (batch, head); each
// wavefront owns 32 of them as the N dimension of its MFMA tiles and streams
// the keys in tiles of 64, carrying the running state (m, l, acc) of the
// max -> sum-exp -> weighted-sum cascade.  acc stays unnormalised (Eq. (8))
// and is divided by l once in the epilogue.
//
//   S^T = K Q^T        A = K tile (LDS), B = Q^T (registers, loaded once)
//   O^T += V^T P^T     A = V^T (LDS transpose reads of the V tile), B = P^T
//
// Computing the scores transposed makes the accumulator layout of S^T (lane =
// query column, registers = key rows) coincide with the B-operand layout of
// the second product, so probabilities go from fp32 accumulators to bf16
// operands without leaving their lane.
//
// Data movement: K and V tiles go from HBM straight into LDS with 128-bit
// direct-to-LDS loads (no staging registers), double-buffered, one barrier per
// tile.  Rows are XOR-swizzled in 16-byte slots so that both the 128-bit
// A-operand reads of K and the 64-bit transpose reads of V are free of bank
// conflicts.  Two workgroups fit on a compute unit, so the softmax VALU work
// of one overlaps the MFMA work of the other.
//
// The reference point m of the state is only advanced when a tile's row max
// exceeds it by more than kTau (in log2 units): (m, l, acc) with any common
// reference gives the same O = acc / l, exponentials stay below 2^kTau, and
// the rescale of acc (the correction step of the incremental form) is skipped
// on almost every tile.
#include <type_traits>

#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

namespace {

// NW wavefronts of 32 query rows each per workgroup: 4 (two workgroups per CU) or 8 (one
// workgroup per CU; half the K/V loads and LDS traffic per MFMA)
constexpr int kBK = 64;   // keys per tile
constexpr float kTau = 8.0f;

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;

// 16-byte slot swizzles (slot = piece ^ f(row)).
template <int D>
__device__ __forceinline__ int fK(int row) {
  return (D == 128) ? (row & 15) : ((row >> 1) & 7);
}
template <int D>
__device__ __forceinline__ int fV(int row) {
  return (D == 128) ? (((row & 3) << 2) | ((row >> 2) & 3))
                    : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

__device__ __forceinline__ void wait_vmem_all() {
  // vmcnt(0), expcnt and lgkmcnt untouched (gfx9 encoding)
  __builtin_amdgcn_s_waitcnt(0x0F70);
}

}  // namespace

template <int D, int NW, bool PAIRED>
__global__ __launch_bounds__(NW * kWave, NW == 4 ? 2 : 1) void attention_bf16_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    bf16_t* __restrict__ o, Strides4 sq, Strides4 sk, Strides4 sv, Strides4 so, int Hq, int Hkv,
    int Lq, int Lk, float scale_log2e, int causal, int n_qtiles) {
  constexpr bool paired = PAIRED;
  constexpr int KS = D / 16;                 // contraction steps of S^T = K Q^T
  constexpr int DT = D / 32;                 // 32-row tiles of O^T
  constexpr int P = D / 8;                   // 16-byte slots per K/V row
  constexpr int ROWB = D * 2;                // bytes per K/V row
  constexpr int TILEB = kBK * ROWB;          // bytes per K or V tile
  constexpr int ROWS_PER_LD = 1024 / ROWB;   // rows covered by one wavefront load
  constexpr int kWaves = NW;
  constexpr int kBQ = 32 * NW;               // query rows per workgroup
  constexpr int LD_PER_WAVE = kBK / ROWS_PER_LD / kWaves;

  // Two K/V slots.  Layout: the K slots, then the V slots; the K address registers point at the
  // first K slot, the V registers at the first V slot.
  constexpr int NS = 2;
  __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * NS * TILEB];  // [K,V][slot]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int i32 = lane & 31;
  const int hh = lane >> 5;

  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Renumber
  // them so that an XCD owns a contiguous range of heads: the query tiles of one head
  // then share that head's K/V in one L2.
  //  - no mask: head-major inside the XCD, so all query tiles of a head run together and
  //    each K/V tile is fetched into the L2 once;
  //  - causal mask, one tile per workgroup: query-tile-major, heaviest first.  The late query
  //    tiles see the most keys; starting all of them before any light tile keeps the tail of
  //    the launch short;
  //  - causal mask, two tiles per workgroup (PAIRED): all workgroups are equally heavy, so the
  //    head-major order of the unmasked case applies.
  int qt, bh;
  const int n_units = paired ? n_qtiles / 2 : n_qtiles;  // workgroups per head
  const int n_bh = gridDim.x / n_units;
  if ((n_bh & 7) == 0) {
    const int hx = n_bh >> 3;            // heads per XCD
    const int xcd = blockIdx.x & 7;
    const int j = blockIdx.x >> 3;       // arrival order inside the XCD
    if (causal && !paired) {
      qt = n_qtiles - 1 - j / hx;
      bh = xcd * hx + j % hx;
    } else {
      qt = j % n_units;
      bh = xcd * hx + j / n_units;
    }
  } else {
    qt = n_units - 1 - (int)(blockIdx.x / n_bh);
    bh = blockIdx.x % n_bh;
  }
  // (integer division runs on the vector unit even for wave-uniform operands: hand the results
  // back to the scalar unit here, once, so that everything derived from them, the K/V base
  // pointers of the direct-to-LDS loads above all, is scalar)
  qt = __builtin_amdgcn_readfirstlane(qt);
  bh = __builtin_amdgcn_readfirstlane(bh);
  const int h = __builtin_amdgcn_readfirstlane(bh % Hq);
  const int b = __builtin_amdgcn_readfirstlane(bh / Hq);
  const int hk = __builtin_amdgcn_readfirstlane(h / (Hq / Hkv));
  const bf16_t* qb = q + (int64_t)b * sq.b + (int64_t)h * sq.h;
  const bf16_t* kb = k + (int64_t)b * sk.b + (int64_t)hk * sk.h;
  const bf16_t* vb = v + (int64_t)b * sv.b + (int64_t)hk * sv.h;

  const bool scale_negative = scale_log2e < 0.f, scale_zero = scale_log2e == 0.f;
  scale_log2e = scale_zero ? 1.0f : fabsf(scale_log2e);

  // ---- direct-to-LDS load geometry: this lane's row / slot in each of its loads ----
  // load e of a wavefront covers rows (wave * LD_PER_WAVE + e) * ROWS_PER_LD + lane / P, one
  // 16-byte slot per lane; the slot holds the piece that the swizzle puts there
  auto ld_row = [&](int e, int ln) { return (wave * LD_PER_WAVE + e) * ROWS_PER_LD + ln / P; };
  auto ld_col = [&](int e, int ln, int is_v) {  // element offset inside the global row
    const int row = ld_row(e, ln), slot = ln % P;
    return 8 * (slot ^ (is_v ? fV<D>(row) : fK<D>(row)));
  };
  uint32_t ld_koff[LD_PER_WAVE], ld_voff[LD_PER_WAVE];  // byte offsets from the tile's first row
#pragma unroll
  for (int e = 0; e < LD_PER_WAVE; ++e) {
    ld_koff[e] = (uint32_t)(((int64_t)ld_row(e, lane) * sk.l + ld_col(e, lane, 0)) * 2);
    ld_voff[e] = (uint32_t)(((int64_t)ld_row(e, lane) * sv.l + ld_col(e, lane, 1)) * 2);
  }
  // byte offsets stay below 2^32 inside one 64-row tile only if the row stride does
  const bool small_stride = sk.l < (1 << 24) && sv.l < (1 << 24);
  // One direct-to-LDS load of this wavefront's share of the tile at key0: load e of K
  // (is_v = 0) or of V (is_v = 1) into buffer buf.
  const uint32_t lds_base =
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;
  // LDS address of this wavefront's first load in K slot 0, on the scalar unit
  const uint32_t dma_base = __builtin_amdgcn_readfirstlane(lds_base + wave * LD_PER_WAVE * 1024);
  auto issue_one = [&](int key0, int buf, int e, int is_v) {
    const uint32_t dst_addr = dma_base + is_v * NS * TILEB + buf * TILEB + e * 1024;
    const bf16_t* base = is_v ? vb : kb;
    const int64_t ld = is_v ? sv.l : sk.l;
    if (key0 + kBK <= Lk && small_stride) {
      // full tile: uniform tile base + per-lane 32-bit offset, no per-load address math
      // (raw instruction: scalar base + 32-bit lane offset, LDS destination in M0)
      const char* tile = reinterpret_cast<const char*>(base) + (int64_t)key0 * ld * 2;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(dst_addr), "v"(is_v ? ld_voff[e] : ld_koff[e]), "s"(tile)
                   : "memory", "m0");
    } else {
      // ragged last tile: rows past the end re-read the last key (masked later).  The same raw
      // instruction with a 64-bit lane address: every direct-to-LDS load of this kernel goes
      // through one mechanism, so M0 is only ever written here, in statements that declare it
      // as clobbered.
      // (an opaque copy of the lane number: the address pieces of this rare path are then
      // computed here, not ahead of the loop, where they would occupy registers all along)
      int ln = lane;
      asm volatile("" : "+v"(ln));
      const int key = min(key0 + ld_row(e, ln), Lk - 1);
      const bf16_t* src = base + (int64_t)key * ld + ld_col(e, ln, is_v);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                   :
                   : "s"(dst_addr), "v"(src)
                   : "memory", "m0");
    }
  };
  auto issue_loads = [&](int key0, int buf) {
#pragma unroll
    for (int e = 0; e < LD_PER_WAVE; ++e) {
      issue_one(key0, buf, e, 0);
      issue_one(key0, buf, e, 1);
    }
  };

  // The first K/V tile of the workgroup's first query tile is requested here, before the rest of
  // the set-up (LDS read offsets, Q fragments, masks): the trip to memory then overlaps it.
  {
    const int last_row0 = min(Lq - 1, qt * kBQ + kBQ - 1);
    const int wg_last0 = causal ? min(Lk - 1, last_row0 + (Lk - Lq)) : Lk - 1;
    if (wg_last0 >= 0) issue_loads(0, 0);
  }

  // ---- LDS read offsets (loop invariant) ----
  // K fragment of contraction step kk: row i32 (+ 32 rt), slot (2 kk + hh) ^ fK.  The slot index
  // is an XOR and the row pitch is a multiple of 256, so step kk's address is step 0's with
  // kk << 5 XOR-ed in: one register instead of one per step.
  uint32_t koff0 = i32 * ROWB + ((hh ^ fK<D>(i32)) << 4);  // LDS byte address in slot 0; + rt * 32 * ROWB
  static_assert(ROWB % 256 == 0 || (KS - 1) << 5 < ROWB, "kk << 5 stays inside the row");
  // transpose reads of V: lane = 32hh + 16g2 + 4j + a reads 8 bytes of key row
  // (16u + 8w + 4hh + j) at head-dim offset 32t + 16g2 + 4a; the 16-lane group gets,
  // in lane 4a + e, keys j = 0..3 of head-dim 32t + 16g2 + 4a + e.
  // (head-dim tile t enters the slot index as 4 t under an XOR: its address is tile 0's with
  // t << 6 XOR-ed in)
  uint32_t voff0[2];  // [w2], tile t = 0; + u * 16 * ROWB
  {
    const int i16 = lane & 15, g2 = (lane >> 4) & 1;
    const int j = i16 >> 2, a = i16 & 3;
#pragma unroll
    for (int w2 = 0; w2 < 2; ++w2) {
      const int row = 8 * w2 + 4 * hh + j;
      const int piece = 2 * g2 + (a >> 1);
      voff0[w2] = row * ROWB + (((piece ^ fV<D>(row)) & (P - 1)) << 4) + 8 * (a & 1);
    }
  }

  voff0[0] += lds_base + NS * TILEB;
  voff0[1] += lds_base + NS * TILEB;
  koff0 += lds_base;

  // Under a causal mask a workgroup may own two query tiles of its head, the one that sees the
  // most keys paired with the one that sees the fewest and so on inwards: every workgroup of the
  // launch then does the same amount of work.
#pragma nounroll
  for (int pass = 0; pass < (PAIRED ? 2 : 1); ++pass) {
  if (pass) {
    qt = n_qtiles - 1 - qt;
    __syncthreads();  // the last tile of the first pass has been read by every wavefront
  }
  const int q0 = qt * kBQ;
  // Q^T fragments: slot (hh, e) of step kk stands for d = 16kk + 8hh + e
  const int my_q = q0 + wave * 32 + i32;
  u32x4 qf[KS];
  {
    const bf16_t* qp = qb + (int64_t)min(my_q, Lq - 1) * sq.l + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = *reinterpret_cast<const u32x4*>(qp + 16 * kk);
  }
  // The loop below needs a positive scale (row max taken on raw scores, masked
  // scores set to -inf before scaling): fold the sign of the scale into Q, and
  // turn scale == 0 (uniform weights) into Q = 0 with scale 1.
  if (scale_negative) {
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] ^= 0x80008000u;
  } else if (scale_zero) {
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = u32x4{0u, 0u, 0u, 0u};
  }

  const int shift = Lk - Lq;
  const int my_last = causal ? min(Lk - 1, my_q + shift) : Lk - 1;
  const int wave_min_last = causal ? min(Lk - 1, q0 + wave * 32 + shift) : Lk - 1;
  const int wave_last = causal ? min(Lk - 1, min(Lq - 1, q0 + wave * 32 + 31) + shift) : Lk - 1;
  const int wg_last = causal ? min(Lk - 1, min(Lq - 1, q0 + kBQ - 1) + shift) : Lk - 1;
  const int n_ktiles = wg_last >= 0 ? wg_last / kBK + 1 : 0;

  float m_ref = -INFINITY, l = 0.f;
  f32x16 acc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  // K fragments of one tile: all of them are requested at once (LDS latency is paid once per
  // tile, not once per contraction step), as raw instructions waited for by hand: through the
  // compiler they would wait for the direct-to-LDS loads in flight.
  // (the addresses are formed from an opaque copy of the base, here and for V below: otherwise
  // the compiler forms all of them ahead of the loop and carries them in registers)
#define RF_ISSUE_K(KF, SLOT)                                                              \
  {                                                                                       \
    uint32_t kb_ = koff0;                                                                 \
    asm volatile("" : "+v"(kb_));                                                         \
    _Pragma("unroll") for (int kk = 0; kk < KS; ++kk) {                                   \
      const uint32_t ka_ = kb_ ^ (kk << 5);                                               \
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(KF[kk][0]) : "v"(ka_), "n"((SLOT) * TILEB)); \
      asm volatile("ds_read_b128 %0, %1 offset:%2"                                        \
                   : "=v"(KF[kk][1]) : "v"(ka_), "n"((SLOT) * TILEB + 32 * ROWB));        \
    }                                                                                     \
  }

  // One key tile.  BUF is a compile-time constant so that every LDS access of the tile is a
  // register plus an immediate offset.
  auto tile_step = [&](int kt, auto buf_tag) {
    constexpr int BUF = decltype(buf_tag)::value;
    constexpr int FILL = BUF ^ 1;   // slot of the tile requested during this one
    const int key0 = kt * kBK;
    wait_vmem_all();   // this wavefront's share of tile kt has landed
    __syncthreads();   // everyone's share has landed; everyone is done reading the other slot
    const bool more = kt + 1 < n_ktiles;
    if (key0 > wave_last) {  // nothing visible for this wavefront (uniform): only fetch its share
      if (more) issue_loads(key0 + kBK, FILL);
      return;
    }
    u32x4 kq[KS][2];
    RF_ISSUE_K(kq, BUF)

    // ---- S^T = K Q^T : two 32-key row tiles ----
    f32x16 s[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[rt][r] = 0.f;
    __builtin_amdgcn_sched_barrier(0);
    // The loads of the next tile are issued one at a time between the MFMAs.  Issued in a
    // burst right after the barrier, the eight wavefronts of a CU queue up behind each
    // other in the vector-memory unit and every one of them idles for the whole burst.
    constexpr int kIssueEvery = KS / (2 * LD_PER_WAVE);  // contraction steps per load
    static_assert(kIssueEvery * 2 * LD_PER_WAVE == KS, "loads spread evenly over the contraction steps");
    static_assert(2 * (KS - 1) <= 15, "the wait counts below fit the LDS counter");
    auto st_step = [&](auto kk_tag) {
      constexpr int kk = decltype(kk_tag)::value;
      // the two fragments of this step are back once at most the younger ones are in flight
      u32x4& k0 = kq[kk][0];
      u32x4& k1 = kq[kk][1];
      asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(k0), "+v"(k1) : "n"(2 * (KS - 1 - kk)));
      s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, k0),
                                                     __builtin_bit_cast(bf16x8, qf[kk]), s[0], 0, 0, 0);
      s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, k1),
                                                     __builtin_bit_cast(bf16x8, qf[kk]), s[1], 0, 0, 0);
      if (more && kk % kIssueEvery == 0)
        issue_one(key0 + kBK, FILL, (kk / kIssueEvery) >> 1, (kk / kIssueEvery) & 1);
      __builtin_amdgcn_sched_barrier(0);
    };
    st_step(std::integral_constant<int, 0>{});
    st_step(std::integral_constant<int, 1>{});
    st_step(std::integral_constant<int, 2>{});
    st_step(std::integral_constant<int, 3>{});
    if constexpr (KS > 4) {
      st_step(std::integral_constant<int, 4>{});
      st_step(std::integral_constant<int, 5>{});
      st_step(std::integral_constant<int, 6>{});
      st_step(std::integral_constant<int, 7>{});
    }
    static_assert(KS == 4 || KS == 8, "contraction steps written out above");
    // ---- V^T fragments of the first two contraction steps: requested now, they arrive
    //      while the softmax below runs on the vector ALU ----
    // The transpose reads are issued as raw instructions and waited for by hand:
    // going through the compiler's intrinsic would make it wait for the
    // direct-to-LDS loads of the NEXT tile before every read of this one.
    u32x2 va[2][DT][2];
    uint32_t vb_[2] = {voff0[0], voff0[1]};
    asm volatile("" : "+v"(vb_[0]), "+v"(vb_[1]));
#define RF_ISSUE_V(STAGE, U)                                                              \
  _Pragma("unroll") for (int t = 0; t < DT; ++t) {                                        \
    _Pragma("unroll") for (int w2 = 0; w2 < 2; ++w2) asm volatile(                        \
        "ds_read_b64_tr_b16 %0, %1 offset:%2"                                             \
        : "=v"(va[STAGE][t][w2])                                                          \
        : "v"(vb_[w2] ^ (t << 6)), "n"(BUF * TILEB + (U) * 16 * ROWB));                   \
  }
    // wait until at most PENDING transpose reads are still in flight; the registers of
    // STAGE are tied to the wait so that their uses stay behind it
#define RF_WAIT_V(STAGE, PENDING)                                                         \
  if constexpr (DT == 4)                                                                  \
    asm volatile("s_waitcnt lgkmcnt(%8)"                                                  \
                 : "+v"(va[STAGE][0][0]), "+v"(va[STAGE][0][1]), "+v"(va[STAGE][1][0]),   \
                   "+v"(va[STAGE][1][1]), "+v"(va[STAGE][2][0]), "+v"(va[STAGE][2][1]),   \
                   "+v"(va[STAGE][3][0]), "+v"(va[STAGE][3][1])                           \
                 : "n"(PENDING));                                                         \
  else                                                                                    \
    asm volatile("s_waitcnt lgkmcnt(%4)"                                                  \
                 : "+v"(va[STAGE][0][0]), "+v"(va[STAGE][0][1]), "+v"(va[STAGE][1][0]),   \
                   "+v"(va[STAGE][1][1])                                                  \
                 : "n"(PENDING));
#define RF_PV_STEP(STAGE, U)                                                              \
  _Pragma("unroll") for (int t = 0; t < DT; ++t) {                                        \
    u32x4 a;                                                                              \
    a[0] = va[STAGE][t][0][0]; a[1] = va[STAGE][t][0][1];                                 \
    a[2] = va[STAGE][t][1][0]; a[3] = va[STAGE][t][1][1];                                 \
    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                     \
        __builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, pb[U]), acc[t], 0, 0, 0); \
  }
    RF_ISSUE_V(0, 0)
    RF_ISSUE_V(1, 1)
    // s[rt][r] = raw score(key key0 + 32rt + 8(r/4) + 4hh + r%4, query my_q)
    if (key0 + kBK - 1 > wave_min_last) {  // uniform: tile crosses the mask boundary
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + 32 * rt + 8 * (r >> 2) + 4 * hh + (r & 3);
          s[rt][r] = (key <= my_last) ? s[rt][r] : -INFINITY;
        }
    }
    // ---- stage 1: running max (reference point advanced lazily) ----
    float tmax = -INFINITY;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[rt][r]);
    {
      // lane l <-> lane l^32 through a VALU lane swap (no LDS round trip)
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax),
                                                       false, false);
      tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    const float tmax2 = tmax * scale_log2e;  // log2 units; scale > 0 keeps the order
    if (__builtin_amdgcn_ballot_w64(tmax2 > m_ref + kTau) != 0) {
      const float m_new = fmaxf(m_ref, tmax2);
      const float corr = (m_new == -INFINITY) ? 1.0f : fast_exp2(m_ref - m_new);
      m_ref = m_new;
      l *= corr;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] *= corr;
    }
    // ---- stage 2: running sum of exponentials; P^T packed to bf16 B operands ----
    const float neg_m = (m_ref == -INFINITY) ? 0.f : -m_ref;
    float psum = 0.f, psum1 = 0.f;
    u32x4 pb[4];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r2 = 0; r2 < 8; ++r2) {
        const float p0 = fast_exp2(fmaf(s[rt][2 * r2], scale_log2e, neg_m));
        const float p1 = fast_exp2(fmaf(s[rt][2 * r2 + 1], scale_log2e, neg_m));
        const uint32_t pk = pack_bf16(p0, p1);
        pb[2 * rt + (r2 >> 2)][r2 & 3] = pk;
        // one dot instruction adds the pair; the sum runs over the rounded probabilities,
        // the values the second product sees (two chains: the additions do not wait on each other)
        typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
        const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
        if (rt == 0) psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones, psum, false);
        else psum1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones, psum1, false);
      }
    l += psum + psum1;
    // ---- stage 3: acc += V^T P^T ----
    constexpr int NV = 2 * DT;  // transpose reads per contraction step
    RF_WAIT_V(0, NV)
    RF_PV_STEP(0, 0)
    RF_ISSUE_V(0, 2)
    RF_WAIT_V(1, NV)
    RF_PV_STEP(1, 1)
    RF_ISSUE_V(1, 3)
    RF_WAIT_V(0, NV)
    RF_PV_STEP(0, 2)
    RF_WAIT_V(1, 0)
    RF_PV_STEP(1, 3)
#undef RF_ISSUE_V
#undef RF_WAIT_V
#undef RF_PV_STEP
  };

  if (pass && n_ktiles > 0) issue_loads(0, 0);   // (first pass: requested during the set-up)
  for (int kt = 0; kt < n_ktiles; kt += 2) {
    tile_step(kt, std::integral_constant<int, 0>{});
    if (kt + 1 < n_ktiles) tile_step(kt + 1, std::integral_constant<int, 1>{});
  }

  // ---- epilogue: O = acc / l ----
  // The accumulators hold a query row per lane, four output values at a time: written to
  // memory from there, every store instruction would touch 32 rows with 16 bytes each.  The
  // rows go through LDS instead (the K/V buffers, once every wavefront is done with the last
  // tile; same slot swizzle as a K tile) and leave as whole 16-byte pieces, a full row per 16
  // (or 8) lanes.  A wavefront stages and stores its own 32 rows, so no barrier is needed in
  // between.
  l += __shfl_xor(l, 32, 64);
  const float inv = l > 0.f ? 1.0f / l : 0.f;
  __syncthreads();
  {
    unsigned char* stage = lds + (wave * 32) * ROWB;
    // (opaque copies: the addresses below are the same in both passes of a paired launch, and
    // the compiler would otherwise compute them all up front and carry them through the loop)
    int i32e = i32, lanee = lane;
    asm volatile("" : "+v"(i32e), "+v"(lanee));
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        // acc[t][4r4 + j] = O[my_q][32t + 8r4 + 4hh + j]
        u32x2 w;
        w[0] = pack_bf16(acc[t][4 * r4] * inv, acc[t][4 * r4 + 1] * inv);
        w[1] = pack_bf16(acc[t][4 * r4 + 2] * inv, acc[t][4 * r4 + 3] * inv);
        *reinterpret_cast<u32x2*>(stage + i32e * ROWB + (((4 * t + r4) ^ fK<D>(i32e)) << 4) +
                                  8 * (lanee >> 5)) = w;
      }
    bf16_t* ob = o + (int64_t)b * so.b + (int64_t)h * so.h;
#pragma unroll
    for (int i = 0; i < 32 / ROWS_PER_LD; ++i) {
      const int row = i * ROWS_PER_LD + lanee / P;   // within the wavefront's 32 rows
      const int slot = lanee % P;
      const u32x4 w = *reinterpret_cast<const u32x4*>(stage + row * ROWB + ((slot ^ fK<D>(row)) << 4));
      const int qrow = q0 + wave * 32 + row;
      // (non-temporal: keeps the output out of the way of the K/V tiles in L2; measured 2 % under
      // a causal mask, nothing without one)
      if (qrow < Lq)
        __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(ob + (int64_t)qrow * so.l + 8 * slot));
    }
  }
  }  // pass
}

hipError_t launch_attention_bf16(const void* q, const void* k, const void* v, void* o, Strides4 sq,
                                 Strides4 sk, Strides4 sv, Strides4 so, const AttnShape& a,
                                 hipStream_t s) {
  // Without a mask the larger workgroup wins (fewer loads per MFMA).  Under a causal mask the
  // query tiles of a head see different numbers of keys; a launch with enough heads gives
  // every workgroup two tiles of one head, the heaviest with the lightest and so on inwards,
  // so that all workgroups do the same work: with 256-query tiles if that still leaves one
  // workgroup per compute unit, else with 128-query tiles if that leaves two.  Smaller causal
  // launches keep one 128-query tile per workgroup, heaviest tiles first.
  const int64_t n_bh = (int64_t)a.B * a.Hq;
  auto tiles = [&](int bq) { return (a.Lq + bq - 1) / bq; };
  int nw = a.Lq <= 128 ? 4 : 8;
  int paired = 0;
  if (a.causal) {
    if (nw == 8 && tiles(256) % 2 == 0 && (tiles(256) / 2) * n_bh >= 256) {
      paired = 1;
    } else {
      nw = 4;
      paired = (tiles(128) % 2 == 0 && (tiles(128) / 2) * n_bh >= 512) ? 1 : 0;
    }
  }
  const int n_qtiles = tiles(32 * nw);
  const int64_t grid = (paired ? n_qtiles / 2 : n_qtiles) * n_bh;
  if (grid > INT32_MAX) return hipErrorInvalidValue;
  const float sl2 = a.scale * kLog2e;
#define RF_LAUNCH_ATTN(DD, NWW, PP)                                                               \
  hipLaunchKernelGGL((attention_bf16_kernel<DD, NWW, PP>), dim3((unsigned)grid), dim3(NWW * kWave), 0, s, \
                     (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, sq, sk, sv, so, \
                     a.Hq, a.Hkv, a.Lq, a.Lk, sl2, a.causal, n_qtiles)
  if (a.d == 128) {
    if (paired && nw == 8) RF_LAUNCH_ATTN(128, 8, true);
    else if (paired) RF_LAUNCH_ATTN(128, 4, true);
    else if (nw == 4) RF_LAUNCH_ATTN(128, 4, false);
    else RF_LAUNCH_ATTN(128, 8, false);
  } else if (a.d == 64) {
    if (paired && nw == 8) RF_LAUNCH_ATTN(64, 8, true);
    else if (paired) RF_LAUNCH_ATTN(64, 4, true);
    else if (nw == 4) RF_LAUNCH_ATTN(64, 4, false);
    else RF_LAUNCH_ATTN(64, 8, false);
  } else {
    return hipErrorInvalidValue;
  }
#undef RF_LAUNCH_ATTN
  return hipGetLastError();
}

}  // namespace rf
