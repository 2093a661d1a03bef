// bf16 fused attention without a mask, head dimension 128, 64 query rows per wavefront
// (paper Section 4.3 single-segment strategy; Appendix A.2 incremental forms; Appendix A.4
// tile-level structure).  Same mathematics and operand layouts as attention_bf16.hip:
//
//   S^T = K Q^T        A = K tile (LDS), B = Q^T (registers, loaded once)
//   O^T += V^T P^T     A = V^T (LDS transpose reads of the V tile), B = P^T
//
// What differs is the shape of the work.  A workgroup is four wavefronts, one per SIMD, and
// a wavefront owns two blocks of 32 query rows: every K and V fragment it reads from LDS
// feeds two MFMAs, which halves the LDS read traffic per MFMA of the 32-row kernel.  With a
// single wavefront on a SIMD nothing else hides the softmax arithmetic, so the loop is
// software-pipelined by hand inside the wavefront: iteration j issues the 32 MFMAs of
// S(j+1) = K(j+1) Q^T and then the 32 of O += V(j) P(j), and the vector-ALU work of softmax(j)
// (on S(j), finished one iteration earlier) is cut into single exponentials that are placed,
// by a compile-time schedule, in the gaps between those MFMAs; the row maxima of S(j+1) are
// taken at the end of iteration j.
//
// K and V tiles (64 keys) go from HBM straight into LDS with direct-to-LDS loads, four slots
// each.  A tile is complete one iteration before it is read, so the one barrier of an iteration
// sits after its first MFMAs and the LDS fragment stream (requested four fragments ahead,
// waited for by count) runs on across iterations.
//
// This kernel is a measured variant, reached through the diagnostic interface only: on the
// benchmark shape it is a few per cent slower than the 32-row kernel (which keeps two
// wavefronts on a SIMD).  A single wavefront issues everything in order, one instruction at a
// time: its MFMAs, exponentials, LDS reads, tile requests and waits add up to more issue time
// than the MFMAs take to execute, and removing any one of the three groups (exponentials,
// fragment reads, tile requests) shortens the loop by its full issue time.
#include <type_traits>
#include <utility>

#include "rf_device.h"
#include "rf_launch.h"

namespace rf {

namespace {

constexpr int kWBK = 64;       // keys per tile
constexpr int kWD = 128;       // head dimension
constexpr int kWQ = 256;       // query rows per workgroup (4 wavefronts x 2 blocks of 32)
constexpr float kWTau = 8.0f;  // the reference point of a row moves when its maximum grows by more (log2 units)
constexpr int kWAhead = 4;     // fragments requested ahead of their use (divides 32: the stream runs on across iterations)
constexpr int kWRing = 4;      // LDS slots per operand (K, V)

constexpr int kWRowB = kWD * 2;          // bytes per K/V row
constexpr int kWTileB = kWBK * kWRowB;   // bytes per K or V tile (16 KB)
constexpr int kWSlots = kWD / 8;         // 16-byte slots per row

// 16-byte slot swizzles (slot = piece ^ f(row)), as in the 32-row kernel
__device__ __forceinline__ int wfK(int row) { return row & 15; }
__device__ __forceinline__ int wfV(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// The fragment stream of one iteration: fragments 0..15 are the K fragments of S(j+1) (one
// 128-bit read each), 16..31 the V^T fragments of O += V(j) P(j) (two 64-bit transpose reads
// each); 32.. are fragments 0.. of the next iteration, requested at the end of this one.
constexpr int frag_reads(int g) { return (g & 31) < 16 ? 1 : 2; }
// LDS reads that may still be in flight when fragment g is needed: those of the fragments
// requested after it (g+1 .. g+kWAhead-1)
constexpr int frag_pending(int g) {
  int s = 0;
  for (int h = g + 1; h < g + kWAhead; ++h) s += frag_reads(h);
  return s;
}

// The vector-ALU work of one iteration, as items in dependency order with their cost in issue
// slots.  Item 0, 1: finish the row maximum of block A, B and move its reference point.
// Items 2..65: one exponential each, item 2 + k for contraction step u = k / 16 of the second
// product, block (k / 8) % 2, element k % 8 of the step (the odd elements also pack a pair of
// probabilities and add it to the row sum).  Items 66..73: row maxima of the next tile, eight
// scores of one block each.  An iteration issues 64 MFMAs; item i runs in the gap after MFMA
// item_gap(i): the exponentials spread evenly over gaps 0..55 (step u is then complete before
// MFMA 32 + 8u, the first that needs it), the maxima follow one per gap.
constexpr int kWItems = 74;
constexpr int item_cost(int i) { return i < 2 ? 8 : i < 66 ? (((i - 2) & 1) ? 5 : 3) : 4; }
constexpr int item_gap(int i) {
  if (i >= 66) return 56 + (i - 66);
  int before = 0, total = 0;
  for (int k = 0; k < 66; ++k) {
    if (k < i) before += item_cost(k);
    total += item_cost(k);
  }
  return before * 56 / total;
}
constexpr int gap_first_item(int m) {
  int i = 0;
  while (i < kWItems && item_gap(i) < m) ++i;
  return i;
}
constexpr bool schedule_meets_deadlines() {
  for (int k = 0; k < 64; ++k)
    if (item_gap(2 + k) >= 32 + 8 * (k / 16)) return false;
  return true;
}
static_assert(schedule_meets_deadlines(), "a probability is computed after the MFMA that reads it");

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

// Register files.  The MFMAs are raw instructions and two groups of their operands sit in
// accumulation registers chosen by hand, outside the compiler's register allocation:
//   a[0:127]    O^T accumulators: block x (0, 1), 32-row tile t (0..3) at a[16 (4x + t) ..]
//   a[128:191]  Q^T operands: block x, contraction step kk (0..7) at a[128 + 4 (8x + kk) ..]
// Nothing but MFMAs touches them inside the loop, and the vector registers are left to two
// score buffers, the probabilities and the fragments.  The scores come back in vector
// registers because the softmax reads them.  (Through the compiler's builtin every MFMA of a
// kernel that may use more than 256 registers writes accumulation registers, so the softmax
// would copy every score out; and accumulators that are compiler variables get moved between
// registers where the two unrolled halves of the loop meet, by copies that read them while
// MFMAs are still writing them.)  Every statement that touches these registers lists all of
// them as clobbered, which keeps the compiler from parking anything there across it.
// The compiler does not know these statements are MFMAs and inserts none of the wait states
// that software owes between an MFMA and another kind of instruction that reads its result:
// the explicit s_nop statements below stand wherever such a read follows closely (everywhere
// else dozens of instructions lie between).
#define RF_WIDE_AGPRS \
  "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", \
  "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", \
  "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47", \
  "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63", \
  "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", \
  "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95", \
  "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111", \
  "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127", \
  "a128", "a129", "a130", "a131", "a132", "a133", "a134", "a135", "a136", "a137", "a138", "a139", "a140", "a141", "a142", "a143", \
  "a144", "a145", "a146", "a147", "a148", "a149", "a150", "a151", "a152", "a153", "a154", "a155", "a156", "a157", "a158", "a159", \
  "a160", "a161", "a162", "a163", "a164", "a165", "a166", "a167", "a168", "a169", "a170", "a171", "a172", "a173", "a174", "a175", \
  "a176", "a177", "a178", "a179", "a180", "a181", "a182", "a183", "a184", "a185", "a186", "a187", "a188", "a189", "a190", "a191"
constexpr int kWAccBase = 0, kWQBase = 128;

// S block (vector registers) = or += K fragment x Q^T operand at accumulation register QLO
template <int QLO>
__device__ __forceinline__ void mfma_scores_first(f32x16& d, const u32x4& a) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[%2:%3], 0"
               : "=&v"(d) : "v"(a), "n"(QLO), "n"(QLO + 3) : RF_WIDE_AGPRS);
}
template <int QLO>
__device__ __forceinline__ void mfma_scores(f32x16& d, const u32x4& a) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[%2:%3], %0"
               : "+v"(d) : "v"(a), "n"(QLO), "n"(QLO + 3) : RF_WIDE_AGPRS);
}
// O^T block at accumulation register LO += V^T fragment x P^T fragment
template <int LO>
__device__ __forceinline__ void mfma_out(const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, a[%2:%3]"
               : : "v"(a), "v"(b), "n"(LO), "n"(LO + 15) : RF_WIDE_AGPRS);
}

}  // namespace

__global__ __launch_bounds__(256, 1) void attention_bf16_wide_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    bf16_t* __restrict__ o, Strides4 sq, Strides4 sk, Strides4 sv, Strides4 so, int Hq, int Hkv,
    int Lq, int Lk, float scale_log2e, int n_qtiles) {
  constexpr int KS = kWD / 16;  // contraction steps of S^T = K Q^T
  constexpr int DT = kWD / 32;  // 32-row tiles of O^T

  __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * kWRing * kWTileB];  // K slots, then V slots

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int i32 = lane & 31;
  const int hh = lane >> 5;

  // XCD-aware numbering: an XCD owns a contiguous range of heads, head-major inside, so the
  // query tiles of a head run together and share its K/V in one L2
  int qt, bh;
  {
    const int n_bh = gridDim.x / n_qtiles;
    if ((n_bh & 7) == 0) {
      const int hx = n_bh >> 3;
      const int xcd = blockIdx.x & 7;
      const int j = blockIdx.x >> 3;
      qt = j % n_qtiles;
      bh = xcd * hx + j / n_qtiles;
    } else {
      qt = (int)(blockIdx.x / n_bh);
      bh = blockIdx.x % n_bh;
    }
  }
  const int h = bh % Hq;
  const int b = bh / Hq;
  const int hk = h / (Hq / Hkv);
  const bf16_t* qb = q + (int64_t)b * sq.b + (int64_t)h * sq.h;
  const bf16_t* kb = k + (int64_t)b * sk.b + (int64_t)hk * sk.h;
  const bf16_t* vb = v + (int64_t)b * sv.b + (int64_t)hk * sv.h;

  // Q^T fragments of the wavefront's two row blocks: slot (hh, e) of step kk stands for
  // d = 16kk + 8hh + e
  const int q0 = qt * kWQ + wave * 64;
  const int my_q[2] = {q0 + i32, q0 + 32 + i32};
  const int n_ktiles = (Lk + kWBK - 1) / kWBK;  // >= 1; a ragged tile implies >= 2 (Lk >= 64)
  const bool ragged = (Lk % kWBK) != 0;

  // ---- direct-to-LDS load geometry: four loads of K and four of V per wavefront and tile,
  //      each 4 rows x 256 bytes ----
  uint32_t ld_koff[4], ld_voff[4];  // byte offsets from the tile's first row
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int row = (wave * 4 + e) * 4 + lane / kWSlots;
    const int slot = lane % kWSlots;
    ld_koff[e] = (uint32_t)(((int64_t)row * sk.l + 8 * (slot ^ wfK(row))) * 2);
    ld_voff[e] = (uint32_t)(((int64_t)row * sv.l + 8 * (slot ^ wfV(row))) * 2);
  }
  const uint32_t lds_base =
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;
  // Tile t holds the 64 keys from tile_start(t): 64 t, except that a ragged last tile is moved
  // back to end at the last key (Lk >= 64 is a condition of this kernel), so every tile is
  // loaded whole and in bounds; the keys such a tile shares with its predecessor are masked.
  // Tiles past the end re-read the last tile (nothing consumes them).
  auto tile_ptr = [&](int t, int is_v) {
    const int start = min(t * kWBK, Lk - kWBK);
    return reinterpret_cast<const char*>(is_v ? vb : kb) + (int64_t)start * (is_v ? sv.l : sk.l) * 2;
  };
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(lds_base + wave * 4096);
  // load e of K (is_v = 0) or V (is_v = 1) of the tile at `tile` into slot `slot`: uniform tile
  // base + per-lane 32-bit offset (row pitches below 2^24 elements are a condition of this kernel)
  // (the LDS address is formed in M0 by the statement itself: as a separate value the compiler
  // would keep one scalar register per load and slot alive across the whole loop)
  auto issue_one = [&](const char* tile, auto slot_tag, auto e_tag, auto v_tag) {
    constexpr int is_v = decltype(v_tag)::value;
    constexpr int dst_off = (kWRing * is_v + decltype(slot_tag)::value) * kWTileB + decltype(e_tag)::value * 1024;
    const uint32_t lane_off = is_v ? ld_voff[decltype(e_tag)::value] : ld_koff[decltype(e_tag)::value];
    const uint32_t wave_base = lds_wave;
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(wave_base), "v"(lane_off), "s"(tile), "n"(dst_off)
                 : "memory", "m0", "scc");
  };

  // ---- LDS read addresses (loop invariant; slots and steps are immediate offsets) ----
  uint32_t koff[KS];  // + rt * 32 rows, + K slot
#pragma unroll
  for (int kk = 0; kk < KS; ++kk)
    koff[kk] = lds_base + i32 * kWRowB + (((2 * kk + hh) ^ wfK(i32)) << 4);
  // transpose reads of V: lane = 32hh + 16g2 + 4j + a reads 8 bytes of key row
  // (16u + 8w + 4hh + j) at head-dim offset 32t + 16g2 + 4a
  uint32_t voff[DT][2];  // V slot 0 (the V slots follow the K slots); + u * 16 rows, + V slot
  {
    const int i16 = lane & 15, g2 = (lane >> 4) & 1;
    const int jj = i16 >> 2, a = i16 & 3;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int w2 = 0; w2 < 2; ++w2) {
        const int row = 8 * w2 + 4 * hh + jj;
        const int piece = 4 * t + 2 * g2 + (a >> 1);
        voff[t][w2] = lds_base + kWRing * kWTileB + row * kWRowB +
                      (((piece ^ wfV(row)) & (kWSlots - 1)) << 4) + 8 * (a & 1);
      }
  }

  // ---- running state of the cascade, per row block ----
  float m_ref[2] = {-INFINITY, -INFINITY}, l[2] = {0.f, 0.f};
  float neg_m[2] = {0.f, 0.f};
  float tmax[2] = {-INFINITY, -INFINITY};  // this lane's share of the row maxima of the next S
  f32x16 s[2][2][2];  // [buffer][row block][32-key half]; s[..][rt][r] = raw score(key 32rt + 8(r/4) + 4hh + r%4)
  u32x4 pb[2][4];     // P^T operands of the four contraction steps, per row block
  float psum[2] = {0.f, 0.f};
  const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);

  u32x4 kfr[kWAhead];
  u32x2 vfr[kWAhead][2];

  // tile t >= n - 1 (scores in buffer SB) starts at key Lk - 64: a ragged last tile has the keys
  // masked that the tile before it already covered, a tile past the end all of them
  auto mask_tail = [&](auto sb_tag, int t) {
    constexpr int SB = decltype(sb_tag)::value;
    const int key0 = Lk - kWBK, first_new = t >= n_ktiles ? INT32_MAX : (n_ktiles - 1) * kWBK;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + 32 * rt + 8 * (r >> 2) + 4 * hh + (r & 3);
          s[SB][x][rt][r] = (key >= first_new) ? s[SB][x][rt][r] : -INFINITY;
        }
  };
  // eight of the 32 scores a lane holds per row block: chunk c = 0..3 of block x
  auto max_item = [&](auto sb_tag, auto x_tag, auto c_tag) {
    constexpr int SB = decltype(sb_tag)::value;
    constexpr int x = decltype(x_tag)::value;
    constexpr int C = decltype(c_tag)::value;
    const f32x16& sv_ = s[SB][x][C >> 1];
    constexpr int r0 = 8 * (C & 1);
    const float t0 = fmaxf(fmaxf(sv_[r0], sv_[r0 + 1]), fmaxf(sv_[r0 + 2], sv_[r0 + 3]));
    const float t1 = fmaxf(fmaxf(sv_[r0 + 4], sv_[r0 + 5]), fmaxf(sv_[r0 + 6], sv_[r0 + 7]));
    tmax[x] = fmaxf(tmax[x], fmaxf(t0, t1));
  };
  // finish the row maximum of block X, move its reference point if needed (rare after the
  // first tiles), fold the finished sum of the previous tile into l
  auto cross_lane = [&](auto x_tag) {
    constexpr int x = decltype(x_tag)::value;
    l[x] += psum[x];
    psum[x] = 0.f;
    float t = tmax[x];
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    t = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    tmax[x] = -INFINITY;
    const float tmax2 = t * scale_log2e;  // log2 units; scale > 0 keeps the order
    if (__builtin_amdgcn_ballot_w64(tmax2 > m_ref[x] + kWTau) != 0) {
      const float m_new = fmaxf(m_ref[x], tmax2);
      const float corr = (m_new == -INFINITY) ? 1.0f : fast_exp2(m_ref[x] - m_new);
      m_ref[x] = m_new;
      l[x] *= corr;
      // the last MFMAs into these accumulators were issued a few instructions ago: let them
      // write back, then scale the block's 64 accumulation registers in place
      asm volatile("s_nop 15\n\ts_nop 3" ::: "memory");
      static_for<64>([&](auto i_tag) {
        float tmp;
        const float factor = corr;
        asm volatile("v_accvgpr_read_b32 %0, a[%2]\n\tv_mul_f32 %0, %0, %1\n\tv_accvgpr_write_b32 a[%2], %0"
                     : "=&v"(tmp) : "v"(factor), "n"(kWAccBase + 64 * x + decltype(i_tag)::value) : RF_WIDE_AGPRS);
      });
      neg_m[x] = (m_new == -INFINITY) ? 0.f : -m_new;
    }
  };
  // one exponential: element e = 0..7 of contraction step u of block x
  float p_even[2] = {0.f, 0.f};
  auto exp_item = [&](auto sb_tag, auto k_tag) {
    constexpr int SB = decltype(sb_tag)::value;
    constexpr int K = decltype(k_tag)::value;
    constexpr int u = K >> 4, x = (K >> 3) & 1, e = K & 7;
    const float pv = fast_exp2(fmaf(s[SB][x][u >> 1][8 * (u & 1) + e], scale_log2e, neg_m[x]));
    if constexpr ((e & 1) == 0) {
      p_even[x] = pv;
    } else {
      const uint32_t pk = pack_bf16(p_even[x], pv);
      pb[x][u][e >> 1] = pk;
      // the sum runs over the rounded probabilities, the values the second product sees
      psum[x] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones, psum[x], false);
      // (the sum is only read in the next iteration: without this the compiler collects all
      // these additions at the end of the loop body)
      asm volatile("" : "+v"(psum[x]));
    }
  };

  // fragment g of the stream of the iteration with phase PH (g >= 32: of the next iteration)
  auto issue_frag = [&](auto ph_tag, auto g_tag) {
    constexpr int PH = decltype(ph_tag)::value;
    constexpr int G = decltype(g_tag)::value;
    constexpr int g = G & 31;
    constexpr int ph = (PH + (G >> 5)) % kWRing;
    if constexpr (g < 16) {
      constexpr int kk = g >> 1, rt = g & 1;
      u32x4& d = kfr[g % kWAhead];
      const uint32_t a0 = koff[kk];
      asm volatile("ds_read_b128 %0, %1 offset:%2"
                   : "=v"(d) : "v"(a0), "n"(((ph + 1) % kWRing) * kWTileB + rt * 32 * kWRowB));
    } else {
      constexpr int f = g - 16, u = f >> 2, t = f & 3;
      u32x2& d0 = vfr[g % kWAhead][0];
      u32x2& d1 = vfr[g % kWAhead][1];
      const uint32_t a0 = voff[t][0], a1 = voff[t][1];
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(d0) : "v"(a0), "n"(ph * kWTileB + u * 16 * kWRowB));
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(d1) : "v"(a1), "n"(ph * kWTileB + u * 16 * kWRowB));
    }
  };

  // One iteration, j = PH mod 4: tile j (scores in buffer SB = PH mod 2) gets its softmax and its
  // share of O, tile j+1 its scores (into buffer SB^1).  Tile t of K or V sits in slot t mod 4.
  // The tiles an iteration reads were complete one iteration earlier: the barrier of iteration
  // j (placed after the first MFMAs, so that the wavefronts need not arrive together) comes
  // after each wavefront has seen its own loads of K(j+2) and V(j+1) land, which it requested
  // in iteration j-2; the eight loads of iteration j-1 may still be in flight.  After the
  // barrier nobody reads K(j) or V(j-1) any more, and their slots take the requests for K(j+4)
  // and V(j+3).  The first fragments of iteration j+1 are requested at the end of iteration j.
  auto iteration = [&](int j, auto ph_tag) {
    constexpr int PH = decltype(ph_tag)::value;
    constexpr int SB = PH & 1;
    const std::integral_constant<int, SB> sb_tag{};
    const std::integral_constant<int, SB ^ 1> sb_next{};
    const char* knext = tile_ptr(j + 4, 0);
    const char* vnext = tile_ptr(j + 3, 1);

    static_for<64>([&](auto m_tag) {
      constexpr int M = decltype(m_tag)::value;
      constexpr int G = M >> 1, x = M & 1;
      // ---- MFMA M ----
      if constexpr (G < 16) {
        constexpr int kk = G >> 1, rt = G & 1;
        if constexpr (x == 0)
          asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(kfr[G % kWAhead]) : "n"(frag_pending(G)));
        if constexpr (kk == 0)
          mfma_scores_first<kWQBase + 4 * (8 * x + kk)>(s[SB ^ 1][x][rt], kfr[G % kWAhead]);
        else
          mfma_scores<kWQBase + 4 * (8 * x + kk)>(s[SB ^ 1][x][rt], kfr[G % kWAhead]);
      } else {
        constexpr int f = G - 16, u = f >> 2, t = f & 3;
        if constexpr (x == 0)
          asm volatile("s_waitcnt lgkmcnt(%2)"
                       : "+v"(vfr[G % kWAhead][0]), "+v"(vfr[G % kWAhead][1])
                       : "n"(frag_pending(G)));
        u32x4 a4;
        a4[0] = vfr[G % kWAhead][0][0]; a4[1] = vfr[G % kWAhead][0][1];
        a4[2] = vfr[G % kWAhead][1][0]; a4[3] = vfr[G % kWAhead][1][1];
        mfma_out<kWAccBase + 16 * (4 * x + t)>(a4, pb[x][u]);
      }
      if constexpr (x == 1) {
        issue_frag(ph_tag, std::integral_constant<int, G + kWAhead>{});
        if constexpr (G == 1) {
          asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
          __builtin_amdgcn_s_barrier();
        }
        // requests for K(j+4) and V(j+3): one at every other position from 2 to 16
        if constexpr (G >= 2 && G <= 16 && (G & 1) == 0) {
          constexpr int n = (G - 2) >> 1, e = n & 3, is_v = n >> 2;
          using e_type = std::integral_constant<int, e>;
          if constexpr (is_v) issue_one(vnext, std::integral_constant<int, (PH + 3) % kWRing>{}, e_type{}, std::integral_constant<int, 1>{});
          else issue_one(knext, std::integral_constant<int, PH>{}, e_type{}, std::integral_constant<int, 0>{});
        }
      }
      // ---- the vector-ALU items of this gap ----
      constexpr int first = gap_first_item(M), count = gap_first_item(M + 1) - first;
      static_for<count>([&](auto i_tag) {
        constexpr int I = first + decltype(i_tag)::value;
        if constexpr (I < 2) {
          cross_lane(std::integral_constant<int, I>{});
        } else if constexpr (I < 66) {
          exp_item(sb_tag, std::integral_constant<int, I - 2>{});
        } else {
          if (I == 66 && j + 2 >= n_ktiles && (ragged || j + 1 >= n_ktiles)) mask_tail(sb_next, j + 1);
          max_item(sb_next, std::integral_constant<int, (I - 66) & 1>{}, std::integral_constant<int, (I - 66) / 2>{});
        }
      });
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // ---- prologue: K(0), V(0), K(1) complete; S(0) computed without overlap; then the requests
  //      that iterations -2 and -1 would have made ----
  static_for<4>([&](auto e) { issue_one(tile_ptr(0, 0), std::integral_constant<int, 0>{}, e, std::integral_constant<int, 0>{}); });
  static_for<4>([&](auto e) { issue_one(tile_ptr(0, 1), std::integral_constant<int, 0>{}, e, std::integral_constant<int, 1>{}); });
  static_for<4>([&](auto e) { issue_one(tile_ptr(1, 0), std::integral_constant<int, 1>{}, e, std::integral_constant<int, 0>{}); });
  // Q is fetched behind the first tile requests, so the two trips to memory overlap
  u32x4 qf[2][KS];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const bf16_t* qp = qb + (int64_t)min(my_q[x], Lq - 1) * sq.l + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[x][kk] = *reinterpret_cast<const u32x4*>(qp + 16 * kk);
  }
  // The loop needs a positive scale (row maxima are taken on raw scores): fold the sign of
  // the scale into Q, and turn scale == 0 (uniform weights) into Q = 0 with scale 1.
  if (scale_log2e < 0.f) {
    scale_log2e = -scale_log2e;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) qf[x][kk] ^= 0x80008000u;
  } else if (scale_log2e == 0.f) {
    scale_log2e = 1.0f;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) qf[x][kk] = u32x4{0u, 0u, 0u, 0u};
  }

  // the Q^T operands move to their accumulation registers, the accumulators start at zero
  static_for<2 * KS * 4>([&](auto i_tag) {
    constexpr int I = decltype(i_tag)::value;
    const uint32_t word = qf[I >> 5][(I >> 2) & 7][I & 3];
    asm volatile("v_accvgpr_write_b32 a[%1], %0" : : "v"(word), "n"(kWQBase + I) : RF_WIDE_AGPRS);
  });
  static_for<128>([&](auto i_tag) {
    asm volatile("v_accvgpr_write_b32 a[%0], 0" : : "n"(kWAccBase + decltype(i_tag)::value) : RF_WIDE_AGPRS);
  });

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  static_for<4>([&](auto e) { issue_one(tile_ptr(2, 0), std::integral_constant<int, 2>{}, e, std::integral_constant<int, 0>{}); });
  static_for<4>([&](auto e) { issue_one(tile_ptr(1, 1), std::integral_constant<int, 1>{}, e, std::integral_constant<int, 1>{}); });
  static_for<4>([&](auto e) { issue_one(tile_ptr(3, 0), std::integral_constant<int, 3>{}, e, std::integral_constant<int, 0>{}); });
  static_for<4>([&](auto e) { issue_one(tile_ptr(2, 1), std::integral_constant<int, 2>{}, e, std::integral_constant<int, 1>{}); });
  static_for<2 * KS>([&](auto g_tag) {
    constexpr int kk = decltype(g_tag)::value >> 1, rt = decltype(g_tag)::value & 1;
    const u32x4 a = *reinterpret_cast<const u32x4*>(lds + (koff[kk] - lds_base) + rt * 32 * kWRowB);
    if constexpr (kk == 0) {
      mfma_scores_first<kWQBase + 4 * kk>(s[0][0][rt], a);
      mfma_scores_first<kWQBase + 4 * (8 + kk)>(s[0][1][rt], a);
    } else {
      mfma_scores<kWQBase + 4 * kk>(s[0][0][rt], a);
      mfma_scores<kWQBase + 4 * (8 + kk)>(s[0][1][rt], a);
    }
  });
  // the scores are read right away: let the last MFMAs write them back first
  asm volatile("s_nop 15\n\ts_nop 3" : "+v"(s[0][0][0]), "+v"(s[0][0][1]), "+v"(s[0][1][0]), "+v"(s[0][1][1]));
  static_for<8>([&](auto i) {
    max_item(std::integral_constant<int, 0>{}, std::integral_constant<int, decltype(i)::value & 1>{},
             std::integral_constant<int, decltype(i)::value / 2>{});
  });
  // the first fragments of iteration 0
  static_for<kWAhead>([&](auto g) { issue_frag(std::integral_constant<int, 0>{}, g); });

  // ---- main loop: iterations 0 .. n-1 in groups of four (slots), the last one computes no scores ----
  {
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using P2 = std::integral_constant<int, 2>;
    using P3 = std::integral_constant<int, 3>;
    // (the last iteration also computes scores, of a tile past the end that re-reads the last
    // one, and drops them: one code path per slot phase keeps the register allocation of the
    // loop free of copies, at the price of 32 surplus MFMAs per workgroup)
    // Whole groups of four iterations, one code path per slot phase and a single back edge: the
    // register allocation of the loop then needs no copies.  Iterations past the last tile work
    // on a tile whose keys are all masked, which leaves the state as it is.
    for (int j = 0; j < n_ktiles; j += 4) {
      iteration(j, P0{});
      iteration(j + 1, P1{});
      iteration(j + 2, P2{});
      iteration(j + 3, P3{});
    }
  }
  // the surplus requests and fragment reads of the last iteration land
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");

  // ---- epilogue: O = acc / l, staged through LDS (K slots; every wavefront is past its last
  //      read after the barrier) so that rows leave in whole 16-byte pieces ----
  asm volatile("s_nop 15\n\ts_nop 3" ::: "memory");  // the last MFMAs write back
  __builtin_amdgcn_s_barrier();
  static_for<2>([&](auto x_tag) {
    constexpr int x = decltype(x_tag)::value;
    float lx = l[x] + psum[x];
    lx += __shfl_xor(lx, 32, 64);
    const float inv = lx > 0.f ? 1.0f / lx : 0.f;
    unsigned char* stage = lds + (wave * 64 + 32 * x) * kWRowB;
    static_for<DT * 4>([&](auto i_tag) {
      constexpr int t = decltype(i_tag)::value / 4, r4 = decltype(i_tag)::value & 3;
      // accumulator register 4 r4 + jj of tile t holds O[my_q][32t + 8r4 + 4hh + jj]
      float a4[4];
      static_for<4>([&](auto j_tag) {
        constexpr int jj = decltype(j_tag)::value;
        float word;
        asm volatile("v_accvgpr_read_b32 %0, a[%1]"
                     : "=v"(word) : "n"(kWAccBase + 16 * (4 * x + t) + 4 * r4 + jj));
        a4[jj] = word;
      });
      u32x2 w;
      w[0] = pack_bf16(a4[0] * inv, a4[1] * inv);
      w[1] = pack_bf16(a4[2] * inv, a4[3] * inv);
      *reinterpret_cast<u32x2*>(stage + i32 * kWRowB + (((4 * t + r4) ^ wfK(i32)) << 4) + 8 * hh) = w;
    });
    bf16_t* ob = o + (int64_t)b * so.b + (int64_t)h * so.h;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = 4 * i + lane / kWSlots;   // within the block's 32 rows
      const int slot = lane % kWSlots;
      const u32x4 w = *reinterpret_cast<const u32x4*>(stage + row * kWRowB + ((slot ^ wfK(row)) << 4));
      const int qrow = q0 + 32 * x + row;
      if (qrow < Lq) *reinterpret_cast<u32x4*>(ob + (int64_t)qrow * so.l + 8 * slot) = w;
    }
  });
}

// Takes the shapes the wide kernel is built for: no mask, head dimension 128, at least one
// whole key tile (Lk >= 64), row pitches of K and V below 2^24 elements.  Returns hipErrorInvalidValue otherwise.
hipError_t launch_attention_bf16_wide(const void* q, const void* k, const void* v, void* o,
                                      Strides4 sq, Strides4 sk, Strides4 sv, Strides4 so,
                                      const AttnShape& a, hipStream_t s) {
  if (a.causal || a.d != kWD || a.Lk < kWBK || sk.l >= (1 << 24) || sv.l >= (1 << 24))
    return hipErrorInvalidValue;
  const int n_qtiles = (a.Lq + kWQ - 1) / kWQ;
  const int64_t grid = (int64_t)n_qtiles * a.B * a.Hq;
  if (grid > INT32_MAX) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attention_bf16_wide_kernel, dim3((unsigned)grid), dim3(256), 0, s,
                     (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, sq, sk, sv, so,
                     a.Hq, a.Hkv, a.Lq, a.Lk, a.scale * kLog2e, n_qtiles);
  return hipGetLastError();
}

}  // namespace rf
