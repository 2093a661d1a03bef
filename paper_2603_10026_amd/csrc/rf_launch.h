// Internal launch interface between the C-ABI layer (argument validation) and
// the kernel translation units.  Plain pointers and sizes; every function
// enqueues on `s` and returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rf {

// Rows of length n; pitches in elements.  vec_ok: base pointers and pitches
// allow 128-bit accesses.
hipError_t launch_softmax(const void* x, void* y, bool is_bf16, int64_t rows, int64_t n,
                          int64_t x_pitch, int64_t y_pitch, bool vec_ok, hipStream_t s);

// Strides (in elements) of a [B, H, L, d] tensor whose last axis is contiguous.
struct Strides4 {
  int64_t b, h, l;
};

struct AttnShape {
  int B, Hq, Hkv, Lq, Lk, d;
  float scale;
  int causal;
};

hipError_t launch_attention_f32(const float* q, const float* k, const float* v, float* o,
                                Strides4 sq, Strides4 sk, Strides4 sv, Strides4 so,
                                const AttnShape& a, hipStream_t s);

hipError_t launch_attention_bf16(const void* q, const void* k, const void* v, void* o,
                                 Strides4 sq, Strides4 sk, Strides4 sv, Strides4 so,
                                 const AttnShape& a, hipStream_t s);
// measured variant: 64 query rows per wavefront, one wavefront per SIMD; no mask, head
// dimension 128, Lk >= 64, K/V row pitches below 2^24 (other shapes: hipErrorInvalidValue)
hipError_t launch_attention_bf16_wide(const void* q, const void* k, const void* v, void* o,
                                 Strides4 sq, Strides4 sk, Strides4 sv, Strides4 so,
                                 const AttnShape& a, hipStream_t s);

// Partial states are contiguous: part_m, part_l [B,Hq,Lq,S]; part_acc [B,Hq,Lq,S,d].
hipError_t launch_attention_splitk_bf16(const void* q, const void* k, const void* v,
                                        Strides4 sq, Strides4 sk, Strides4 sv, int num_splits,
                                        float* part_m, float* part_l, float* part_acc,
                                        const AttnShape& a, hipStream_t s);

// Output row (b, h, i) lives at o + b*so.b + h*so.h + i*so.l.
hipError_t launch_merge_states(const float* part_m, const float* part_l, const float* part_acc,
                               void* o, bool o_is_bf16, int B, int Hq, int Lq, int S, int d,
                               Strides4 so, hipStream_t s);

// x [M,K], g [K], w [K,N], y [M,N]; leading dimensions in elements.
hipError_t launch_rmsnorm_gemm_bf16(const void* x, const void* g, const void* w, void* y, int M,
                                    int K, int N, int64_t ldx, int64_t ldw, int64_t ldy,
                                    float eps, hipStream_t s);

// Rows of length n (pitch in elements); mean, var: one float per row.
hipError_t launch_variance(const void* x, bool is_bf16, float* mean, float* var, int64_t rows,
                           int64_t n, int64_t x_pitch, bool vec_ok, hipStream_t s);

// x [S,hd], w [hd,E] bf16; prob, idx [S,topk] with row pitches ldp, ldi; part: fp32
// workspace of moe_num_slices(S, hd) * S * E floats.  hd % 128 == 0, E in {32, 64, 128},
// 1 <= topk <= 16.
int moe_num_slices(int S, int hd);
hipError_t launch_moe_routing(const void* x, const void* w, int S, int hd, int E, int topk,
                              int64_t ldx, int64_t ldw, float* prob, int32_t* idx, int64_t ldp,
                              int64_t ldi, float* part, hipStream_t s);

// The same two kernels with the partial scores in a file-scope device array of
// kMoeStaticScratchBytes bytes instead of a caller's workspace: no allocation anywhere.
constexpr size_t kMoeStaticScratchBytes = (size_t)8 << 20;
hipError_t launch_moe_routing_static(const void* x, const void* w, int S, int hd, int E, int topk,
                                     int64_t ldx, int64_t ldw, float* prob, int32_t* idx,
                                     int64_t ldp, int64_t ldi, hipStream_t s);

// a [M,K] bf16, w [N,K] FP8 (E4M3), c [M,N] bf16; leading dimensions in elements.
// K % 128 == 0, N % 8 == 0.
hipError_t launch_fp8_quant_gemm(const void* a, const void* w, void* c, int M, int K, int N,
                                 int64_t lda, int64_t ldw, int64_t ldc, hipStream_t s);

// Fusion-level study of the softmax cascade (bf16 rows, n % 8 == 0, n <= 8192): level 0 =
// unfused (three kernels; ml_buf holds 2 * rows floats), 1 = fused per lane, 2 = per
// wavefront (the shipped kernel), 3 = per workgroup, 4 = across workgroups (two kernels;
// ml_buf holds 8 * rows floats).
hipError_t launch_softmax_level(const void* x, void* y, int64_t rows, int64_t n, int64_t x_pitch,
                                int64_t y_pitch, int level, float* ml_buf, hipStream_t s);

// Measurement aids: a plain copy of `bytes` (multiple of 16) and an MFMA-only loop
// (workgroups x 4 wavefronts x iters x 32 MFMAs of 32x32x16 bf16; sink holds
// workgroups * 256 floats).
hipError_t launch_diag_copy(const void* src, void* dst, int64_t bytes, hipStream_t s);
constexpr int kDiagReadWorkgroups = 8192;  // the sink holds one 32-bit word per wavefront (4 per workgroup)
hipError_t launch_diag_read(const void* src, int64_t bytes, void* sink, hipStream_t s);
hipError_t launch_diag_mfma(float* sink, int workgroups, int iters, int random_operands,
                            hipStream_t s);

}  // namespace rf
