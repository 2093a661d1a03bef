// C-ABI layer: argument validation on the host, then dispatch to the kernel
// launchers.  No device memory is allocated, freed or retained here.
#include "../../include/rf.h"
#include "../../include/rf_diag.h"

#include <string.h>

#include "rf_launch.h"

static_assert(RF_MOE_ROUTING_NOALLOC_MAX_BYTES == rf::kMoeStaticScratchBytes, "header and kernels agree on the scratch size");

namespace {

inline size_t esize(rf_dtype t) { return t == RF_BF16 ? 2 : t == RF_FP8_E4M3 ? 1 : 4; }  // f32, i32: 4
// `also`: one more dtype this argument may have (-1: none)
inline bool dtype_ok(rf_dtype t, int also) {
  return t == RF_F32 || t == RF_BF16 || (also >= 0 && (int)t == also);
}

// Structural checks common to every tensor argument.
// (integer and FP8 tensors are accepted only where an entry point asks for them)
rf_status check_tensor(const rf_tensor* t, int ndim_min, int ndim_max, int also = -1) {
  if (t == nullptr) return RF_ERR_INVALID_ARG;
  if (t->ndim < ndim_min || t->ndim > ndim_max) return RF_ERR_INVALID_ARG;
  if (!dtype_ok(t->dtype, also)) return RF_ERR_UNSUPPORTED;
  for (int i = 0; i < t->ndim; ++i) {
    if (t->shape[i] < 0 || t->stride[i] < 0) return RF_ERR_INVALID_ARG;
  }
  return RF_OK;
}

int64_t numel(const rf_tensor* t) {
  int64_t n = 1;
  for (int i = 0; i < t->ndim; ++i) n *= t->shape[i];
  return n;
}

bool same_shape(const rf_tensor* a, const rf_tensor* b) {
  if (a->ndim != b->ndim) return false;
  for (int i = 0; i < a->ndim; ++i)
    if (a->shape[i] != b->shape[i]) return false;
  return true;
}

bool is_contiguous(const rf_tensor* t) {
  int64_t expect = 1;
  for (int i = t->ndim - 1; i >= 0; --i) {
    if (t->shape[i] != 1 && t->stride[i] != expect) return false;
    expect *= t->shape[i];
  }
  return true;
}

// 16-byte alignment of the base pointer and of every outer stride.
bool aligned16(const rf_tensor* t) {
  if (reinterpret_cast<uintptr_t>(t->data) % 16 != 0) return false;
  for (int i = 0; i + 1 < t->ndim; ++i)
    if (t->shape[i] > 1 && (t->stride[i] * (int64_t)esize(t->dtype)) % 16 != 0) return false;
  return true;
}

// Leading dims collapse to `rows` rows with a single pitch?
bool collapse_rows(const rf_tensor* t, int64_t* rows, int64_t* pitch) {
  const int nd = t->ndim;
  int64_t r = 1;
  for (int i = 0; i + 1 < nd; ++i) r *= t->shape[i];
  *rows = r;
  if (nd == 1) { *pitch = t->shape[0]; return true; }
  *pitch = t->stride[nd - 2];
  for (int i = nd - 3; i >= 0; --i) {
    if (t->shape[i] == 1) continue;
    if (t->stride[i] != t->stride[i + 1] * t->shape[i + 1]) return false;
  }
  if (r > 1 && *pitch < t->shape[nd - 1]) return false;
  return true;
}

rf::Strides4 strides4(const rf_tensor* t) { return {t->stride[0], t->stride[1], t->stride[2]}; }

struct AttnArgs {
  rf::AttnShape a;
};

// Shared validation of (q, k, v) for the attention entry points.
rf_status check_qkv(const rf_tensor* q, const rf_tensor* k, const rf_tensor* v, rf::AttnShape* a) {
  rf_status st;
  if ((st = check_tensor(q, 4, 4)) != RF_OK) return st;
  if ((st = check_tensor(k, 4, 4)) != RF_OK) return st;
  if ((st = check_tensor(v, 4, 4)) != RF_OK) return st;
  if (q->dtype != k->dtype || q->dtype != v->dtype) return RF_ERR_UNSUPPORTED;
  if (!same_shape(k, v)) return RF_ERR_INVALID_ARG;
  if (q->shape[0] != k->shape[0] || q->shape[3] != k->shape[3]) return RF_ERR_INVALID_ARG;
  if (k->shape[1] <= 0 || q->shape[1] % k->shape[1] != 0) return RF_ERR_INVALID_ARG;
  for (const rf_tensor* t : {q, k, v}) {
    if (t->shape[3] > 1 && t->stride[3] != 1) return RF_ERR_UNSUPPORTED;
    for (int i = 0; i < 4; ++i)
      if (t->shape[i] > INT32_MAX) return RF_ERR_UNSUPPORTED;
  }
  a->B = (int)q->shape[0];
  a->Hq = (int)q->shape[1];
  a->Hkv = (int)k->shape[1];
  a->Lq = (int)q->shape[2];
  a->Lk = (int)k->shape[2];
  a->d = (int)q->shape[3];
  return RF_OK;
}

}  // namespace

extern "C" {

const char* rf_status_string(rf_status s) {
  switch (s) {
    case RF_OK: return "RF_OK";
    case RF_ERR_INVALID_ARG: return "RF_ERR_INVALID_ARG";
    case RF_ERR_UNSUPPORTED: return "RF_ERR_UNSUPPORTED";
    case RF_ERR_ALIGNMENT: return "RF_ERR_ALIGNMENT";
    case RF_ERR_WORKSPACE: return "RF_ERR_WORKSPACE";
    case RF_ERR_LAUNCH: return "RF_ERR_LAUNCH";
  }
  return "RF_ERR_UNKNOWN";
}

int rf_describe_cascade(const char* entry, rf_stage* out, int cap) {
  if (entry == nullptr) return -1;
  static const rf_stage kSoftmax[] = {{RF_RED_MAX, RF_COMB_ADD}, {RF_RED_SUM, RF_COMB_MUL}};
  static const rf_stage kAttention[] = {
      {RF_RED_MAX, RF_COMB_ADD}, {RF_RED_SUM, RF_COMB_MUL}, {RF_RED_SUM, RF_COMB_MUL}};
  static const rf_stage kRms[] = {{RF_RED_SUM, RF_COMB_MUL}, {RF_RED_SUM, RF_COMB_MUL}};
  // max, sum of exponentials, TopK (a max-type reduction, Table 1)
  static const rf_stage kRouting[] = {
      {RF_RED_MAX, RF_COMB_ADD}, {RF_RED_SUM, RF_COMB_MUL}, {RF_RED_MAX, RF_COMB_ADD}};
  // abs-max, then the scaled sum
  static const rf_stage kQuant[] = {{RF_RED_MAX, RF_COMB_ADD}, {RF_RED_SUM, RF_COMB_MUL}};
  const rf_stage* src = nullptr;
  int n = 0;
  if (!strcmp(entry, "rf_safe_softmax")) { src = kSoftmax; n = 2; }
  else if (!strcmp(entry, "rf_cascade_attention") || !strcmp(entry, "rf_cascade_attention_splitk") ||
           !strcmp(entry, "rf_merge_states")) { src = kAttention; n = 3; }
  else if (!strcmp(entry, "rf_rmsnorm_gemm")) { src = kRms; n = 2; }
  else if (!strcmp(entry, "rf_variance")) { src = kRms; n = 2; }  // sum, then sum
  else if (!strcmp(entry, "rf_moe_routing")) { src = kRouting; n = 3; }
  else if (!strcmp(entry, "rf_fp8_quant_gemm")) { src = kQuant; n = 2; }
  else return -1;
  if (out != nullptr)
    for (int i = 0; i < n && i < cap; ++i) out[i] = src[i];
  return n;
}

rf_status rf_safe_softmax(const rf_tensor* x, rf_tensor* y, int axis, rf_stream stream) {
  rf_status st;
  if ((st = check_tensor(x, 1, RF_MAX_DIMS)) != RF_OK) return st;
  if ((st = check_tensor(y, 1, RF_MAX_DIMS)) != RF_OK) return st;
  if (x->dtype != y->dtype) return RF_ERR_UNSUPPORTED;
  if (!same_shape(x, y)) return RF_ERR_INVALID_ARG;
  const int nd = x->ndim;
  if (axis < -nd || axis >= nd) return RF_ERR_INVALID_ARG;
  if (axis != nd - 1 && axis != -1) return RF_ERR_UNSUPPORTED;
  if (numel(x) == 0) return RF_OK;
  if (x->data == nullptr || y->data == nullptr) return RF_ERR_INVALID_ARG;
  if (x->stride[nd - 1] != 1 && x->shape[nd - 1] > 1) return RF_ERR_UNSUPPORTED;
  if (y->stride[nd - 1] != 1 && y->shape[nd - 1] > 1) return RF_ERR_UNSUPPORTED;
  int64_t rows, xp, yp, rows_y;
  if (!collapse_rows(x, &rows, &xp) || !collapse_rows(y, &rows_y, &yp)) return RF_ERR_UNSUPPORTED;
  const int64_t n = x->shape[nd - 1];
  if (rows > INT32_MAX) return RF_ERR_UNSUPPORTED;
  const size_t es = esize(x->dtype);
  const bool vec_ok = reinterpret_cast<uintptr_t>(x->data) % 16 == 0 &&
                      reinterpret_cast<uintptr_t>(y->data) % 16 == 0 && (xp * es) % 16 == 0 &&
                      (yp * es) % 16 == 0;
  hipError_t e = rf::launch_softmax(x->data, y->data, x->dtype == RF_BF16, rows, n, xp, yp, vec_ok,
                                    (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_variance(const rf_tensor* x, rf_tensor* mean, rf_tensor* var, rf_stream stream) {
  rf_status st;
  if ((st = check_tensor(x, 1, RF_MAX_DIMS)) != RF_OK) return st;
  if ((st = check_tensor(mean, 1, RF_MAX_DIMS)) != RF_OK) return st;
  if ((st = check_tensor(var, 1, RF_MAX_DIMS)) != RF_OK) return st;
  if (mean->dtype != RF_F32 || var->dtype != RF_F32) return RF_ERR_UNSUPPORTED;
  const int nd = x->ndim;
  // outputs: x.shape without its last axis ([1] for a 1-D x), contiguous
  if (!same_shape(mean, var)) return RF_ERR_INVALID_ARG;
  if (nd == 1) {
    if (mean->ndim != 1 || mean->shape[0] != 1) return RF_ERR_INVALID_ARG;
  } else {
    if (mean->ndim != nd - 1) return RF_ERR_INVALID_ARG;
    for (int i = 0; i < nd - 1; ++i)
      if (mean->shape[i] != x->shape[i]) return RF_ERR_INVALID_ARG;
  }
  if (!is_contiguous(mean) || !is_contiguous(var)) return RF_ERR_UNSUPPORTED;
  const int64_t n = x->shape[nd - 1];
  int64_t rows, xp;
  if (!collapse_rows(x, &rows, &xp)) return RF_ERR_UNSUPPORTED;
  if (rows == 0) return RF_OK;
  if (n == 0) return RF_ERR_INVALID_ARG;  // the variance of nothing is not defined
  if (x->data == nullptr || mean->data == nullptr || var->data == nullptr) return RF_ERR_INVALID_ARG;
  if (x->stride[nd - 1] != 1 && n > 1) return RF_ERR_UNSUPPORTED;
  if (rows > INT32_MAX) return RF_ERR_UNSUPPORTED;
  const size_t es = esize(x->dtype);
  const bool vec_ok = reinterpret_cast<uintptr_t>(x->data) % 16 == 0 && (xp * es) % 16 == 0;
  hipError_t e = rf::launch_variance(x->data, x->dtype == RF_BF16, (float*)mean->data,
                                     (float*)var->data, rows, n, xp, vec_ok, (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

size_t rf_moe_routing_workspace_bytes(int64_t S, int64_t hd, int64_t E) {
  if (S <= 0 || hd <= 0 || E <= 0 || S > INT32_MAX || hd > INT32_MAX) return 0;
  return (size_t)rf::moe_num_slices((int)S, (int)hd) * (size_t)S * (size_t)E * sizeof(float);
}

namespace {
// Argument checks shared by the two MoE routing entry points (everything but the workspace).
rf_status check_moe_routing(const rf_tensor* x, const rf_tensor* w, int topk, const rf_tensor* prob,
                            const rf_tensor* idx, bool* empty) {
  rf_status st;
  *empty = false;
  if ((st = check_tensor(x, 2, 2)) != RF_OK) return st;
  if ((st = check_tensor(w, 2, 2)) != RF_OK) return st;
  if ((st = check_tensor(prob, 2, 2)) != RF_OK) return st;
  if ((st = check_tensor(idx, 2, 2, RF_I32)) != RF_OK) return st;
  if (x->dtype != RF_BF16 || w->dtype != RF_BF16 || prob->dtype != RF_F32 || idx->dtype != RF_I32)
    return RF_ERR_UNSUPPORTED;
  const int64_t S = x->shape[0], hd = x->shape[1], E = w->shape[1];
  if (w->shape[0] != hd) return RF_ERR_INVALID_ARG;
  if (topk < 1 || topk > E) return RF_ERR_INVALID_ARG;
  if (prob->shape[0] != S || prob->shape[1] != topk || !same_shape(prob, idx)) return RF_ERR_INVALID_ARG;
  if (S == 0) { *empty = true; return RF_OK; }
  if (hd == 0 || hd % 128 != 0 || (E != 32 && E != 64 && E != 128) || topk > 16)
    return RF_ERR_UNSUPPORTED;
  if (S > INT32_MAX || hd > INT32_MAX) return RF_ERR_UNSUPPORTED;
  for (const rf_tensor* t : {x, w, (const rf_tensor*)prob, (const rf_tensor*)idx})
    if (t->shape[1] > 1 && t->stride[1] != 1) return RF_ERR_UNSUPPORTED;
  if (x->data == nullptr || w->data == nullptr || prob->data == nullptr || idx->data == nullptr)
    return RF_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(w)) return RF_ERR_ALIGNMENT;
  if (reinterpret_cast<uintptr_t>(prob->data) % 4 != 0 || reinterpret_cast<uintptr_t>(idx->data) % 4 != 0)
    return RF_ERR_ALIGNMENT;
  if (S * x->stride[0] * 2 >= ((int64_t)1 << 32) || 128 * w->stride[0] * 2 >= ((int64_t)1 << 32))
    return RF_ERR_UNSUPPORTED;
  return RF_OK;
}
}  // namespace

rf_status rf_moe_routing(const rf_tensor* x, const rf_tensor* w, int topk, rf_tensor* prob,
                         rf_tensor* idx, void* workspace, size_t workspace_bytes,
                         rf_stream stream) {
  bool empty;
  rf_status st = check_moe_routing(x, w, topk, prob, idx, &empty);
  if (st != RF_OK || empty) return st;
  const int64_t S = x->shape[0], hd = x->shape[1], E = w->shape[1];
  if (workspace == nullptr || reinterpret_cast<uintptr_t>(workspace) % 16 != 0 ||
      workspace_bytes < rf_moe_routing_workspace_bytes(S, hd, E))
    return RF_ERR_WORKSPACE;
  hipError_t e = rf::launch_moe_routing(x->data, w->data, (int)S, (int)hd, (int)E, topk,
                                        x->stride[0], w->stride[0], (float*)prob->data,
                                        (int32_t*)idx->data, prob->stride[0], idx->stride[0],
                                        (float*)workspace, (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_moe_routing_noalloc(const rf_tensor* x, const rf_tensor* w, int topk, rf_tensor* prob,
                                 rf_tensor* idx, rf_stream stream) {
  bool empty;
  rf_status st = check_moe_routing(x, w, topk, prob, idx, &empty);
  if (st != RF_OK || empty) return st;
  const int64_t S = x->shape[0], hd = x->shape[1], E = w->shape[1];
  if (rf_moe_routing_workspace_bytes(S, hd, E) > RF_MOE_ROUTING_NOALLOC_MAX_BYTES) return RF_ERR_WORKSPACE;
  hipError_t e = rf::launch_moe_routing_static(x->data, w->data, (int)S, (int)hd, (int)E, topk,
                                               x->stride[0], w->stride[0], (float*)prob->data,
                                               (int32_t*)idx->data, prob->stride[0], idx->stride[0],
                                               (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_fp8_quant_gemm(const rf_tensor* a, const rf_tensor* w, rf_tensor* c, rf_stream stream) {
  rf_status st;
  if ((st = check_tensor(a, 2, 2)) != RF_OK) return st;
  if ((st = check_tensor(w, 2, 2, RF_FP8_E4M3)) != RF_OK) return st;
  if ((st = check_tensor(c, 2, 2)) != RF_OK) return st;
  if (a->dtype != RF_BF16 || w->dtype != RF_FP8_E4M3 || c->dtype != RF_BF16) return RF_ERR_UNSUPPORTED;
  const int64_t M = a->shape[0], K = a->shape[1], N = w->shape[0];
  if (w->shape[1] != K || c->shape[0] != M || c->shape[1] != N) return RF_ERR_INVALID_ARG;
  if (M == 0 || N == 0) return RF_OK;
  if (K == 0 || K % 128 != 0 || N % 8 != 0) return RF_ERR_UNSUPPORTED;
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX) return RF_ERR_UNSUPPORTED;
  for (const rf_tensor* t : {a, w, (const rf_tensor*)c})
    if (t->shape[1] > 1 && t->stride[1] != 1) return RF_ERR_UNSUPPORTED;
  if (a->data == nullptr || w->data == nullptr || c->data == nullptr) return RF_ERR_INVALID_ARG;
  if (!aligned16(a) || !aligned16(w) || !aligned16(c)) return RF_ERR_ALIGNMENT;
  if (128 * a->stride[0] * 2 >= ((int64_t)1 << 32) || N * w->stride[0] >= ((int64_t)1 << 32))
    return RF_ERR_UNSUPPORTED;
  hipError_t e = rf::launch_fp8_quant_gemm(a->data, w->data, c->data, (int)M, (int)K, (int)N,
                                           a->stride[0], w->stride[0], c->stride[0],
                                           (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_cascade_attention(const rf_tensor* q, const rf_tensor* k, const rf_tensor* v,
                               rf_tensor* o, float scale, int causal, rf_stream stream) {
  rf::AttnShape a{};
  rf_status st;
  if ((st = check_qkv(q, k, v, &a)) != RF_OK) return st;
  if ((st = check_tensor(o, 4, 4)) != RF_OK) return st;
  if (o->dtype != q->dtype) return RF_ERR_UNSUPPORTED;
  if (!same_shape(o, q)) return RF_ERR_INVALID_ARG;
  if (o->shape[3] > 1 && o->stride[3] != 1) return RF_ERR_UNSUPPORTED;
  if (a.d != 64 && a.d != 128) return RF_ERR_UNSUPPORTED;
  if (numel(q) == 0) return RF_OK;
  if (q->data == nullptr || o->data == nullptr) return RF_ERR_INVALID_ARG;
  if (a.Lk > 0 && (k->data == nullptr || v->data == nullptr)) return RF_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(o) || (a.Lk > 0 && (!aligned16(k) || !aligned16(v))))
    return RF_ERR_ALIGNMENT;
  a.scale = scale;
  a.causal = causal != 0;
  hipError_t e;
  if (q->dtype == RF_F32)
    e = rf::launch_attention_f32((const float*)q->data, (const float*)k->data,
                                 (const float*)v->data, (float*)o->data, strides4(q), strides4(k),
                                 strides4(v), strides4(o), a, (hipStream_t)stream);
  else
    e = rf::launch_attention_bf16(q->data, k->data, v->data, o->data, strides4(q), strides4(k),
                                  strides4(v), strides4(o), a, (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_diag_attention_wide(const rf_tensor* q, const rf_tensor* k, const rf_tensor* v,
                                 rf_tensor* o, float scale, rf_stream stream) {
  rf::AttnShape a{};
  rf_status st;
  if ((st = check_qkv(q, k, v, &a)) != RF_OK) return st;
  if ((st = check_tensor(o, 4, 4)) != RF_OK) return st;
  if (o->dtype != q->dtype) return RF_ERR_UNSUPPORTED;
  if (!same_shape(o, q)) return RF_ERR_INVALID_ARG;
  if (o->shape[3] > 1 && o->stride[3] != 1) return RF_ERR_UNSUPPORTED;
  if (q->dtype != RF_BF16 || a.d != 128 || a.Lk < 64) return RF_ERR_UNSUPPORTED;
  if (k->stride[2] >= (1 << 24) || v->stride[2] >= (1 << 24)) return RF_ERR_UNSUPPORTED;
  if (numel(q) == 0) return RF_OK;
  if (q->data == nullptr || o->data == nullptr || k->data == nullptr || v->data == nullptr)
    return RF_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(o) || !aligned16(k) || !aligned16(v)) return RF_ERR_ALIGNMENT;
  a.scale = scale;
  a.causal = false;
  const hipError_t e = rf::launch_attention_bf16_wide(q->data, k->data, v->data, o->data, strides4(q),
                                                      strides4(k), strides4(v), strides4(o), a,
                                                      (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_cascade_attention_splitk(const rf_tensor* q, const rf_tensor* k, const rf_tensor* v,
                                      int num_splits, rf_tensor* part_m, rf_tensor* part_l,
                                      rf_tensor* part_acc, float scale, int causal,
                                      rf_stream stream) {
  rf::AttnShape a{};
  rf_status st;
  if ((st = check_qkv(q, k, v, &a)) != RF_OK) return st;
  if (num_splits < 1) return RF_ERR_INVALID_ARG;
  if (q->dtype != RF_BF16) return RF_ERR_UNSUPPORTED;
  if (a.d != 128) return RF_ERR_UNSUPPORTED;
  if ((st = check_tensor(part_m, 4, 4)) != RF_OK) return st;
  if ((st = check_tensor(part_l, 4, 4)) != RF_OK) return st;
  if ((st = check_tensor(part_acc, 5, 5)) != RF_OK) return st;
  if (part_m->dtype != RF_F32 || part_l->dtype != RF_F32 || part_acc->dtype != RF_F32)
    return RF_ERR_WORKSPACE;
  const int64_t want[5] = {a.B, a.Hq, a.Lq, num_splits, a.d};
  for (int i = 0; i < 4; ++i)
    if (part_m->shape[i] != want[i] || part_l->shape[i] != want[i]) return RF_ERR_WORKSPACE;
  for (int i = 0; i < 5; ++i)
    if (part_acc->shape[i] != want[i]) return RF_ERR_WORKSPACE;
  if (!is_contiguous(part_m) || !is_contiguous(part_l) || !is_contiguous(part_acc))
    return RF_ERR_WORKSPACE;
  if (numel(q) == 0) return RF_OK;
  if (q->data == nullptr || part_m->data == nullptr || part_l->data == nullptr ||
      part_acc->data == nullptr)
    return RF_ERR_INVALID_ARG;
  if (a.Lk > 0 && (k->data == nullptr || v->data == nullptr)) return RF_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(part_acc) || (a.Lk > 0 && (!aligned16(k) || !aligned16(v))))
    return RF_ERR_ALIGNMENT;
  a.scale = scale;
  a.causal = causal != 0;
  hipError_t e = rf::launch_attention_splitk_bf16(
      q->data, k->data, v->data, strides4(q), strides4(k), strides4(v), num_splits,
      (float*)part_m->data, (float*)part_l->data, (float*)part_acc->data, a, (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_merge_states(const rf_tensor* part_m, const rf_tensor* part_l,
                          const rf_tensor* part_acc, rf_tensor* o, rf_stream stream) {
  rf_status st;
  if ((st = check_tensor(part_m, 4, 4)) != RF_OK) return st;
  if ((st = check_tensor(part_l, 4, 4)) != RF_OK) return st;
  if ((st = check_tensor(part_acc, 5, 5)) != RF_OK) return st;
  if ((st = check_tensor(o, 4, 4)) != RF_OK) return st;
  if (part_m->dtype != RF_F32 || part_l->dtype != RF_F32 || part_acc->dtype != RF_F32)
    return RF_ERR_WORKSPACE;
  if (!same_shape(part_m, part_l)) return RF_ERR_WORKSPACE;
  for (int i = 0; i < 4; ++i)
    if (part_acc->shape[i] != part_m->shape[i]) return RF_ERR_WORKSPACE;
  if (!is_contiguous(part_m) || !is_contiguous(part_l) || !is_contiguous(part_acc))
    return RF_ERR_WORKSPACE;
  const int64_t S = part_m->shape[3], d = part_acc->shape[4];
  for (int i = 0; i < 3; ++i)
    if (o->shape[i] != part_m->shape[i] || o->shape[i] > INT32_MAX) return RF_ERR_INVALID_ARG;
  if (o->shape[3] != d) return RF_ERR_INVALID_ARG;
  if (o->shape[3] > 1 && o->stride[3] != 1) return RF_ERR_UNSUPPORTED;
  if (numel(o) == 0) return RF_OK;
  if (S < 1) return RF_ERR_INVALID_ARG;
  if (d % 4 != 0 || d > 1024 || S > INT32_MAX) return RF_ERR_UNSUPPORTED;
  if (part_m->data == nullptr || part_l->data == nullptr || part_acc->data == nullptr ||
      o->data == nullptr)
    return RF_ERR_INVALID_ARG;
  if (!aligned16(part_acc)) return RF_ERR_ALIGNMENT;
  for (int i = 0; i < 3; ++i)
    if (o->shape[i] > 1 && (o->stride[i] * (int64_t)esize(o->dtype)) % 8 != 0)
      return RF_ERR_ALIGNMENT;
  if (reinterpret_cast<uintptr_t>(o->data) % 8 != 0) return RF_ERR_ALIGNMENT;
  hipError_t e = rf::launch_merge_states(
      (const float*)part_m->data, (const float*)part_l->data, (const float*)part_acc->data, o->data,
      o->dtype == RF_BF16, (int)o->shape[0], (int)o->shape[1], (int)o->shape[2], (int)S, (int)d,
      strides4(o), (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_rmsnorm_gemm(const rf_tensor* x, const rf_tensor* g, const rf_tensor* w, rf_tensor* y,
                          float eps, rf_stream stream) {
  rf_status st;
  if ((st = check_tensor(x, 2, 2)) != RF_OK) return st;
  if ((st = check_tensor(g, 1, 1)) != RF_OK) return st;
  if ((st = check_tensor(w, 2, 2)) != RF_OK) return st;
  if ((st = check_tensor(y, 2, 2)) != RF_OK) return st;
  if (x->dtype != RF_BF16 || g->dtype != RF_BF16 || w->dtype != RF_BF16 || y->dtype != RF_BF16)
    return RF_ERR_UNSUPPORTED;
  const int64_t M = x->shape[0], K = x->shape[1], N = w->shape[1];
  if (g->shape[0] != K || w->shape[0] != K || y->shape[0] != M || y->shape[1] != N)
    return RF_ERR_INVALID_ARG;
  if ((K > 1 && x->stride[1] != 1) || (N > 1 && (w->stride[1] != 1 || y->stride[1] != 1)) ||
      (K > 1 && g->stride[0] != 1))
    return RF_ERR_UNSUPPORTED;
  if (M > INT32_MAX || K > INT32_MAX || N > INT32_MAX) return RF_ERR_UNSUPPORTED;
  if (M == 0 || N == 0) return RF_OK;
  if (K == 0 || K % 64 != 0 || N % 8 != 0) return RF_ERR_UNSUPPORTED;
  if (x->data == nullptr || g->data == nullptr || w->data == nullptr || y->data == nullptr)
    return RF_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(g) || !aligned16(w) || !aligned16(y)) return RF_ERR_ALIGNMENT;
  // the kernel addresses a 128-row tile of x and a 64-row tile of w with 32-bit byte offsets
  if (x->stride[0] >= (1 << 24) || w->stride[0] >= (1 << 24)) return RF_ERR_UNSUPPORTED;
  hipError_t e = rf::launch_rmsnorm_gemm_bf16(x->data, g->data, w->data, y->data, (int)M, (int)K,
                                              (int)N, x->stride[0], w->stride[0], y->stride[0], eps,
                                              (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_diag_softmax_level(const rf_tensor* x, rf_tensor* y, int level, float* ml_buf,
                                rf_stream stream) {
  rf_status st;
  if ((st = check_tensor(x, 2, 2)) != RF_OK) return st;
  if ((st = check_tensor(y, 2, 2)) != RF_OK) return st;
  if (x->dtype != RF_BF16 || y->dtype != RF_BF16) return RF_ERR_UNSUPPORTED;
  if (!same_shape(x, y)) return RF_ERR_INVALID_ARG;
  if (level < 0 || level > 4) return RF_ERR_INVALID_ARG;
  const int64_t rows = x->shape[0], n = x->shape[1];
  if (rows == 0 || n == 0) return RF_OK;
  if (n % 8 != 0 || n > 8192 || rows > INT32_MAX) return RF_ERR_UNSUPPORTED;
  if ((n > 1 && (x->stride[1] != 1 || y->stride[1] != 1))) return RF_ERR_UNSUPPORTED;
  if (x->data == nullptr || y->data == nullptr || ((level == 0 || level == 4) && ml_buf == nullptr)) return RF_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(y)) return RF_ERR_ALIGNMENT;
  hipError_t e = rf::launch_softmax_level(x->data, y->data, rows, n, x->stride[0], y->stride[0], level,
                                          ml_buf, (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_diag_copy(const void* src, void* dst, int64_t bytes, rf_stream stream) {
  if (bytes < 0) return RF_ERR_INVALID_ARG;
  if (bytes == 0) return RF_OK;
  if (src == nullptr || dst == nullptr) return RF_ERR_INVALID_ARG;
  if (bytes % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(dst) % 16 != 0)
    return RF_ERR_ALIGNMENT;
  hipError_t e = rf::launch_diag_copy(src, dst, bytes, (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_diag_read(const void* src, int64_t bytes, void* sink, rf_stream stream) {
  if (bytes < 0) return RF_ERR_INVALID_ARG;
  if (bytes == 0) return RF_OK;
  if (src == nullptr || sink == nullptr) return RF_ERR_INVALID_ARG;
  if (bytes % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(sink) % 4 != 0)
    return RF_ERR_ALIGNMENT;
  hipError_t e = rf::launch_diag_read(src, bytes, sink, (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

rf_status rf_diag_mfma(float* sink, int workgroups, int iters, int random_operands,
                       rf_stream stream) {
  if (sink == nullptr || workgroups < 1 || iters < 0 || workgroups > (1 << 20))
    return RF_ERR_INVALID_ARG;
  hipError_t e = rf::launch_diag_mfma(sink, workgroups, iters, random_operands != 0,
                                      (hipStream_t)stream);
  return e == hipSuccess ? RF_OK : RF_ERR_LAUNCH;
}

}  // extern "C"
