// C ABI of the MaskKV library: argument validation and marshalling only; all arithmetic is in the kernels.
#include <math.h>
#include <mutex>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "kernels.hpp"

namespace maskkv {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int check_launch(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return MASKKV_OK;
  set_error("%s: %s", what, hipGetErrorString(e));
  return MASKKV_EHIP;
}

namespace {

int elem_bytes(const maskkv_desc* d) { return d->dtype == MASKKV_BF16 ? 2 : 4; }

int check_desc(const maskkv_desc* d, Lens* lens) {
  if (!d) {
    set_error("desc is NULL");
    return MASKKV_EINVAL;
  }
  if (d->dtype != MASKKV_F32 && d->dtype != MASKKV_BF16) {
    set_error("dtype %d is neither MASKKV_F32 nor MASKKV_BF16", d->dtype);
    return MASKKV_EDTYPE;
  }
  if (d->d != 64 && d->d != 128) {
    set_error("head_dim %d unsupported (64 or 128)", d->d);
    return MASKKV_ESHAPE;
  }
  if (d->B < 1 || d->B > MASKKV_MAX_BATCH) {
    set_error("B = %d outside 1..%d", d->B, MASKKV_MAX_BATCH);
    return MASKKV_ESHAPE;
  }
  if (d->H < 1 || d->H > 65535 || (int64_t)d->B * d->H > 65535) {
    set_error("H = %d (B*H = %lld) outside 1..65535", d->H, (long long)d->B * d->H);
    return MASKKV_ESHAPE;
  }
  if (d->n_resp < 1 || d->n_query < 1 || d->P_max < 0 || d->q_per_kv < 0 || d->q_per_kv > 64) {
    set_error("n_resp = %d, n_query = %d must be >= 1, P_max = %d >= 0, q_per_kv = %d in 0..64", d->n_resp, d->n_query,
              d->P_max, d->q_per_kv);
    return MASKKV_EINVAL;
  }
  if ((int64_t)d->n_query * query_heads_per_kv(d) > (1 << 20) || (int64_t)d->n_resp * query_heads_per_kv(d) > (1 << 20)) {
    set_error("more than 2^20 query rows per key/value head (n_query %d, n_resp %d, q_per_kv %d)", d->n_query,
              d->n_resp, d->q_per_kv);
    return MASKKV_ESHAPE;
  }
  if ((int64_t)d->P_max + d->n_resp > (1 << 30)) {
    set_error("sequence length %lld too large", (long long)d->P_max + d->n_resp);
    return MASKKV_ESHAPE;
  }
  for (int b = 0; b < MASKKV_MAX_BATCH; ++b) lens->P[b] = 0;
  for (int b = 0; b < d->B; ++b) {
    const int p = d->prompt_len ? d->prompt_len[b] : d->P_max;
    if (p < 0 || p > d->P_max) {
      set_error("prompt_len[%d] = %d outside 0..P_max = %d", b, p, d->P_max);
      return MASKKV_EINVAL;
    }
    lens->P[b] = p;
  }
  return MASKKV_OK;
}

int make_view(const maskkv_desc* d, const maskkv_tensor* t, const char* name, View* v) {
  if (!t || !t->ptr) {
    set_error("%s is NULL", name);
    return MASKKV_EINVAL;
  }
  const int64_t eb = elem_bytes(d);
  if (t->stride_t < d->d || t->stride_h < 0 || t->stride_b < 0) {
    set_error("%s: strides (b=%lld, h=%lld, t=%lld) invalid for head_dim %d", name, (long long)t->stride_b,
              (long long)t->stride_h, (long long)t->stride_t, d->d);
    return MASKKV_EINVAL;
  }
  if (t->stride_t * eb > (int64_t)1 << 24) {  // kernels keep row offsets inside a 64-row tile in 32 bits
    set_error("%s: token stride of %lld bytes exceeds the supported 16 MiB", name, (long long)(t->stride_t * eb));
    return MASKKV_EINVAL;
  }
  if (((uintptr_t)t->ptr & 15) || ((t->stride_b * eb) & 15) || ((t->stride_h * eb) & 15) || ((t->stride_t * eb) & 15)) {
    set_error("%s: pointer and strides must be multiples of 16 bytes", name);
    return MASKKV_EINVAL;
  }
  v->ptr = reinterpret_cast<char*>(t->ptr);
  v->stride_h = t->stride_h * eb;
  v->stride_t = t->stride_t * eb;
  for (int b = 0; b < MASKKV_MAX_BATCH; ++b) v->boff[b] = 0;
  for (int b = 0; b < d->B; ++b) {
    const int64_t s = t->seq_start ? t->seq_start[b] : 0;
    if (s < 0) {
      set_error("%s: seq_start[%d] negative", name, b);
      return MASKKV_EINVAL;
    }
    v->boff[b] = ((int64_t)b * t->stride_b + s * t->stride_t) * eb;
  }
  return MASKKV_OK;
}

int check_workspace(const char* what, void* ws, size_t have, size_t need) {
  if (need == 0) return MASKKV_OK;
  if (!ws || have < need) {
    set_error("%s: workspace of %zu bytes given, %zu needed", what, ws ? have : (size_t)0, need);
    return MASKKV_EWORKSPACE;
  }
  if ((uintptr_t)ws & 255) {
    set_error("%s: workspace must be 256-byte aligned", what);
    return MASKKV_EWORKSPACE;
  }
  return MASKKV_OK;
}

float pick_scale(const maskkv_desc* d, float scale) { return scale > 0.f ? scale : 1.0f / sqrtf((float)d->d); }

// ---- static scratch of maskkv_score_static: one copy per GPU for the life of the process
constexpr size_t kStaticScratchBytes = MASKKV_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU (null: not asked for yet)

// Device address of this GPU's copy of `scratch` (the array's name is only a host-side handle: kernels are always
// given this pointer).  Resolved once per device, with that device current.
int static_scratch(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_error("score_static: hipGetDevice: %s (device %d)", hipGetErrorString(e), dev);
    (void)hipGetLastError();
    return MASKKV_EHIP;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      set_error("score_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
      (void)hipGetLastError();
      return MASKKV_EHIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return MASKKV_OK;
}

}  // namespace
}  // namespace maskkv

namespace maskkv {

// maskkv_score with optional stage marks (see kernels.hpp).
int score_entry(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full, float scale,
                float* scores, int64_t score_stride, float* prompt_mass, void* workspace, size_t workspace_bytes,
                void* stream, void* const* events) {
  Lens lens;
  View q, k;
  if (int e = check_desc(desc, &lens)) return e;
  if (int e = make_view(desc, Q_mask, "Q_mask", &q)) return e;
  if (int e = make_view(desc, K_full, "K_full", &k)) return e;
  if (!scores || score_stride < desc->P_max) {
    set_error("scores is NULL or score_stride %lld < P_max %d", (long long)score_stride, desc->P_max);
    return MASKKV_EINVAL;
  }
  if (int e = check_workspace("score", workspace, workspace_bytes, score_workspace_bytes(desc, lens))) return e;
  return launch_score(desc, q, k, lens, pick_scale(desc, scale), scores, score_stride, prompt_mass, workspace,
                      reinterpret_cast<hipStream_t>(stream), events);
}

}  // namespace maskkv

using namespace maskkv;

extern "C" {

int maskkv_version(void) { return MASKKV_VERSION; }

const char* maskkv_strerror(int status) {
  switch (status) {
    case MASKKV_OK: return "ok";
    case MASKKV_EINVAL: return "invalid argument";
    case MASKKV_ESHAPE: return "unsupported shape";
    case MASKKV_EDTYPE: return "unsupported dtype";
    case MASKKV_EWORKSPACE: return "workspace missing, too small or misaligned";
    case MASKKV_EHIP: return "HIP launch failed";
    case MASKKV_ECAPACITY: return "output capacity too small";
    default: return "unknown status";
  }
}

const char* maskkv_last_error(void) { return g_err; }

int maskkv_score_workspace_bytes(const maskkv_desc* desc, size_t* bytes) {
  Lens lens;
  if (int e = check_desc(desc, &lens)) return e;
  if (!bytes) {
    set_error("bytes is NULL");
    return MASKKV_EINVAL;
  }
  *bytes = score_workspace_bytes(desc, lens);
  return MASKKV_OK;
}

int maskkv_score(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full, float scale,
                 float* scores, int64_t score_stride, float* prompt_mass, void* workspace, size_t workspace_bytes,
                 void* stream) {
  return score_entry(desc, Q_mask, K_full, scale, scores, score_stride, prompt_mass, workspace, workspace_bytes,
                     stream, nullptr);
}

int maskkv_score_given_lse(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full,
                           float scale, const float* row_lse, float* scores, int64_t score_stride,
                           float* prompt_mass, void* workspace, size_t workspace_bytes, void* stream) {
  Lens lens;
  View q, k;
  if (int e = check_desc(desc, &lens)) return e;
  if (int e = make_view(desc, Q_mask, "Q_mask", &q)) return e;
  if (int e = make_view(desc, K_full, "K_full", &k)) return e;
  if (!row_lse || !scores || score_stride < desc->P_max) {
    set_error("row_lse or scores is NULL, or score_stride %lld < P_max %d", (long long)score_stride, desc->P_max);
    return MASKKV_EINVAL;
  }
  if (int e = check_workspace("score_given_lse", workspace, workspace_bytes, score_workspace_bytes(desc, lens)))
    return e;
  return launch_score(desc, q, k, lens, pick_scale(desc, scale), scores, score_stride, prompt_mass, workspace,
                      reinterpret_cast<hipStream_t>(stream), nullptr, row_lse);
}

int maskkv_score_static(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full, float scale,
                        float* scores, int64_t score_stride, float* prompt_mass, void* stream) {
  Lens lens;
  View q, k;
  if (int e = check_desc(desc, &lens)) return e;
  if (int e = make_view(desc, Q_mask, "Q_mask", &q)) return e;
  if (int e = make_view(desc, K_full, "K_full", &k)) return e;
  if (!scores || score_stride < desc->P_max) {
    set_error("scores is NULL or score_stride %lld < P_max %d", (long long)score_stride, desc->P_max);
    return MASKKV_EINVAL;
  }
  const size_t need = score_workspace_bytes(desc, lens);
  if (need > kStaticScratchBytes) {
    set_error("score_static: this description needs %zu bytes of scratch, the static array holds %zu; use maskkv_score "
              "with a caller workspace", need, kStaticScratchBytes);
    return MASKKV_EWORKSPACE;
  }
  void* ws = nullptr;
  if (int e = static_scratch(&ws)) return e;
  return launch_score(desc, q, k, lens, pick_scale(desc, scale), scores, score_stride, prompt_mass, ws,
                      reinterpret_cast<hipStream_t>(stream), nullptr);
}

int maskkv_select_workspace_bytes(const maskkv_desc* desc, size_t* bytes) {
  Lens lens;
  if (int e = check_desc(desc, &lens)) return e;
  if (!bytes) {
    set_error("bytes is NULL");
    return MASKKV_EINVAL;
  }
  *bytes = select_workspace_bytes(desc);
  return MASKKV_OK;
}

// Validation of maskkv_select: everything the host can know.
static int check_select(const maskkv_desc* desc, const Lens& lens, const float* scores, int64_t score_stride,
                        int pool_window, int pool_mode, const int32_t* budgets, const int32_t* budgets_host,
                        const int32_t* idx, const int32_t* cu_budget, int64_t capacity) {
  if (!scores || !budgets || !cu_budget || score_stride < desc->P_max) {
    set_error("select: scores, budgets or cu_budget NULL, or score_stride %lld < P_max %d", (long long)score_stride,
              desc->P_max);
    return MASKKV_EINVAL;
  }
  if (pool_window < 1 || pool_window > 63 || (pool_window & 1) == 0) {
    set_error("pool_window %d must be odd and in 1..63", pool_window);
    return MASKKV_EINVAL;
  }
  if (pool_mode != MASKKV_POOL_MEAN && pool_mode != MASKKV_POOL_MAX) {
    set_error("pool_mode %d unknown", pool_mode);
    return MASKKV_EINVAL;
  }
  if (capacity < 0 || capacity > 0x7FFFFFFF || (capacity > 0 && !idx)) {
    set_error("select: capacity %lld invalid or idx NULL", (long long)capacity);
    return MASKKV_EINVAL;
  }
  if (desc->P_max > select_max_prompt()) {
    set_error("select: prompts above %lld tokens are not supported (P_max = %d)", (long long)select_max_prompt(),
              desc->P_max);
    return MASKKV_ESHAPE;
  }
  int64_t worst = 0;  // the prefix sums of the clamped budgets are 32-bit
  for (int b = 0; b < desc->B; ++b) worst += (int64_t)desc->H * lens.P[b];
  if (worst > 0x7FFFFFFF) {
    set_error("select: B*H*P = %lld kept rows in the worst case do not fit 32-bit offsets", (long long)worst);
    return MASKKV_ESHAPE;
  }
  if (budgets_host) {
    int64_t sum = 0;
    for (int b = 0; b < desc->B; ++b)
      for (int h = 0; h < desc->H; ++h) {
        const int32_t k = budgets_host[b * desc->H + h];
        if (k < 0) {
          set_error("select: budget %d of (sequence %d, head %d) is negative", k, b, h);
          return MASKKV_EINVAL;
        }
        sum += k < lens.P[b] ? k : lens.P[b];
      }
    if (sum > capacity) {
      set_error("select: the budgets keep %lld rows, capacity is %lld", (long long)sum, (long long)capacity);
      return MASKKV_ECAPACITY;
    }
  }
  return MASKKV_OK;
}

int maskkv_select(const maskkv_desc* desc, const float* scores, int64_t score_stride, int pool_window, int pool_mode,
                  const int32_t* budgets, const int32_t* budgets_host, int32_t* idx, int32_t* cu_budget,
                  int64_t capacity, void* workspace, size_t workspace_bytes, void* stream) {
  Lens lens;
  if (int e = check_desc(desc, &lens)) return e;
  if (int e = check_select(desc, lens, scores, score_stride, pool_window, pool_mode, budgets, budgets_host, idx,
                           cu_budget, capacity))
    return e;
  if (int e = check_workspace("select", workspace, workspace_bytes, select_workspace_bytes(desc))) return e;
  return launch_select(desc, lens, scores, score_stride, pool_window, pool_mode, budgets, idx, cu_budget, capacity,
                       workspace, reinterpret_cast<hipStream_t>(stream));
}

int maskkv_compact(const maskkv_desc* desc, const maskkv_tensor* K, const maskkv_tensor* V, const int32_t* idx,
                   const int32_t* cu_budget, int64_t capacity, void* Kc, void* Vc, void* stream) {
  Lens lens;
  View k, v;
  if (int e = check_desc(desc, &lens)) return e;
  if (int e = make_view(desc, K, "K", &k)) return e;
  if (int e = make_view(desc, V, "V", &v)) return e;
  if (!cu_budget || capacity < 0 || capacity > 0x7FFFFFFF || (capacity > 0 && (!idx || !Kc || !Vc))) {
    set_error("compact: cu_budget NULL, capacity %lld invalid, or idx/Kc/Vc NULL", (long long)capacity);
    return MASKKV_EINVAL;
  }
  if (((uintptr_t)Kc & 15) || ((uintptr_t)Vc & 15)) {
    set_error("compact: Kc and Vc must be 16-byte aligned");
    return MASKKV_EINVAL;
  }
  return launch_compact(desc, lens, k, v, idx, cu_budget, capacity, Kc, Vc, reinterpret_cast<hipStream_t>(stream));
}

int maskkv_attend_workspace_bytes(const maskkv_desc* desc, int full, size_t* bytes) {
  Lens lens;
  if (int e = check_desc(desc, &lens)) return e;
  if (!bytes) {
    set_error("bytes is NULL");
    return MASKKV_EINVAL;
  }
  *bytes = attend_workspace_bytes(desc, full != 0);
  return MASKKV_OK;
}

int maskkv_attend(const maskkv_desc* desc, const maskkv_tensor* Q_resp, const void* Kc, const void* Vc,
                  const int32_t* cu_budget, int64_t capacity, const maskkv_tensor* K_resp,
                  const maskkv_tensor* V_resp, float scale, const maskkv_tensor* O, float* lse, void* workspace,
                  size_t workspace_bytes, void* stream) {
  Lens lens;
  View q, k2, v2, o;
  if (int e = check_desc(desc, &lens)) return e;
  if (int e = make_view(desc, Q_resp, "Q_resp", &q)) return e;
  if (int e = make_view(desc, K_resp, "K_resp", &k2)) return e;
  if (int e = make_view(desc, V_resp, "V_resp", &v2)) return e;
  if (int e = make_view(desc, O, "O", &o)) return e;
  if (!cu_budget || capacity < 0 || capacity > 0x7FFFFFFF || (capacity > 0 && (!Kc || !Vc))) {
    set_error("attend: cu_budget NULL, capacity %lld invalid, or Kc/Vc NULL", (long long)capacity);
    return MASKKV_EINVAL;
  }
  if (((uintptr_t)Kc & 15) || ((uintptr_t)Vc & 15)) {
    set_error("attend: Kc and Vc must be 16-byte aligned");
    return MASKKV_EINVAL;
  }
  if (int e = check_workspace("attend", workspace, workspace_bytes, attend_workspace_bytes(desc, false))) return e;
  return launch_attend(desc, lens, false, q, Kc, Vc, cu_budget, capacity, k2, v2, pick_scale(desc, scale), o, lse,
                       workspace, reinterpret_cast<hipStream_t>(stream));
}

int maskkv_attend_full(const maskkv_desc* desc, const maskkv_tensor* Q_resp, const maskkv_tensor* K_full,
                       const maskkv_tensor* V_full, float scale, const maskkv_tensor* O, float* lse, void* workspace,
                       size_t workspace_bytes, void* stream) {
  Lens lens;
  View q, k2, v2, o;
  if (int e = check_desc(desc, &lens)) return e;
  if (int e = make_view(desc, Q_resp, "Q_resp", &q)) return e;
  if (int e = make_view(desc, K_full, "K_full", &k2)) return e;
  if (int e = make_view(desc, V_full, "V_full", &v2)) return e;
  if (int e = make_view(desc, O, "O", &o)) return e;
  if (int e = check_workspace("attend_full", workspace, workspace_bytes, attend_workspace_bytes(desc, true))) return e;
  return launch_attend(desc, lens, true, q, nullptr, nullptr, nullptr, 0, k2, v2, pick_scale(desc, scale), o, lse,
                       workspace, reinterpret_cast<hipStream_t>(stream));
}

int maskkv_head_budgets(const maskkv_desc* desc, const float* prompt_mass, int32_t k_l, float alpha, int32_t* budgets,
                        void* stream) {
  Lens lens;
  if (int e = check_desc(desc, &lens)) return e;
  if (!prompt_mass || !budgets || k_l < 0 || !(alpha >= 0.f && alpha <= 1.f)) {
    set_error("head_budgets: NULL pointer, k_l %d < 0 or alpha %g outside [0, 1]", k_l, (double)alpha);
    return MASKKV_EINVAL;
  }
  return launch_head_budgets(desc, prompt_mass, k_l, alpha, budgets, reinterpret_cast<hipStream_t>(stream));
}

int maskkv_layer_importance_workspace_bytes(size_t* bytes) {
  if (!bytes) {
    set_error("bytes is NULL");
    return MASKKV_EINVAL;
  }
  *bytes = layer_importance_workspace_bytes();
  return MASKKV_OK;
}

int maskkv_layer_importance(const void* h_in, const void* h_out, int64_t n_tokens, int32_t hidden, int32_t dtype,
                            int64_t row_stride, float* importance, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (dtype != MASKKV_F32 && dtype != MASKKV_BF16) {
    set_error("dtype %d is neither MASKKV_F32 nor MASKKV_BF16", dtype);
    return MASKKV_EDTYPE;
  }
  const int64_t eb = dtype == MASKKV_BF16 ? 2 : 4;
  if (!h_in || !h_out || !importance || n_tokens < 1 || hidden < 8 || (hidden & 7) || row_stride < hidden) {
    set_error("layer_importance: NULL pointer, n_tokens %lld < 1, hidden %d not a positive multiple of 8, or "
              "row_stride %lld < hidden", (long long)n_tokens, hidden, (long long)row_stride);
    return MASKKV_EINVAL;
  }
  if (((uintptr_t)h_in & 15) || ((uintptr_t)h_out & 15) || ((row_stride * eb) & 15) || ((hidden * eb) & 15)) {
    set_error("layer_importance: pointers, rows and row stride must be multiples of 16 bytes");
    return MASKKV_EINVAL;
  }
  if (int e = check_workspace("layer_importance", workspace, workspace_bytes, layer_importance_workspace_bytes()))
    return e;
  return launch_layer_importance(h_in, h_out, n_tokens, hidden, dtype, row_stride * eb, importance, workspace,
                                 reinterpret_cast<hipStream_t>(stream));
}

int maskkv_value_shift(const void* V_now, const void* V_prev, int64_t n_tokens, int32_t width, int32_t dtype,
                       int64_t row_stride, float delta, float* cos, int32_t* refresh, int32_t* count, void* stream) {
  if (dtype != MASKKV_F32 && dtype != MASKKV_BF16) {
    set_error("dtype %d is neither MASKKV_F32 nor MASKKV_BF16", dtype);
    return MASKKV_EDTYPE;
  }
  const int64_t eb = dtype == MASKKV_BF16 ? 2 : 4;
  if (!V_now || !V_prev || !cos || !refresh || !count || n_tokens < 1 || n_tokens > 0x7FFFFFFF || width < 8 ||
      (width & 7) || row_stride < width || !(delta == delta)) {
    set_error("value_shift: NULL pointer, n_tokens %lld outside 1..2^31-1, width %d not a positive multiple of 8, "
              "row_stride %lld < width, or delta is NaN", (long long)n_tokens, width, (long long)row_stride);
    return MASKKV_EINVAL;
  }
  if (((uintptr_t)V_now & 15) || ((uintptr_t)V_prev & 15) || ((row_stride * eb) & 15)) {
    set_error("value_shift: pointers and row stride must be multiples of 16 bytes");
    return MASKKV_EINVAL;
  }
  return launch_value_shift(V_now, V_prev, n_tokens, width, dtype, row_stride * eb, delta, cos, refresh, count,
                            reinterpret_cast<hipStream_t>(stream));
}

int maskkv_layer_budgets(const float* importance, int32_t n_layers, int64_t k_p, float beta, const int32_t* boundary,
                         int32_t n_boundary, int64_t* k_l) {
  if (!importance || !k_l || n_layers < 1 || k_p < 0 || !(beta >= 0.f && beta <= 1.f) || n_boundary < 0 ||
      (n_boundary > 0 && !boundary)) {
    set_error("layer_budgets: NULL pointer, n_layers %d < 1, k_p %lld < 0, beta %g outside [0, 1] or bad boundary list",
              n_layers, (long long)k_p, (double)beta);
    return MASKKV_EINVAL;
  }
  // group membership: 1 = boundary
  int first_last[2] = {0, n_layers - 1};
  const int32_t* bl = boundary ? boundary : first_last;
  const int nbl = boundary ? n_boundary : (n_layers > 1 ? 2 : 1);
  int n_b = 0;
  double imp_b = 0.0, imp_m = 0.0;
  for (int l = 0; l < n_layers; ++l) {
    if (!(importance[l] >= 0.f)) {
      set_error("layer_budgets: importance[%d] = %g is negative or NaN", l, (double)importance[l]);
      return MASKKV_EINVAL;
    }
    bool is_b = false;
    for (int i = 0; i < nbl; ++i) {
      if (bl[i] < 0 || bl[i] >= n_layers) {
        set_error("layer_budgets: boundary layer %d outside 0..%d", bl[i], n_layers - 1);
        return MASKKV_EINVAL;
      }
      is_b = is_b || bl[i] == l;
    }
    if (is_b) {
      ++n_b;
      imp_b += (double)importance[l];
    } else {
      imp_m += (double)importance[l];
    }
    k_l[l] = is_b ? 1 : 0;  // remembered until the shares are known
  }
  if (!(imp_b + imp_m > 0.0)) {
    set_error("layer_budgets: the importances sum to zero");
    return MASKKV_EINVAL;
  }
  const int n_m = n_layers - n_b;
  const int64_t k_base = (int64_t)floor((double)beta * (double)k_p / (double)n_layers);
  const double k_imp = (double)(k_p - (int64_t)n_layers * k_base);
  const double part_b = k_imp * imp_b / (imp_b + imp_m);
  const double part_m = k_imp - part_b;
  const int64_t share_b = n_b > 0 ? (int64_t)floor(part_b / n_b) : 0;
  const int64_t share_m = n_m > 0 ? (int64_t)floor(part_m / n_m) : 0;
  for (int l = 0; l < n_layers; ++l) k_l[l] = k_base + (k_l[l] ? share_b : share_m);
  return MASKKV_OK;
}

}  // extern "C"
