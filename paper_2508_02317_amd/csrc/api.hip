// Host-side entry points of the grouped expert FFN plus the library's error reporting.
// Argument validation happens here, before anything is launched.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <atomic>
#include "moe_common.h"

namespace moe {

static thread_local char g_error[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

// ---- launch bookkeeping ---------------------------------------------------------------------------
namespace {
thread_local hipError_t g_call_error = hipSuccess;    // first failed launch of the entry point running on this thread
thread_local char g_call_where[64] = "";
thread_local const char* g_call_entry = "";
thread_local hipStream_t g_call_stream = nullptr;
std::atomic<moe_launch_hook_t> g_hook{nullptr};
std::atomic<void*> g_hook_user{nullptr};
}  // namespace

void begin_call(const char* entry, hipStream_t stream) {
  (void)hipGetLastError();                             // an error left by an unrelated earlier call is not this call's
  g_call_error = hipSuccess;
  g_call_where[0] = 0;
  g_call_entry = entry;
  g_call_stream = stream;
  if (moe_launch_hook_t h = g_hook.load(std::memory_order_acquire)) h(entry, 2, stream, g_hook_user.load(std::memory_order_acquire));
}

void note_hip_failure(const char* what, hipError_t err) {
  if (err == hipSuccess || g_call_error != hipSuccess) return;
  g_call_error = err;
  snprintf(g_call_where, sizeof(g_call_where), "%s", what);
}

bool launch_begin(const char* name, hipStream_t stream) {
  if (g_call_error != hipSuccess) return false;
  if (moe_launch_hook_t h = g_hook.load(std::memory_order_acquire)) h(name, 0, stream, g_hook_user.load(std::memory_order_acquire));
  return true;
}

void launch_end(const char* name, hipStream_t stream) {
  note_hip_failure(name, hipGetLastError());
  if (moe_launch_hook_t h = g_hook.load(std::memory_order_acquire)) h(name, 1, stream, g_hook_user.load(std::memory_order_acquire));
}

int32_t end_call() {
  if (moe_launch_hook_t h = g_hook.load(std::memory_order_acquire)) h(g_call_entry, 3, g_call_stream, g_hook_user.load(std::memory_order_acquire));
  if (g_call_error == hipSuccess) return MOE_OK;
  return fail(MOE_ERR_HIP, "%s: launch of %s failed: %s (kernels enqueued before it still run; none after it was launched)", g_call_entry,
              g_call_where, hipGetErrorString(g_call_error));
}

static int32_t check_ffn_dims(const char* who, int dtype, int P, int d, int f, int E) {
  MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_ERR_UNSUPPORTED, "%s: unknown dtype %d", who, dtype);
  MOE_REQUIRE(P >= 0 && d > 0 && f > 0 && E > 0, MOE_ERR_INVALID_ARG, "%s: need P >= 0, d, f, E > 0 (P=%d d=%d f=%d E=%d)", who, P, d, f, E);
  MOE_REQUIRE(E <= kMaxExperts, MOE_ERR_UNSUPPORTED, "%s: E=%d above the built maximum %d", who, E, kMaxExperts);
  MOE_REQUIRE(d % 8 == 0 && f % 8 == 0, MOE_ERR_UNSUPPORTED, "%s: d=%d and f=%d must be multiples of 8", who, d, f);
  MOE_REQUIRE(static_cast<int64_t>(E) * d * f <= (int64_t{1} << 40), MOE_ERR_UNSUPPORTED, "%s: weights too large", who);
  return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" const char* moe_version(void) { return "0.1.0"; }
extern "C" const char* moe_last_error(void) { return g_error; }

extern "C" int32_t moe_set_launch_hook(moe_launch_hook_t hook, void* user) {
  g_hook.store(nullptr, std::memory_order_release);    // never pair the new user pointer with the old function
  g_hook_user.store(user, std::memory_order_release);
  g_hook.store(hook, std::memory_order_release);
  return MOE_OK;
}

extern "C" size_t moe_grouped_gemm_swiglu_fwd_workspace_bytes(int dtype, int P, int d, int f, int E) {
  if (P < 0 || d <= 0 || f <= 0 || E <= 0) return 0;
  return dtype == MOE_BF16 ? ffn_fwd_ws_bytes_bf16(P, d, f, E) : ffn_fwd_ws_bytes_f32(P, d, f, E);
}

extern "C" size_t moe_grouped_gemm_swiglu_bwd_workspace_bytes(int dtype, int P, int d, int f, int E, int have_saved) {
  if (P < 0 || d <= 0 || f <= 0 || E <= 0) return 0;
  return dtype == MOE_BF16 ? ffn_bwd_ws_bytes_bf16(P, d, f, E, have_saved) : ffn_bwd_ws_bytes_f32(P, d, f, E, have_saved);
}

extern "C" int32_t moe_grouped_gemm_swiglu_fwd(const void* xp, const void* w_gate, const void* w_up,
                                               const void* w_down, int dtype, int P, int d, int f, int E,
                                               const int32_t* offsets, void* g_save, void* u_save,
                                               void* act, void* yp, void* ws, size_t ws_bytes, void* stream) {
  if (int32_t rc = check_ffn_dims("ffn_fwd", dtype, P, d, f, E)) return rc;
  MOE_REQUIRE((g_save == nullptr) == (u_save == nullptr), MOE_ERR_INVALID_ARG, "ffn_fwd: g_save and u_save must both be given or both be null");
  if (P == 0) return MOE_OK;
  MOE_REQUIRE(xp && w_gate && w_up && w_down && offsets && act && yp, MOE_ERR_INVALID_ARG, "ffn_fwd: null pointer");
  MOE_REQUIRE(aligned16(xp) && aligned16(w_gate) && aligned16(w_up) && aligned16(w_down) && aligned16(act) && aligned16(yp) &&
              aligned16(g_save) && aligned16(u_save), MOE_ERR_INVALID_ARG, "ffn_fwd: tensors must be 16-byte aligned");
  const size_t need = moe_grouped_gemm_swiglu_fwd_workspace_bytes(dtype, P, d, f, E);
  MOE_REQUIRE(ws && ws_bytes >= need && aligned16(ws), MOE_ERR_WORKSPACE, "ffn_fwd: workspace null, misaligned or smaller than %zu bytes", need);
  FfnFwdArgs a{xp, w_gate, w_up, w_down, P, d, f, E, offsets, g_save, u_save, act, yp, ws, static_cast<hipStream_t>(stream)};
  begin_call("moe_grouped_gemm_swiglu_fwd", static_cast<hipStream_t>(stream));
  if (dtype == MOE_BF16) ffn_fwd_bf16(a); else ffn_fwd_f32(a);
  return end_call();
}

extern "C" int32_t moe_grouped_gemm_swiglu_bwd(const void* dyp, const void* xp, const void* g_save,
                                               const void* u_save, const void* act, const void* w_gate,
                                               const void* w_up, const void* w_down, int dtype, int P, int d,
                                               int f, int E, const int32_t* offsets, void* dxp, void* dw_gate,
                                               void* dw_up, void* dw_down, void* ws, size_t ws_bytes, void* stream) {
  if (int32_t rc = check_ffn_dims("ffn_bwd", dtype, P, d, f, E)) return rc;
  MOE_REQUIRE((g_save == nullptr) == (u_save == nullptr), MOE_ERR_INVALID_ARG, "ffn_bwd: g_save and u_save must both be given or both be null");
  MOE_REQUIRE(offsets && dw_gate && dw_up && dw_down, MOE_ERR_INVALID_ARG, "ffn_bwd: null offsets or weight-gradient pointer");
  MOE_REQUIRE(P == 0 || (dyp && xp && act && w_gate && w_up && w_down && dxp), MOE_ERR_INVALID_ARG, "ffn_bwd: null pointer");
  MOE_REQUIRE(aligned16(dyp) && aligned16(xp) && aligned16(act) && aligned16(g_save) && aligned16(u_save) && aligned16(w_gate) &&
              aligned16(w_up) && aligned16(w_down) && aligned16(dxp) && aligned16(dw_gate) && aligned16(dw_up) && aligned16(dw_down),
              MOE_ERR_INVALID_ARG, "ffn_bwd: tensors must be 16-byte aligned");
  const size_t need = moe_grouped_gemm_swiglu_bwd_workspace_bytes(dtype, P, d, f, E, g_save != nullptr);
  MOE_REQUIRE(ws && ws_bytes >= need && aligned16(ws), MOE_ERR_WORKSPACE, "ffn_bwd: workspace null, misaligned or smaller than %zu bytes", need);
  FfnBwdArgs a{dyp, xp, g_save, u_save, act, w_gate, w_up, w_down, P, d, f, E, offsets, dxp, dw_gate, dw_up, dw_down, ws,
               static_cast<hipStream_t>(stream)};
  begin_call("moe_grouped_gemm_swiglu_bwd", static_cast<hipStream_t>(stream));
  if (dtype == MOE_BF16) ffn_bwd_bf16(a); else ffn_bwd_f32(a);
  return end_call();
}

// ---- grouped FFN reading its rows by token (no expert-ordered copies) -------------------------------------
static int32_t check_gather_dims(const char* who, int dtype, int T, int k, int P, int d) {
  MOE_REQUIRE(T >= 0 && k > 0 && static_cast<int64_t>(T) * k == P, MOE_ERR_INVALID_ARG, "%s: need P == T * k (T=%d k=%d P=%d)", who, T, k, P);
  // the kernels address a token's row with a 32-bit byte offset
  MOE_REQUIRE(static_cast<int64_t>(T) * d * elem_size(dtype) < (int64_t{1} << 32) - 65536, MOE_ERR_UNSUPPORTED,
              "%s: T * d * element size must stay below 4 GiB (T=%d d=%d)", who, T, d);
  return MOE_OK;
}

extern "C" size_t moe_grouped_gemm_swiglu_fwd_gather_workspace_bytes(int dtype, int P, int d, int f, int E) {
  if (P < 0 || d <= 0 || f <= 0 || E <= 0) return 0;
  return dtype == MOE_BF16 ? ffn_fwd_gather_ws_bytes_bf16(P, d, f, E) : ffn_fwd_gather_ws_bytes_f32(P, d, f, E);
}

extern "C" size_t moe_grouped_gemm_swiglu_bwd_gather_workspace_bytes(int dtype, int P, int d, int f, int E, int have_saved) {
  if (P < 0 || d <= 0 || f <= 0 || E <= 0) return 0;
  return dtype == MOE_BF16 ? ffn_bwd_gather_ws_bytes_bf16(P, d, f, E, have_saved) : ffn_bwd_gather_ws_bytes_f32(P, d, f, E, have_saved);
}

extern "C" int32_t moe_grouped_gemm_swiglu_fwd_gather(const void* x, int T, int k, const int32_t* pair_of_row, const float* topk_w,
                                                      const void* w_gate, const void* w_up, const void* w_down, int dtype, int P,
                                                      int d, int f, int E, const int32_t* offsets, void* g_save, void* u_save,
                                                      void* act, void* yp, void* ws, size_t ws_bytes, void* stream) {
  if (int32_t rc = check_ffn_dims("ffn_fwd_gather", dtype, P, d, f, E)) return rc;
  if (int32_t rc = check_gather_dims("ffn_fwd_gather", dtype, T, k, P, d)) return rc;
  MOE_REQUIRE((g_save == nullptr) == (u_save == nullptr), MOE_ERR_INVALID_ARG, "ffn_fwd_gather: g_save and u_save must both be given or both be null");
  if (P == 0) return MOE_OK;
  MOE_REQUIRE(x && pair_of_row && w_gate && w_up && w_down && offsets && act && yp, MOE_ERR_INVALID_ARG, "ffn_fwd_gather: null pointer");
  MOE_REQUIRE(aligned16(x) && aligned16(w_gate) && aligned16(w_up) && aligned16(w_down) && aligned16(act) && aligned16(yp) &&
              aligned16(g_save) && aligned16(u_save), MOE_ERR_INVALID_ARG, "ffn_fwd_gather: tensors must be 16-byte aligned");
  const size_t need = moe_grouped_gemm_swiglu_fwd_gather_workspace_bytes(dtype, P, d, f, E);
  MOE_REQUIRE(ws && ws_bytes >= need && aligned16(ws), MOE_ERR_WORKSPACE, "ffn_fwd_gather: workspace null, misaligned or smaller than %zu bytes", need);
  FfnFwdGatherArgs a{x, T, k, pair_of_row, w_gate, w_up, w_down, P, d, f, E, offsets, g_save, u_save, act, yp, ws,
                     static_cast<hipStream_t>(stream), topk_w};
  begin_call("moe_grouped_gemm_swiglu_fwd_gather", static_cast<hipStream_t>(stream));
  if (dtype == MOE_BF16) ffn_fwd_gather_bf16(a); else ffn_fwd_gather_f32(a);
  return end_call();
}

extern "C" int32_t moe_grouped_gemm_swiglu_bwd_gather(const void* dy, const void* x, int T, int k, const float* topk_w,
                                                      const int32_t* pair_of_row, const void* g_save, const void* u_save,
                                                      const void* act_w, const void* w_gate, const void* w_up, const void* w_down,
                                                      int dtype, int P, int d, int f, int E, const int32_t* offsets, void* dxp,
                                                      void* dw_gate, void* dw_up, void* dw_down, float* dtopk_w, void* ws,
                                                      size_t ws_bytes, void* stream) {
  if (int32_t rc = check_ffn_dims("ffn_bwd_gather", dtype, P, d, f, E)) return rc;
  if (int32_t rc = check_gather_dims("ffn_bwd_gather", dtype, T, k, P, d)) return rc;
  MOE_REQUIRE((g_save == nullptr) == (u_save == nullptr), MOE_ERR_INVALID_ARG, "ffn_bwd_gather: g_save and u_save must both be given or both be null");
  MOE_REQUIRE(offsets && dw_gate && dw_up && dw_down, MOE_ERR_INVALID_ARG, "ffn_bwd_gather: null offsets or weight-gradient pointer");
  MOE_REQUIRE(P == 0 || (dy && x && topk_w && pair_of_row && w_gate && w_up && w_down && dxp && dtopk_w), MOE_ERR_INVALID_ARG,
              "ffn_bwd_gather: null pointer");
  MOE_REQUIRE(aligned16(dy) && aligned16(x) && aligned16(g_save) && aligned16(u_save) && aligned16(act_w) && aligned16(w_gate) && aligned16(w_up) &&
              aligned16(w_down) && aligned16(dxp) && aligned16(dw_gate) && aligned16(dw_up) && aligned16(dw_down),
              MOE_ERR_INVALID_ARG, "ffn_bwd_gather: tensors must be 16-byte aligned");
  const size_t need = moe_grouped_gemm_swiglu_bwd_gather_workspace_bytes(dtype, P, d, f, E, g_save != nullptr);
  MOE_REQUIRE(ws && ws_bytes >= need && aligned16(ws), MOE_ERR_WORKSPACE, "ffn_bwd_gather: workspace null, misaligned or smaller than %zu bytes", need);
  FfnBwdGatherArgs a{dy, x, T, k, topk_w, pair_of_row, g_save, u_save, w_gate, w_up, w_down, P, d, f, E, offsets, dxp, dw_gate,
                     dw_up, dw_down, dtopk_w, ws, static_cast<hipStream_t>(stream), act_w};
  begin_call("moe_grouped_gemm_swiglu_bwd_gather", static_cast<hipStream_t>(stream));
  if (dtype == MOE_BF16) ffn_bwd_gather_bf16(a); else ffn_bwd_gather_f32(a);
  return end_call();
}

// ---- 8-bit operands ----------------------------------------------------------------------------------
extern "C" int32_t moe_mx8_quantise(const void* src, int64_t rows, int K, void* codes, void* scales, void* stream) {
  MOE_REQUIRE(rows >= 0 && K > 0, MOE_ERR_INVALID_ARG, "mx8_quantise: need rows >= 0 and K > 0 (rows=%lld K=%d)", static_cast<long long>(rows), K);
  MOE_REQUIRE(K % 128 == 0, MOE_ERR_UNSUPPORTED, "mx8_quantise: K=%d must be a multiple of 128 (four 32-element blocks per packed scale word)", K);
  MOE_REQUIRE(rows * (K / 8) < (int64_t{1} << 39), MOE_ERR_UNSUPPORTED, "mx8_quantise: matrix too large");
  if (rows == 0) return MOE_OK;
  MOE_REQUIRE(src && codes && scales, MOE_ERR_INVALID_ARG, "mx8_quantise: null pointer");
  MOE_REQUIRE(aligned16(src) && aligned16(codes) && aligned16(scales), MOE_ERR_INVALID_ARG, "mx8_quantise: tensors must be 16-byte aligned");
  Mx8QuantArgs a{src, static_cast<long>(rows), K, codes, scales, static_cast<hipStream_t>(stream)};
  begin_call("moe_mx8_quantise", static_cast<hipStream_t>(stream));
  mx8_quantise(a);
  return end_call();
}

static int32_t check_mx8_dims(int P, int d, int f, int E, int T, int k, bool gathered) {
  if (int32_t rc = check_ffn_dims("ffn_fwd_mx8", MOE_BF16, P, d, f, E)) return rc;
  MOE_REQUIRE(d % 128 == 0 && f % 128 == 0, MOE_ERR_UNSUPPORTED, "ffn_fwd_mx8: d=%d and f=%d must be multiples of 128", d, f);
  if (gathered) {
    MOE_REQUIRE(T >= 0 && k >= 1 && static_cast<int64_t>(T) * k == P, MOE_ERR_INVALID_ARG, "ffn_fwd_mx8: P=%d is not T*k (T=%d k=%d)", P, T, k);
    MOE_REQUIRE(static_cast<int64_t>(T) * d < (int64_t{1} << 32), MOE_ERR_UNSUPPORTED, "ffn_fwd_mx8: T*d must fit 32 bits (rows are addressed with 32-bit byte offsets)");
  }
  return MOE_OK;
}

extern "C" size_t moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(int P, int d, int f, int E) {
  if (P < 0 || d <= 0 || f <= 0 || E <= 0) return 0;
  return ffn_fwd_mx8_ws_bytes(P, d, f, E);
}

extern "C" int32_t moe_grouped_gemm_swiglu_fwd_mx8(const void* xq, const void* xs, int T, int k, const int32_t* pair_of_row,
                                                   const void* wgq, const void* wgs, const void* wuq, const void* wus,
                                                   const void* wdq, const void* wds, int P, int d, int f, int E,
                                                   const int32_t* offsets, void* actq, void* acts, void* yp, void* ws,
                                                   size_t ws_bytes, void* stream) {
  if (int32_t rc = check_mx8_dims(P, d, f, E, T, k, pair_of_row != nullptr)) return rc;
  if (P == 0) return MOE_OK;
  MOE_REQUIRE(xq && xs && wgq && wgs && wuq && wus && wdq && wds && offsets && actq && acts && yp, MOE_ERR_INVALID_ARG, "ffn_fwd_mx8: null pointer");
  MOE_REQUIRE(aligned16(xq) && aligned16(xs) && aligned16(wgq) && aligned16(wgs) && aligned16(wuq) && aligned16(wus) && aligned16(wdq) &&
              aligned16(wds) && aligned16(actq) && aligned16(acts) && aligned16(yp), MOE_ERR_INVALID_ARG, "ffn_fwd_mx8: tensors must be 16-byte aligned");
  const size_t need = moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(P, d, f, E);
  MOE_REQUIRE(ws && ws_bytes >= need && aligned16(ws), MOE_ERR_WORKSPACE, "ffn_fwd_mx8: workspace null, misaligned or smaller than %zu bytes", need);
  FfnFwdMx8Args a{xq, xs, T, k, pair_of_row, wgq, wgs, wuq, wus, wdq, wds, P, d, f, E, offsets, actq, acts, yp, ws, static_cast<hipStream_t>(stream)};
  begin_call("moe_grouped_gemm_swiglu_fwd_mx8", static_cast<hipStream_t>(stream));
  ffn_fwd_mx8(a);
  return end_call();
}

extern "C" int32_t moe_grouped_gemm_down_mx8(const void* actq, const void* acts, const void* wdq, const void* wds, int P, int d, int f,
                                            int E, const int32_t* offsets, void* yp, void* ws, size_t ws_bytes, void* stream) {
  if (int32_t rc = check_mx8_dims(P, d, f, E, 0, 1, false)) return rc;
  if (P == 0) return MOE_OK;
  MOE_REQUIRE(actq && acts && wdq && wds && offsets && yp, MOE_ERR_INVALID_ARG, "down_mx8: null pointer");
  MOE_REQUIRE(aligned16(actq) && aligned16(acts) && aligned16(wdq) && aligned16(wds) && aligned16(yp), MOE_ERR_INVALID_ARG,
              "down_mx8: tensors must be 16-byte aligned");
  const size_t need = moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(P, d, f, E);
  MOE_REQUIRE(ws && ws_bytes >= need && aligned16(ws), MOE_ERR_WORKSPACE, "down_mx8: workspace null, misaligned or smaller than %zu bytes", need);
  FfnFwdMx8Args a{nullptr, nullptr, P, 1, nullptr, nullptr, nullptr, nullptr, nullptr, wdq, wds, P, d, f, E, offsets,
                  const_cast<void*>(actq), const_cast<void*>(acts), yp, ws, static_cast<hipStream_t>(stream)};
  begin_call("moe_grouped_gemm_down_mx8", static_cast<hipStream_t>(stream));
  ffn_fwd_mx8(a);
  return end_call();
}

// ---- router linear -----------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t* p, size_t n) {
  const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

static int32_t check_router_dims(const char* who, int dtype, int T, int d, int E) {
  MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_ERR_UNSUPPORTED, "%s: unknown dtype %d", who, dtype);
  MOE_REQUIRE(T >= 0 && d > 0 && E > 0, MOE_ERR_INVALID_ARG, "%s: need T >= 0, d, E > 0 (T=%d d=%d E=%d)", who, T, d, E);
  MOE_REQUIRE(E <= kMaxExperts, MOE_ERR_UNSUPPORTED, "%s: E=%d above the built maximum %d", who, E, kMaxExperts);
  MOE_REQUIRE(dtype == MOE_F32 || (d % 8 == 0 && E % 8 == 0), MOE_ERR_UNSUPPORTED, "%s: d=%d and E=%d must be multiples of 8 for bf16", who, d, E);
  return MOE_OK;
}

extern "C" size_t moe_router_logits_workspace_bytes(int dtype, int T, int d, int E) {
  if (T <= 0 || d <= 0 || E <= 0) return 256;
  return dtype == MOE_BF16 ? router_fwd_ws_bytes_bf16(T, d, E) : 256;
}

extern "C" size_t moe_router_bwd_workspace_bytes(int dtype, int T, int d, int E) {
  if (T <= 0 || d <= 0 || E <= 0) return 256;
  return dtype == MOE_BF16 ? router_bwd_ws_bytes_bf16(T, d, E) : 256;
}

extern "C" int32_t moe_router_logits(const void* x, const void* w_router, int dtype, int T, int d, int E, float* logits,
                                     void* ws, size_t ws_bytes, void* stream) {
  if (int32_t rc = check_router_dims("router_logits", dtype, T, d, E)) return rc;
  if (T == 0) return MOE_OK;
  MOE_REQUIRE(x && w_router && logits, MOE_ERR_INVALID_ARG, "router_logits: null pointer");
  MOE_REQUIRE(aligned16(x) && aligned16(w_router) && aligned16(logits), MOE_ERR_INVALID_ARG, "router_logits: tensors must be 16-byte aligned");
  const size_t need = moe_router_logits_workspace_bytes(dtype, T, d, E);
  MOE_REQUIRE(ws && ws_bytes >= need && aligned16(ws), MOE_ERR_WORKSPACE, "router_logits: workspace null, misaligned or smaller than %zu bytes", need);
  RouterFwdArgs a{x, w_router, T, d, E, logits, ws, static_cast<hipStream_t>(stream)};
  begin_call("moe_router_logits", static_cast<hipStream_t>(stream));
  if (dtype == MOE_BF16) router_fwd_bf16(a); else router_fwd_f32(a);
  return end_call();
}

extern "C" int32_t moe_router_bwd(const float* dlogits, const void* x, const void* w_router, int dtype, int T, int d, int E,
                                  int accumulate, void* dx, void* dw_router, void* ws, size_t ws_bytes, void* stream) {
  if (int32_t rc = check_router_dims("router_bwd", dtype, T, d, E)) return rc;
  MOE_REQUIRE(w_router && dw_router, MOE_ERR_INVALID_ARG, "router_bwd: null weight or weight-gradient pointer");
  MOE_REQUIRE(T == 0 || (dlogits && x && dx), MOE_ERR_INVALID_ARG, "router_bwd: null pointer");
  MOE_REQUIRE(aligned16(dlogits) && aligned16(x) && aligned16(w_router) && aligned16(dx) && aligned16(dw_router), MOE_ERR_INVALID_ARG,
              "router_bwd: tensors must be 16-byte aligned");
  const size_t need = moe_router_bwd_workspace_bytes(dtype, T, d, E);
  MOE_REQUIRE(ws && ws_bytes >= need && aligned16(ws), MOE_ERR_WORKSPACE, "router_bwd: workspace null, misaligned or smaller than %zu bytes", need);
  if (T == 0) {   // no rows: the weight gradient is all zeros (a fill kernel, not a memset node: callers may capture this)
    const size_t words = static_cast<size_t>(E) * d * elem_size(dtype) / 4;
    begin_call("moe_router_bwd", static_cast<hipStream_t>(stream));
    MOE_LAUNCH("zero_dw_router", zero_words_kernel, dim3(static_cast<unsigned>((words + 255) / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
               static_cast<uint32_t*>(dw_router), words);
    return end_call();
  }
  RouterBwdArgs a{dlogits, x, w_router, T, d, E, accumulate != 0, dx, dw_router, ws, static_cast<hipStream_t>(stream)};
  begin_call("moe_router_bwd", static_cast<hipStream_t>(stream));
  if (dtype == MOE_BF16) router_bwd_bf16(a); else router_bwd_f32(a);
  return end_call();
}

