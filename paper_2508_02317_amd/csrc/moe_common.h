// Shared host/device helpers of libmoe (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "moe.h"

namespace moe {

// ---- host-side error reporting ---------------------------------------------------------
int32_t fail(int32_t code, const char* fmt, ...);   // records the message, returns code

#define MOE_REQUIRE(cond, code, ...) \
  do { if (!(cond)) return ::moe::fail((code), __VA_ARGS__); } while (0)

// ---- launching ------------------------------------------------------------------------------
// Every kernel goes through MOE_LAUNCH.  An entry point calls begin_call() once its arguments are
// validated: that forgets whatever error an earlier, unrelated HIP call left behind on this thread.
// The status of each launch is then read straight after it; after the first failure the remaining
// launches of the call are skipped, and end_call() reports the kernel that failed.
// A harness may install a hook (moe_set_launch_hook) that is told about every launch, before and
// after it is enqueued, with the stream it goes to -- that is all the library offers for timing.
void begin_call(const char* entry, hipStream_t stream);
int32_t end_call();                                  // MOE_ERR_HIP if a launch of this call failed
bool launch_begin(const char* name, hipStream_t stream);   // false: an earlier launch of this call failed
void launch_end(const char* name, hipStream_t stream);
void note_hip_failure(const char* what, hipError_t err);   // first failure of the call wins
#define MOE_LAUNCH(name, kern, grid, block, shmem, stream, ...)            \
  do {                                                                     \
    if (::moe::launch_begin(name, stream)) {                               \
      hipLaunchKernelGGL(kern, grid, block, shmem, stream, __VA_ARGS__);   \
      ::moe::launch_end(name, stream);                                     \
    }                                                                      \
  } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int elem_size(int dtype) { return dtype == MOE_BF16 ? 2 : 4; }

constexpr int kMaxExperts = 1024;
constexpr int kMaxTopK = 64;

// ---- bf16 <-> f32 on the device ---------------------------------------------------------
typedef uint16_t bf16_t;   // raw bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(static_cast<uint32_t>(v) << 16);
}
// round to nearest, ties to even (inputs are finite on this path)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}
// two floats -> packed bf16 pair with the hardware converter (v_cvt_pk_bf16_f32, round to nearest even)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fast variants (bf16 path: the result is rounded to 8 bits of mantissa anyway)
__device__ __forceinline__ float sigmoid_fast(float g) { return 1.0f / (1.0f + __expf(-g)); }
// accurate variants (fp32 path)
__device__ __forceinline__ float sigmoid_acc(float g) { return 1.0f / (1.0f + expf(-g)); }

// ---- wave64 reductions -------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// ---- internal launchers of the grouped expert FFN (one per element type) -------------------
// All pointers are device pointers; arguments are already validated by the C entry points.
struct FfnFwdArgs {
  const void *xp, *w_gate, *w_up, *w_down;
  int P, d, f, E;
  const int32_t* offsets;
  void *g_save, *u_save, *act, *yp;   // g_save/u_save/act may be null (not written then)
  void* ws;
  hipStream_t stream;
};
struct FfnBwdArgs {
  const void *dyp, *xp, *g_save, *u_save, *act, *w_gate, *w_up, *w_down;
  int P, d, f, E;
  const int32_t* offsets;
  void *dxp, *dw_gate, *dw_up, *dw_down;
  void* ws;
  hipStream_t stream;
};
// the variants that read the layer input / the output gradient by token (P == T * k)
struct FfnFwdGatherArgs {
  const void* x;                      // [T, d]
  int T, k;
  const int32_t* pair_of_row;         // [P]
  const void *w_gate, *w_up, *w_down;
  int P, d, f, E;
  const int32_t* offsets;
  void *g_save, *u_save, *act, *yp;   // g_save/u_save may be null
  void* ws;
  hipStream_t stream;
  const float* topk_w;                // [T, k] or null; given: act and yp leave scaled by the row's combine weight
};
struct FfnBwdGatherArgs {
  const void *dy, *x;                 // [T, d]
  int T, k;
  const float* topk_w;                // [T, k]
  const int32_t* pair_of_row;         // [P]
  const void *g_save, *u_save, *w_gate, *w_up, *w_down;
  int P, d, f, E;
  const int32_t* offsets;
  void *dxp, *dw_gate, *dw_up, *dw_down;
  float* dtopk_w;                     // [T, k]
  void* ws;
  hipStream_t stream;
  const void* act_w;                  // [P, f] or null: w * act as the weighted forward left it (null: formed here)
};
// 8-bit (MXFP8) operands: quantiser and forward products
struct Mx8QuantArgs {
  const void* src;                    // [rows, K] bf16
  long rows; int K;
  void *codes, *scales;               // [rows, K] E4M3 codes; [K/128][rows] packed scale words
  hipStream_t stream;
};
struct FfnFwdMx8Args {
  const void *xq, *xs;                // [T, d] codes and [d/128][T] scales (pair_of_row given) or [P, d] and [d/128][P]
  int T, k;
  const int32_t* pair_of_row;         // [P] or null
  const void *wgq, *wgs, *wuq, *wus, *wdq, *wds;
  int P, d, f, E;
  const int32_t* offsets;
  void *actq, *acts, *yp;
  void* ws;
  hipStream_t stream;
};
void mx8_quantise(const Mx8QuantArgs& a);
size_t ffn_fwd_mx8_ws_bytes(int P, int d, int f, int E);
void ffn_fwd_mx8(const FfnFwdMx8Args& a);
size_t ffn_fwd_gather_ws_bytes_bf16(int P, int d, int f, int E);
size_t ffn_bwd_gather_ws_bytes_bf16(int P, int d, int f, int E, int have_saved);
void ffn_fwd_gather_bf16(const FfnFwdGatherArgs& a);
void ffn_bwd_gather_bf16(const FfnBwdGatherArgs& a);
size_t ffn_fwd_gather_ws_bytes_f32(int P, int d, int f, int E);
size_t ffn_bwd_gather_ws_bytes_f32(int P, int d, int f, int E, int have_saved);
void ffn_fwd_gather_f32(const FfnFwdGatherArgs& a);
void ffn_bwd_gather_f32(const FfnBwdGatherArgs& a);
size_t ffn_fwd_ws_bytes_bf16(int P, int d, int f, int E);
size_t ffn_bwd_ws_bytes_bf16(int P, int d, int f, int E, int have_saved);
void ffn_fwd_bf16(const FfnFwdArgs& a);
void ffn_bwd_bf16(const FfnBwdArgs& a);
size_t ffn_fwd_ws_bytes_f32(int P, int d, int f, int E);
size_t ffn_bwd_ws_bytes_f32(int P, int d, int f, int E, int have_saved);
void ffn_fwd_f32(const FfnFwdArgs& a);
void ffn_bwd_f32(const FfnBwdArgs& a);

// ---- router linear (gemm_bf16.hip: bf16 MFMA; gemm_f32.hip: fp32 reference-speed kernels) --------
struct RouterFwdArgs {
  const void *x, *w_router;    // [T, d], [E, d]
  int T, d, E;
  float* logits;               // [T, E]
  void* ws;
  hipStream_t stream;
};
struct RouterBwdArgs {
  const float* dlogits;        // [T, E]
  const void *x, *w_router;
  int T, d, E;
  int accumulate;              // add to dx instead of overwriting it
  void *dx, *dw_router;        // [T, d], [E, d]
  void* ws;
  hipStream_t stream;
};
size_t router_fwd_ws_bytes_bf16(int T, int d, int E);
size_t router_bwd_ws_bytes_bf16(int T, int d, int E);
void router_fwd_bf16(const RouterFwdArgs& a);
void router_bwd_bf16(const RouterBwdArgs& a);
void router_fwd_f32(const RouterFwdArgs& a);
void router_bwd_f32(const RouterBwdArgs& a);

}  // namespace moe
