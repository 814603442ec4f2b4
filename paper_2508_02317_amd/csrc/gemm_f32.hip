// fp32 variant of the grouped SwiGLU expert FFN (Sec. 3.2.5; stacked weights of App. B.6).
//
// This element type exists for the small full-precision parity configuration; its sizes
// are launch-latency bound, so the kernels are written for exactness and clarity: one
// thread per output element, a sequential fp32 FMA chain over the reduction index, no
// tiling.  The bf16 MFMA path lives in gemm_bf16.hip.
#include "moe_common.h"

namespace moe {

constexpr int kF32Threads = 256;

// expert whose row segment [offsets[e], offsets[e+1]) contains row r
__device__ __forceinline__ int expert_of_row(const int32_t* __restrict__ offsets, int E, int r) {
  int lo = 0, hi = E;          // invariant: offsets[lo] <= r < offsets[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (offsets[mid] <= r) lo = mid; else hi = mid;
  }
  return lo;
}

// G = xp Wg^T, U = xp Wu^T, act = silu(G) * U          one thread per (row, n)
// Every kernel here that reads one row per routed pair takes an optional list of source rows: with it the
// operand is the token-major matrix and row r reads its row row_src[r] (no expert-ordered copy exists).
__global__ __launch_bounds__(kF32Threads) void f32_gate_up_kernel(
    const float* __restrict__ xp, const float* __restrict__ wg, const float* __restrict__ wu,
    int P, int d, int f, int E, const int32_t* __restrict__ offsets,
    float* __restrict__ G, float* __restrict__ U, float* __restrict__ act, const int32_t* __restrict__ row_src,
    const float* __restrict__ row_w) {
  const size_t i = static_cast<size_t>(blockIdx.x) * kF32Threads + threadIdx.x;
  if (i >= static_cast<size_t>(P) * f) return;
  const int r = static_cast<int>(i / f), n = static_cast<int>(i % f);
  const int e = expert_of_row(offsets, E, r);
  const float* x = xp + static_cast<size_t>(row_src ? row_src[r] : r) * d;   // row_src: xp is token-major
  const float* g_row = wg + (static_cast<size_t>(e) * f + n) * d;
  const float* u_row = wu + (static_cast<size_t>(e) * f + n) * d;
  float g = 0.0f, u = 0.0f;
  for (int c = 0; c < d; ++c) { g = fmaf(x[c], g_row[c], g); u = fmaf(x[c], u_row[c], u); }
  if (G) G[i] = g;
  if (U) U[i] = u;
  if (act) act[i] = (row_w ? row_w[r] : 1.0f) * (g * sigmoid_acc(g) * u);      // row_w: the activation carries the combine weight
}

// yp = act Wd^T                                         one thread per (row, c)
__global__ __launch_bounds__(kF32Threads) void f32_down_kernel(
    const float* __restrict__ act, const float* __restrict__ wd, int P, int d, int f, int E,
    const int32_t* __restrict__ offsets, float* __restrict__ yp) {
  const size_t i = static_cast<size_t>(blockIdx.x) * kF32Threads + threadIdx.x;
  if (i >= static_cast<size_t>(P) * d) return;
  const int r = static_cast<int>(i / d), c = static_cast<int>(i % d);
  const int e = expert_of_row(offsets, E, r);
  const float* a = act + static_cast<size_t>(r) * f;
  const float* w = wd + (static_cast<size_t>(e) * d + c) * f;
  float s = 0.0f;
  for (int n = 0; n < f; ++n) s = fmaf(a[n], w[n], s);
  yp[i] = s;
}

// dA = dyp Wd;  dG = dA * U * silu'(G);  dU = dA * silu(G)      one thread per (row, n)
__global__ __launch_bounds__(kF32Threads) void f32_dact_kernel(
    const float* __restrict__ dyp, const float* __restrict__ wd, const float* __restrict__ G,
    const float* __restrict__ U, int P, int d, int f, int E, const int32_t* __restrict__ offsets,
    float* __restrict__ dG, float* __restrict__ dU, const int32_t* __restrict__ row_src,
    const float* __restrict__ row_w, float* __restrict__ dA_unscaled, float* __restrict__ act_w) {
  const size_t i = static_cast<size_t>(blockIdx.x) * kF32Threads + threadIdx.x;
  if (i >= static_cast<size_t>(P) * f) return;
  const int r = static_cast<int>(i / f), n = static_cast<int>(i % f);
  const int e = expert_of_row(offsets, E, r);
  const float* dy = dyp + static_cast<size_t>(row_src ? row_src[r] : r) * d;
  const float* w = wd + static_cast<size_t>(e) * d * f + n;
  float da = 0.0f;
  for (int c = 0; c < d; ++c) da = fmaf(dy[c], w[static_cast<size_t>(c) * f], da);
  const float g = G[i], u = U[i];
  const float s = sigmoid_acc(g);
  if (row_w) {   // the rows of dyp are w_r * dy[token]: scale the product instead, and keep what the combine backward needs
    dA_unscaled[i] = da;
    if (act_w) act_w[i] = row_w[r] * (g * s * u);
    da *= row_w[r];
  }
  dG[i] = da * u * (s * (1.0f + g * (1.0f - s)));
  dU[i] = da * (g * s);
}

// gradient of the combine weights: dw[pair_of_row[r]] = <dy[token(r)] Wd, act[r]> = <dy[token(r)], yp[r]>
// one wavefront per row, lanes stride over the columns
__global__ __launch_bounds__(kF32Threads) void f32_dw_kernel(
    const float* __restrict__ dA_unscaled, const float* __restrict__ G, const float* __restrict__ U, int P, int f,
    const int32_t* __restrict__ pair_of_row, float* __restrict__ dw) {
  const int r = blockIdx.x * (kF32Threads / 64) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (r >= P) return;
  float s = 0.0f;
  for (int n = lane; n < f; n += 64) {
    const size_t i = static_cast<size_t>(r) * f + n;
    const float g = G[i];
    s = fmaf(g * sigmoid_acc(g) * U[i], dA_unscaled[i], s);
  }
  s = wave_sum(s);
  if (lane == 0) dw[min(max(pair_of_row[r], 0), P - 1)] = s;
}

__global__ __launch_bounds__(kF32Threads) void f32_row_token_kernel(const int32_t* __restrict__ pair_of_row, const float* __restrict__ topk_w,
                                                                    int P, int T, int k, int32_t* __restrict__ row_token,
                                                                    float* __restrict__ row_w) {
  const int r = blockIdx.x * kF32Threads + threadIdx.x;
  if (r >= P) return;
  const int pair = min(max(pair_of_row[r], 0), P - 1);
  row_token[r] = min(pair / k, T - 1);
  if (row_w) row_w[r] = topk_w[pair];
}

// dxp = dG Wg + dU Wu                                    one thread per (row, c)
__global__ __launch_bounds__(kF32Threads) void f32_dx_kernel(
    const float* __restrict__ dG, const float* __restrict__ dU, const float* __restrict__ wg,
    const float* __restrict__ wu, int P, int d, int f, int E, const int32_t* __restrict__ offsets,
    float* __restrict__ dxp) {
  const size_t i = static_cast<size_t>(blockIdx.x) * kF32Threads + threadIdx.x;
  if (i >= static_cast<size_t>(P) * d) return;
  const int r = static_cast<int>(i / d), c = static_cast<int>(i % d);
  const int e = expert_of_row(offsets, E, r);
  const float* dg = dG + static_cast<size_t>(r) * f;
  const float* du = dU + static_cast<size_t>(r) * f;
  const float* g_col = wg + static_cast<size_t>(e) * f * d + c;
  const float* u_col = wu + static_cast<size_t>(e) * f * d + c;
  float s = 0.0f;
  for (int n = 0; n < f; ++n) s = fmaf(dg[n], g_col[static_cast<size_t>(n) * d], s);
  for (int n = 0; n < f; ++n) s = fmaf(du[n], u_col[static_cast<size_t>(n) * d], s);
  dxp[i] = s;
}

// out[e][i][j] = sum over the expert's rows of lhs[r,i] * rhs[r,j]      one thread per (e,i,j)
__global__ __launch_bounds__(kF32Threads) void f32_wgrad_kernel(
    const float* __restrict__ lhs, int li, const float* __restrict__ rhs, int lj, int E, int P,
    const int32_t* __restrict__ offsets, float* __restrict__ out, const int32_t* __restrict__ lhs_src,
    const int32_t* __restrict__ rhs_src) {
  const size_t idx = static_cast<size_t>(blockIdx.x) * kF32Threads + threadIdx.x;
  const size_t per = static_cast<size_t>(li) * lj;
  if (idx >= per * E) return;
  const int e = static_cast<int>(idx / per);
  const int i = static_cast<int>((idx % per) / lj), j = static_cast<int>(idx % lj);
  float s = 0.0f;
  const int begin = min(max(offsets[e], 0), P), end = min(offsets[e + 1], P);
  for (int r = begin; r < end; ++r)
    s = fmaf(lhs[static_cast<size_t>(lhs_src ? lhs_src[r] : r) * li + i], rhs[static_cast<size_t>(rhs_src ? rhs_src[r] : r) * lj + j], s);
  out[idx] = s;
}

static unsigned blocks_for(size_t n) { return static_cast<unsigned>((n + kF32Threads - 1) / kF32Threads); }

size_t ffn_fwd_ws_bytes_f32(int, int, int, int) { return 256; }

size_t ffn_bwd_ws_bytes_f32(int P, int d, int f, int E, int have_saved) {
  (void)d; (void)E;
  const size_t pf = align_up(static_cast<size_t>(P) * f * sizeof(float), 256);
  return 256 + (have_saved ? 2 : 4) * pf;     // dG, dU (+ recomputed G, U)
}

void ffn_fwd_f32(const FfnFwdArgs& a) {
  const size_t pf = static_cast<size_t>(a.P) * a.f, pd = static_cast<size_t>(a.P) * a.d;
  if (a.P == 0) return;
  MOE_LAUNCH("f32_gate_up", f32_gate_up_kernel, dim3(blocks_for(pf)), dim3(kF32Threads), 0, a.stream,
                     static_cast<const float*>(a.xp), static_cast<const float*>(a.w_gate),
                     static_cast<const float*>(a.w_up), a.P, a.d, a.f, a.E, a.offsets,
                     static_cast<float*>(a.g_save), static_cast<float*>(a.u_save), static_cast<float*>(a.act),
                     static_cast<const int32_t*>(nullptr), static_cast<const float*>(nullptr));
  if (a.yp)
    MOE_LAUNCH("f32_down", f32_down_kernel, dim3(blocks_for(pd)), dim3(kF32Threads), 0, a.stream,
                       static_cast<const float*>(a.act), static_cast<const float*>(a.w_down), a.P, a.d, a.f, a.E,
                       a.offsets, static_cast<float*>(a.yp));
}

void ffn_bwd_f32(const FfnBwdArgs& a) {
  const size_t pf = static_cast<size_t>(a.P) * a.f, pd = static_cast<size_t>(a.P) * a.d;
  const size_t pf_bytes = align_up(pf * sizeof(float), 256);
  char* ws = static_cast<char*>(a.ws);
  float* dG = reinterpret_cast<float*>(ws);
  float* dU = reinterpret_cast<float*>(ws + pf_bytes);
  const float* G = static_cast<const float*>(a.g_save);
  const float* U = static_cast<const float*>(a.u_save);
  if (a.P > 0) {
    if (!G) {   // recompute the pre-activations
      float* Gr = reinterpret_cast<float*>(ws + 2 * pf_bytes);
      float* Ur = reinterpret_cast<float*>(ws + 3 * pf_bytes);
      MOE_LAUNCH("f32_gate_up", f32_gate_up_kernel, dim3(blocks_for(pf)), dim3(kF32Threads), 0, a.stream,
                         static_cast<const float*>(a.xp), static_cast<const float*>(a.w_gate),
                         static_cast<const float*>(a.w_up), a.P, a.d, a.f, a.E, a.offsets, Gr, Ur,
                         static_cast<float*>(nullptr), static_cast<const int32_t*>(nullptr), static_cast<const float*>(nullptr));
      G = Gr; U = Ur;
    }
    MOE_LAUNCH("f32_dact", f32_dact_kernel, dim3(blocks_for(pf)), dim3(kF32Threads), 0, a.stream,
                       static_cast<const float*>(a.dyp), static_cast<const float*>(a.w_down), G, U, a.P, a.d, a.f, a.E,
                       a.offsets, dG, dU, static_cast<const int32_t*>(nullptr), static_cast<const float*>(nullptr),
                       static_cast<float*>(nullptr), static_cast<float*>(nullptr));
    MOE_LAUNCH("f32_dx", f32_dx_kernel, dim3(blocks_for(pd)), dim3(kF32Threads), 0, a.stream, dG, dU,
                       static_cast<const float*>(a.w_gate), static_cast<const float*>(a.w_up), a.P, a.d, a.f, a.E,
                       a.offsets, static_cast<float*>(a.dxp));
  }
  const size_t per = static_cast<size_t>(a.d) * a.f * a.E;
  // with P == 0 every segment is empty and the kernels only write zeros (dG/dU are not read)
  MOE_LAUNCH("f32_wgrad", f32_wgrad_kernel, dim3(blocks_for(per)), dim3(kF32Threads), 0, a.stream,
                     static_cast<const float*>(a.dyp), a.d, static_cast<const float*>(a.act), a.f, a.E, a.P, a.offsets,
                     static_cast<float*>(a.dw_down), static_cast<const int32_t*>(nullptr),
                     static_cast<const int32_t*>(nullptr));
  MOE_LAUNCH("f32_wgrad", f32_wgrad_kernel, dim3(blocks_for(per)), dim3(kF32Threads), 0, a.stream,
                     static_cast<const float*>(dG), a.f, static_cast<const float*>(a.xp), a.d, a.E, a.P, a.offsets,
                     static_cast<float*>(a.dw_gate), static_cast<const int32_t*>(nullptr),
                     static_cast<const int32_t*>(nullptr));
  MOE_LAUNCH("f32_wgrad", f32_wgrad_kernel, dim3(blocks_for(per)), dim3(kF32Threads), 0, a.stream,
                     static_cast<const float*>(dU), a.f, static_cast<const float*>(a.xp), a.d, a.E, a.P, a.offsets,
                     static_cast<float*>(a.dw_up), static_cast<const int32_t*>(nullptr),
                     static_cast<const int32_t*>(nullptr));
}

// ---- the variants that read the layer input / the output gradient by token -------------------------
// workspace: [256 | row_token P i32 | row_w P f32 | dG | dU | dA_unscaled | act_w | (G | U)], each aligned to 256
static size_t f32_list_bytes(int P) { return align_up(static_cast<size_t>(P) * 4, 256); }
size_t ffn_fwd_gather_ws_bytes_f32(int P, int, int, int) { return 256 + 2 * f32_list_bytes(P); }
size_t ffn_bwd_gather_ws_bytes_f32(int P, int d, int f, int E, int have_saved) {
  (void)d; (void)E;
  const size_t pf = align_up(static_cast<size_t>(P) * f * sizeof(float), 256);
  return 256 + 2 * f32_list_bytes(P) + (have_saved ? 4 : 6) * pf;
}

void ffn_fwd_gather_f32(const FfnFwdGatherArgs& a) {
  if (a.P == 0) return;
  const size_t pf = static_cast<size_t>(a.P) * a.f, pd = static_cast<size_t>(a.P) * a.d;
  int32_t* row_token = reinterpret_cast<int32_t*>(static_cast<char*>(a.ws) + 256);
  float* row_w = a.topk_w ? reinterpret_cast<float*>(static_cast<char*>(a.ws) + 256 + f32_list_bytes(a.P)) : nullptr;
  MOE_LAUNCH("f32_row_token", f32_row_token_kernel, dim3(blocks_for(a.P)), dim3(kF32Threads), 0, a.stream, a.pair_of_row,
             a.topk_w, a.P, a.T, a.k, row_token, row_w);
  MOE_LAUNCH("f32_gate_up", f32_gate_up_kernel, dim3(blocks_for(pf)), dim3(kF32Threads), 0, a.stream,
             static_cast<const float*>(a.x), static_cast<const float*>(a.w_gate), static_cast<const float*>(a.w_up), a.P, a.d, a.f,
             a.E, a.offsets, static_cast<float*>(a.g_save), static_cast<float*>(a.u_save), static_cast<float*>(a.act),
             static_cast<const int32_t*>(row_token), static_cast<const float*>(row_w));
  MOE_LAUNCH("f32_down", f32_down_kernel, dim3(blocks_for(pd)), dim3(kF32Threads), 0, a.stream, static_cast<const float*>(a.act),
             static_cast<const float*>(a.w_down), a.P, a.d, a.f, a.E, a.offsets, static_cast<float*>(a.yp));
}

void ffn_bwd_gather_f32(const FfnBwdGatherArgs& a) {
  const size_t pf = static_cast<size_t>(a.P) * a.f, pd = static_cast<size_t>(a.P) * a.d;
  const size_t pf_bytes = align_up(pf * sizeof(float), 256), lb = f32_list_bytes(a.P);
  char* ws = static_cast<char*>(a.ws) + 256;
  int32_t* row_token = reinterpret_cast<int32_t*>(ws);
  float* row_w = reinterpret_cast<float*>(ws + lb);
  char* big = ws + 2 * lb;
  float* dG = reinterpret_cast<float*>(big);
  float* dU = reinterpret_cast<float*>(big + pf_bytes);
  float* dA = reinterpret_cast<float*>(big + 2 * pf_bytes);
  float* act_w_ws = reinterpret_cast<float*>(big + 3 * pf_bytes);
  const float* act_w = a.act_w ? static_cast<const float*>(a.act_w) : act_w_ws;
  const float* G = static_cast<const float*>(a.g_save);
  const float* U = static_cast<const float*>(a.u_save);
  if (a.P > 0) {
    MOE_LAUNCH("f32_row_token", f32_row_token_kernel, dim3(blocks_for(a.P)), dim3(kF32Threads), 0, a.stream, a.pair_of_row,
               a.topk_w, a.P, a.T, a.k, row_token, row_w);
    if (!G) {   // recompute the pre-activations
      float* Gr = reinterpret_cast<float*>(big + 4 * pf_bytes);
      float* Ur = reinterpret_cast<float*>(big + 5 * pf_bytes);
      MOE_LAUNCH("f32_gate_up", f32_gate_up_kernel, dim3(blocks_for(pf)), dim3(kF32Threads), 0, a.stream,
                 static_cast<const float*>(a.x), static_cast<const float*>(a.w_gate), static_cast<const float*>(a.w_up), a.P, a.d,
                 a.f, a.E, a.offsets, Gr, Ur, static_cast<float*>(nullptr), static_cast<const int32_t*>(row_token), static_cast<const float*>(nullptr));
      G = Gr; U = Ur;
    }
    MOE_LAUNCH("f32_dact", f32_dact_kernel, dim3(blocks_for(pf)), dim3(kF32Threads), 0, a.stream, static_cast<const float*>(a.dy),
               static_cast<const float*>(a.w_down), G, U, a.P, a.d, a.f, a.E, a.offsets, dG, dU,
               static_cast<const int32_t*>(row_token), static_cast<const float*>(row_w), dA, a.act_w ? static_cast<float*>(nullptr) : act_w_ws);
    MOE_LAUNCH("f32_dw", f32_dw_kernel, dim3(blocks_for(static_cast<size_t>(a.P) * 64)), dim3(kF32Threads), 0, a.stream, static_cast<const float*>(dA), G, U,
               a.P, a.f, a.pair_of_row, a.dtopk_w);
    MOE_LAUNCH("f32_dx", f32_dx_kernel, dim3(blocks_for(pd)), dim3(kF32Threads), 0, a.stream, dG, dU,
               static_cast<const float*>(a.w_gate), static_cast<const float*>(a.w_up), a.P, a.d, a.f, a.E, a.offsets,
               static_cast<float*>(a.dxp));
  }
  const size_t per = static_cast<size_t>(a.d) * a.f * a.E;
  const int32_t* none = nullptr;
  const int32_t* rt = row_token;
  MOE_LAUNCH("f32_wgrad", f32_wgrad_kernel, dim3(blocks_for(per)), dim3(kF32Threads), 0, a.stream, static_cast<const float*>(a.dy), a.d,
             static_cast<const float*>(act_w), a.f, a.E, a.P, a.offsets, static_cast<float*>(a.dw_down), rt, none);
  MOE_LAUNCH("f32_wgrad", f32_wgrad_kernel, dim3(blocks_for(per)), dim3(kF32Threads), 0, a.stream, static_cast<const float*>(dG), a.f,
             static_cast<const float*>(a.x), a.d, a.E, a.P, a.offsets, static_cast<float*>(a.dw_gate), none, rt);
  MOE_LAUNCH("f32_wgrad", f32_wgrad_kernel, dim3(blocks_for(per)), dim3(kF32Threads), 0, a.stream, static_cast<const float*>(dU), a.f,
             static_cast<const float*>(a.x), a.d, a.E, a.P, a.offsets, static_cast<float*>(a.dw_up), none, rt);
}

// ---- router linear, fp32 element type: one thread per output, sequential FMA ----------------------
__global__ __launch_bounds__(kF32Threads) void f32_router_logits_kernel(const float* __restrict__ x, const float* __restrict__ wr,
                                                                        int T, int d, int E, float* __restrict__ logits) {
  const long i = static_cast<long>(blockIdx.x) * kF32Threads + threadIdx.x;
  if (i >= static_cast<long>(T) * E) return;
  const int t = static_cast<int>(i / E), e = static_cast<int>(i % E);
  const float* xr = x + static_cast<long>(t) * d;
  const float* w = wr + static_cast<long>(e) * d;
  float acc = 0.0f;
  for (int c = 0; c < d; ++c) acc = fmaf(xr[c], w[c], acc);
  logits[i] = acc;
}
__global__ __launch_bounds__(kF32Threads) void f32_router_dx_kernel(const float* __restrict__ dz, const float* __restrict__ wr,
                                                                    int T, int d, int E, int accumulate, float* __restrict__ dx) {
  const long i = static_cast<long>(blockIdx.x) * kF32Threads + threadIdx.x;
  if (i >= static_cast<long>(T) * d) return;
  const int t = static_cast<int>(i / d), c = static_cast<int>(i % d);
  float acc = 0.0f;
  for (int e = 0; e < E; ++e) acc = fmaf(dz[static_cast<long>(t) * E + e], wr[static_cast<long>(e) * d + c], acc);
  dx[i] = accumulate ? dx[i] + acc : acc;
}
__global__ __launch_bounds__(kF32Threads) void f32_router_dw_kernel(const float* __restrict__ dz, const float* __restrict__ x,
                                                                    int T, int d, int E, float* __restrict__ dwr) {
  const long i = static_cast<long>(blockIdx.x) * kF32Threads + threadIdx.x;
  if (i >= static_cast<long>(E) * d) return;
  const int e = static_cast<int>(i / d), c = static_cast<int>(i % d);
  float acc = 0.0f;
  for (int t = 0; t < T; ++t) acc = fmaf(dz[static_cast<long>(t) * E + e], x[static_cast<long>(t) * d + c], acc);
  dwr[i] = acc;
}

void router_fwd_f32(const RouterFwdArgs& a) {
  MOE_LAUNCH("f32_router_logits", f32_router_logits_kernel, dim3(blocks_for(static_cast<size_t>(a.T) * a.E)), dim3(kF32Threads), 0,
             a.stream, static_cast<const float*>(a.x), static_cast<const float*>(a.w_router), a.T, a.d, a.E, a.logits);
}
void router_bwd_f32(const RouterBwdArgs& a) {
  if (a.T > 0)
    MOE_LAUNCH("f32_router_dx", f32_router_dx_kernel, dim3(blocks_for(static_cast<size_t>(a.T) * a.d)), dim3(kF32Threads), 0, a.stream,
               a.dlogits, static_cast<const float*>(a.w_router), a.T, a.d, a.E, a.accumulate, static_cast<float*>(a.dx));
  MOE_LAUNCH("f32_router_dw", f32_router_dw_kernel, dim3(blocks_for(static_cast<size_t>(a.E) * a.d)), dim3(kF32Threads), 0, a.stream,
             a.dlogits, static_cast<const float*>(a.x), a.T, a.d, a.E, static_cast<float*>(a.dw_router));
}

}  // namespace moe
