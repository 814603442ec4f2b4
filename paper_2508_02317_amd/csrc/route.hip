// Top-k softmax routing and its backward (Sec. 3.2.3: tokens are routed to experts).
//
// One wavefront owns one token at a time.  Lane l holds the logits of experts l, l+64, ...
// as 64-bit keys (order-preserving float bits in the high word, the complemented expert
// index in the low word), so a single wave-wide max implements "largest logit, ties to
// the lower index" (taken word by word with row shifts and row broadcasts, see wave_max_key).
// k rounds of that max give the slots in order.  Each workgroup keeps
// an LDS histogram of the experts it selected and writes it to its own row of the
// workspace; a second one-block kernel sums the rows (counts) and prefix-scans them
// (offsets).  No float atomics, no global atomics: the result is deterministic.
#include <mutex>
#include <type_traits>
#include "moe_common.h"

namespace moe {

constexpr int kRouteThreads = 1024;                // 16 waves: few histogram rows for the scan, many waves in flight
constexpr int kRouteWaves = kRouteThreads / 64;
constexpr int kRouteMaxBlocks = 1024;

// Largest 32-bit value of the wave, in every lane (as a scalar).  Data-parallel primitives only: four shifts inside
// each row of 16 lanes, then the row results are passed on to the next rows; lane 63 ends up with the maximum of all
// 64.  Lanes shifted in from outside a row contribute 0, the identity of an unsigned maximum.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  auto dpp = [](uint32_t old, uint32_t x, auto ctrl, auto rows) {
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(static_cast<int>(old), static_cast<int>(x), decltype(ctrl)::value,
                                                             decltype(rows)::value, 0xF, decltype(rows)::value == 0xF));
  };
  typedef std::integral_constant<int, 0xF> AllRows;
  v = max(v, dpp(0u, v, std::integral_constant<int, 0x111>{}, AllRows{}));     // row_shr:1
  v = max(v, dpp(0u, v, std::integral_constant<int, 0x112>{}, AllRows{}));     // row_shr:2
  v = max(v, dpp(0u, v, std::integral_constant<int, 0x114>{}, AllRows{}));     // row_shr:4
  v = max(v, dpp(0u, v, std::integral_constant<int, 0x118>{}, AllRows{}));     // row_shr:8: lane 15 of a row holds the row's maximum
  v = max(v, dpp(v, v, std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xA>{}));   // row_bcast:15 into rows 1 and 3
  v = max(v, dpp(v, v, std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xC>{}));   // row_bcast:31 into rows 2 and 3
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), 63));
}
// Largest 64-bit key of the wave from the lane's VPL keys: first the largest high word, then the largest low word
// among the keys that have it (the order of 64-bit integers, without 64-bit exchanges between lanes).
template <int VPL>
__device__ __forceinline__ uint64_t wave_max_key(const uint64_t (&key)[VPL]) {
  uint32_t hi = 0u;
#pragma unroll
  for (int i = 0; i < VPL; ++i) hi = max(hi, static_cast<uint32_t>(key[i] >> 32));
  hi = wave_max_u32(hi);
  uint32_t lo = 0u;
#pragma unroll
  for (int i = 0; i < VPL; ++i)
    if (static_cast<uint32_t>(key[i] >> 32) == hi) lo = max(lo, static_cast<uint32_t>(key[i]));
  lo = wave_max_u32(lo);
  return (static_cast<uint64_t>(hi) << 32) | lo;
}
// float -> uint32 whose unsigned order equals the float order (-0 folded into +0 first)
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  uint32_t u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(uint32_t o) {
  uint32_t u = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
  return __uint_as_float(u);
}

template <int VPL>   // logits held per lane; E <= 64 * VPL
__global__ __launch_bounds__(kRouteThreads) void route_topk_kernel(
    const float* __restrict__ logits, int T, int E, int k, int renorm,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int32_t* __restrict__ block_hist) {
  __shared__ int32_t hist[kMaxExperts];
  for (int e = threadIdx.x; e < E; e += kRouteThreads) hist[e] = 0;
  __syncthreads();

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int waves_total = gridDim.x * kRouteWaves;
  for (int t = blockIdx.x * kRouteWaves + wave; t < T; t += waves_total) {
    const float* z = logits + static_cast<size_t>(t) * E;
    uint64_t key[VPL];
    float zloc[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      int e = lane + 64 * i;
      if (e < E) {
        zloc[i] = z[e] + 0.0f;
        key[i] = (static_cast<uint64_t>(ordered_bits(zloc[i])) << 32) | static_cast<uint32_t>(~e);
      } else {
        zloc[i] = 0.0f;
        key[i] = 0;   // below every real key (real keys have a non-zero low word)
      }
    }
    int my_idx = 0;
    float my_z = 0.0f;
    float zmax = 0.0f;
    for (int j = 0; j < k; ++j) {
      const uint64_t best = wave_max_key<VPL>(key);
      int e_sel = static_cast<int>(~static_cast<uint32_t>(best));
      float z_sel = from_ordered_bits(static_cast<uint32_t>(best >> 32));
      if (j == 0) zmax = z_sel;
      if (lane == j) { my_idx = e_sel; my_z = z_sel; }
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (lane + 64 * i == e_sel) key[i] = 0;
    }
    // softmax weights: exp(z - max) over the selected (renorm) or over all experts
    float ex = lane < k ? expf(my_z - zmax) : 0.0f;
    float denom;
    if (renorm) {
      denom = wave_sum(ex);
    } else {
      float s = 0.0f;
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (lane + 64 * i < E) s += expf(zloc[i] - zmax);
      denom = wave_sum(s);
    }
    if (lane < k) {
      topk_idx[static_cast<size_t>(t) * k + lane] = my_idx;
      topk_w[static_cast<size_t>(t) * k + lane] = ex / denom;
      atomicAdd(&hist[my_idx], 1);
    }
  }
  __syncthreads();
  int32_t* out = block_hist + static_cast<size_t>(blockIdx.x) * E;
  for (int e = threadIdx.x; e < E; e += kRouteThreads) out[e] = hist[e];
}

// counts[e] = sum over workgroup rows; offsets = exclusive scan.  One block of 1024 threads:
// thread (g, c) sums rows g, g+G, ... of column c, then the groups are folded through LDS.
__global__ __launch_bounds__(1024) void route_scan_kernel(
    const int32_t* __restrict__ block_hist, int nblk, int E, int epad,
    int32_t* __restrict__ counts, int32_t* __restrict__ offsets) {
  __shared__ int32_t part[1024];
  __shared__ int32_t scan[kMaxExperts];
  const int groups = 1024 / epad;
  const int c = threadIdx.x % epad;
  const int g = threadIdx.x / epad;
  int32_t s = 0;
  if (c < E) {
#pragma unroll 8
    for (int b = g; b < nblk; b += groups) s += block_hist[static_cast<size_t>(b) * E + c];
  }
  part[threadIdx.x] = s;
  __syncthreads();
  if (g == 0) {
    for (int q = 1; q < groups; ++q) s += part[q * epad + c];
    scan[c] = c < E ? s : 0;
    if (c < E) counts[c] = s;
  }
  __syncthreads();
  // Hillis-Steele inclusive scan over epad (<= 1024) entries
  const int tid = static_cast<int>(threadIdx.x);
  for (int o = 1; o < epad; o <<= 1) {
    int32_t v = 0;
    if (tid < epad && tid >= o) v = scan[tid - o];
    __syncthreads();
    if (tid < epad) scan[tid] += v;
    __syncthreads();
  }
  if (tid < E) offsets[tid + 1] = scan[tid];
  if (tid == 0) offsets[0] = 0;
}

// histogram of an already known assignment (pre-routed rows): same per-workgroup rows as above
__global__ __launch_bounds__(kRouteThreads) void pair_hist_kernel(
    const int32_t* __restrict__ idx, int n_pairs, int E, int32_t* __restrict__ block_hist) {
  __shared__ int32_t hist[kMaxExperts];
  for (int e = threadIdx.x; e < E; e += kRouteThreads) hist[e] = 0;
  __syncthreads();
  for (int p = blockIdx.x * kRouteThreads + threadIdx.x; p < n_pairs; p += gridDim.x * kRouteThreads) {
    const int e = min(max(idx[p], 0), E - 1);
    atomicAdd(&hist[e], 1);
  }
  __syncthreads();
  int32_t* out = block_hist + static_cast<size_t>(blockIdx.x) * E;
  for (int e = threadIdx.x; e < E; e += kRouteThreads) out[e] = hist[e];
}

template <int VPL>
__global__ __launch_bounds__(kRouteThreads) void route_bwd_kernel(
    const float* __restrict__ dw, const float* __restrict__ topk_w, const int32_t* __restrict__ topk_idx,
    const float* __restrict__ logits, int T, int E, int k, int renorm, float* __restrict__ dlogits) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int waves_total = gridDim.x * kRouteWaves;
  for (int t = blockIdx.x * kRouteWaves + wave; t < T; t += waves_total) {
    int my_idx = -1;
    float my_w = 0.0f, my_dw = 0.0f;
    if (lane < k) {
      my_idx = topk_idx[static_cast<size_t>(t) * k + lane];
      my_w = topk_w[static_cast<size_t>(t) * k + lane];
      my_dw = dw[static_cast<size_t>(t) * k + lane];
    }
    const float s = wave_sum(my_w * my_dw);          // sum_m w_m dw_m
    const float my_val = my_w * (my_dw - s);          // value at a selected expert
    float out[VPL];
    if (renorm) {
#pragma unroll
      for (int i = 0; i < VPL; ++i) out[i] = 0.0f;
    } else {
      const float* z = logits + static_cast<size_t>(t) * E;
      float zl[VPL];
      float m = -INFINITY;
#pragma unroll
      for (int i = 0; i < VPL; ++i) {
        int e = lane + 64 * i;
        zl[i] = e < E ? z[e] : -INFINITY;
        m = fmaxf(m, zl[i]);
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
      float sum = 0.0f;
#pragma unroll
      for (int i = 0; i < VPL; ++i) {
        zl[i] = (lane + 64 * i < E) ? expf(zl[i] - m) : 0.0f;
        sum += zl[i];
      }
      sum = wave_sum(sum);
#pragma unroll
      for (int i = 0; i < VPL; ++i) out[i] = -(zl[i] / sum) * s;   // unselected: -p_e * s
    }
    for (int j = 0; j < k; ++j) {
      int e_j = __shfl(my_idx, j, 64);
      float v_j = __shfl(my_val, j, 64);
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (lane + 64 * i == e_j) out[i] = v_j;
    }
    float* dz = dlogits + static_cast<size_t>(t) * E;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      int e = lane + 64 * i;
      if (e < E) dz[e] = out[i];
    }
  }
}

static int route_blocks(int T) {
  int b = ceil_div(T, kRouteWaves * 2);   // about 2 tokens per wave: the per-token chain of wave reductions is latency-bound, so many waves
  return b < 1 ? 1 : (b > kRouteMaxBlocks ? kRouteMaxBlocks : b);
}

// ---- scratch of the entry point that takes no workspace -----------------------------------------------
// moe_route_topk_noalloc keeps the per-workgroup histograms in this array instead of a caller's workspace.
// Every GPU the library runs on holds its own copy (2 MiB) at its own address until the process ends.  In host
// code the array's name is only a handle: the device address comes from hipGetSymbolAddress, once per device
// with that device current, and that pointer is what the kernels are given.
constexpr int kStaticHistInts = 1 << 19;
static __device__ __align__(256) int32_t scratch[kStaticHistInts];

constexpr int kMaxScratchDevices = 64;
static std::mutex g_scratch_mutex;
static int32_t* g_scratch_ptr[kMaxScratchDevices] = {};

// device address of `scratch` on the current device (null + message on failure)
static int32_t* scratch_on_current_device(const char* who) {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess || dev < 0 || dev >= kMaxScratchDevices) {
    fail(MOE_ERR_HIP, "%s: cannot identify the current device (%s)", who, hipGetErrorString(err));
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess || !p) {
      fail(MOE_ERR_HIP, "%s: hipGetSymbolAddress of the static scratch failed on device %d (%s)", who, dev, hipGetErrorString(err));
      return nullptr;
    }
    g_scratch_ptr[dev] = static_cast<int32_t*>(p);
  }
  return g_scratch_ptr[dev];
}

static int32_t check_route_dims(int T, int E, int k) {
  MOE_REQUIRE(T >= 0 && E > 0 && k > 0, MOE_ERR_INVALID_ARG, "route: need T >= 0, E > 0, k > 0 (T=%d E=%d k=%d)", T, E, k);
  MOE_REQUIRE(k <= E, MOE_ERR_INVALID_ARG, "route: k=%d exceeds E=%d", k, E);
  MOE_REQUIRE(E <= kMaxExperts, MOE_ERR_UNSUPPORTED, "route: E=%d above the built maximum %d", E, kMaxExperts);
  MOE_REQUIRE(k <= kMaxTopK, MOE_ERR_UNSUPPORTED, "route: k=%d above the built maximum %d", k, kMaxTopK);
  MOE_REQUIRE(static_cast<int64_t>(T) * k <= INT32_MAX, MOE_ERR_UNSUPPORTED, "route: T*k does not fit in int32");
  return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" size_t moe_route_topk_workspace_bytes(int T, int E, int k) {
  (void)k;
  if (T < 0 || E <= 0) return 0;
  return align_up(static_cast<size_t>(route_blocks(T)) * E * sizeof(int32_t), 256);
}

// the two launches of the routing call; hist: route_blocks(T) rows of E counters, every one of them written by
// the first kernel before the second reads it (nothing has to be cleared)
static void launch_route_topk(const float* logits, int T, int E, int k, int renorm, int32_t* topk_idx, float* topk_w,
                              int32_t* counts, int32_t* offsets, int32_t* hist, hipStream_t s) {
  const int nblk = route_blocks(T);
  const int vpl = ceil_div(E, 64);
#define MOE_LAUNCH_ROUTE(V) \
  MOE_LAUNCH("route_topk", route_topk_kernel<V>, dim3(nblk), dim3(kRouteThreads), 0, s, logits, T, E, k, renorm, topk_idx, topk_w, hist)
  if (vpl <= 1) MOE_LAUNCH_ROUTE(1);
  else if (vpl <= 2) MOE_LAUNCH_ROUTE(2);
  else if (vpl <= 4) MOE_LAUNCH_ROUTE(4);
  else if (vpl <= 8) MOE_LAUNCH_ROUTE(8);
  else MOE_LAUNCH_ROUTE(16);
#undef MOE_LAUNCH_ROUTE
  int epad = 64;
  while (epad < E) epad <<= 1;
  MOE_LAUNCH("route_scan", route_scan_kernel, dim3(1), dim3(1024), 0, s, hist, nblk, E, epad, counts, offsets);
}

extern "C" int32_t moe_route_topk(const float* logits, int T, int E, int k, int renorm,
                                  int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets,
                                  void* ws, size_t ws_bytes, void* stream) {
  if (int32_t rc = check_route_dims(T, E, k)) return rc;
  MOE_REQUIRE(counts && offsets, MOE_ERR_INVALID_ARG, "route: counts/offsets must not be null");
  MOE_REQUIRE(T == 0 || (logits && topk_idx && topk_w), MOE_ERR_INVALID_ARG, "route: null logits/topk_idx/topk_w");
  MOE_REQUIRE(ws && ws_bytes >= moe_route_topk_workspace_bytes(T, E, k) && aligned16(ws), MOE_ERR_WORKSPACE,
              "route: workspace null, misaligned or smaller than %zu bytes", moe_route_topk_workspace_bytes(T, E, k));
  hipStream_t s = static_cast<hipStream_t>(stream);
  begin_call("moe_route_topk", s);
  launch_route_topk(logits, T, E, k, renorm, topk_idx, topk_w, counts, offsets, static_cast<int32_t*>(ws), s);
  return end_call();
}

extern "C" size_t moe_route_topk_noalloc_max_bytes(void) { return static_cast<size_t>(kStaticHistInts) * sizeof(int32_t); }

extern "C" int32_t moe_route_topk_noalloc(const float* logits, int T, int E, int k, int renorm,
                                          int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets,
                                          void* stream) {
  if (int32_t rc = check_route_dims(T, E, k)) return rc;
  MOE_REQUIRE(counts && offsets, MOE_ERR_INVALID_ARG, "route_noalloc: counts/offsets must not be null");
  MOE_REQUIRE(T == 0 || (logits && topk_idx && topk_w), MOE_ERR_INVALID_ARG, "route_noalloc: null logits/topk_idx/topk_w");
  const size_t need = moe_route_topk_workspace_bytes(T, E, k);
  MOE_REQUIRE(need <= moe_route_topk_noalloc_max_bytes(), MOE_ERR_UNSUPPORTED,
              "route_noalloc: T=%d, E=%d needs %zu bytes of histogram rows, the static scratch holds %zu; "
              "use moe_route_topk with a workspace", T, E, need, moe_route_topk_noalloc_max_bytes());
  int32_t* hist = scratch_on_current_device("route_noalloc");
  if (!hist) return MOE_ERR_HIP;
  hipStream_t s = static_cast<hipStream_t>(stream);
  begin_call("moe_route_topk_noalloc", s);
  launch_route_topk(logits, T, E, k, renorm, topk_idx, topk_w, counts, offsets, hist, s);
  return end_call();
}

static int hist_blocks(int n_pairs) {
  int b = ceil_div(n_pairs, kRouteThreads * 4);
  return b < 1 ? 1 : (b > kRouteMaxBlocks ? kRouteMaxBlocks : b);
}

extern "C" size_t moe_expert_offsets_workspace_bytes(int n_pairs, int E) {
  if (n_pairs < 0 || E <= 0) return 0;
  return align_up(static_cast<size_t>(hist_blocks(n_pairs)) * E * sizeof(int32_t), 256);
}

extern "C" int32_t moe_expert_offsets(const int32_t* topk_idx, int n_pairs, int E, int32_t* counts,
                                      int32_t* offsets, void* ws, size_t ws_bytes, void* stream) {
  MOE_REQUIRE(n_pairs >= 0 && E > 0, MOE_ERR_INVALID_ARG, "expert_offsets: need n_pairs >= 0, E > 0");
  MOE_REQUIRE(E <= kMaxExperts, MOE_ERR_UNSUPPORTED, "expert_offsets: E=%d above the built maximum %d", E, kMaxExperts);
  MOE_REQUIRE(counts && offsets && (n_pairs == 0 || topk_idx), MOE_ERR_INVALID_ARG, "expert_offsets: null pointer");
  MOE_REQUIRE(ws && ws_bytes >= moe_expert_offsets_workspace_bytes(n_pairs, E) && aligned16(ws), MOE_ERR_WORKSPACE,
              "expert_offsets: workspace null, misaligned or smaller than %zu bytes", moe_expert_offsets_workspace_bytes(n_pairs, E));
  hipStream_t s = static_cast<hipStream_t>(stream);
  begin_call("moe_expert_offsets", s);
  const int nblk = hist_blocks(n_pairs);
  int32_t* hist = static_cast<int32_t*>(ws);
  MOE_LAUNCH("pair_hist", pair_hist_kernel, dim3(nblk), dim3(kRouteThreads), 0, s, topk_idx, n_pairs, E, hist);
  int epad = 64;
  while (epad < E) epad <<= 1;
  MOE_LAUNCH("route_scan", route_scan_kernel, dim3(1), dim3(1024), 0, s, hist, nblk, E, epad, counts, offsets);
  return end_call();
}

extern "C" int32_t moe_route_topk_bwd(const float* dw, const float* topk_w, const int32_t* topk_idx,
                                      const float* logits, int T, int E, int k, int renorm,
                                      float* dlogits, void* stream) {
  if (int32_t rc = check_route_dims(T, E, k)) return rc;
  if (T == 0) return MOE_OK;
  MOE_REQUIRE(dw && topk_w && topk_idx && dlogits, MOE_ERR_INVALID_ARG, "route_bwd: null pointer");
  MOE_REQUIRE(renorm || logits, MOE_ERR_INVALID_ARG, "route_bwd: logits required when renorm == 0");
  hipStream_t s = static_cast<hipStream_t>(stream);
  begin_call("moe_route_topk_bwd", s);
  const int nblk = route_blocks(T);
  const int vpl = ceil_div(E, 64);
#define MOE_LAUNCH_RBWD(V) \
  MOE_LAUNCH("route_bwd", route_bwd_kernel<V>, dim3(nblk), dim3(kRouteThreads), 0, s, dw, topk_w, topk_idx, logits, T, E, k, renorm, dlogits)
  if (vpl <= 1) MOE_LAUNCH_RBWD(1);
  else if (vpl <= 2) MOE_LAUNCH_RBWD(2);
  else if (vpl <= 4) MOE_LAUNCH_RBWD(4);
  else if (vpl <= 8) MOE_LAUNCH_RBWD(8);
  else MOE_LAUNCH_RBWD(16);
#undef MOE_LAUNCH_RBWD
  return end_call();
}
