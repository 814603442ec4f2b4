// Token permutation into expert-contiguous rows and the weighted un-permute / combine,
// forward and backward (the local halves of the dispatch / return of Sec. 3.2.3).
//
// The permutation is a stable counting sort of the P = T*k (token, slot) pairs by expert:
//   1. each workgroup takes a contiguous chunk of pairs, ranks every pair among the
//      earlier pairs of the same expert inside the chunk and writes the chunk's
//      per-expert histogram (expert-major, so step 2 reads contiguously);
//   2. one wavefront per expert prefix-scans its histogram over the chunks and adds the
//      expert's segment offset;
//   3. one wavefront per token adds chunk base and in-chunk rank, writes both maps and
//      copies the token's row to each of its k destination rows (the source row is read
//      once and kept in registers).
// Integer work only; no atomics decide an order, so the result is the stable order.
//
// The movers are pure HBM traffic: every lane moves 16 bytes per access and rows are
// traversed contiguously.
#include "moe_common.h"

namespace moe {

constexpr int kChunkPairs = 256;     // pairs ranked by one workgroup
constexpr int kMoverThreads = 256;

// ---- step 1: in-chunk ranks + chunk histogram ---------------------------------------------
__global__ __launch_bounds__(kChunkPairs) void permute_rank_kernel(
    const int32_t* __restrict__ topk_idx, int P, int E, int nchunks,
    int32_t* __restrict__ rank_in_chunk, int32_t* __restrict__ chunk_hist /* [E][nchunks] */) {
  __shared__ int32_t idx_s[kChunkPairs];
  __shared__ int32_t hist[kMaxExperts];
  const int chunk = blockIdx.x;
  const int p = chunk * kChunkPairs + threadIdx.x;
  for (int e = threadIdx.x; e < E; e += kChunkPairs) hist[e] = 0;
  const int my = p < P ? min(max(topk_idx[p], 0), E - 1) : -1;   // out-of-range ids cannot leave the histogram
  idx_s[threadIdx.x] = my;
  __syncthreads();
  if (p < P) {
    int rank = 0;
    for (int q = 0; q < static_cast<int>(threadIdx.x); ++q) rank += (idx_s[q] == my);
    rank_in_chunk[p] = rank;
    atomicAdd(&hist[my], 1);           // integer count: order-independent
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += kChunkPairs)
    chunk_hist[static_cast<size_t>(e) * nchunks + chunk] = hist[e];
}

// ---- step 2: per expert, exclusive scan over chunks, plus the segment offset --------------
__global__ __launch_bounds__(256) void permute_scan_kernel(
    int32_t* __restrict__ chunk_hist /* in: counts, out: bases */, int nchunks, int E,
    const int32_t* __restrict__ offsets) {
  const int lane = threadIdx.x & 63;
  const int e = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (e >= E) return;
  int32_t* col = chunk_hist + static_cast<size_t>(e) * nchunks;
  int32_t carry = offsets[e];
  for (int base = 0; base < nchunks; base += 64) {
    int c = base + lane;
    int32_t v = c < nchunks ? col[c] : 0;
    int32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      int32_t up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (c < nchunks) col[c] = carry + incl - v;
    carry += __shfl(incl, 63, 64);
  }
}

// ---- step 3: maps + row gather ------------------------------------------------------------

// The combine kernels stream their rows: every source piece is read once and every destination piece written
// once, to be consumed by a later kernel.  Non-temporal accesses keep them from displacing what the neighbouring
// kernels share through the L2 (measured: 5-8 % on combine_fwd, 2 % on the kernels that follow).  The gather of
// the permutation is faster with ordinary accesses and keeps them.
typedef unsigned int mover_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_stream(const uint4* p) {
  const mover_u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const mover_u32x4*>(p));
  return make_uint4(w.x, w.y, w.z, w.w);
}
__device__ __forceinline__ void store16_stream(uint4* p, const uint4& v) {
  const mover_u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<mover_u32x4*>(p));
}

// One wave per token; a row is d*elem bytes = n16 sixteen-byte pieces.
__global__ __launch_bounds__(kMoverThreads) void permute_gather_kernel(
    const uint4* __restrict__ x, int T, int k, int E, int n16, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ rank_in_chunk, const int32_t* __restrict__ chunk_base, int nchunks,
    uint4* __restrict__ xp, int32_t* __restrict__ row_of_pair, int32_t* __restrict__ pair_of_row) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * (kMoverThreads / 64) + (threadIdx.x >> 6);
  if (t >= T) return;
  // lanes 0..k-1 resolve the k destination rows of this token
  int my_row = 0;
  if (lane < k) {
    int p = t * k + lane;
    int e = min(max(topk_idx[p], 0), E - 1);
    my_row = chunk_base[static_cast<size_t>(e) * nchunks + p / kChunkPairs] + rank_in_chunk[p];
    my_row = min(max(my_row, 0), T * k - 1);     // stays in bounds even if offsets are inconsistent
    row_of_pair[p] = my_row;
    pair_of_row[my_row] = p;
  }
  const uint4* src = x + static_cast<size_t>(t) * n16;
  for (int c0 = 0; c0 < n16; c0 += 256) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      int c = c0 + u * 64 + lane;
      if (c < n16) v[u] = src[c];
    }
    for (int j = 0; j < k; ++j) {
      int row = __shfl(my_row, j, 64);
      uint4* dst = xp + static_cast<size_t>(row) * n16;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        int c = c0 + u * 64 + lane;
        if (c < n16) dst[c] = v[u];
      }
    }
  }
}

// ---- element helpers: a 16-byte piece as fp32 values --------------------------------------
template <int DT> struct Piece;
template <> struct Piece<MOE_BF16> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float* f) {
    return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
  }
};
template <> struct Piece<MOE_F32> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float* f) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
};

// ---- combine forward: y[t] = sum_j w[t,j] * yp[row(t,j)] ------------------------------------
// One thread per PPT 16-byte pieces of y (a workgroup covers PPT x 256 consecutive pieces, piece u of a thread 256
// pieces after piece u-1, so every access of a wave is 1 KiB contiguous).  The slot indices and weights of the tokens
// are fetched first, then KB slots x PPT pieces are all in flight together before the fp32 sums, which run in slot
// order (the same order on every run).
template <int DT, int KB, int PPT>
__global__ __launch_bounds__(kMoverThreads) void combine_fwd_kernel(
    const uint4* __restrict__ yp, int T, int k, int n16, const float* __restrict__ topk_w,
    const int32_t* __restrict__ row_of_pair, uint4* __restrict__ y) {
  constexpr int N = Piece<DT>::N;
  const size_t total = static_cast<size_t>(T) * n16;
  const size_t first = static_cast<size_t>(blockIdx.x) * (kMoverThreads * PPT) + threadIdx.x;
  const int last = T * k - 1;
  float acc[PPT][N];
  int t[PPT], c[PPT];
#pragma unroll
  for (int u = 0; u < PPT; ++u) {
    const size_t piece = min(first + static_cast<size_t>(u) * kMoverThreads, total - 1);   // pieces past the end repeat the last one (not stored)
    t[u] = static_cast<int>(piece / n16);
    c[u] = static_cast<int>(piece % n16);
#pragma unroll
    for (int i = 0; i < N; ++i) acc[u][i] = 0.0f;
  }
  for (int j = 0; j < k; j += KB) {
    int r[PPT][KB];
    float wj[PPT][KB];
#pragma unroll
    for (int u = 0; u < PPT; ++u) {
      const int32_t* rows = row_of_pair + static_cast<size_t>(t[u]) * k;
      const float* w = topk_w ? topk_w + static_cast<size_t>(t[u]) * k : nullptr;
#pragma unroll
      for (int q = 0; q < KB; ++q) {                     // slots beyond k repeat the last one with weight 0
        const int jq = min(j + q, k - 1);
        r[u][q] = min(max(rows[jq], 0), last);
        wj[u][q] = j + q < k ? (w ? w[jq] : 1.0f) : 0.0f;
      }
    }
    uint4 v[PPT][KB];
#pragma unroll
    for (int u = 0; u < PPT; ++u)
#pragma unroll
      for (int q = 0; q < KB; ++q) v[u][q] = load16_stream(yp + static_cast<size_t>(r[u][q]) * n16 + c[u]);
#pragma unroll
    for (int u = 0; u < PPT; ++u)
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        if (j + q < k) {
          float f[N];
          Piece<DT>::unpack(v[u][q], f);
#pragma unroll
          for (int i = 0; i < N; ++i) acc[u][i] = fmaf(wj[u][q], f[i], acc[u][i]);
        }
      }
  }
#pragma unroll
  for (int u = 0; u < PPT; ++u) {
    const size_t piece = first + static_cast<size_t>(u) * kMoverThreads;
    if (piece < total) store16_stream(y + piece, Piece<DT>::pack(acc[u]));
  }
}

// ---- combine backward: dyp[row] = w * dy[t];  dw[t,j] = <dy[t], yp[row]> --------------------
// One wave per token.  The token's row of dy is read once per 256-piece stretch and kept in registers; the matching
// pieces of up to KB slots' yp rows are requested together, then each slot's dyp pieces are written and its dot
// product accumulated; the KB dot products are reduced across the wave at the end, all in a fixed order.
template <int DT, int KB>
__global__ __launch_bounds__(kMoverThreads) void combine_bwd_kernel(
    const uint4* __restrict__ dy, const uint4* __restrict__ yp, int T, int k, int n16,
    const float* __restrict__ topk_w, const int32_t* __restrict__ row_of_pair,
    uint4* __restrict__ dyp, float* __restrict__ dw) {
  constexpr int N = Piece<DT>::N;
  constexpr int PL = 4;                                  // pieces per lane and stretch
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * (kMoverThreads / 64) + (threadIdx.x >> 6);
  if (t >= T) return;
  const uint4* dyr = dy + static_cast<size_t>(t) * n16;
  int my_row = 0;
  float my_w = 0.0f;
  if (lane < k) {
    my_row = min(max(row_of_pair[static_cast<size_t>(t) * k + lane], 0), T * k - 1);
    my_w = topk_w[static_cast<size_t>(t) * k + lane];
  }
  float my_dot = 0.0f;
  for (int j0 = 0; j0 < k; j0 += KB) {
    int row[KB];
    float wj[KB], dot[KB];
#pragma unroll
    for (int q = 0; q < KB; ++q) {                       // slots beyond k repeat the last one; nothing of theirs is stored
      const int jq = min(j0 + q, k - 1);
      row[q] = __shfl(my_row, jq, 64);
      wj[q] = __shfl(my_w, jq, 64);
      dot[q] = 0.0f;
    }
    for (int c0 = 0; c0 < n16; c0 += 64 * PL) {
      uint4 a[PL], b[KB][PL];
#pragma unroll
      for (int u = 0; u < PL; ++u) {
        const int c = min(c0 + u * 64 + lane, n16 - 1);
        a[u] = dyr[c];
      }
#pragma unroll
      for (int q = 0; q < KB; ++q)
#pragma unroll
        for (int u = 0; u < PL; ++u) {
          const int c = min(c0 + u * 64 + lane, n16 - 1);
          b[q][u] = load16_stream(yp + static_cast<size_t>(row[q]) * n16 + c);
        }
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        if (j0 + q < k) {
#pragma unroll
          for (int u = 0; u < PL; ++u) {
            const int c = c0 + u * 64 + lane;
            if (c < n16) {
              float fa[N], fb[N], fo[N];
              Piece<DT>::unpack(a[u], fa);
              Piece<DT>::unpack(b[q][u], fb);
#pragma unroll
              for (int i = 0; i < N; ++i) { dot[q] = fmaf(fa[i], fb[i], dot[q]); fo[i] = wj[q] * fa[i]; }
              store16_stream(dyp + static_cast<size_t>(row[q]) * n16 + c, Piece<DT>::pack(fo));
            }
          }
        }
      }
    }
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      const float d = wave_sum(dot[q]);
      if (lane == j0 + q) my_dot = d;
    }
  }
  if (lane < k) dw[static_cast<size_t>(t) * k + lane] = my_dot;
}

static int32_t check_mover_dims(const char* who, int dtype, int T, int d, int k) {
  MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_ERR_UNSUPPORTED, "%s: unknown dtype %d", who, dtype);
  MOE_REQUIRE(T >= 0 && d > 0 && k > 0, MOE_ERR_INVALID_ARG, "%s: need T >= 0, d > 0, k > 0 (T=%d d=%d k=%d)", who, T, d, k);
  MOE_REQUIRE(k <= kMaxTopK, MOE_ERR_UNSUPPORTED, "%s: k=%d above the built maximum %d", who, k, kMaxTopK);
  MOE_REQUIRE(d % 8 == 0, MOE_ERR_UNSUPPORTED, "%s: d=%d must be a multiple of 8", who, d);
  MOE_REQUIRE(static_cast<int64_t>(T) * k <= INT32_MAX, MOE_ERR_UNSUPPORTED, "%s: T*k does not fit in int32", who);
  return MOE_OK;
}

static size_t permute_ws_layout(int T, int E, int k, size_t* hist_off) {
  const size_t P = static_cast<size_t>(T) * k;
  const size_t nchunks = (P + kChunkPairs - 1) / kChunkPairs;
  const size_t rank_bytes = align_up(P * sizeof(int32_t), 256);
  if (hist_off) *hist_off = rank_bytes;
  return rank_bytes + align_up(nchunks * E * sizeof(int32_t), 256) + 256;
}

}  // namespace moe

using namespace moe;

extern "C" size_t moe_permute_workspace_bytes(int T, int E, int k) {
  if (T < 0 || E <= 0 || k <= 0) return 0;
  return permute_ws_layout(T, E, k, nullptr);
}

extern "C" int32_t moe_permute(const void* x, int dtype, int T, int d, int E, int k,
                               const int32_t* topk_idx, const int32_t* offsets,
                               void* xp, int32_t* row_of_pair, int32_t* pair_of_row,
                               void* ws, size_t ws_bytes, void* stream) {
  if (int32_t rc = check_mover_dims("permute", dtype, T, d, k)) return rc;
  MOE_REQUIRE(E > 0 && k <= E, MOE_ERR_INVALID_ARG, "permute: need E > 0 and k <= E (E=%d k=%d)", E, k);
  MOE_REQUIRE(E <= kMaxExperts, MOE_ERR_UNSUPPORTED, "permute: E=%d above the built maximum %d", E, kMaxExperts);
  if (T == 0) return MOE_OK;
  MOE_REQUIRE(topk_idx && offsets && row_of_pair && pair_of_row, MOE_ERR_INVALID_ARG, "permute: null pointer");
  MOE_REQUIRE((x == nullptr) == (xp == nullptr), MOE_ERR_INVALID_ARG, "permute: x and xp must both be given, or both be null for the maps alone");
  MOE_REQUIRE(aligned16(x) && aligned16(xp), MOE_ERR_INVALID_ARG, "permute: x / xp must be 16-byte aligned");
  size_t hist_off = 0;
  const size_t need = permute_ws_layout(T, E, k, &hist_off);
  MOE_REQUIRE(ws && ws_bytes >= need && aligned16(ws), MOE_ERR_WORKSPACE, "permute: workspace null, misaligned or smaller than %zu bytes", need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  begin_call("moe_permute", s);
  const int P = T * k;
  const int nchunks = ceil_div(P, kChunkPairs);
  int32_t* rank = static_cast<int32_t*>(ws);
  int32_t* hist = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + hist_off);
  const int n16 = x ? d * elem_size(dtype) / 16 : 0;     // no rows to copy: the gather kernel only writes the two maps
  MOE_LAUNCH("permute_rank", permute_rank_kernel, dim3(nchunks), dim3(kChunkPairs), 0, s, topk_idx, P, E, nchunks, rank, hist);
  MOE_LAUNCH("permute_scan", permute_scan_kernel, dim3(ceil_div(E, 4)), dim3(256), 0, s, hist, nchunks, E, offsets);
  MOE_LAUNCH(x ? "permute_gather" : "permute_maps", permute_gather_kernel, dim3(ceil_div(T, kMoverThreads / 64)), dim3(kMoverThreads), 0, s,
                     static_cast<const uint4*>(x), T, k, E, n16, topk_idx, rank, hist, nchunks,
                     static_cast<uint4*>(xp), row_of_pair, pair_of_row);
  return end_call();
}

extern "C" int32_t moe_unpermute_combine_fwd(const void* yp, int dtype, int T, int d, int k,
                                             const float* topk_w, const int32_t* row_of_pair,
                                             void* y, void* stream) {
  if (int32_t rc = check_mover_dims("combine_fwd", dtype, T, d, k)) return rc;
  if (T == 0) return MOE_OK;
  MOE_REQUIRE(yp && row_of_pair && y, MOE_ERR_INVALID_ARG, "combine_fwd: null pointer");
  MOE_REQUIRE(aligned16(yp) && aligned16(y), MOE_ERR_INVALID_ARG, "combine_fwd: yp / y must be 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  begin_call("moe_unpermute_combine_fwd", s);
  const int n16 = d * elem_size(dtype) / 16;
  const size_t total = static_cast<size_t>(T) * n16;
  // KB slots of a token x PPT pieces in flight per thread.  Measured: with one slot per token (rows delivered by an
  // expert-parallel dispatch) more pieces per thread are slower (0.56 of the HBM peak with eight against 0.62 with one:
  // the launch is 27 us long and fewer, fatter threads fill the chip later), so PPT stays 1.
#define MOE_COMBINE_FWD(DT, KB, PPT) \
  MOE_LAUNCH("combine_fwd", (combine_fwd_kernel<DT, KB, PPT>), dim3(static_cast<unsigned>((total + kMoverThreads * PPT - 1) / (kMoverThreads * PPT))), \
             dim3(kMoverThreads), 0, s, static_cast<const uint4*>(yp), T, k, n16, topk_w, row_of_pair, static_cast<uint4*>(y))
  if (dtype == MOE_BF16) {
    if (k >= 8) MOE_COMBINE_FWD(MOE_BF16, 8, 1); else if (k >= 3) MOE_COMBINE_FWD(MOE_BF16, 4, 1);
    else if (k == 2) MOE_COMBINE_FWD(MOE_BF16, 2, 1); else MOE_COMBINE_FWD(MOE_BF16, 1, 1);
  } else {
    if (k >= 8) MOE_COMBINE_FWD(MOE_F32, 8, 1); else if (k >= 3) MOE_COMBINE_FWD(MOE_F32, 4, 1);
    else if (k == 2) MOE_COMBINE_FWD(MOE_F32, 2, 1); else MOE_COMBINE_FWD(MOE_F32, 1, 1);
  }
#undef MOE_COMBINE_FWD
  return end_call();
}

extern "C" int32_t moe_unpermute_combine_bwd(const void* dy, const void* yp, int dtype, int T, int d, int k,
                                             const float* topk_w, const int32_t* row_of_pair,
                                             void* dyp, float* dw, void* stream) {
  if (int32_t rc = check_mover_dims("combine_bwd", dtype, T, d, k)) return rc;
  if (T == 0) return MOE_OK;
  MOE_REQUIRE(dy && yp && topk_w && row_of_pair && dyp && dw, MOE_ERR_INVALID_ARG, "combine_bwd: null pointer");
  MOE_REQUIRE(aligned16(dy) && aligned16(yp) && aligned16(dyp), MOE_ERR_INVALID_ARG, "combine_bwd: dy / yp / dyp must be 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  begin_call("moe_unpermute_combine_bwd", s);
  const int n16 = d * elem_size(dtype) / 16;
  const unsigned blocks = static_cast<unsigned>(ceil_div(T, kMoverThreads / 64));
#define MOE_COMBINE_BWD(DT, KB) \
  MOE_LAUNCH("combine_bwd", (combine_bwd_kernel<DT, KB>), dim3(blocks), dim3(kMoverThreads), 0, s, static_cast<const uint4*>(dy), \
             static_cast<const uint4*>(yp), T, k, n16, topk_w, row_of_pair, static_cast<uint4*>(dyp), dw)
  if (dtype == MOE_BF16) {
    if (k >= 4) MOE_COMBINE_BWD(MOE_BF16, 4); else if (k >= 2) MOE_COMBINE_BWD(MOE_BF16, 2); else MOE_COMBINE_BWD(MOE_BF16, 1);
  } else {
    if (k >= 4) MOE_COMBINE_BWD(MOE_F32, 4); else if (k >= 2) MOE_COMBINE_BWD(MOE_F32, 2); else MOE_COMBINE_BWD(MOE_F32, 1);
  }
#undef MOE_COMBINE_BWD
  return end_call();
}
