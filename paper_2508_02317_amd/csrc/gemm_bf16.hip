// bf16 MFMA grouped GEMMs of the SwiGLU expert FFN, forward and backward
// (Sec. 3.2.5 SwiGLU among the efficient kernels; App. B.6 stacked expert-major weights).
//
// One kernel skeleton serves all nine matrix products of the layer:
//   * a 128 x 128 output tile per 256-thread workgroup (2 x 2 wavefronts, each 64 x 64 =
//     2 x 2 MFMA tiles of v_mfma_f32_32x32x16_bf16, fp32 accumulators);
//   * the reduction dimension is walked in 64-wide slabs, double-buffered in LDS; the
//     global loads of slab i+1 are issued before the MFMAs of slab i;
//   * both operand tiles live in LDS as [128 rows][64 k] bf16 with the 16-byte column
//     pieces XOR-swizzled by the row, so that the 16-byte MFMA operand reads are
//     bank-conflict free;
//   * an operand whose reduction index is the slow (strided) axis in memory -- the
//     weight in the two "backward data" products and both operands of the weight-gradient
//     products -- is transposed in registers on its way into LDS, so the MFMA inner loop
//     is identical for all variants.
// Row-grouped products (rows of the activation matrix belong to experts) take their
// (expert, row-tile) list from a small schedule built on the device from `offsets`, so no
// host synchronisation is needed; weight-gradient products are grouped along the
// reduction dimension instead and have a host-known grid.
// Workgroup ids are remapped so that consecutive tiles -- which share an expert's weights
// -- run on the same XCD and hit its L2.
#include "moe_common.h"

namespace moe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kGemmThreads = 256;
constexpr int kTileBytes = BM * BK * 2;                 // one operand tile in LDS (16 KiB)
constexpr int kLdsBytes = 4 * kTileBytes;               // A and B, double-buffered
constexpr int kXcds = 8;

// byte offset of (row, 16-byte piece) inside a swizzled [128][64] bf16 tile
__device__ __forceinline__ int swz(int row, int piece) { return row * (BK * 2) + ((piece ^ (row & 7)) << 4); }

// One 128-row operand tile: element (row, k).  Two 64-row halves with their own base so
// that the gate and the up projection can share one tile.
//   k-contiguous: half[h] + row * ld + k          k-strided: half[h] + k * ld + row
struct Operand {
  const bf16_t* half[2];
  long ld;
  int valid[2];      // rows of each half that exist (others read as zero)
};

// ---- global -> register -> LDS staging ---------------------------------------------------
template <bool KS> struct Stager;

// reduction index contiguous in memory: 4 independent 16-byte loads, stored as they are
template <> struct Stager<false> {
  const bf16_t* ptr[4];
  bool row_ok[4];
  int lds_off[4];
  int kpiece;
  uint4 v[4];
  __device__ __forceinline__ void init(const Operand& op, int tid) {
    kpiece = tid & 7;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (tid >> 3) + 32 * i;
      const int rh = row & 63;
      const bool upper = i >= 2;            // rows 64..127 are loads 2 and 3
      row_ok[i] = rh < (upper ? op.valid[1] : op.valid[0]);
      ptr[i] = (upper ? op.half[1] : op.half[0]) + static_cast<long>(rh) * op.ld + kpiece * 8;
      lds_off[i] = swz(row, kpiece);
    }
  }
  __device__ __forceinline__ void load(int k0, int K) {
    const bool k_ok = k0 + kpiece * 8 < K;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[i] = make_uint4(0, 0, 0, 0);
      if (row_ok[i] && k_ok) v[i] = *reinterpret_cast<const uint4*>(ptr[i] + k0);
    }
  }
  __device__ __forceinline__ void store(char* tile) const {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(tile + lds_off[i]) = v[i];
  }
};

// reduction index strided: thread (nb, kq) loads k = 4kq..4kq+3 for rows 8nb..8nb+7,
// transposes the 4 x 8 block in registers and stores eight 8-byte pieces
template <> struct Stager<true> {
  const bf16_t* ptr;
  long ld;
  bool row_ok;
  int nb, kq;
  uint4 v[4];
  __device__ __forceinline__ void init(const Operand& op, int tid) {
    nb = tid & 15;
    kq = tid >> 4;
    const int row = nb * 8;
    const int rh = row & 63;
    const bool upper = row >= 64;
    row_ok = rh < (upper ? op.valid[1] : op.valid[0]);          // valid counts are multiples of 8
    ld = op.ld;
    ptr = (upper ? op.half[1] : op.half[0]) + rh + static_cast<long>(kq * 4) * ld;
  }
  __device__ __forceinline__ void load(int k0, int K) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[i] = make_uint4(0, 0, 0, 0);
      if (row_ok && k0 + kq * 4 + i < K) v[i] = *reinterpret_cast<const uint4*>(ptr + static_cast<long>(k0 + i) * ld);
    }
  }
  __device__ __forceinline__ void store(char* tile) const {
    const uint32_t in[4][4] = {{v[0].x, v[0].y, v[0].z, v[0].w}, {v[1].x, v[1].y, v[1].z, v[1].w},
                               {v[2].x, v[2].y, v[2].z, v[2].w}, {v[3].x, v[3].y, v[3].z, v[3].w}};
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      // rotate the row visited at step s by the lane's block id to spread LDS banks
      const int n = (s + nb) & 7;
      uint32_t lo, hi;
      // word n>>1 of every k-row, half n&1
      uint32_t w0 = 0, w1 = 0, w2 = 0, w3 = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if ((n >> 1) == q) { w0 = in[0][q]; w1 = in[1][q]; w2 = in[2][q]; w3 = in[3][q]; }
      }
      if (n & 1) {
        lo = (w0 >> 16) | (w1 & 0xFFFF0000u);
        hi = (w2 >> 16) | (w3 & 0xFFFF0000u);
      } else {
        lo = (w0 & 0xFFFFu) | (w1 << 16);
        hi = (w2 & 0xFFFFu) | (w3 << 16);
      }
      const int row = nb * 8 + n;
      *reinterpret_cast<uint2*>(tile + swz(row, kq >> 1) + (kq & 1) * 8) = make_uint2(lo, hi);
    }
  }
};

// ---- MFMA over one staged 64-wide slab ----------------------------------------------------
// a_row[mi] / b_row[ni]: first tile row of this wave's mi-th / ni-th 32-row fragment
__device__ __forceinline__ void mma_slab(const char* tileA, const char* tileB, const int (&a_row)[2],
                                         const int (&b_row)[2], int lane, f32x16 (&acc)[2][2]) {
  const int r = lane & 31, kh = lane >> 5;
#pragma unroll
  for (int kk = 0; kk < BK / 16; ++kk) {
    bf16x8 a[2], b[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a[i] = *reinterpret_cast<const bf16x8*>(tileA + swz(a_row[i] + r, 2 * kk + kh));
      b[i] = *reinterpret_cast<const bf16x8*>(tileB + swz(b_row[i] + r, 2 * kk + kh));
    }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
  }
}

// acc += A(128 x K) * B(128 x K)^T, both staged through LDS.  Ends with a barrier, so it
// can be called again (second reduction segment) right away.
template <bool A_KS, bool B_KS>
__device__ __forceinline__ void mainloop(const Operand& opA, const Operand& opB, int K, char* lds,
                                         const int (&a_row)[2], const int (&b_row)[2], f32x16 (&acc)[2][2]) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int ktiles = (K + BK - 1) / BK;
  if (ktiles <= 0) return;
  Stager<A_KS> sa;
  Stager<B_KS> sb;
  sa.init(opA, tid);
  sb.init(opB, tid);
  char* const tA = lds;                       // two A buffers, then two B buffers
  char* const tB = lds + 2 * kTileBytes;
  sa.load(0, K);
  sb.load(0, K);
  sa.store(tA);
  sb.store(tB);
  __syncthreads();
  for (int kt = 0; kt < ktiles; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < ktiles;
    if (more) {
      sa.load((kt + 1) * BK, K);
      sb.load((kt + 1) * BK, K);
    }
    mma_slab(tA + cur * kTileBytes, tB + cur * kTileBytes, a_row, b_row, lane, acc);
    if (more) {
      sa.store(tA + (cur ^ 1) * kTileBytes);
      sb.store(tB + (cur ^ 1) * kTileBytes);
    }
    __syncthreads();
  }
}

// ---- device-built schedule of (expert, row tile) for row-grouped products -----------------
struct RowTiles {
  int32_t* count;        // [1] number of row tiles
  int32_t* expert;       // [max_tiles]
  int32_t* row0;         // [max_tiles]
  int max_tiles;
};

__global__ __launch_bounds__(1024) void build_row_tiles_kernel(const int32_t* __restrict__ offsets, int E, int P,
                                                                RowTiles rt) {
  __shared__ int32_t scan[kMaxExperts];
  const int e = threadIdx.x;
  int begin = 0, end = 0, nt = 0;
  if (e < E) {
    begin = min(max(offsets[e], 0), P);
    end = min(max(offsets[e + 1], begin), P);
    nt = (end - begin + BM - 1) / BM;
  }
  scan[e] = nt;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    int v = e >= o ? scan[e - o] : 0;
    __syncthreads();
    scan[e] += v;
    __syncthreads();
  }
  // offsets that are not a monotone scan ending at P cannot overflow the lists
  const int first = scan[e] - nt;
  for (int i = 0; i < nt && first + i < rt.max_tiles; ++i) {
    rt.expert[first + i] = e;
    rt.row0[first + i] = begin + i * BM;
  }
  if (e == 1023) rt.count[0] = min(scan[1023], rt.max_tiles);
}

// workgroup id -> virtual tile id such that consecutive virtual ids share an XCD
__device__ __forceinline__ int xcd_remap(int b, int total) {
  const int per = (total + kXcds - 1) / kXcds;
  const int v = (b % kXcds) * per + b / kXcds;
  return (b / kXcds < per && v < total) ? v : -1;
}

// ---- accumulator coordinates ----------------------------------------------------------------
// element i (0..15) of a 32x32 MFMA tile held by `lane`: row 8*(i/4) + 4*(lane/32) + i%4, col lane%32
__device__ __forceinline__ int acc_row(int lane, int i) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

// ============================================================================================
// Row-grouped kernels
// ============================================================================================
enum { kGateUp = 0, kDown = 1, kDAct = 2, kDX = 3 };

struct RowArgs {
  const bf16_t* a;         // activation operand [P, lda]
  long lda;
  const bf16_t* w0;        // first weight  [E, ...]
  const bf16_t* w1;        // second weight (gate/up kinds) or null
  long w_expert_stride;    // elements between experts
  long ldw;                // row pitch of one expert's weight matrix
  int K;                   // reduction length per segment
  int N;                   // output columns
  const int32_t* offsets;
  int P;
  RowTiles rt;
  int n_tiles_n;
  bf16_t* out0;            // kGateUp: G (may be null)   kDown/kDX: output     kDAct: dGU
  bf16_t* out1;            // kGateUp: U (may be null)
  bf16_t* out2;            // kGateUp: act (may be null)
  long ldo;
  const bf16_t* g;         // kDAct: saved pre-activations
  const bf16_t* u;
};

template <int KIND>
__global__ __launch_bounds__(kGemmThreads) void row_grouped_kernel(RowArgs p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int n_row_tiles = p.rt.count[0];
  const int v = xcd_remap(blockIdx.x, n_row_tiles * p.n_tiles_n);
  if (v < 0) return;
  const int mt = v / p.n_tiles_n, nt = v % p.n_tiles_n;
  const int e = p.rt.expert[mt];
  const int row0 = p.rt.row0[mt];
  const int row_end = min(p.offsets[e + 1], p.P);
  const int rows = min(BM, row_end - row0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

  const int a_row[2] = {wm * 64, wm * 64 + 32};
  Operand opA, opB;
  opA.ld = p.lda;
  opA.valid[0] = min(rows, 64);
  opA.valid[1] = max(rows - 64, 0);

  if (KIND == kGateUp) {
    // tile columns: 64 gate columns n0.. and the matching 64 up columns
    const int n0 = nt * 64;
    const int ncols = min(64, p.N - n0);
    const int b_row[2] = {wn * 32, 64 + wn * 32};
    opA.half[0] = p.a + static_cast<long>(row0) * p.lda;
    opA.half[1] = opA.half[0] + 64 * p.lda;
    opB.ld = p.ldw;
    opB.half[0] = p.w0 + e * p.w_expert_stride + static_cast<long>(n0) * p.ldw;
    opB.half[1] = p.w1 + e * p.w_expert_stride + static_cast<long>(n0) * p.ldw;
    opB.valid[0] = opB.valid[1] = ncols;
    mainloop<false, false>(opA, opB, p.K, lds, a_row, b_row, acc);
    const int col = n0 + wn * 32 + (lane & 31);
    if (wn * 32 + (lane & 31) < ncols) {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = wm * 64 + mi * 32 + acc_row(lane, i);
          if (r < rows) {
            const float g = acc[mi][0][i], u = acc[mi][1][i];
            const long o = static_cast<long>(row0 + r) * p.ldo + col;
            if (p.out0) p.out0[o] = f32_to_bf16(g);
            if (p.out1) p.out1[o] = f32_to_bf16(u);
            if (p.out2) p.out2[o] = f32_to_bf16(g * sigmoid_fast(g) * u);
          }
        }
    }
    return;
  }

  const int n0 = nt * BN;
  const int ncols = min(BN, p.N - n0);
  const int b_row[2] = {wn * 64, wn * 64 + 32};
  opB.ld = p.ldw;
  opB.valid[0] = min(ncols, 64);
  opB.valid[1] = max(ncols - 64, 0);
  if (KIND == kDown) {
    // yp = act * Wd[e]^T : weight rows are output columns, reduction contiguous
    opA.half[0] = p.a + static_cast<long>(row0) * p.lda;
    opA.half[1] = opA.half[0] + 64 * p.lda;
    opB.half[0] = p.w0 + e * p.w_expert_stride + static_cast<long>(n0) * p.ldw;
    opB.half[1] = opB.half[0] + 64 * p.ldw;
    mainloop<false, false>(opA, opB, p.K, lds, a_row, b_row, acc);
  } else if (KIND == kDAct) {
    // dA = dyp * Wd[e] : weight is [K = d, N = f], reduction strided
    opA.half[0] = p.a + static_cast<long>(row0) * p.lda;
    opA.half[1] = opA.half[0] + 64 * p.lda;
    opB.half[0] = p.w0 + e * p.w_expert_stride + n0;
    opB.half[1] = opB.half[0] + 64;
    mainloop<false, true>(opA, opB, p.K, lds, a_row, b_row, acc);
  } else {
    // dxp = dG * Wg[e] + dU * Wu[e] : two reduction segments over the columns of [dG | dU]
    opA.half[0] = p.a + static_cast<long>(row0) * p.lda;
    opA.half[1] = opA.half[0] + 64 * p.lda;
    opB.half[0] = p.w0 + e * p.w_expert_stride + n0;
    opB.half[1] = opB.half[0] + 64;
    mainloop<false, true>(opA, opB, p.K, lds, a_row, b_row, acc);
    opA.half[0] += p.K;
    opA.half[1] += p.K;
    opB.half[0] = p.w1 + e * p.w_expert_stride + n0;
    opB.half[1] = opB.half[0] + 64;
    mainloop<false, true>(opA, opB, p.K, lds, a_row, b_row, acc);
  }

#pragma unroll
  for (int ni = 0; ni < 2; ++ni) {
    const int cl = wn * 64 + ni * 32 + (lane & 31);
    if (cl >= ncols) continue;
    const int col = n0 + cl;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int r = wm * 64 + mi * 32 + acc_row(lane, i);
        if (r >= rows) continue;
        const float val = acc[mi][ni][i];
        if (KIND == kDAct) {
          const long gi = static_cast<long>(row0 + r) * p.N + col;
          const float g = bf16_to_f32(p.g[gi]), u = bf16_to_f32(p.u[gi]);
          const float s = sigmoid_fast(g);
          const long o = static_cast<long>(row0 + r) * p.ldo + col;
          p.out0[o] = f32_to_bf16(val * u * (s * (1.0f + g * (1.0f - s))));
          p.out0[o + p.N] = f32_to_bf16(val * (g * s));
        } else {
          p.out0[static_cast<long>(row0 + r) * p.ldo + col] = f32_to_bf16(val);
        }
      }
  }
}

// ============================================================================================
// Weight-gradient kernel: out[e] (M x N) = lhs[rows of e, M]^T * rhs[rows of e, N]
// Output rows below `m_split` go to out0[e], the rest to out1[e] (gate / up share one launch).
// ============================================================================================
struct WgradArgs {
  const bf16_t* lhs; long ld_lhs; int M;
  const bf16_t* rhs; long ld_rhs; int N;
  const int32_t* offsets; int E; int P;
  int tiles_m, tiles_n;
  bf16_t* out0; bf16_t* out1; int m_split;     // out1 rows are (m - m_split)
};

template <int WHICH>   // 0: dW_down, 1: [dW_gate; dW_up] (separate symbols so profiles tell them apart)
__global__ __launch_bounds__(kGemmThreads) void wgrad_kernel(WgradArgs p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int per_e = p.tiles_m * p.tiles_n;
  const int v = xcd_remap(blockIdx.x, per_e * p.E);
  if (v < 0) return;
  const int e = v / per_e, mt = (v % per_e) / p.tiles_n, nt = v % p.tiles_n;
  const int begin = min(max(p.offsets[e], 0), p.P);
  const int end = min(max(p.offsets[e + 1], begin), p.P);
  const int m0 = mt * BM, n0 = nt * BN;
  const int mrows = min(BM, p.M - m0), ncols = min(BN, p.N - n0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

  const int a_row[2] = {wm * 64, wm * 64 + 32};
  const int b_row[2] = {wn * 64, wn * 64 + 32};
  Operand opA, opB;
  opA.ld = p.ld_lhs;
  opA.half[0] = p.lhs + static_cast<long>(begin) * p.ld_lhs + m0;
  opA.half[1] = opA.half[0] + 64;
  opA.valid[0] = min(mrows, 64);
  opA.valid[1] = max(mrows - 64, 0);
  opB.ld = p.ld_rhs;
  opB.half[0] = p.rhs + static_cast<long>(begin) * p.ld_rhs + n0;
  opB.half[1] = opB.half[0] + 64;
  opB.valid[0] = min(ncols, 64);
  opB.valid[1] = max(ncols - 64, 0);
  mainloop<true, true>(opA, opB, end - begin, lds, a_row, b_row, acc);

#pragma unroll
  for (int ni = 0; ni < 2; ++ni) {
    const int cl = wn * 64 + ni * 32 + (lane & 31);
    if (cl >= ncols) continue;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int rl = wm * 64 + mi * 32 + acc_row(lane, i);
        if (rl >= mrows) continue;
        const int m = m0 + rl;
        bf16_t* out = m < p.m_split ? p.out0 + (static_cast<long>(e) * p.m_split + m) * p.N
                                    : p.out1 + (static_cast<long>(e) * (p.M - p.m_split) + (m - p.m_split)) * p.N;
        out[n0 + cl] = f32_to_bf16(acc[mi][ni][i]);
      }
  }
}

// ============================================================================================
// Host side
// ============================================================================================
static int max_row_tiles(int P, int E) { return ceil_div(P, BM) + E; }

struct WsLayout {
  size_t tiles_count, tiles_expert, tiles_row0, dgu, g, u, total;
};
static WsLayout ws_layout(int P, int f, int E, bool need_dgu, bool need_gu) {
  WsLayout w{};
  size_t off = 0;
  w.tiles_count = off; off += 256;
  const size_t t = align_up(static_cast<size_t>(max_row_tiles(P, E)) * sizeof(int32_t), 256);
  w.tiles_expert = off; off += t;
  w.tiles_row0 = off; off += t;
  const size_t pf = align_up(static_cast<size_t>(P) * f * 2, 256);
  w.dgu = off; if (need_dgu) off += 2 * pf;
  w.g = off; if (need_gu) off += pf;
  w.u = off; if (need_gu) off += pf;
  w.total = off + 256;
  return w;
}

size_t ffn_fwd_ws_bytes_bf16(int P, int d, int f, int E) { (void)d; return ws_layout(P, f, E, false, false).total; }
size_t ffn_bwd_ws_bytes_bf16(int P, int d, int f, int E, int have_saved) {
  (void)d;
  return ws_layout(P, f, E, true, !have_saved).total;
}

static RowTiles row_tiles_at(void* ws, const WsLayout& w, int P, int E) {
  char* b = static_cast<char*>(ws);
  RowTiles rt;
  rt.max_tiles = max_row_tiles(P, E);
  rt.count = reinterpret_cast<int32_t*>(b + w.tiles_count);
  rt.expert = reinterpret_cast<int32_t*>(b + w.tiles_expert);
  rt.row0 = reinterpret_cast<int32_t*>(b + w.tiles_row0);
  return rt;
}

static unsigned padded_grid(int tiles) { return static_cast<unsigned>(ceil_div(tiles < 1 ? 1 : tiles, kXcds) * kXcds); }

template <int KIND>
static void launch_row(const RowArgs& p, int P, int E, hipStream_t s) {
  static const char* const names[4] = {"ffn_gate_up", "ffn_down", "ffn_dact", "ffn_dx"};
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&row_grouped_kernel<KIND>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    attr_set = true;
  }
  const unsigned grid = padded_grid(max_row_tiles(P, E) * p.n_tiles_n);
  MOE_LAUNCH(names[KIND], row_grouped_kernel<KIND>, dim3(grid), dim3(kGemmThreads), kLdsBytes, s, p);
}

template <int WHICH>
static void launch_wgrad(const WgradArgs& p, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_kernel<WHICH>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    attr_set = true;
  }
  const unsigned grid = padded_grid(p.tiles_m * p.tiles_n * p.E);
  MOE_LAUNCH(WHICH == 0 ? "wgrad_down" : "wgrad_gate_up", wgrad_kernel<WHICH>, dim3(grid), dim3(kGemmThreads), kLdsBytes, s, p);
}

static void launch_gate_up(const void* xp, const void* wg, const void* wu, int P, int d, int f, int E,
                           const int32_t* offsets, const RowTiles& rt, void* G, void* U, void* act, hipStream_t s) {
  RowArgs p{};
  p.a = static_cast<const bf16_t*>(xp); p.lda = d;
  p.w0 = static_cast<const bf16_t*>(wg); p.w1 = static_cast<const bf16_t*>(wu);
  p.w_expert_stride = static_cast<long>(f) * d; p.ldw = d;
  p.K = d; p.N = f; p.offsets = offsets; p.P = P; p.rt = rt; p.n_tiles_n = ceil_div(f, 64);
  p.out0 = static_cast<bf16_t*>(G); p.out1 = static_cast<bf16_t*>(U); p.out2 = static_cast<bf16_t*>(act); p.ldo = f;
  launch_row<kGateUp>(p, P, E, s);
}

void ffn_fwd_bf16(const FfnFwdArgs& a) {
  const WsLayout w = ws_layout(a.P, a.f, a.E, false, false);
  const RowTiles rt = row_tiles_at(a.ws, w, a.P, a.E);
  MOE_LAUNCH("build_row_tiles", build_row_tiles_kernel, dim3(1), dim3(1024), 0, a.stream, a.offsets, a.E, a.P, rt);
  launch_gate_up(a.xp, a.w_gate, a.w_up, a.P, a.d, a.f, a.E, a.offsets, rt, a.g_save, a.u_save, a.act, a.stream);
  RowArgs p{};
  p.a = static_cast<const bf16_t*>(a.act); p.lda = a.f;
  p.w0 = static_cast<const bf16_t*>(a.w_down); p.w_expert_stride = static_cast<long>(a.d) * a.f; p.ldw = a.f;
  p.K = a.f; p.N = a.d; p.offsets = a.offsets; p.P = a.P; p.rt = rt; p.n_tiles_n = ceil_div(a.d, BN);
  p.out0 = static_cast<bf16_t*>(a.yp); p.ldo = a.d;
  launch_row<kDown>(p, a.P, a.E, a.stream);
}

void ffn_bwd_bf16(const FfnBwdArgs& a) {
  const bool recompute = a.g_save == nullptr;
  const WsLayout w = ws_layout(a.P, a.f, a.E, true, recompute);
  const RowTiles rt = row_tiles_at(a.ws, w, a.P, a.E);
  char* base = static_cast<char*>(a.ws);
  bf16_t* dgu = reinterpret_cast<bf16_t*>(base + w.dgu);       // [P, 2f] = [dG | dU]
  const bf16_t* G = static_cast<const bf16_t*>(a.g_save);
  const bf16_t* U = static_cast<const bf16_t*>(a.u_save);
  MOE_LAUNCH("build_row_tiles", build_row_tiles_kernel, dim3(1), dim3(1024), 0, a.stream, a.offsets, a.E, a.P, rt);
  if (recompute) {
    bf16_t* Gr = reinterpret_cast<bf16_t*>(base + w.g);
    bf16_t* Ur = reinterpret_cast<bf16_t*>(base + w.u);
    launch_gate_up(a.xp, a.w_gate, a.w_up, a.P, a.d, a.f, a.E, a.offsets, rt, Gr, Ur, nullptr, a.stream);
    G = Gr; U = Ur;
  }
  {  // dA = dyp Wd, fused with the SwiGLU derivative -> [dG | dU]
    RowArgs p{};
    p.a = static_cast<const bf16_t*>(a.dyp); p.lda = a.d;
    p.w0 = static_cast<const bf16_t*>(a.w_down); p.w_expert_stride = static_cast<long>(a.d) * a.f; p.ldw = a.f;
    p.K = a.d; p.N = a.f; p.offsets = a.offsets; p.P = a.P; p.rt = rt; p.n_tiles_n = ceil_div(a.f, BN);
    p.out0 = dgu; p.ldo = 2L * a.f; p.g = G; p.u = U;
    launch_row<kDAct>(p, a.P, a.E, a.stream);
  }
  {  // dxp = dG Wg + dU Wu
    RowArgs p{};
    p.a = dgu; p.lda = 2L * a.f;
    p.w0 = static_cast<const bf16_t*>(a.w_gate); p.w1 = static_cast<const bf16_t*>(a.w_up);
    p.w_expert_stride = static_cast<long>(a.f) * a.d; p.ldw = a.d;
    p.K = a.f; p.N = a.d; p.offsets = a.offsets; p.P = a.P; p.rt = rt; p.n_tiles_n = ceil_div(a.d, BN);
    p.out0 = static_cast<bf16_t*>(a.dxp); p.ldo = a.d;
    launch_row<kDX>(p, a.P, a.E, a.stream);
  }
  {  // dWd[e] = dyp^T act
    WgradArgs p{};
    p.lhs = static_cast<const bf16_t*>(a.dyp); p.ld_lhs = a.d; p.M = a.d;
    p.rhs = static_cast<const bf16_t*>(a.act); p.ld_rhs = a.f; p.N = a.f;
    p.offsets = a.offsets; p.E = a.E; p.P = a.P;
    p.tiles_m = ceil_div(a.d, BM); p.tiles_n = ceil_div(a.f, BN);
    p.out0 = static_cast<bf16_t*>(a.dw_down); p.out1 = p.out0; p.m_split = a.d;
    launch_wgrad<0>(p, a.stream);
  }
  {  // [dWg[e]; dWu[e]] = [dG | dU]^T xp
    WgradArgs p{};
    p.lhs = dgu; p.ld_lhs = 2L * a.f; p.M = 2 * a.f;
    p.rhs = static_cast<const bf16_t*>(a.xp); p.ld_rhs = a.d; p.N = a.d;
    p.offsets = a.offsets; p.E = a.E; p.P = a.P;
    p.tiles_m = ceil_div(2 * a.f, BM); p.tiles_n = ceil_div(a.d, BN);
    p.out0 = static_cast<bf16_t*>(a.dw_gate); p.out1 = static_cast<bf16_t*>(a.dw_up); p.m_split = a.f;
    launch_wgrad<1>(p, a.stream);
  }
}

}  // namespace moe
