// bf16 MFMA grouped GEMMs of the SwiGLU expert FFN, forward and backward
// (Sec. 3.2.5 SwiGLU among the efficient kernels; App. B.6 stacked expert-major weights).
//
// One kernel skeleton serves all nine matrix products of the layer:
//   * a BM x BN output tile per 256-thread workgroup: 2 x 2 wavefronts, each owning a
//     WM x WN sub-tile made of 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16, fp32
//     accumulators kept in registers for the whole reduction);
//   * the reduction dimension is walked in BK-wide slabs, double-buffered in LDS; the
//     global loads of slab i+1 are issued before the MFMAs of slab i, and one barrier
//     per slab separates writers from readers;
//   * an operand whose reduction index is contiguous in memory is staged as
//     [rows][BK] and read with 16-byte LDS loads; an operand whose reduction index is the
//     slow axis in memory (the weight in the two backward-data products, both operands of
//     the weight-gradient products) is staged untransposed as [BK][rows] and read with
//     the transposing LDS load ds_read_b64_tr_b16, which hands every lane four
//     consecutive reduction elements of its own row.  Both layouts are XOR-swizzled so
//     that each group of lanes the LDS serves in one cycle covers all 64 banks.
// Row-grouped products (rows of the activation matrix belong to experts) take their
// (expert, row-tile) list from a small schedule built on the device from `offsets`, so no
// host synchronisation is needed; weight-gradient products are grouped along the
// reduction dimension instead and have a host-known grid.
// Workgroup ids are remapped so that consecutive tiles -- which share an expert's weights
// -- run on the same XCD and hit its L2.
#include <cstdlib>
#include "moe_common.h"

namespace moe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kGemmThreads = 256;
constexpr int kXcds = 8;

// ---- tile shapes ------------------------------------------------------------------------------
template <int BM_, int BN_, int BK_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_;
  static constexpr int WM = BM / 2, WN = BN / 2;          // 2 x 2 waves
  static constexpr int MI = WM / 32, NI = WN / 32;        // MFMA tiles per wave
  static constexpr int kABytes = BM * BK * 2, kBBytes = BN * BK * 2;
  static constexpr int kLdsBytes = 2 * (kABytes + kBBytes);
};

// One operand tile of ROWS rows: element (row, k).  Two halves of ROWS/2 rows with their own
// base so that the gate and the up projection can share one tile.
//   k-contiguous: half[h] + row * ld + k          k-strided: half[h] + k * ld + row
struct Operand {
  const bf16_t* half[2];
  long ld;
  int valid[2];      // rows of each half that exist (others read as zero); multiples of 8 if k-strided
};

// ---- LDS layouts ---------------------------------------------------------------------------------
// k-contiguous operand: [ROWS][BK]; the 16-byte pieces of a row are XORed with the index of the
// 256-byte line the row lives in, so 16 consecutive rows read at one piece index hit 64 banks.
template <int BK>
__device__ __forceinline__ int kc_off(int row, int piece) {
  constexpr int PPR = BK / 8;                    // pieces per row
  constexpr int RPL = 256 / (BK * 2);            // rows per 256-byte line
  return row * (BK * 2) + ((piece ^ ((row / RPL) & (PPR - 1))) << 4);
}
// k-strided operand: [BK][ROWS]; the 64-byte chunks of a k-row are XORed with k & 3, so the four
// k-rows a transposing read touches lie in different banks.
template <int ROWS>
__device__ __forceinline__ int ks_off(int k, int piece) {
  return k * (ROWS * 2) + (((((piece >> 2) ^ (k & 3)) << 2) | (piece & 3)) << 4);
}

// ---- global -> register -> LDS staging -------------------------------------------------------------
template <bool KS, int ROWS, int BK> struct Stager;

template <int ROWS, int BK> struct Stager<false, ROWS, BK> {
  static constexpr int PPR = BK / 8;
  static constexpr int N = ROWS * PPR / kGemmThreads;        // 16-byte loads per thread
  static constexpr int RSTEP = kGemmThreads / PPR;           // rows covered by one pass
  const bf16_t* ptr[N];
  int lds_off[N];
  bool ok[N];
  int kpiece;
  uint4 v[N];
  __device__ __forceinline__ void init(const Operand& op, int tid) {
    kpiece = tid % PPR;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int row = tid / PPR + RSTEP * i;
      const bool upper = (RSTEP * i) >= ROWS / 2;            // RSTEP divides ROWS/2: compile-time per i
      const int rh = row - (upper ? ROWS / 2 : 0);
      ok[i] = rh < (upper ? op.valid[1] : op.valid[0]);
      ptr[i] = (upper ? op.half[1] : op.half[0]) + static_cast<long>(rh) * op.ld + kpiece * 8;
      lds_off[i] = kc_off<BK>(row, kpiece);
    }
  }
  __device__ __forceinline__ void load(int k0, int K) {
    const bool k_ok = k0 + kpiece * 8 < K;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      v[i] = make_uint4(0, 0, 0, 0);
      if (ok[i] && k_ok) v[i] = *reinterpret_cast<const uint4*>(ptr[i] + k0);
    }
  }
  __device__ __forceinline__ void store(char* tile) const {
#pragma unroll
    for (int i = 0; i < N; ++i) *reinterpret_cast<uint4*>(tile + lds_off[i]) = v[i];
  }
};

template <int ROWS, int BK> struct Stager<true, ROWS, BK> {
  static constexpr int PPK = ROWS / 8;                       // 16-byte pieces per k-row
  static constexpr int N = BK * PPK / kGemmThreads;
  static constexpr int KSTEP = kGemmThreads / PPK;           // k-rows covered by one pass
  const bf16_t* ptr;
  long ld;
  bool ok;
  int krow, piece;
  uint4 v[N];
  __device__ __forceinline__ void init(const Operand& op, int tid) {
    piece = tid % PPK;
    krow = tid / PPK;
    const int row = piece * 8;
    const bool upper = row >= ROWS / 2;
    const int rh = row - (upper ? ROWS / 2 : 0);
    ok = rh < (upper ? op.valid[1] : op.valid[0]);
    ld = op.ld;
    ptr = (upper ? op.half[1] : op.half[0]) + rh + static_cast<long>(krow) * ld;
  }
  __device__ __forceinline__ void load(int k0, int K) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      v[i] = make_uint4(0, 0, 0, 0);
      if (ok && k0 + krow + KSTEP * i < K) v[i] = *reinterpret_cast<const uint4*>(ptr + static_cast<long>(k0 + KSTEP * i) * ld);
    }
  }
  __device__ __forceinline__ void store(char* tile) const {
#pragma unroll
    for (int i = 0; i < N; ++i) *reinterpret_cast<uint4*>(tile + ks_off<ROWS>(krow + KSTEP * i, piece)) = v[i];
  }
};

// ---- MFMA operand fragments ----------------------------------------------------------------------------
// Fragment = 32 rows x 16 k: lane l holds row l%32, k = 8*(l/32) .. +7 of the 16-wide step kk.
template <bool KS, int ROWS, int BK>
__device__ __forceinline__ bf16x8 read_frag(const char* tile, int row_base, int kk, int lane) {
  if constexpr (!KS) {
    return *reinterpret_cast<const bf16x8*>(tile + kc_off<BK>(row_base + (lane & 31), 2 * kk + (lane >> 5)));
  } else {
    // Transposing read: within each group of 16 lanes, lane i receives element i%4 of the 8-byte
    // rows addressed by lanes i/4, i/4+4, i/4+8, i/4+12.  Lane s therefore addresses k-row s/4 at
    // columns 4*(s%4)..+3 of its group's 16 columns, and ends up with 4 consecutive k of column s.
    const int s = lane & 15;
    const int col = row_base + 16 * ((lane >> 4) & 1) + 4 * (s & 3);     // multiple of 4
    const int k = kk * 16 + 8 * (lane >> 5) + (s >> 2);
    const int piece = col >> 3, sub = (col & 4) * 2;                       // 8-byte half of the piece
    typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        (lds_bf16x4*)(tile + ks_off<ROWS>(k, piece) + sub));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        (lds_bf16x4*)(tile + ks_off<ROWS>(k + 4, piece) + sub));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }
}

// acc += sum over segments of A_s(BM x K) * B_s(BN x K)^T for this wave's sub-tile (segments differ
// only in their base pointers), operands staged
// through LDS.  a_row[mi] / b_row[ni]: first tile row of the wave's mi-th / ni-th 32-row fragment.
// Every slab ends with a barrier, so the next segment can start writing LDS right away.
template <class T, bool A_KS, bool B_KS>
__device__ __forceinline__ void mainloop(const Operand* opA, const Operand* opB, int nseg, int K, char* lds,
                                         const int (&a_row)[T::MI], const int (&b_row)[T::NI],
                                         f32x16 (&acc)[T::MI][T::NI]) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int ktiles = (K + T::BK - 1) / T::BK;
  if (ktiles <= 0) return;
  char* const tA = lds;                              // two A buffers, then two B buffers
  char* const tB = lds + 2 * T::kABytes;
#pragma nounroll
  for (int seg = 0; seg < nseg; ++seg) {
    Stager<A_KS, T::BM, T::BK> sa;
    Stager<B_KS, T::BN, T::BK> sb;
    {   // pick the segment's operands field by field: no dynamically indexed copies
      Operand oa, ob;
      oa.half[0] = seg ? opA[1].half[0] : opA[0].half[0];
      oa.half[1] = seg ? opA[1].half[1] : opA[0].half[1];
      oa.ld = opA[0].ld;
      oa.valid[0] = opA[0].valid[0];
      oa.valid[1] = opA[0].valid[1];
      ob.half[0] = seg ? opB[1].half[0] : opB[0].half[0];
      ob.half[1] = seg ? opB[1].half[1] : opB[0].half[1];
      ob.ld = opB[0].ld;
      ob.valid[0] = opB[0].valid[0];
      ob.valid[1] = opB[0].valid[1];
      sa.init(oa, tid);
      sb.init(ob, tid);
    }
    sa.load(0, K);
    sb.load(0, K);
    sa.store(tA);
    sb.store(tB);
    __syncthreads();
#pragma nounroll
    for (int kt = 0; kt < ktiles; ++kt) {
      const int cur = kt & 1;
      const bool more = kt + 1 < ktiles;
      if (more) {
        sa.load((kt + 1) * T::BK, K);
        sb.load((kt + 1) * T::BK, K);
      }
      const char* bufA = tA + cur * T::kABytes;
      const char* bufB = tB + cur * T::kBBytes;
#pragma unroll
      for (int kk = 0; kk < T::BK / 16; ++kk) {
        bf16x8 a[T::MI], b[T::NI];
#pragma unroll
        for (int i = 0; i < T::MI; ++i) a[i] = read_frag<A_KS, T::BM, T::BK>(bufA, a_row[i], kk, lane);
#pragma unroll
        for (int i = 0; i < T::NI; ++i) b[i] = read_frag<B_KS, T::BN, T::BK>(bufB, b_row[i], kk, lane);
#pragma unroll
        for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < T::NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
      }
      if (more) {
        sa.store(tA + (cur ^ 1) * T::kABytes);
        sb.store(tB + (cur ^ 1) * T::kBBytes);
      }
      __syncthreads();
    }
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
                                                                int bm, RowTiles rt) {
  __shared__ int32_t scan[kMaxExperts];
  const int e = threadIdx.x;
  int begin = 0, end = 0, nt = 0;
  if (e < E) {
    begin = min(max(offsets[e], 0), P);
    end = min(max(offsets[e + 1], begin), P);
    nt = (end - begin + bm - 1) / bm;
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
    rt.row0[first + i] = begin + i * bm;
  }
  if (e == 1023) rt.count[0] = min(scan[1023], rt.max_tiles);
}

// workgroup id -> virtual tile id such that consecutive virtual ids share an XCD
__device__ __forceinline__ int xcd_remap(int b, int total) {
  const int per = (total + kXcds - 1) / kXcds;
  const int v = (b % kXcds) * per + b / kXcds;
  return (b / kXcds < per && v < total) ? v : -1;
}

// element i (0..15) of a 32x32 MFMA tile held by `lane`: row 8*(i/4) + 4*(lane/32) + i%4, col lane%32
__device__ __forceinline__ int acc_row(int lane, int i) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

template <class T>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[T::MI][T::NI]) {
#pragma unroll
  for (int i = 0; i < T::MI; ++i)
#pragma unroll
    for (int j = 0; j < T::NI; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;
}

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
  bf16_t* out0;            // kGateUp: G (may be null)   kDown/kDX: output     kDAct: [dG | dU]
  bf16_t* out1;            // kGateUp: U (may be null)
  bf16_t* out2;            // kGateUp: act (may be null)
  long ldo;
  const bf16_t* g;         // kDAct: saved pre-activations
  const bf16_t* u;
};

template <int KIND, class T>
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void row_grouped_kernel(RowArgs p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int BM = T::BM, BN = T::BN, WM = T::WM, WN = T::WN, MI = T::MI, NI = T::NI;
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

  f32x16 acc[MI][NI];
  zero_acc<T>(acc);

  int a_row[MI];
#pragma unroll
  for (int i = 0; i < MI; ++i) a_row[i] = wm * WM + i * 32;
  Operand opsA[2], opsB[2];
  Operand& opA = opsA[0];
  Operand& opB = opsB[0];
  opA.ld = p.lda;
  opA.valid[0] = min(rows, BM / 2);
  opA.valid[1] = max(rows - BM / 2, 0);
  opA.half[0] = p.a + static_cast<long>(row0) * p.lda;
  opA.half[1] = opA.half[0] + (BM / 2) * p.lda;
  opB.ld = p.ldw;

  if constexpr (KIND == kGateUp) {
    // tile columns: BN/2 gate columns n0.. and the matching BN/2 up columns; each wave gets the
    // same gate and up columns so the SwiGLU product needs no exchange between lanes
    constexpr int HN = BN / 2, HW = WN / 2, HI = NI / 2;
    const int n0 = nt * HN;
    const int ncols = min(HN, p.N - n0);
    int b_row[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) b_row[i] = (i < HI ? 0 : HN) + wn * HW + (i % HI) * 32;
    opB.half[0] = p.w0 + e * p.w_expert_stride + static_cast<long>(n0) * p.ldw;
    opB.half[1] = p.w1 + e * p.w_expert_stride + static_cast<long>(n0) * p.ldw;
    opB.valid[0] = opB.valid[1] = ncols;
    mainloop<T, false, false>(opsA, opsB, 1, p.K, lds, a_row, b_row, acc);
#pragma unroll
    for (int ni = 0; ni < HI; ++ni) {
      const int cl = wn * HW + ni * 32 + (lane & 31);
      if (cl >= ncols) continue;
      const int col = n0 + cl;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = wm * WM + mi * 32 + acc_row(lane, i);
          if (r < rows) {
            const float g = acc[mi][ni][i], u = acc[mi][ni + HI][i];
            const long o = static_cast<long>(row0 + r) * p.ldo + col;
            if (p.out0) p.out0[o] = f32_to_bf16(g);
            if (p.out1) p.out1[o] = f32_to_bf16(u);
            if (p.out2) p.out2[o] = f32_to_bf16(g * sigmoid_fast(g) * u);
          }
        }
    }
    return;
  } else {
    const int n0 = nt * BN;
    const int ncols = min(BN, p.N - n0);
    int b_row[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) b_row[i] = wn * WN + i * 32;
    opB.valid[0] = min(ncols, BN / 2);
    opB.valid[1] = max(ncols - BN / 2, 0);
    if constexpr (KIND == kDown) {
      // yp = act * Wd[e]^T : weight rows are output columns, reduction contiguous
      opB.half[0] = p.w0 + e * p.w_expert_stride + static_cast<long>(n0) * p.ldw;
      opB.half[1] = opB.half[0] + (BN / 2) * p.ldw;
      mainloop<T, false, false>(opsA, opsB, 1, p.K, lds, a_row, b_row, acc);
    } else if constexpr (KIND == kDAct) {
      // dA = dyp * Wd[e] : weight is [K = d, N = f], reduction strided
      opB.half[0] = p.w0 + e * p.w_expert_stride + n0;
      opB.half[1] = opB.half[0] + BN / 2;
      mainloop<T, false, true>(opsA, opsB, 1, p.K, lds, a_row, b_row, acc);
    } else {
      // dxp = dG * Wg[e] + dU * Wu[e] : two reduction segments over the columns of [dG | dU]
      opB.half[0] = p.w0 + e * p.w_expert_stride + n0;
      opB.half[1] = opB.half[0] + BN / 2;
      opsA[1] = opA;
      opsA[1].half[0] += p.K;
      opsA[1].half[1] += p.K;
      opsB[1] = opB;
      opsB[1].half[0] = p.w1 + e * p.w_expert_stride + n0;
      opsB[1].half[1] = opsB[1].half[0] + BN / 2;
      mainloop<T, false, true>(opsA, opsB, 2, p.K, lds, a_row, b_row, acc);
    }

#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int cl = wn * WN + ni * 32 + (lane & 31);
      if (cl >= ncols) continue;
      const int col = n0 + cl;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = wm * WM + mi * 32 + acc_row(lane, i);
          if (r >= rows) continue;
          const float val = acc[mi][ni][i];
          if constexpr (KIND == kDAct) {
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

template <int WHICH, class T>   // WHICH 0: dW_down, 1: [dW_gate; dW_up] (separate symbols so profiles tell them apart)
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void wgrad_kernel(WgradArgs p) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int BM = T::BM, BN = T::BN, WM = T::WM, WN = T::WN, MI = T::MI, NI = T::NI;
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

  f32x16 acc[MI][NI];
  zero_acc<T>(acc);
  int a_row[MI], b_row[NI];
#pragma unroll
  for (int i = 0; i < MI; ++i) a_row[i] = wm * WM + i * 32;
#pragma unroll
  for (int i = 0; i < NI; ++i) b_row[i] = wn * WN + i * 32;
  Operand opA, opB;
  opA.ld = p.ld_lhs;
  opA.half[0] = p.lhs + static_cast<long>(begin) * p.ld_lhs + m0;
  opA.half[1] = opA.half[0] + BM / 2;
  opA.valid[0] = min(mrows, BM / 2);
  opA.valid[1] = max(mrows - BM / 2, 0);
  opB.ld = p.ld_rhs;
  opB.half[0] = p.rhs + static_cast<long>(begin) * p.ld_rhs + n0;
  opB.half[1] = opB.half[0] + BN / 2;
  opB.valid[0] = min(ncols, BN / 2);
  opB.valid[1] = max(ncols - BN / 2, 0);
  mainloop<T, true, true>(&opA, &opB, 1, end - begin, lds, a_row, b_row, acc);

#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int cl = wn * WN + ni * 32 + (lane & 31);
    if (cl >= ncols) continue;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int rl = wm * WM + mi * 32 + acc_row(lane, i);
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
// Tile shapes in use.  Row-grouped products keep the row (token) side at 128 so that experts
// with a few hundred rows waste little; the weight side is 256 wide.
typedef Tile<128, 128, 64> TileRowSmall;
typedef Tile<128, 256, 32> TileRow;
typedef Tile<128, 256, 32> TileWgrad;

static int tile_choice() {           // 0 = default; MOE_GEMM_TILE=1 selects the 128x128x64 variant
  static int choice = -1;
  if (choice < 0) {
    const char* s = getenv("MOE_GEMM_TILE");
    choice = s ? atoi(s) : 0;
  }
  return choice;
}

constexpr int kRowBM = 128;          // both row-grouped tile types use 128 rows
static int max_row_tiles(int P, int E) { return ceil_div(P, kRowBM) + E; }

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

template <int KIND, class T>
static void launch_row_t(RowArgs p, int P, int E, hipStream_t s) {
  static const char* const names[4] = {"ffn_gate_up", "ffn_down", "ffn_dact", "ffn_dx"};
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&row_grouped_kernel<KIND, T>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
    attr_set = true;
  }
  p.n_tiles_n = ceil_div(p.N, KIND == kGateUp ? T::BN / 2 : T::BN);
  const unsigned grid = padded_grid(max_row_tiles(P, E) * p.n_tiles_n);
  MOE_LAUNCH(names[KIND], (row_grouped_kernel<KIND, T>), dim3(grid), dim3(kGemmThreads), T::kLdsBytes, s, p);
}

template <int KIND>
static void launch_row(const RowArgs& p, int P, int E, hipStream_t s) {
  if (tile_choice() == 1) launch_row_t<KIND, TileRowSmall>(p, P, E, s);
  else launch_row_t<KIND, TileRow>(p, P, E, s);
}

template <int WHICH, class T>
static void launch_wgrad_t(WgradArgs p, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_kernel<WHICH, T>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
    attr_set = true;
  }
  p.tiles_m = ceil_div(p.M, T::BM);
  p.tiles_n = ceil_div(p.N, T::BN);
  const unsigned grid = padded_grid(p.tiles_m * p.tiles_n * p.E);
  MOE_LAUNCH(WHICH == 0 ? "wgrad_down" : "wgrad_gate_up", (wgrad_kernel<WHICH, T>), dim3(grid), dim3(kGemmThreads),
             T::kLdsBytes, s, p);
}

template <int WHICH>
static void launch_wgrad(const WgradArgs& p, hipStream_t s) {
  if (tile_choice() == 1) launch_wgrad_t<WHICH, TileRowSmall>(p, s);
  else launch_wgrad_t<WHICH, TileWgrad>(p, s);
}

static void launch_gate_up(const void* xp, const void* wg, const void* wu, int P, int d, int f, int E,
                           const int32_t* offsets, const RowTiles& rt, void* G, void* U, void* act, hipStream_t s) {
  RowArgs p{};
  p.a = static_cast<const bf16_t*>(xp); p.lda = d;
  p.w0 = static_cast<const bf16_t*>(wg); p.w1 = static_cast<const bf16_t*>(wu);
  p.w_expert_stride = static_cast<long>(f) * d; p.ldw = d;
  p.K = d; p.N = f; p.offsets = offsets; p.P = P; p.rt = rt;
  p.out0 = static_cast<bf16_t*>(G); p.out1 = static_cast<bf16_t*>(U); p.out2 = static_cast<bf16_t*>(act); p.ldo = f;
  launch_row<kGateUp>(p, P, E, s);
}

void ffn_fwd_bf16(const FfnFwdArgs& a) {
  const WsLayout w = ws_layout(a.P, a.f, a.E, false, false);
  const RowTiles rt = row_tiles_at(a.ws, w, a.P, a.E);
  MOE_LAUNCH("build_row_tiles", build_row_tiles_kernel, dim3(1), dim3(1024), 0, a.stream, a.offsets, a.E, a.P, kRowBM, rt);
  launch_gate_up(a.xp, a.w_gate, a.w_up, a.P, a.d, a.f, a.E, a.offsets, rt, a.g_save, a.u_save, a.act, a.stream);
  RowArgs p{};
  p.a = static_cast<const bf16_t*>(a.act); p.lda = a.f;
  p.w0 = static_cast<const bf16_t*>(a.w_down); p.w_expert_stride = static_cast<long>(a.d) * a.f; p.ldw = a.f;
  p.K = a.f; p.N = a.d; p.offsets = a.offsets; p.P = a.P; p.rt = rt;
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
  MOE_LAUNCH("build_row_tiles", build_row_tiles_kernel, dim3(1), dim3(1024), 0, a.stream, a.offsets, a.E, a.P, kRowBM, rt);
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
    p.K = a.d; p.N = a.f; p.offsets = a.offsets; p.P = a.P; p.rt = rt;
    p.out0 = dgu; p.ldo = 2L * a.f; p.g = G; p.u = U;
    launch_row<kDAct>(p, a.P, a.E, a.stream);
  }
  {  // dxp = dG Wg + dU Wu
    RowArgs p{};
    p.a = dgu; p.lda = 2L * a.f;
    p.w0 = static_cast<const bf16_t*>(a.w_gate); p.w1 = static_cast<const bf16_t*>(a.w_up);
    p.w_expert_stride = static_cast<long>(a.f) * a.d; p.ldw = a.d;
    p.K = a.f; p.N = a.d; p.offsets = a.offsets; p.P = a.P; p.rt = rt;
    p.out0 = static_cast<bf16_t*>(a.dxp); p.ldo = a.d;
    launch_row<kDX>(p, a.P, a.E, a.stream);
  }
  {  // dWd[e] = dyp^T act
    WgradArgs p{};
    p.lhs = static_cast<const bf16_t*>(a.dyp); p.ld_lhs = a.d; p.M = a.d;
    p.rhs = static_cast<const bf16_t*>(a.act); p.ld_rhs = a.f; p.N = a.f;
    p.offsets = a.offsets; p.E = a.E; p.P = a.P;
    p.out0 = static_cast<bf16_t*>(a.dw_down); p.out1 = p.out0; p.m_split = a.d;
    launch_wgrad<0>(p, a.stream);
  }
  {  // [dWg[e]; dWu[e]] = [dG | dU]^T xp
    WgradArgs p{};
    p.lhs = dgu; p.ld_lhs = 2L * a.f; p.M = 2 * a.f;
    p.rhs = static_cast<const bf16_t*>(a.xp); p.ld_rhs = a.d; p.N = a.d;
    p.offsets = a.offsets; p.E = a.E; p.P = a.P;
    p.out0 = static_cast<bf16_t*>(a.dw_gate); p.out1 = static_cast<bf16_t*>(a.dw_up); p.m_split = a.f;
    launch_wgrad<1>(p, a.stream);
  }
}

}  // namespace moe
