// bf16 MFMA grouped GEMMs of the SwiGLU expert FFN, forward and backward
// (Sec. 3.2.5 SwiGLU among the efficient kernels; App. B.6 stacked expert-major weights).
//
// One kernel skeleton serves all nine matrix products of the layer:
//   * a BM x BN output tile per 256-thread workgroup: 2 x 2 wavefronts, each owning a
//     WM x WN sub-tile made of 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16, fp32
//     accumulators kept in registers for the whole reduction);
//   * the reduction dimension is walked in BK-wide slabs through a 3-stage LDS ring that is
//     filled by direct global->LDS loads (no staging registers); two to three slabs are in
//     flight behind the one being multiplied, the MFMA operands are double-buffered in
//     registers one reduction step ahead, and one barrier per slab separates writers from
//     readers;
//   * results leave through LDS as well, so that all global stores (and the loads of the
//     saved pre-activations in the fused SwiGLU derivative) are 16 bytes per lane and
//     contiguous along rows;
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

constexpr int kXcds = 8;

// ---- tile shapes ------------------------------------------------------------------------------
template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int STAGES_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_;
  static constexpr int WGM = WGM_, WGN = WGN_;            // grid of wavefronts over the tile
  static constexpr int kWaves = WGM * WGN, kThreads = 64 * kWaves;
  static constexpr int WM = BM / WGM, WN = BN / WGN;      // sub-tile of one wavefront
  static constexpr int MI = WM / 32, NI = WN / 32;        // MFMA tiles per wave
  static constexpr int kABytes = BM * BK * 2, kBBytes = BN * BK * 2;
  static constexpr int kStageBytes = kABytes + kBBytes;
  static constexpr int kStages = STAGES_;                 // LDS ring: one slab being read, the others in flight
  static constexpr int kLdsBytes = kStages * kStageBytes;
  static constexpr int kBlocksPerCu = 2 * kLdsBytes <= 160 * 1024 ? 2 : 1;   // by LDS capacity
  static constexpr int kWavesPerSimd = kBlocksPerCu * kWaves / 4;
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
template <bool KS, int ROWS, int BK, int THREADS> struct Stager;

template <int ROWS, int BK, int THREADS> struct Stager<false, ROWS, BK, THREADS> {
  static constexpr int PPR = BK / 8;
  static constexpr int N = ROWS * PPR / THREADS;             // 16-byte loads per thread
  static constexpr int RSTEP = THREADS / PPR;                // rows covered by one pass
  static_assert(N >= 1 && (ROWS / 2) % RSTEP == 0, "tile too small for this many threads");
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

template <int ROWS, int BK, int THREADS> struct Stager<true, ROWS, BK, THREADS> {
  static constexpr int PPK = ROWS / 8;                       // 16-byte pieces per k-row
  static constexpr int N = BK * PPK / THREADS;
  static constexpr int KSTEP = THREADS / PPK;                // k-rows covered by one pass
  static_assert(N >= 1, "tile too small for this many threads");
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

// ---- global -> LDS without passing through registers -----------------------------------------------
// One wave instruction (global_load_lds_dwordx4) moves 64 x 16 bytes into 1 KiB of consecutive LDS;
// the swizzles above are applied on the global side: each lane fetches the piece that belongs in its
// LDS slot.  Rows that do not exist are redirected to the tile's first row: they only feed output
// rows / columns that are never stored.  The reduction range is NOT checked here, so this path is
// used for full slabs only; a partial last slab goes through the register Stager, which zero-fills.
template <bool KS, int ROWS, int BK, int WAVES> struct Dma {
  static constexpr int CHUNKS = ROWS * BK * 2 / 1024;
  static constexpr int N = CHUNKS / WAVES;                   // chunks per wave
  static_assert(N >= 1 && CHUNKS % WAVES == 0, "tile too small for this many waves");
  const bf16_t* ptr[N];
  long step;                                                 // elements per slab
  __device__ __forceinline__ void init(const Operand& op, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = wave * N + i;
      if constexpr (!KS) {
        constexpr int PPR = BK / 8, RPC = 1024 / (BK * 2), RPL = 256 / (BK * 2);
        const int row = c * RPC + lane / PPR;
        const int piece = (lane % PPR) ^ ((row / RPL) & (PPR - 1));
        const bool upper = row >= ROWS / 2;
        const int rh = row - (upper ? ROWS / 2 : 0);
        const bool ok = rh < (upper ? op.valid[1] : op.valid[0]);
        const bf16_t* base = ok ? (upper ? op.half[1] : op.half[0]) + static_cast<long>(rh) * op.ld : op.half[0];
        ptr[i] = base + piece * 8;
      } else {
        constexpr int PPK = ROWS / 8, KPC = 1024 / (ROWS * 2);
        const int k = c * KPC + lane / PPK;
        const int phys = lane % PPK;
        const int piece = ((((phys >> 2) ^ (k & 3)) << 2) | (phys & 3));
        const int col = piece * 8;
        const bool upper = col >= ROWS / 2;
        const int ch = col - (upper ? ROWS / 2 : 0);
        const bool ok = ch < (upper ? op.valid[1] : op.valid[0]);
        ptr[i] = (ok ? (upper ? op.half[1] : op.half[0]) + ch : op.half[0]) + static_cast<long>(k) * op.ld;
      }
    }
    step = KS ? static_cast<long>(BK) * op.ld : BK;
  }
  // enqueue this wave's share of slab `slab` into the operand tile at `tile` (LDS)
  __device__ __forceinline__ void issue(int slab, char* tile, int wave) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(ptr[i] + slab * step),
          (__attribute__((address_space(3))) void*)(tile + (wave * N + i) * 1024), 16, 0, 0);
    }
  }
};

// s_waitcnt that waits only for the vector-memory counter to drop to n (gfx9 encoding:
// vmcnt = imm[3:0] | imm[15:14] << 4, expcnt = imm[6:4], lgkmcnt = imm[11:8])
template <int n> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14));
}

// s_waitcnt that waits only for the LDS / scalar-memory counter to reach zero
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14)); }

// the MFMA operands of one 16-wide reduction step for this wave's sub-tile
template <class T> struct Frags {
  bf16x8 a[T::MI];
  bf16x8 b[T::NI];
};
// mi_n / ni_n: how many of the wave's 32-row / 32-column fragments hold at least one row / column
// that exists (wave-uniform).  Fragments beyond them are neither read nor multiplied, so a tile
// that sticks out of its expert's row segment costs MFMA time only for the rows it really has.
template <class T, bool A_KS, bool B_KS>
__device__ __forceinline__ void load_frags(Frags<T>& f, const char* bufA, const char* bufB, int kk,
                                           const int (&a_row)[T::MI], const int (&b_row)[T::NI], int lane,
                                           int mi_n, int ni_n) {
#pragma unroll
  for (int i = 0; i < T::MI; ++i)
    if (i < mi_n) f.a[i] = read_frag<A_KS, T::BM, T::BK>(bufA, a_row[i], kk, lane);
#pragma unroll
  for (int i = 0; i < T::NI; ++i)
    if (i < ni_n) f.b[i] = read_frag<B_KS, T::BN, T::BK>(bufB, b_row[i], kk, lane);
}
template <class T>
__device__ __forceinline__ void mma(const Frags<T>& f, f32x16 (&acc)[T::MI][T::NI], int mi_n, int ni_n) {
#pragma unroll
  for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < T::NI; ++ni)
      if (mi < mi_n && ni < ni_n)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[mi], f.b[ni], acc[mi][ni], 0, 0, 0);
}

// wait until at most `slabs` slabs' worth of this wave's direct loads are still in flight
template <int L, int MAXS>
__device__ __forceinline__ void wait_slabs_in_flight(int slabs) {
  if constexpr (MAXS == 0) {
    wait_vmcnt<0>();
  } else {
    if (slabs >= MAXS) wait_vmcnt<MAXS * L>();
    else wait_slabs_in_flight<L, MAXS - 1>(slabs);
  }
}

// acc += sum over segments of A_s(BM x K) * B_s(BN x K)^T for this wave's sub-tile (segments differ
// only in their base pointers).  a_row[mi] / b_row[ni]: first tile row of the wave's mi-th / ni-th
// 32-row fragment.
//
// Full slabs stream through an S-stage LDS ring filled by direct global->LDS loads, and the MFMA
// operands are double-buffered in registers, so that every LDS read is issued one reduction step
// ahead of the MFMAs that consume it.  Per slab kt:
//     read step 1.. of slab kt (into the other register set) | MFMAs of the steps already loaded
//     wait: own LDS reads of slab kt complete, own loads of slab kt+1 landed
//     barrier: slab kt+1 is visible to all, and nobody reads the stage of slab kt any more
//     refill that stage with slab kt+S; read step 0 of slab kt+1 | MFMAs of the last step of slab kt
// so up to S-1 slabs are in flight behind the slab being multiplied: the global-memory latency a
// workgroup can hide is (S-1) slabs of MFMA time.
template <class T, bool A_KS, bool B_KS>
__device__ __forceinline__ void mainloop(const Operand* opA, const Operand* opB, int nseg, int K, char* lds,
                                         const int (&a_row)[T::MI], const int (&b_row)[T::NI], int mi_n, int ni_n,
                                         int rot, f32x16 (&acc)[T::MI][T::NI]) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS destinations stay scalar
  if (K <= 0) return;
  const int nfull = K / T::BK;
  const int tail = K - nfull * T::BK;
  typedef Dma<A_KS, T::BM, T::BK, T::kWaves> DmaA;
  typedef Dma<B_KS, T::BN, T::BK, T::kWaves> DmaB;
  constexpr int L = DmaA::N + DmaB::N;                 // loads per thread per slab
  constexpr int S = T::kStages;
  constexpr int STEPS = T::BK / 16;                    // reduction steps per slab (even)
  static_assert((S - 1) * L < 64, "vmcnt is a 6-bit counter");
#pragma nounroll
  for (int seg = 0; seg < nseg; ++seg) {
    Operand oa, ob;                                    // picked field by field: no dynamically indexed copies
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
    if (nfull > 0) {
      DmaA da;
      DmaB db;
      da.init(oa, wave, lane);
      db.init(ob, wave, lane);
      // The full slabs are visited in rotated order, starting at slab `rot`: workgroups of
      // different experts then stream different offsets of their rows at the same time, which
      // spreads the traffic over the memory channels instead of camping on a few of them.
      int next_slab = rot % nfull;                     // next slab to request
#pragma unroll
      for (int s0 = 0; s0 < S; ++s0)
        if (s0 < nfull) {
          da.issue(next_slab, lds + s0 * T::kStageBytes, wave);
          db.issue(next_slab, lds + s0 * T::kStageBytes + T::kABytes, wave);
          next_slab = next_slab + 1 == nfull ? 0 : next_slab + 1;
        }
      wait_slabs_in_flight<L, S - 1>(nfull - 1);       // slab 0 has landed
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      Frags<T> f0, f1;                                 // even / odd reduction steps
      load_frags<T, A_KS, B_KS>(f0, lds, lds + T::kABytes, 0, a_row, b_row, lane, mi_n, ni_n);
      int stage = 0;
#pragma nounroll
      for (int kt = 0; kt < nfull; ++kt) {
        char* buf = lds + stage * T::kStageBytes;
#pragma unroll
        for (int kk = 0; kk + 2 < STEPS; kk += 2) {    // all but the last two steps of the slab
          load_frags<T, A_KS, B_KS>(f1, buf, buf + T::kABytes, kk + 1, a_row, b_row, lane, mi_n, ni_n);
          mma<T>(f0, acc, mi_n, ni_n);
          load_frags<T, A_KS, B_KS>(f0, buf, buf + T::kABytes, kk + 2, a_row, b_row, lane, mi_n, ni_n);
          mma<T>(f1, acc, mi_n, ni_n);
        }
        load_frags<T, A_KS, B_KS>(f1, buf, buf + T::kABytes, STEPS - 1, a_row, b_row, lane, mi_n, ni_n);
        __builtin_amdgcn_sched_barrier(0);
        mma<T>(f0, acc, mi_n, ni_n);
        __builtin_amdgcn_sched_barrier(0);
        wait_lgkmcnt0();                               // this wave no longer needs the stage of slab kt
        if (kt + 1 < nfull) wait_slabs_in_flight<L, S - 2>(nfull - 2 - kt);   // slab kt+1 has landed
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (kt + S < nfull) {
          da.issue(next_slab, buf, wave);
          db.issue(next_slab, buf + T::kABytes, wave);
          next_slab = next_slab + 1 == nfull ? 0 : next_slab + 1;
        }
        stage = stage == S - 1 ? 0 : stage + 1;
        if (kt + 1 < nfull) {
          const char* nxt = lds + stage * T::kStageBytes;
          load_frags<T, A_KS, B_KS>(f0, nxt, nxt + T::kABytes, 0, a_row, b_row, lane, mi_n, ni_n);
        }
        __builtin_amdgcn_sched_barrier(0);
        mma<T>(f1, acc, mi_n, ni_n);
      }
    }
    if (tail) {
      // partial last slab: through registers, zero-filled beyond K.  Every stage is free here: all
      // loads have landed and every wave finished its LDS reads before the last barrier.
      Stager<A_KS, T::BM, T::BK, T::kThreads> sa;
      Stager<B_KS, T::BN, T::BK, T::kThreads> sb;
      sa.init(oa, tid);
      sb.init(ob, tid);
      sa.load(nfull * T::BK, K);
      sb.load(nfull * T::BK, K);
      sa.store(lds);
      sb.store(lds + T::kABytes);
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < STEPS; ++kk) {
        Frags<T> f;
        load_frags<T, A_KS, B_KS>(f, lds, lds + T::kABytes, kk, a_row, b_row, lane, mi_n, ni_n);
        mma<T>(f, acc, mi_n, ni_n);
      }
    }
    __syncthreads();                                   // all reads done before anything refills the ring
  }
}

// element i (0..15) of a 32x32 MFMA tile held by `lane`: row 8*(i/4) + 4*(lane/32) + i%4, col lane%32
__device__ __forceinline__ int acc_row(int lane, int i) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

// ---- epilogue: accumulators -> LDS (fp32) -> 16-byte row-contiguous global accesses -----------------
// The MFMA result layout gives a lane one column and four consecutive rows; written out directly
// that means 2-byte accesses.  Each wave instead parks a 32-row strip of its sub-tile in its own
// quarter of the (now idle) LDS ring and reads it back row-major, 8 consecutive columns per lane.
template <class T> struct Strip {
  static constexpr int LD = T::WN + 8;                 // floats per staged row: 4 rows shift the banks by 32
  static constexpr int kBytes = 32 * LD * 4;
  static_assert(T::kWaves * kBytes <= T::kLdsBytes, "staging strips must fit in the LDS ring");
};

template <class T>
__device__ __forceinline__ void park_strip(const f32x16 (&acc_mi)[T::NI], float* strip, int lane) {
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
    for (int i = 0; i < 16; ++i)
      strip[acc_row(lane, i) * Strip<T>::LD + ni * 32 + (lane & 31)] = acc_mi[ni][i];
}

__device__ __forceinline__ void read8(const float* p, float (&v)[8]) {
  const float4 x = *reinterpret_cast<const float4*>(p), y = *reinterpret_cast<const float4*>(p + 4);
  v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
}
__device__ __forceinline__ uint4 pack8(const float (&v)[8]) {
  return make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
}
__device__ __forceinline__ void unpack8(const uint4& w, float (&v)[8]) {
  v[0] = bf16_lo(w.x); v[1] = bf16_hi(w.x); v[2] = bf16_lo(w.y); v[3] = bf16_hi(w.y);
  v[4] = bf16_lo(w.z); v[5] = bf16_hi(w.z); v[6] = bf16_lo(w.w); v[7] = bf16_hi(w.w);
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
__global__ __launch_bounds__(T::kThreads) __attribute__((amdgpu_waves_per_eu(T::kWavesPerSimd, T::kWavesPerSimd))) void row_grouped_kernel(RowArgs p) {
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
  const int wm = wave / T::WGN, wn = wave % T::WGN;

  f32x16 acc[MI][NI];
  zero_acc<T>(acc);

  int a_row[MI];
#pragma unroll
  for (int i = 0; i < MI; ++i) a_row[i] = wm * WM + i * 32;
  // fragments of this wave that hold rows of the expert (wave-uniform)
  const int mi_n = __builtin_amdgcn_readfirstlane(min(MI, max(0, (rows - wm * WM + 31) / 32)));
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
    mainloop<T, false, false>(opsA, opsB, 1, p.K, lds, a_row, b_row, mi_n, NI, e * 13, acc);
    // strip columns: [0, HW) gate, [WN/2 + 0, ...) up -- both halves hold the same output columns
    float* strip = reinterpret_cast<float*>(lds + wave * Strip<T>::kBytes);
    constexpr int LPR = HW / 8;                        // lanes per output row (8 columns each)
    constexpr int RPP = 64 / LPR;                      // rows per pass
    const int cl = wn * HW + (lane % LPR) * 8;         // first of this lane's 8 columns inside the tile
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      if (mi >= mi_n) break;
      park_strip<T>(acc[mi], strip, lane);
      if (cl < ncols) {
#pragma unroll
        for (int pass = 0; pass < 32 / RPP; ++pass) {
          const int rs = pass * RPP + lane / LPR;
          const int r = wm * WM + mi * 32 + rs;
          if (r < rows) {
            float g[8], u[8], a[8];
            read8(strip + rs * Strip<T>::LD + (lane % LPR) * 8, g);
            read8(strip + rs * Strip<T>::LD + WN / 2 + (lane % LPR) * 8, u);
#pragma unroll
            for (int q = 0; q < 8; ++q) a[q] = g[q] * sigmoid_fast(g[q]) * u[q];
            const long o = static_cast<long>(row0 + r) * p.ldo + n0 + cl;
            if (p.out0) *reinterpret_cast<uint4*>(p.out0 + o) = pack8(g);
            if (p.out1) *reinterpret_cast<uint4*>(p.out1 + o) = pack8(u);
            if (p.out2) *reinterpret_cast<uint4*>(p.out2 + o) = pack8(a);
          }
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
      mainloop<T, false, false>(opsA, opsB, 1, p.K, lds, a_row, b_row, mi_n, NI, e * 13, acc);
    } else if constexpr (KIND == kDAct) {
      // dA = dyp * Wd[e] : weight is [K = d, N = f], reduction strided
      opB.half[0] = p.w0 + e * p.w_expert_stride + n0;
      opB.half[1] = opB.half[0] + BN / 2;
      mainloop<T, false, true>(opsA, opsB, 1, p.K, lds, a_row, b_row, mi_n, NI, e * 13, acc);
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
      mainloop<T, false, true>(opsA, opsB, 2, p.K, lds, a_row, b_row, mi_n, NI, e * 13, acc);
    }

    float* strip = reinterpret_cast<float*>(lds + wave * Strip<T>::kBytes);
    constexpr int LPR = WN / 8;                        // lanes per output row (8 columns each)
    constexpr int RPP = 64 / LPR;                      // rows per pass
    const int cl = wn * WN + (lane % LPR) * 8;         // first of this lane's 8 columns inside the tile
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      if (mi >= mi_n) break;
      park_strip<T>(acc[mi], strip, lane);
      if (cl < ncols) {
#pragma unroll
        for (int pass = 0; pass < 32 / RPP; ++pass) {
          const int rs = pass * RPP + lane / LPR;
          const int r = wm * WM + mi * 32 + rs;
          if (r < rows) {
            float v[8];
            read8(strip + rs * Strip<T>::LD + (lane % LPR) * 8, v);
            if constexpr (KIND == kDAct) {
              const long gi = static_cast<long>(row0 + r) * p.N + n0 + cl;
              float g[8], u[8], dg[8], du[8];
              unpack8(*reinterpret_cast<const uint4*>(p.g + gi), g);
              unpack8(*reinterpret_cast<const uint4*>(p.u + gi), u);
#pragma unroll
              for (int q = 0; q < 8; ++q) {
                const float sg = sigmoid_fast(g[q]);
                dg[q] = v[q] * u[q] * (sg * (1.0f + g[q] * (1.0f - sg)));
                du[q] = v[q] * (g[q] * sg);
              }
              const long o = static_cast<long>(row0 + r) * p.ldo + n0 + cl;
              *reinterpret_cast<uint4*>(p.out0 + o) = pack8(dg);
              *reinterpret_cast<uint4*>(p.out0 + o + p.N) = pack8(du);
            } else {
              *reinterpret_cast<uint4*>(p.out0 + static_cast<long>(row0 + r) * p.ldo + n0 + cl) = pack8(v);
            }
          }
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
__global__ __launch_bounds__(T::kThreads) __attribute__((amdgpu_waves_per_eu(T::kWavesPerSimd, T::kWavesPerSimd))) void wgrad_kernel(WgradArgs p) {
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
  const int wm = wave / T::WGN, wn = wave % T::WGN;

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
  mainloop<T, true, true>(&opA, &opB, 1, end - begin, lds, a_row, b_row, MI, NI, e * 13, acc);

  float* strip = reinterpret_cast<float*>(lds + wave * Strip<T>::kBytes);
  constexpr int LPR = WN / 8;
  constexpr int RPP = 64 / LPR;
  const int cl = wn * WN + (lane % LPR) * 8;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    park_strip<T>(acc[mi], strip, lane);
    if (cl < ncols) {
#pragma unroll
      for (int pass = 0; pass < 32 / RPP; ++pass) {
        const int rs = pass * RPP + lane / LPR;
        const int rl = wm * WM + mi * 32 + rs;
        if (rl < mrows) {
          float v[8];
          read8(strip + rs * Strip<T>::LD + (lane % LPR) * 8, v);
          const int m = m0 + rl;
          bf16_t* out = m < p.m_split ? p.out0 + (static_cast<long>(e) * p.m_split + m) * p.N
                                      : p.out1 + (static_cast<long>(e) * (p.M - p.m_split) + (m - p.m_split)) * p.N;
          *reinterpret_cast<uint4*>(out + n0 + cl) = pack8(v);
        }
      }
    }
  }
}

// ============================================================================================
// Host side
// ============================================================================================
// Tile shapes in use.  Row-grouped products keep the row (token) side at 128 so that experts
// with a few hundred rows waste little; the weight side is 256 wide.
typedef Tile<128, 256, 32, 2, 2, 3> TileRow;           // 72 KiB of LDS: two 4-wave workgroups per CU
typedef Tile<128, 256, 32, 2, 2, 3> TileWgrad;
typedef Tile<256, 256, 32, 2, 4, 5> TileBig;           // 160 KiB of LDS: one 8-wave workgroup per CU

// 0 = default.  MOE_GEMM_TILE=1 in the environment selects the 256 x 256 variant for every product
// (a tuning knob; the measured difference on the 30B-class shapes is a few percent either way).
static int tile_choice() {
  static int choice = -1;
  if (choice < 0) {
    const char* s = getenv("MOE_GEMM_TILE");
    choice = s ? atoi(s) : 0;
  }
  return choice;
}

static int row_bm() { return tile_choice() == 1 ? TileBig::BM : TileRow::BM; }
// bound used for workspace sizing: the smallest row tile gives the longest list
static int max_row_tiles(int P, int E) { return ceil_div(P, 128) + E; }

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
  const unsigned grid = padded_grid((ceil_div(P, T::BM) + E) * p.n_tiles_n);
  MOE_LAUNCH(names[KIND], (row_grouped_kernel<KIND, T>), dim3(grid), dim3(T::kThreads), T::kLdsBytes, s, p);
}

template <int KIND>
static void launch_row(const RowArgs& p, int P, int E, hipStream_t s) {
  if (tile_choice() == 1) launch_row_t<KIND, TileBig>(p, P, E, s);
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
  MOE_LAUNCH(WHICH == 0 ? "wgrad_down" : "wgrad_gate_up", (wgrad_kernel<WHICH, T>), dim3(grid), dim3(T::kThreads),
             T::kLdsBytes, s, p);
}

template <int WHICH>
static void launch_wgrad(const WgradArgs& p, hipStream_t s) {
  if (tile_choice() == 1) launch_wgrad_t<WHICH, TileBig>(p, s);
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
  MOE_LAUNCH("build_row_tiles", build_row_tiles_kernel, dim3(1), dim3(1024), 0, a.stream, a.offsets, a.E, a.P, row_bm(), rt);
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
  MOE_LAUNCH("build_row_tiles", build_row_tiles_kernel, dim3(1), dim3(1024), 0, a.stream, a.offsets, a.E, a.P, row_bm(), rt);
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
