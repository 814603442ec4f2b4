// bf16 MFMA grouped GEMMs of the SwiGLU expert FFN, forward and backward
// (Sec. 3.2.5 SwiGLU among the efficient kernels; App. B.6 stacked expert-major weights).
//
// One kernel skeleton serves all nine matrix products of the layer (and the three of the router):
//   * a BM x BN output tile per workgroup, a grid of WGM x WGN wavefronts over it, each owning a
//     WM x WN sub-tile made of 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16, fp32 accumulators kept in
//     registers for the whole reduction); the default is 256 x 256 with 2 x 4 wavefronts of 128 x 64;
//   * the reduction dimension is walked in BK-wide slabs through an S-stage LDS ring that is
//     filled by direct global->LDS loads (no staging registers); S-1 slabs are in flight behind the
//     one being multiplied, the MFMA operands are double-buffered in registers one reduction step
//     ahead, and one barrier per slab separates writers from readers; a partial last slab reads
//     zeros for the reduction indices it does not have;
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
// host synchronisation is needed.  Weight-gradient products reduce over an expert's rows
// instead: a second device-built schedule cuts long experts into bounded chunks whose fp32
// partial tiles a small kernel adds in chunk order (no float atomics).
// Workgroup ids are remapped so that consecutive tiles -- which share an expert's weights
// -- run on the same XCD (workgroup b runs on XCD b mod 8) and hit its L2.
// The router linear (logits, its weight gradient, its part of the input gradient) runs on
// the same skeleton with a single segment of all rows.
#include <algorithm>
#include <mutex>
#include <type_traits>
#include <utility>
#include "moe_common.h"

namespace moe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kXcds = 8;

// ---- tile shapes ------------------------------------------------------------------------------
template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int STAGES_A_, int STAGES_B_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_;
  static constexpr int WGM = WGM_, WGN = WGN_;            // grid of wavefronts over the tile
  static constexpr int kWaves = WGM * WGN, kThreads = 64 * kWaves;
  static constexpr int WM = BM / WGM, WN = BN / WGN;      // sub-tile of one wavefront
  static constexpr int MI = WM / 32, NI = WN / 32;        // MFMA tiles per wave
  static constexpr int kABytes = BM * BK * 2, kBBytes = BN * BK * 2;
  // LDS ring: each operand has its own ring of slab buffers (SA for the row side, SB for the column side); slab kt
  // lives in buffer kt % SA and kt % SB.  One slab is being multiplied, the others are in flight.  With 64 KiB per
  // slab only 2.5 slabs fit the 160 KiB of a CU: SA = 2, SB = 3, which is what keeps the CU's window of outstanding
  // L2 requests full across the barrier that separates two slabs (with 2 + 2 it drains at every slab).  The deeper
  // ring goes to the side with fewer fragments per wave: its third buffer lies beyond the 16-bit immediate offset of
  // the LDS instructions and costs one more address register per fragment.
  static constexpr int SA = STAGES_A_, SB = STAGES_B_;
  static constexpr int kBBase = SA * kABytes;             // the column side's buffers follow the row side's
  static constexpr int kLdsBytes = SA * kABytes + SB * kBBytes;
  // Epilogue staging strips (one per wave, 32 rows x (WN + 4) floats) reuse the ring from its start once it is idle.
  static constexpr int kStripBytes = 32 * (WN + 4) * 4;
  static constexpr int kStripBase = 0;
  static constexpr int kLdsAlloc = kWaves * kStripBytes > kLdsBytes ? kWaves * kStripBytes : kLdsBytes;
  static_assert(kLdsAlloc <= 160 * 1024, "a CU has 160 KiB of LDS");
  static constexpr int kBlocksPerCu = 2 * kLdsAlloc <= 160 * 1024 ? 2 : 1;   // by LDS capacity
  static constexpr int kWavesPerSimd = kBlocksPerCu * kWaves / 4;
};

// One operand tile of ROWS rows: element (row, k).  Two halves of ROWS/2 rows with their own
// base so that the gate and the up projection can share one tile.
//   k-contiguous: half[h] + row * ld + k          k-strided: half[h] + k * ld + row
struct Operand {
  const bf16_t* half[2];
  long ld;
  int valid[2];      // rows of each half that exist (others read as zero); multiples of 8 if k-strided
  // Gathered operands (the matrix is [*, ld] and never copied into expert order): logical row r of the
  // operand -- a tile row if k-contiguous, a reduction index if k-strided -- is memory row gather[grow + r]
  // of half[0]; half[1] is not used, and every byte offset (row * ld * 2) must fit in 32 bits.
  const int32_t* gather;
  int grow;
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

// ---- MFMA operand fragments ----------------------------------------------------------------------------
// Fragment = 32 rows x 16 k: lane l holds row l%32, k = 8*(l/32) .. +7 of the 16-wide step kk.
// frag_off: this lane's byte offset inside the operand tile, computed once per kernel for step 0; the main
// loop derives the other steps with one XOR (or a constant) and adds compile-time stage offsets.
template <bool KS, int ROWS, int BK>
__device__ __forceinline__ int frag_off(int row_base, int kk, int lane) {
  if constexpr (!KS) {
    return kc_off<BK>(row_base + (lane & 31), 2 * kk + (lane >> 5));
  } else {
    // Transposing read: within each group of 16 lanes, lane i receives element i%4 of the 8-byte
    // rows addressed by lanes i/4, i/4+4, i/4+8, i/4+12.  Lane s therefore addresses k-row s/4 at
    // columns 4*(s%4)..+3 of its group's 16 columns, and ends up with 4 consecutive k of column s.
    const int s = lane & 15;
    const int col = row_base + 16 * ((lane >> 4) & 1) + 4 * (s & 3);     // multiple of 4
    const int k = kk * 16 + 8 * (lane >> 5) + (s >> 2);
    return ks_off<ROWS>(k, col >> 3) + (col & 4) * 2;                     // 8-byte half of the piece
  }
}
// One fragment: 16 bytes per lane at LDS address `addr` + IMM (a compile-time constant: buffer, reduction step or
// fragment).  Both kinds of read are assembly statements on purpose.
//   * The compiler orders every LDS read it knows to be one behind all outstanding direct global->LDS loads (it
//     cannot tell which bytes they will write): it puts a wait for *all* of this wave's loads in front of the first
//     such read of every slab, which serialises the ring -- the slabs just requested would have to land before the
//     slab in hand may be read.  The ring needs no such wait: a buffer is read only after the counted wait and the
//     barrier that follow its own loads.
//   * The address register and the 16-bit immediate are chosen here, so no address arithmetic is left in the slab
//     loop (every vector instruction there takes issue slots from the MFMAs of both waves of the SIMD).
// The results arrive asynchronously; they are consumed only after settle() below, which names them as operands.
template <bool KS, int ROWS, int IMM>
__device__ __forceinline__ bf16x8 lds_read_frag(uint32_t addr) {
  static_assert(IMM >= 0 && IMM + (KS ? 4 * ROWS * 2 : 0) < 65536, "the immediate offset of an LDS instruction has 16 bits");
  if constexpr (!KS) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(IMM));
    return v;
  } else {
    // k + 4 has the same swizzle (k & 3 unchanged): a constant 4 k-rows further
    bf16x4 lo, hi;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(IMM));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(IMM + 4 * ROWS * 2));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }
}

// ---- global -> LDS without passing through registers -----------------------------------------------
// One wave instruction (global_load_lds_dwordx4) moves 64 x 16 bytes into 1 KiB of consecutive LDS;
// the swizzles above are applied on the global side: each lane fetches the piece that belongs in its
// LDS slot.  Addresses are a wave-uniform base (advanced per slab with scalar arithmetic) plus a
// 32-bit per-lane offset.  Rows that do not exist are redirected to the tile's first row: they only
// feed output rows / columns that are never stored.  Reduction indices beyond K (last, partial
// slab only) are redirected to a block of zeros, so they contribute nothing.
template <bool KS, int ROWS, int BK, int WAVES, bool GATHER = false> struct Dma {
  static constexpr int CHUNKS = ROWS * BK * 2 / 1024;
  static constexpr int N = CHUNKS / WAVES;                   // chunks per wave
  static_assert(N >= 1 && CHUNKS % WAVES == 0, "tile too small for this many waves");
  static constexpr int KPC = KS ? 1024 / (ROWS * 2) : 1;      // k-strided: reduction rows per chunk
  static constexpr int NR = N * KPC;                         // k-strided: reduction rows per wave and slab (consecutive)
  const char* base[N];       // wave-uniform
  uint32_t voff[N];          // per lane, bytes
  uint32_t kpack[(N + 3) / 4];   // per lane: reduction index inside the slab of this lane's piece of chunk i, 8 bits each
                                 // (only the partial last slab needs it: packed to keep registers for the main loop)
  __device__ __forceinline__ void set_kidx(int i, int k) { kpack[i / 4] |= static_cast<uint32_t>(k) << (8 * (i % 4)); }
  __device__ __forceinline__ int kidx(int i) const { return static_cast<int>((kpack[i / 4] >> (8 * (i % 4))) & 255u); }
  long step;                 // bytes per slab (uniform)
  // gathered k-strided operand: the memory rows of the wave's NR reduction rows of the next slab to be
  // issued, fetched with scalar loads one slab ahead (they do not touch the vector-memory counter
  // that orders the ring)
  typedef __attribute__((address_space(4))) const int32_t* RowList;
  typedef int32_t RowVec __attribute__((ext_vector_type(KS && GATHER ? NR : 1)));   // a value, not an array: stays in scalar registers
  RowList rows;              // wave-uniform: gather + grow + wave * NR
  RowVec next_row;
  uint32_t ld2;              // bytes per memory row
  int lq;                    // per lane: which of the KPC rows of a chunk this lane loads
  __device__ __forceinline__ void fetch_rows(int slab) {
    if constexpr (KS && GATHER) {
      RowList r = rows + slab * BK;
#pragma unroll
      for (int j = 0; j < NR; ++j) next_row[j] = r[j];
    }
  }
  __device__ __forceinline__ void init(const Operand& op, int wave, int lane) {
    const bf16_t* const h0 = op.half[0];                     // scalars, so that the selects below stay selects
    const bf16_t* const h1 = op.half[1];
    const int v0 = op.valid[0], v1 = op.valid[1];
    static_assert(BK <= 256, "reduction indices are packed in 8 bits");
#pragma unroll
    for (int i = 0; i < (N + 3) / 4; ++i) kpack[i] = 0u;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = wave * N + i;                            // wave-uniform
      if constexpr (!KS) {
        constexpr int PPR = BK / 8, RPC = 1024 / (BK * 2), RPL = 256 / (BK * 2);
        static_assert((ROWS / 2) % RPC == 0, "a chunk must not straddle the two halves");
        const int row = c * RPC + lane / PPR;
        const int piece = (lane % PPR) ^ ((row / RPL) & (PPR - 1));
        const bool upper = c * RPC >= ROWS / 2;              // uniform
        const int rh = row - (upper ? ROWS / 2 : 0);
        const int valid = upper ? v1 : v0;
        if constexpr (GATHER) {
          // rows that do not exist read the tile's first row (it exists)
          const int mrow = op.gather[op.grow + (rh < valid ? row : 0)];
          base[i] = reinterpret_cast<const char*>(h0);
          voff[i] = static_cast<uint32_t>(mrow) * static_cast<uint32_t>(op.ld * 2) + piece * 16;
        } else {
          // the chunk's base stays the upper half only if the chunk holds at least one row that exists
          // (uniform); single missing rows are redirected through the per-lane offset
          const bool chunk_any = (c * RPC - (upper ? ROWS / 2 : 0)) < valid;
          const bool own_base = !upper || chunk_any;
          base[i] = reinterpret_cast<const char*>((own_base && upper) ? h1 : h0);
          const bool own_row = own_base && rh < valid;
          voff[i] = static_cast<uint32_t>((own_row ? static_cast<long>(rh) * op.ld : 0) * 2 + piece * 16);
        }
        set_kidx(i, piece * 8);
      } else {
        constexpr int PPK = ROWS / 8;
        const int k = c * KPC + lane / PPK;
        const int phys = lane % PPK;
        const int piece = ((((phys >> 2) ^ (k & 3)) << 2) | (phys & 3));
        const int col = piece * 8;
        const bool upper = col >= ROWS / 2;
        const int ch = col - (upper ? ROWS / 2 : 0);
        const bool ok = ch < (upper ? v1 : v0);
        // k-strided operands are never dual: half[1] is half[0] shifted by ROWS/2 columns
        base[i] = reinterpret_cast<const char*>(h0);
        if constexpr (GATHER) voff[i] = static_cast<uint32_t>((ok ? col : 0) * 2);
        else voff[i] = static_cast<uint32_t>(((ok ? col : 0) + static_cast<long>(k) * op.ld) * 2);
        set_kidx(i, k);
      }
    }
    step = (KS ? (GATHER ? 0L : static_cast<long>(BK) * op.ld) : BK) * 2;
    // the bases are the same in every lane: say so, to get scalar base + 32-bit lane offset addressing
    // (no 64-bit per-lane address arithmetic, fewer registers held across the main loop)
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const uint64_t b64 = reinterpret_cast<uint64_t>(base[i]);
      const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64));
      const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(b64 >> 32));
      base[i] = reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
    }
    if constexpr (KS && GATHER) {
      rows = reinterpret_cast<RowList>(reinterpret_cast<uintptr_t>(op.gather + op.grow + wave * NR));
      ld2 = static_cast<uint32_t>(op.ld * 2);
      lq = lane / (ROWS / 8);
      fetch_rows(0);
    }
  }
  // byte offset of this lane's piece of chunk i from the wave-uniform base
  __device__ __forceinline__ uint32_t lane_off(int i) const {
    if constexpr (KS && GATHER) {
      int32_t mrow = next_row[i * KPC];
#pragma unroll
      for (int q = 1; q < KPC; ++q) mrow = lq == q ? next_row[i * KPC + q] : mrow;
      return static_cast<uint32_t>(mrow) * ld2 + voff[i];
    } else {
      return voff[i];
    }
  }
  // enqueue this wave's share of slab `slab` into the operand tile at `tile` (LDS); slabs are issued in order
  __device__ __forceinline__ void issue(int slab, char* tile, int wave) {
#pragma unroll
    for (int i = 0; i < N; ++i) issue_one(i, slab, tile, wave);
    fetch_rows(slab + 1);
  }
  // one of the N loads of a full slab (the caller enqueues all N, in order, then fetch_rows(slab + 1))
  __device__ __forceinline__ void issue_one(int i, int slab, char* tile, int wave) {
    const char* g = base[i] + slab * step + lane_off(i);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                     (__attribute__((address_space(3))) void*)(tile + (wave * N + i) * 1024), 16, 0, 0);
  }
  // the same for the last, partial slab: pieces whose reduction index is >= K read zeros
  __device__ __forceinline__ void issue_tail(int slab, int K, const char* zeros, char* tile, int wave) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const bool in_range = slab * BK + kidx(i) < K;
      uint32_t off = lane_off(i);
      asm volatile("" : "+v"(off));                          // the 64-bit per-lane address is formed here, not kept in registers across the slab loop
      const char* g = in_range ? base[i] + slab * step + off : zeros;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                       (__attribute__((address_space(3))) void*)(tile + (wave * N + i) * 1024), 16, 0, 0);
    }
    fetch_rows(slab + 1);
  }
};

// s_waitcnt that waits only for the vector-memory counter to drop to n (gfx9 encoding:
// vmcnt = imm[3:0] | imm[15:14] << 4, expcnt = imm[6:4], lgkmcnt = imm[11:8])
template <int n> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14));
}
// s_waitcnt that waits only for the LDS / scalar-memory counter to reach zero
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14)); }

// wait until at most n of this wave's direct loads are still in flight; n is a multiple of STEP and at most MAX
// (the hardware wait takes an immediate: one comparison per candidate, the steady-state value first)
template <int MAX, int STEP>
__device__ __forceinline__ void wait_loads_in_flight(int n) {
  if constexpr (MAX <= 0) {
    wait_vmcnt<0>();
  } else {
    if (n >= MAX) wait_vmcnt<MAX>();
    else wait_loads_in_flight<MAX - STEP, STEP>(n);
  }
}

// the MFMA operands of one 16-wide reduction step for this wave's sub-tile
template <class T> struct Frags {
  bf16x8 a[T::MI];
  bf16x8 b[T::NI];
};
// Per-lane LDS addresses of the fragments, set up once per tile.  The wave's fragments of one side lie a constant
// number of tile rows apart (FR rows, normally 32), and
//   * in a k-contiguous tile a fragment FR rows further is a constant number of bytes further (the swizzle of a row
//     repeats every 16 rows), while the reduction step moves the piece index by 2*KK, which the swizzle turns into
//     an XOR of the address: one register per step, the fragment in the immediate;
//   * in a k-strided tile the step is a constant number of bytes (16 reduction rows; the swizzle k & 3 is unchanged)
//     but a fragment 32 columns further is not (its 64-byte chunk index is XORed with k & 3): one register per
//     fragment, the step in the immediate.
// A buffer that starts 64 KiB or more into its side's ring is out of reach of the immediate: `far` holds the same
// addresses 64 KiB further (only the third buffer of a three-deep ring needs them).
template <class T, bool A_KS, bool B_KS> struct FragAddrs {
  static constexpr int STEPS = T::BK / 16;
  static constexpr int NA = A_KS ? T::MI : STEPS, NB = B_KS ? T::NI : STEPS;
  static constexpr bool A_FAR = (T::SA - 1) * T::kABytes >= 65536, B_FAR = (T::SB - 1) * T::kBBytes >= 65536;
  uint32_t a[NA], b[NB];
  uint32_t a_far[A_FAR ? NA : 1], b_far[B_FAR ? NB : 1];
};
// Fragment I of one side at reduction step KK, from the buffer that starts OFF bytes into the side's ring; FR: tile
// rows between the wave's fragments; near / far: the side's address registers.
template <bool KS, int ROWS, int BK, int FR, int OFF, int KK, int I, int N>
__device__ __forceinline__ bf16x8 read_side(const uint32_t (&near)[N], const uint32_t* far) {
  constexpr int FAR = OFF >= 65536 ? 65536 : 0;
  if constexpr (KS) return lds_read_frag<true, ROWS, OFF - FAR + KK * 16 * ROWS * 2>(FAR ? far[I] : near[I]);
  else return lds_read_frag<false, ROWS, OFF - FAR + I * FR * BK * 2>(FAR ? far[KK] : near[KK]);
}
template <class T, bool A_KS, bool B_KS, int FRA, int FRB, int OFF_A, int OFF_B, int KK, int... IA, int... IB>
__device__ __forceinline__ void load_frags_seq(Frags<T>& f, const FragAddrs<T, A_KS, B_KS>& fa, std::integer_sequence<int, IA...>,
                                               std::integer_sequence<int, IB...>) {
  ((f.a[IA] = read_side<A_KS, T::BM, T::BK, FRA, OFF_A, KK, IA>(fa.a, fa.a_far)), ...);
  ((f.b[IB] = read_side<B_KS, T::BN, T::BK, FRB, OFF_B, KK, IB>(fa.b, fa.b_far)), ...);
}
// OFF_A / OFF_B: where the slab's buffers start in their side's ring; FRA / FRB: tile rows between the wave's fragments.
template <class T, bool A_KS, bool B_KS, int FRA, int FRB, int OFF_A, int OFF_B, int KK>
__device__ __forceinline__ void load_frags(Frags<T>& f, const FragAddrs<T, A_KS, B_KS>& fa) {
  static_assert((T::BK / 16 - 1) * 32 < T::BK * 2, "the step bits must lie inside a row");
  load_frags_seq<T, A_KS, B_KS, FRA, FRB, OFF_A, OFF_B, KK>(f, fa, std::make_integer_sequence<int, T::MI>{}, std::make_integer_sequence<int, T::NI>{});
}
// Wait until this wave's LDS reads have delivered, with the fragments as operands of the wait: the registers a
// transposing read (an assembly statement, see read_frag) is filling stay reserved until here on every path --
// the compiler must neither reuse them earlier nor move a consumer above the wait.
template <class T>
__device__ __forceinline__ void settle(Frags<T>& f) {
  static_assert(T::MI + T::NI <= 8, "one operand per fragment");
  if constexpr (T::MI == 4 && T::NI == 2) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.a[2]), "+v"(f.a[3]), "+v"(f.b[0]), "+v"(f.b[1]));
  } else if constexpr (T::MI == 2 && T::NI == 2) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.b[0]), "+v"(f.b[1]));
  } else {
    static_assert(T::MI == 1 && T::NI == 2, "add the operand list of this wave shape");
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.a[0]), "+v"(f.b[0]), "+v"(f.b[1]));
  }
}

// MFMAs number FROM .. TO-1 (row-major over the wave's MI x NI fragments) of one reduction step
template <class T, int FROM, int TO>
__device__ __forceinline__ void mma(const Frags<T>& f, f32x16 (&acc)[T::MI][T::NI]) {
#pragma unroll
  for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < T::NI; ++ni)
      if (mi * T::NI + ni >= FROM && mi * T::NI + ni < TO)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[ni], f.a[mi], acc[mi][ni], 0, 0, 0);   // transposed tile, see Strip
}

// acc += sum over segments of A_s(BM x K) * B_s(BN x K)^T for this wave's sub-tile (segments differ
// only in their base pointers).  a_row[mi] / b_row[ni]: first tile row of the wave's mi-th / ni-th
// 32-row fragment.
//
// Slabs stream through the two LDS rings (SA buffers for the A side, SB <= SA for the B side) filled by direct
// global->LDS loads, and the MFMA operands are double-buffered in registers, so that every LDS read is issued
// one reduction step ahead of the MFMAs that consume it.  Per slab kt:
//     read step 1.. of slab kt (into the other register set) | MFMAs of the steps already loaded
//     wait: own LDS reads of slab kt complete, own loads of slab kt+1 landed (later slabs stay in flight)
//     barrier: slab kt+1 is visible to all, and nobody reads the buffers of slab kt any more
//     refill them with B of slab kt+SB, then A of slab kt+SA; read step 0 of slab kt+1 | MFMAs of the last step
// Loads complete in the order they were enqueued, and the refill enqueues the slab that is needed first first, so
// "slab kt+1 has landed" is a wait for all but the loads enqueued after it -- an immediate count.  The loop over
// slabs is unrolled lcm(SA, SB) times so that every LDS address is "register + constant" and no address arithmetic
// competes with the MFMAs for issue slots.  What limits the stream is the number of L2 requests a CU can have
// outstanding (about 128 lines, whatever is in flight in the rings): 64-byte row pieces (BK = 32) give about
// 30 bytes per clock and CU on L2 hits, 128-byte pieces (BK = 64) about 60; the rings only have to keep that
// window full, which a ring that drains at every slab (SA = SB = 2) does not.
template <class T, bool A_KS, bool B_KS, bool A_GATHER = false, bool B_GATHER = false, int FRB = 32>
struct MainLoop {
  static constexpr int FRA = 32;                       // tile rows between the wave's fragments, A side and B side
  typedef Dma<A_KS, T::BM, T::BK, T::kWaves, A_GATHER> DmaA;
  typedef Dma<B_KS, T::BN, T::BK, T::kWaves, B_GATHER> DmaB;
  static constexpr int NA = DmaA::N, NB = DmaB::N;     // loads per thread per slab and side
  static constexpr int SA = T::SA, SB = T::SB;
  static_assert(SA >= 2 && SB >= 2, "one slab being multiplied, at least one in flight");
  static constexpr int U = (SA % SB == 0) ? SA : SA * SB;   // slabs per unrolled trip: buffer indices are compile-time
  static constexpr int STEPS = T::BK / 16;             // reduction steps per slab (even)
  static constexpr int kMaxAhead = (SA - 1) * NA + (SB - 1) * NB;   // most loads ever in flight behind slab 0
  static constexpr int kStep = NA == NB ? NA : 1;
  static_assert(kMaxAhead < 64, "vmcnt is a 6-bit counter");

  DmaA da;
  DmaB db;
  FragAddrs<T, A_KS, B_KS> fa;
  Frags<T> f0, f1;                                     // even / odd reduction steps
  char* lds;
  uint32_t lds32;                                      // the ring's start as an LDS address
  const char* zeros;
  int nslabs, nfull, K, wave;

  __device__ __forceinline__ char* buf_a(int stage) const { return lds + stage * T::kABytes; }
  __device__ __forceinline__ char* buf_b(int stage) const { return lds + T::kBBase + stage * T::kBBytes; }
  // LDS reads: the B side's fragment offsets already contain kBBase, so that every buffer but the last of a
  // three-deep ring is reached with the 16-bit immediate offset of the LDS instruction
  __device__ __forceinline__ void issue_a(int slab, int stage) {
    if (slab < nfull) da.issue(slab, buf_a(stage), wave);
    else da.issue_tail(slab, K, zeros, buf_a(stage), wave);
  }
  __device__ __forceinline__ void issue_b(int slab, int stage) {
    if (slab < nfull) db.issue(slab, buf_b(stage), wave);
    else db.issue_tail(slab, K, zeros, buf_b(stage), wave);
  }
  // loads enqueued so far for slabs beyond kt + 1 (they may stay in flight when slab kt + 1 is needed)
  __device__ __forceinline__ int loads_beyond(int kt) const {
    const int rest = nslabs - 2 - kt;                  // slabs that exist beyond kt + 1
    return max(0, min(SA - 2, rest)) * NA + max(0, min(SB - 2, rest)) * NB;
  }

  // Steps KK .. STEPS-2 of the slab in buffers SGA / SGB.  Every step first waits for its own operands, then issues
  // the LDS reads of the next step and only then its MFMAs, so each read has a whole step of MFMAs (plus the other
  // wave on the SIMD) to complete.  Even steps multiply f0, odd steps f1.
  template <int SGA, int SGB, int KK>
  __device__ __forceinline__ void steps(f32x16 (&acc)[T::MI][T::NI]) {
    if constexpr (KK + 1 < STEPS) {
      settle<T>((KK & 1) ? f1 : f0);
      __builtin_amdgcn_sched_barrier(0);
      load_frags<T, A_KS, B_KS, FRA, FRB, SGA * T::kABytes, SGB * T::kBBytes, KK + 1>((KK & 1) ? f0 : f1, fa);
      __builtin_amdgcn_sched_barrier(0);
      mma<T, 0, T::MI * T::NI>((KK & 1) ? f1 : f0, acc);
      __builtin_amdgcn_sched_barrier(0);
      steps<SGA, SGB, KK + 1>(acc);
    }
  }

  // ACTIVE = false: a wave whose sub-tile holds no row of the expert (the tile sticks out of the
  // row segment) only takes part in the loads and barriers; its SIMD time goes to the other waves.
  template <int STG, bool ACTIVE>
  __device__ __forceinline__ void slab_body(int kt, f32x16 (&acc)[T::MI][T::NI]) {
    constexpr int SGA = STG % SA, SGB = STG % SB, NXA = (STG + 1) % SA, NXB = (STG + 1) % SB;
    constexpr int ALL = T::MI * T::NI;
    if constexpr (ACTIVE) {
      steps<SGA, SGB, 0>(acc);                         // every step but the last: fetch the next step, multiply this one
      settle<T>(f1);                                   // last step is in f1; this wave no longer needs the buffers of slab kt
      __builtin_amdgcn_sched_barrier(0);
    }
    if (kt + 1 < nslabs) wait_loads_in_flight<(SA - 2) * NA + (SB - 2) * NB, kStep>(loads_beyond(kt));   // slab kt+1 has landed
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // Products that read an operand transposed start with the last step's MFMAs (their LDS reads and the refill then
    // issue under those MFMAs); the others first fetch and refill (measured: 1-3 % either way).
    constexpr bool MMA_FIRST = A_KS || B_KS;
    if constexpr (ACTIVE && MMA_FIRST) {
      mma<T, 0, ALL>(f1, acc);
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (ACTIVE) {
      if (kt + 1 < nslabs) load_frags<T, A_KS, B_KS, FRA, FRB, NXA * T::kABytes, NXB * T::kBBytes, 0>(f0, fa);
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (SB <= SA) {                          // the side whose slab is needed sooner goes first
      if (kt + SB < nslabs) issue_b(kt + SB, SGB);
      if (kt + SA < nslabs) issue_a(kt + SA, SGA);
    } else {
      if (kt + SA < nslabs) issue_a(kt + SA, SGA);
      if (kt + SB < nslabs) issue_b(kt + SB, SGB);
    }
    if constexpr (ACTIVE && !MMA_FIRST) {
      __builtin_amdgcn_sched_barrier(0);
      mma<T, 0, ALL>(f1, acc);
    }
  }

  // The same for a wave with rows, when every slab the body touches is a full one that exists (slabs kt + 1, kt + SA and
  // kt + SB below nfull): nothing branches, and the refill and the first LDS reads of the next slab are spread between
  // the MFMAs of the last step, one group per MFMA -- they issue while the matrix pipe is busy with the MFMA before
  // them instead of holding it up after the barrier.
  template <int STG>
  __device__ __forceinline__ void slab_interior(int kt, f32x16 (&acc)[T::MI][T::NI]) {
    constexpr int SGA = STG % SA, SGB = STG % SB, NXA = (STG + 1) % SA, NXB = (STG + 1) % SB;
    constexpr int ALL = T::MI * T::NI;
    constexpr int LOADS = NA + NB;
    constexpr int GAPS = ALL - 1;                      // the first gap takes the LDS reads, the others the loads
    constexpr int PER = (LOADS + GAPS - 1) / GAPS;
    static_assert(GAPS >= 1, "a wave has at least two MFMA tiles");
    steps<SGA, SGB, 0>(acc);
    settle<T>(f1);
    __builtin_amdgcn_sched_barrier(0);
    wait_vmcnt<(SA - 2) * NA + (SB - 2) * NB>();       // slab kt+1 has landed
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    mma_one<0>(acc);
    __builtin_amdgcn_sched_barrier(0);
    load_frags<T, A_KS, B_KS, FRA, FRB, NXA * T::kABytes, NXB * T::kBBytes, 0>(f0, fa);
    __builtin_amdgcn_sched_barrier(0);
    interior_gaps<SGA, SGB, 1, PER>(kt, acc);
  }
  // MFMA number M of the last step (operands in f1)
  template <int M>
  __device__ __forceinline__ void mma_one(f32x16 (&acc)[T::MI][T::NI]) { mma<T, M, M + 1>(f1, acc); }
  // load number J of the refill: the side whose slab is needed sooner comes first
  template <int SGA, int SGB, int J>
  __device__ __forceinline__ void refill_one(int kt) {
    constexpr bool B_FIRST = SB <= SA;
    constexpr int N1 = B_FIRST ? NB : NA;
    if constexpr (J < N1) {
      if constexpr (B_FIRST) db.issue_one(J, kt + SB, buf_b(SGB), wave); else da.issue_one(J, kt + SA, buf_a(SGA), wave);
      if constexpr (J == N1 - 1) { if constexpr (B_FIRST) db.fetch_rows(kt + SB + 1); else da.fetch_rows(kt + SA + 1); }
    } else if constexpr (J < NA + NB) {
      if constexpr (B_FIRST) da.issue_one(J - N1, kt + SA, buf_a(SGA), wave); else db.issue_one(J - N1, kt + SB, buf_b(SGB), wave);
      if constexpr (J == NA + NB - 1) { if constexpr (B_FIRST) da.fetch_rows(kt + SA + 1); else db.fetch_rows(kt + SB + 1); }
    }
  }
  template <int SGA, int SGB, int J, int JEND>
  __device__ __forceinline__ void refill_range(int kt) {
    if constexpr (J < JEND) { refill_one<SGA, SGB, J>(kt); refill_range<SGA, SGB, J + 1, JEND>(kt); }
  }
  template <int SGA, int SGB, int M, int PER>
  __device__ __forceinline__ void interior_gaps(int kt, f32x16 (&acc)[T::MI][T::NI]) {
    if constexpr (M < T::MI * T::NI) {
      mma_one<M>(acc);
      __builtin_amdgcn_sched_barrier(0);
      refill_range<SGA, SGB, (M - 1) * PER, M * PER>(kt);
      __builtin_amdgcn_sched_barrier(0);
      interior_gaps<SGA, SGB, M + 1, PER>(kt, acc);
    }
  }
  template <int STG>
  __device__ __forceinline__ void interior_trip(int& kt, f32x16 (&acc)[T::MI][T::NI]) {
    if constexpr (STG < U) {
      slab_interior<STG>(kt, acc);
      ++kt;
      interior_trip<STG + 1>(kt, acc);
    }
  }

  template <int STG, bool ACTIVE>
  __device__ __forceinline__ void run_from(int& kt, f32x16 (&acc)[T::MI][T::NI]) {
    if constexpr (STG < U) {
      if (kt < nslabs) {
        slab_body<STG, ACTIVE>(kt, acc);
        ++kt;
        run_from<STG + 1, ACTIVE>(kt, acc);
      }
    }
  }

  template <bool ACTIVE>
  __device__ __forceinline__ void stream(f32x16 (&acc)[T::MI][T::NI]) {
    if constexpr (ACTIVE) load_frags<T, A_KS, B_KS, FRA, FRB, 0, 0, 0>(f0, fa);
    int kt = 0;
    if constexpr (ACTIVE) {
#pragma nounroll
      while (kt + U + (SA > SB ? SA : SB) <= nfull) {  // trips that only touch full slabs: the branch-free bodies
        interior_trip<0>(kt, acc);
      }
    }
#pragma nounroll
    while (kt + U <= nslabs) {                         // U slabs per trip: buffers are compile-time
      run_from<0, ACTIVE>(kt, acc);
    }
    run_from<0, ACTIVE>(kt, acc);                      // the remaining < U slabs
    if constexpr (ACTIVE) settle<T>(f0);               // nothing is in flight into a register when the epilogue starts
  }

  // reduction length, LDS ring and the per-lane fragment offsets of this wave's sub-tile
  __device__ __forceinline__ void prepare(int K_, char* lds_, const bf16_t* zeros_, const int (&a_row)[T::MI],
                                          const int (&b_row)[T::NI]) {
    const int tid = threadIdx.x, lane = tid & 63;
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS destinations stay scalar
    lds = lds_; zeros = reinterpret_cast<const char*>(zeros_); K = K_;
    lds32 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char*)lds_));
    nfull = K > 0 ? K / T::BK : 0;
    nslabs = K > 0 ? (K + T::BK - 1) / T::BK : 0;
    typedef FragAddrs<T, A_KS, B_KS> FA;
#pragma unroll
    for (int i = 0; i < FA::NA; ++i) {                 // k-strided: fragment i at step 0; k-contiguous: fragment 0 at step i
      if constexpr (A_KS) fa.a[i] = lds32 + frag_off<true, T::BM, T::BK>(a_row[i], 0, lane);
      else fa.a[i] = lds32 + frag_off<false, T::BM, T::BK>(a_row[0], i, lane);
      if constexpr (FA::A_FAR) fa.a_far[i] = fa.a[i] + 65536;
    }
#pragma unroll
    for (int i = 0; i < FA::NB; ++i) {
      if constexpr (B_KS) fa.b[i] = lds32 + T::kBBase + frag_off<true, T::BN, T::BK>(b_row[i], 0, lane);
      else fa.b[i] = lds32 + T::kBBase + frag_off<false, T::BN, T::BK>(b_row[0], i, lane);
      if constexpr (FA::B_FAR) fa.b_far[i] = fa.b[i] + 65536;
    }
  }
  // point the loads at the operands of a segment and fill both rings, slab by slab (A before B), as far as they go.
  // The rings must be idle.
  __device__ __forceinline__ void start(const Operand& oa, const Operand& ob) {
    const int lane = threadIdx.x & 63;
    da.init(oa, wave, lane);
    db.init(ob, wave, lane);
#pragma unroll
    for (int s0 = 0; s0 < (SA > SB ? SA : SB); ++s0) {
      if (s0 < SA && s0 < nslabs) issue_a(s0, s0);
      if (s0 < SB && s0 < nslabs) issue_b(s0, s0);
    }
  }
  // multiply the segment whose first slabs have been enqueued by start()
  __device__ __forceinline__ void go(bool active, f32x16 (&acc)[T::MI][T::NI]) {
    if (nslabs <= 0) return;
    const int rest = nslabs - 1;                       // slabs beyond slab 0 that start() enqueued
    wait_loads_in_flight<kMaxAhead, kStep>(min(SA - 1, rest) * NA + min(SB - 1, rest) * NB);   // slab 0 has landed
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (active) stream<true>(acc); else stream<false>(acc);
    __syncthreads();                                   // all reads done before anything refills the rings
  }

  __device__ __forceinline__ void run(const Operand* opA, const Operand* opB, int nseg, int K_, char* lds_,
                                      const bf16_t* zeros_, const int (&a_row)[T::MI], const int (&b_row)[T::NI],
                                      bool active, f32x16 (&acc)[T::MI][T::NI]) {
    prepare(K_, lds_, zeros_, a_row, b_row);
    if (K <= 0) return;
#pragma nounroll
    for (int seg = 0; seg < nseg; ++seg) {
      Operand oa, ob;                                  // picked field by field: no dynamically indexed copies
      oa.half[0] = seg ? opA[1].half[0] : opA[0].half[0];
      oa.half[1] = seg ? opA[1].half[1] : opA[0].half[1];
      oa.ld = opA[0].ld;
      oa.valid[0] = opA[0].valid[0];
      oa.valid[1] = opA[0].valid[1];
      oa.gather = opA[0].gather;
      oa.grow = opA[0].grow;
      ob.half[0] = seg ? opB[1].half[0] : opB[0].half[0];
      ob.half[1] = seg ? opB[1].half[1] : opB[0].half[1];
      ob.ld = opB[0].ld;
      ob.valid[0] = opB[0].valid[0];
      ob.valid[1] = opB[0].valid[1];
      ob.gather = opB[0].gather;
      ob.grow = opB[0].grow;
      start(oa, ob);
      go(active, acc);
    }
  }
};

// ---- epilogue: accumulators -> LDS (fp32) -> 16-byte row-contiguous global accesses -----------------
// The products are accumulated transposed (mma() hands the MFMA the weight-side fragment as its first
// operand): of the 32x32 tile (mi, ni) a lane then holds tile row lane%32 and, for g = 0..3, the four
// consecutive columns 8g + 4*(lane/32) .. +3 in elements 4g .. 4g+3.  Each wave parks a 32-row strip of its
// sub-tile in its own quarter of the (now idle) LDS ring with 16-byte writes -- 4 per MFMA tile instead of
// 16 four-byte ones; a wave can have only 15 LDS operations outstanding and the other workgroup of the CU
// keeps the LDS busy, so the number of operations is what the epilogue costs -- and reads it back
// row-major, 8 consecutive columns per lane.
template <class T> struct Strip {
  static constexpr int LD = T::WN + 4;                 // floats per staged row: consecutive rows shift the banks by 4, so the 16 lanes
                                                       // the LDS serves per cycle (16 rows, 16 bytes each) cover all 64 banks
  static constexpr int kBytes = T::kStripBytes;
  static_assert(kBytes == 32 * LD * 4 && T::kStripBase + T::kWaves * kBytes <= T::kLdsAlloc, "staging strips must fit in the LDS allocation");
  static_assert(LD % 64 == 4, "bank rotation of the parked rows");
};

template <class T>
__device__ __forceinline__ void park_strip(const f32x16 (&acc_mi)[T::NI], float* strip, int lane) {
  float* row = strip + (lane & 31) * Strip<T>::LD + 4 * (lane >> 5);
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<float4*>(row + ni * 32 + 8 * g) =
          make_float4(acc_mi[ni][4 * g], acc_mi[ni][4 * g + 1], acc_mi[ni][4 * g + 2], acc_mi[ni][4 * g + 3]);
}

// The same for results that leave as bf16 with no further arithmetic: rounded before they are parked, so the strip
// holds 2 instead of 4 bytes per element and the LDS moves half the bytes both ways.  Rows are WN * 2 bytes with
// no padding; the 16-byte pieces of a row are XORed with the row index, which keeps the row-major 16-byte reads
// free of bank conflicts (16 lanes = 256 consecutive bytes) and spreads the 32 rows of a parking write over
// 16 different pieces.
template <class T>
__device__ __forceinline__ void park_strip_bf16(const f32x16 (&acc_mi)[T::NI], char* strip, int lane) {
  constexpr int PPR = T::WN / 8;                       // 16-byte pieces per staged row
  const int r = lane & 31;
  char* row = strip + r * (T::WN * 2) + 8 * (lane >> 5);
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<uint2*>(row + (((ni * 4 + g) ^ (r & (PPR - 1))) << 4)) =
          make_uint2(pack_bf16x2(acc_mi[ni][4 * g], acc_mi[ni][4 * g + 1]), pack_bf16x2(acc_mi[ni][4 * g + 2], acc_mi[ni][4 * g + 3]));
}
// 8 consecutive columns (piece `piece` of staged row `row`) of a strip parked by park_strip_bf16
template <class T>
__device__ __forceinline__ uint4 read_strip_bf16(const char* strip, int row, int piece) {
  return *reinterpret_cast<const uint4*>(strip + row * (T::WN * 2) + ((piece ^ (row & (T::WN / 8 - 1))) << 4));
}

// sum over each aligned group of LANES (8 or 16) consecutive lanes, left in every lane of the group; data-parallel
// primitives (register moves between lanes), fixed order of additions
template <int LANES>
__device__ __forceinline__ float row_group_sum(float v) {
  static_assert(LANES == 8 || LANES == 16, "groups of 8 or 16 lanes");
  auto dpp = [](float x, auto ctrl) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xF, 0xF, true));
  };
  v += dpp(v, std::integral_constant<int, 0xB1>{});          // quad_perm [1,0,3,2]
  v += dpp(v, std::integral_constant<int, 0x4E>{});          // quad_perm [2,3,0,1]
  v += dpp(v, std::integral_constant<int, 0x141>{});         // row_half_mirror: the other quad of the 8 lanes
  if constexpr (LANES == 16) v += dpp(v, std::integral_constant<int, 0x140>{});   // row_mirror: the other 8 lanes
  return v;
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

// Results are written once and read by a later kernel: a non-temporal store keeps them from displacing the
// operand panels that concurrently running tiles share through the L2 (measured: 2 % of the step).
__device__ __forceinline__ void store16(void* p, const uint4& v) {
  typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t*>(p));
}
__device__ __forceinline__ void store16(void* p, float a, float b, float c, float d) {
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  const f32x4_t w = {a, b, c, d};
  __builtin_nontemporal_store(w, reinterpret_cast<f32x4_t*>(p));
}

// ---- device-built schedule of (expert, row tile) for row-grouped products -----------------
struct RowTiles {
  int32_t* count;        // [1] number of row tiles
  int32_t* expert;       // [max_tiles]
  int32_t* row0;         // [max_tiles]
  int max_tiles;
  uint32_t* zeros;       // [64] block of zeros the GEMM kernels read for out-of-range reduction indices
};

__device__ __forceinline__ void build_row_tiles(const int32_t* __restrict__ offsets, int E, int P, int bm, RowTiles rt) {
  __shared__ int32_t scan[kMaxExperts];     // inclusive scan of the row tiles per expert
  __shared__ int32_t first_row[kMaxExperts];
  const int e = threadIdx.x;
  if (e < 64) rt.zeros[e] = 0u;
  int begin = 0, end = 0, nt = 0;
  if (e < E) {                                       // offsets == null: one segment holding all P rows
    begin = offsets ? min(max(offsets[e], 0), P) : 0;
    end = offsets ? min(max(offsets[e + 1], begin), P) : P;
    nt = (end - begin + bm - 1) / bm;
  }
  scan[e] = nt;
  first_row[e] = begin;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    int v = e >= o ? scan[e - o] : 0;
    __syncthreads();
    scan[e] += v;
    __syncthreads();
  }
  // offsets that are not a monotone scan ending at P cannot overflow the lists
  const int total = min(scan[1023], rt.max_tiles);
  // every thread writes the tiles t, t + 1024, ...: the expert of tile t is the first whose inclusive scan exceeds t
  for (int t = threadIdx.x; t < total; t += 1024) {
    int lo = 0, hi = E - 1;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (scan[mid] > t) hi = mid; else lo = mid + 1;
    }
    const int before = lo > 0 ? scan[lo - 1] : 0;
    rt.expert[t] = lo;
    rt.row0[t] = first_row[lo] + (t - before) * bm;
  }
  if (e == 1023) rt.count[0] = total;
}
__global__ __launch_bounds__(1024) void build_row_tiles_kernel(const int32_t* __restrict__ offsets, int E, int P,
                                                                int bm, RowTiles rt) {
  build_row_tiles(offsets, E, P, bm, rt);
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

// Hands back its argument through an empty asm: values derived from the result cannot be computed before
// this point, so the epilogue's per-lane indices do not occupy registers during the main loop.
__device__ __forceinline__ int not_before_here(int v) { asm volatile("" : "+v"(v)); return v; }

// ============================================================================================
// Row-grouped kernels
// ============================================================================================
enum { kGateUp = 0, kDown = 1, kDAct = 2, kDX = 3, kRouterFwd = 4, kRouterDx = 5 };

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
  bf16_t* out0;            // kGateUp: G (may be null)   kDown/kDX/kRouterDx: output     kDAct: [dG | dU]
  bf16_t* out1;            // kGateUp: U (may be null)
  bf16_t* out2;            // kGateUp: act (may be null)
  long ldo;
  float* out_f32;          // kRouterFwd: fp32 output
  int accumulate;          // kRouterDx: add to what out0 holds
  const bf16_t* g;         // kDAct: saved pre-activations
  const bf16_t* u;
  const bf16_t* zeros;     // at least 16 zero bytes (source of out-of-range reduction indices)
  // FUSED kernels: `a` is the token-major matrix [T, lda] and row r of the product reads a[row_token[r]]
  const int32_t* row_token;    // [P (+ padding)]
  const float* row_w;          // kDAct: combine weight of each row; the product's rows are scaled by it
                               // kGateUp (may be null): the activation leaves scaled by it
  bf16_t* act_w;               // kDAct: [P, N] out, row_w * silu(G) * U; null: not written (the forward left it)
  float* dw_partial;           // kDAct: [n_tiles_n * WGN][P] out, partial sums of <silu(G) * U, unscaled dA> per row
};

// FUSED (kGateUp and kDAct only): the activation rows are gathered from the token-major matrix while the
// tiles are loaded, so no expert-ordered copy of it exists.  For kDAct that matrix is the gradient of the
// layer output, and the rest of the combine backward rides in the epilogue:
//   dA = w_r * (dy[token(r)] Wd)              the combine weight scales the product's rows
//   d w_r = <dy[token(r)], yp[r]> = <dy[token(r)] Wd, act[r]>    reduced over the columns of the tile
//   act_w[r] = w_r * act[r]                   the operand with which dWd = dy[token]^T act_w needs no dyp
template <int KIND, class T, bool FUSED = false>
__global__ __launch_bounds__(T::kThreads) __attribute__((amdgpu_waves_per_eu(T::kWavesPerSimd, T::kWavesPerSimd))) void row_grouped_kernel(RowArgs p) {
  static_assert(!FUSED || KIND == kGateUp || KIND == kDAct, "only the two products that read activations by token are fused");
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int BM = T::BM, BN = T::BN, WM = T::WM, WN = T::WN, MI = T::MI, NI = T::NI;
  const int n_row_tiles = p.rt.count[0];
  const int v = xcd_remap(blockIdx.x, n_row_tiles * p.n_tiles_n);
  if (v < 0) return;
  const int mt = v / p.n_tiles_n, nt = v % p.n_tiles_n;
  const int e = p.rt.expert[mt];
  const int row0 = p.rt.row0[mt];
  const int row_end = p.offsets ? min(p.offsets[e + 1], p.P) : p.P;
  const int rows = min(BM, row_end - row0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / T::WGN, wn = wave % T::WGN;

  f32x16 acc[MI][NI];
  zero_acc<T>(acc);

  int a_row[MI];
#pragma unroll
  for (int i = 0; i < MI; ++i) a_row[i] = wm * WM + i * 32;
  // 32-row fragments of this wave that hold rows of the expert (wave-uniform); a wave without any
  // skips the arithmetic, and the epilogue skips strips without rows
  const int mi_n = __builtin_amdgcn_readfirstlane(min(MI, max(0, (rows - wm * WM + 31) / 32)));
  Operand opsA[2], opsB[2];
  Operand& opA = opsA[0];
  Operand& opB = opsB[0];
  opA.ld = p.lda;
  opA.valid[0] = min(rows, BM / 2);
  opA.valid[1] = max(rows - BM / 2, 0);
  opA.half[0] = FUSED ? p.a : p.a + static_cast<long>(row0) * p.lda;
  opA.half[1] = FUSED ? p.a : opA.half[0] + (BM / 2) * p.lda;
  opA.gather = FUSED ? p.row_token : nullptr;
  opA.grow = row0;
  opB.ld = p.ldw;
  opB.gather = nullptr;
  opB.grow = 0;

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
    static_assert(HI == 1, "the wave's gate fragment and its up fragment: two fragments BN/2 tile rows apart");
    { MainLoop<T, false, false, FUSED, false, HN> ml; ml.run(opsA, opsB, 1, p.K, lds, p.zeros, a_row, b_row, mi_n > 0, acc); }
    // strip columns: [0, HW) gate, [WN/2 + 0, ...) up -- both halves hold the same output columns
    float* strip = reinterpret_cast<float*>(lds + T::kStripBase + wave * Strip<T>::kBytes);
    const int el = not_before_here(lane);             // this lane, for the epilogue
    constexpr int LPR = HW / 8;                        // lanes per output row (8 columns each)
    constexpr int RPP = 64 / LPR;                      // rows per pass
    const int cl = wn * HW + (el % LPR) * 8;         // first of this lane's 8 columns inside the tile
    // All LDS reads of a strip are issued before the first is used: one LDS latency per strip, not per pass
    // (the other workgroup of the CU keeps the LDS busy, so that latency is several hundred cycles).
    constexpr int NP = 32 / RPP;                       // passes per strip
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      if (mi >= mi_n) break;
      park_strip<T>(acc[mi], strip, el);
      float g[NP][8], u[NP][8], wr[NP];
#pragma unroll
      for (int pass = 0; pass < NP; ++pass) {           // the rows' combine weights, if the activation is to carry them
        const int r = wm * WM + mi * 32 + pass * RPP + el / LPR;
        wr[pass] = p.row_w ? p.row_w[row0 + (r < rows ? r : 0)] : 1.0f;
      }
#pragma unroll
      for (int pass = 0; pass < NP; ++pass) {
        const int rs = pass * RPP + el / LPR;
        read8(strip + rs * Strip<T>::LD + (el % LPR) * 8, g[pass]);
        read8(strip + rs * Strip<T>::LD + WN / 2 + (el % LPR) * 8, u[pass]);
      }
#pragma unroll
      for (int pass = 0; pass < NP; ++pass) {
        const int r = wm * WM + mi * 32 + pass * RPP + el / LPR;
        if (cl < ncols && r < rows) {
          float a[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) a[q] = wr[pass] * (g[pass][q] * sigmoid_fast(g[pass][q]) * u[pass][q]);
          const long o = static_cast<long>(row0 + r) * p.ldo + n0 + cl;
          if (p.out0) store16(p.out0 + o, pack8(g[pass]));
          if (p.out1) store16(p.out1 + o, pack8(u[pass]));
          if (p.out2) store16(p.out2 + o, pack8(a));
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
    if constexpr (KIND == kDown || KIND == kRouterFwd) {
      // yp = act * Wd[e]^T (logits = x * Wr^T): weight rows are output columns, reduction contiguous
      opB.half[0] = p.w0 + e * p.w_expert_stride + static_cast<long>(n0) * p.ldw;
      opB.half[1] = opB.half[0] + (BN / 2) * p.ldw;
      { MainLoop<T, false, false> ml; ml.run(opsA, opsB, 1, p.K, lds, p.zeros, a_row, b_row, mi_n > 0, acc); }
    } else if constexpr (KIND == kDAct || KIND == kRouterDx) {
      // dA = dyp * Wd[e] (dx = dz * Wr): weight is [K, N], reduction strided
      opB.half[0] = p.w0 + e * p.w_expert_stride + n0;
      opB.half[1] = opB.half[0] + BN / 2;
      { MainLoop<T, false, true, FUSED, false> ml; ml.run(opsA, opsB, 1, p.K, lds, p.zeros, a_row, b_row, mi_n > 0, acc); }
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
      { MainLoop<T, false, true> ml; ml.run(opsA, opsB, 2, p.K, lds, p.zeros, a_row, b_row, mi_n > 0, acc); }
    }

    float* strip = reinterpret_cast<float*>(lds + T::kStripBase + wave * Strip<T>::kBytes);
    const int el = not_before_here(lane);             // this lane, for the epilogue
    constexpr int LPR = WN / 8;                        // lanes per output row (8 columns each)
    constexpr int RPP = 64 / LPR;                      // rows per pass
    const int cl = wn * WN + (el % LPR) * 8;         // first of this lane's 8 columns inside the tile
    // All LDS reads of a strip -- and, for the SwiGLU derivative, the loads of the saved G and U of the
    // strip -- are issued before the first is used: one latency per batch, not one per pass.
    constexpr int NP = 32 / RPP;                       // passes per strip
    if constexpr (KIND == kDAct) {
      constexpr int CH = NP;                           // passes per batch of G / U loads: the whole strip (the fragment registers are free now)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        if (mi >= mi_n) break;
        park_strip<T>(acc[mi], strip, el);
#pragma unroll
        for (int p0 = 0; p0 < NP; p0 += CH) {
          uint4 gq[CH], uq[CH];
          float v[CH][8], wr[CH];
#pragma unroll
          for (int c = 0; c < CH; ++c) {               // rows / columns that do not exist read the tile's first element
            const int r = wm * WM + mi * 32 + (p0 + c) * RPP + el / LPR;
            const long gi = static_cast<long>(row0 + (r < rows ? r : 0)) * p.N + n0 + (cl < ncols ? cl : 0);
            gq[c] = *reinterpret_cast<const uint4*>(p.g + gi);
            uq[c] = *reinterpret_cast<const uint4*>(p.u + gi);
            if constexpr (FUSED) wr[c] = p.row_w[row0 + (r < rows ? r : 0)];
          }
#pragma unroll
          for (int c = 0; c < CH; ++c)
            read8(strip + ((p0 + c) * RPP + el / LPR) * Strip<T>::LD + (el % LPR) * 8, v[c]);
#pragma unroll
          for (int c = 0; c < CH; ++c) {
            const int r = wm * WM + mi * 32 + (p0 + c) * RPP + el / LPR;
            const bool live = cl < ncols && r < rows;
            float g[8], u[8], dg[8], du[8];
            unpack8(gq[c], g);
            unpack8(uq[c], u);
            const long gi = static_cast<long>(row0 + r) * p.N + n0 + cl;
            const long o = static_cast<long>(row0 + r) * p.ldo + n0 + cl;
            if constexpr (FUSED) {
              float part = 0.0f, aw[8];
#pragma unroll
              for (int q = 0; q < 8; ++q) {
                const float sg = sigmoid_fast(g[q]);
                const float act = g[q] * sg * u[q];
                part = fmaf(act, v[c][q], part);
                const float da = wr[c] * v[c][q];
                dg[q] = da * u[q] * (sg * (1.0f + g[q] * (1.0f - sg)));
                du[q] = da * (g[q] * sg);
                aw[q] = wr[c] * act;
              }
              if (live) {
                store16(p.out0 + o, pack8(dg));
                store16(p.out0 + o + p.N, pack8(du));
                if (p.act_w) store16(p.act_w + gi, pack8(aw));
              } else {
                part = 0.0f;
              }
              // the LPR lanes of a row add up their columns; every (column slot, row) is written exactly once
              part = row_group_sum<LPR>(part);
              if (r < rows && el % LPR == 0) p.dw_partial[static_cast<long>(nt * T::WGN + wn) * p.P + row0 + r] = part;
            } else {
#pragma unroll
              for (int q = 0; q < 8; ++q) {
                const float sg = sigmoid_fast(g[q]);
                dg[q] = v[c][q] * u[q] * (sg * (1.0f + g[q] * (1.0f - sg)));
                du[q] = v[c][q] * (g[q] * sg);
              }
              if (live) {
                store16(p.out0 + o, pack8(dg));
                store16(p.out0 + o + p.N, pack8(du));
              }
            }
          }
        }
      }
      return;
    }
    if constexpr (KIND == kDown || KIND == kDX) {      // rounded and stored as they are: staged as bf16
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        if (mi >= mi_n) break;
        park_strip_bf16<T>(acc[mi], reinterpret_cast<char*>(strip), el);
        uint4 v[NP];
#pragma unroll
        for (int pass = 0; pass < NP; ++pass)
          v[pass] = read_strip_bf16<T>(reinterpret_cast<const char*>(strip), pass * RPP + el / LPR, el % LPR);
#pragma unroll
        for (int pass = 0; pass < NP; ++pass) {
          const int r = wm * WM + mi * 32 + pass * RPP + el / LPR;
          if (cl < ncols && r < rows) store16(p.out0 + static_cast<long>(row0 + r) * p.ldo + n0 + cl, v[pass]);
        }
      }
      return;
    }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      if (mi >= mi_n) break;
      park_strip<T>(acc[mi], strip, el);
      float v[NP][8];
#pragma unroll
      for (int pass = 0; pass < NP; ++pass)
        read8(strip + (pass * RPP + el / LPR) * Strip<T>::LD + (el % LPR) * 8, v[pass]);
#pragma unroll
      for (int pass = 0; pass < NP; ++pass) {
        const int r = wm * WM + mi * 32 + pass * RPP + el / LPR;
        if (cl < ncols && r < rows) {
          if constexpr (KIND == kRouterFwd) {
            float* o = p.out_f32 + static_cast<long>(row0 + r) * p.ldo + n0 + cl;
            store16(o, v[pass][0], v[pass][1], v[pass][2], v[pass][3]);
            store16(o + 4, v[pass][4], v[pass][5], v[pass][6], v[pass][7]);
          } else {                                     // kRouterDx
            bf16_t* o = p.out0 + static_cast<long>(row0 + r) * p.ldo + n0 + cl;
            if (p.accumulate) {
              float old[8];
              unpack8(*reinterpret_cast<const uint4*>(o), old);
#pragma unroll
              for (int q = 0; q < 8; ++q) v[pass][q] += old[q];
            }
            store16(o, pack8(v[pass]));
          }
        }
      }
    }
  }
}

// ============================================================================================
// Weight-gradient kernels: out[e] (M x N) = lhs[rows of e, M]^T * rhs[rows of e, N]
// Output rows below `m_split` go to out0[e], the rest to out1[e] (gate / up share one launch).
//
// The reduction runs over the rows of an expert, so its length follows the routing.  Under skewed
// routing a few experts own most rows; to keep every workgroup's share bounded, the rows of an expert
// are cut into chunks of at most `chunk_rows`, one work item per (chunk, output tile).  An expert with a
// single chunk is written directly.  The chunks of a split expert leave fp32 partial tiles in the
// workspace, and a second kernel adds them in chunk order and rounds once -- the same result on every
// run, unlike atomic accumulation.  Items are ordered by descending expert size so the long ones start first.
// ============================================================================================
struct WgradItems {
  int32_t* count;        // [2]: number of items, number of split experts
  int32_t* expert;       // [max_items]
  int32_t* k0;           // [max_items] first row of the chunk
  int32_t* k1;           // [max_items] one past its last row
  int32_t* slot;         // [max_items] partial-tile slot, or -1: write the result directly
  int32_t* split_expert; // [max_split]
  int32_t* split_slot0;  // [max_split]
  int32_t* split_n;      // [max_split]
  int max_items, max_split, max_slots;
};

__device__ __forceinline__ void build_wgrad_items(const int32_t* __restrict__ offsets, int E, int P, int chunk_rows, WgradItems it) {
  __shared__ int32_t cnt[kMaxExperts];      // rows per expert
  __shared__ int32_t order[kMaxExperts];    // expert at each rank (descending size, ties by index)
  __shared__ int32_t scan_items[kMaxExperts];
  __shared__ int32_t scan_slots[kMaxExperts];
  __shared__ int32_t scan_split[kMaxExperts];
  const int e = threadIdx.x;
  int begin = 0, c = -1;
  if (e < E) {                                       // offsets == null: one segment holding all P rows
    begin = offsets ? min(max(offsets[e], 0), P) : 0;
    c = (offsets ? min(max(offsets[e + 1], begin), P) : P) - begin;
  }
  cnt[e] = c;
  __syncthreads();
  if (e < E) {
    int rank = 0;
    for (int o = 0; o < E; ++o) rank += (cnt[o] > c || (cnt[o] == c && o < e)) ? 1 : 0;
    order[rank] = e;
  }
  __syncthreads();
  // thread r now speaks for the expert of rank r
  int my_e = -1, my_n = 0, my_c = 0;
  if (e < E) {
    my_e = order[e];
    my_c = cnt[my_e];
    my_n = max(1, (my_c + chunk_rows - 1) / chunk_rows);
  }
  const int split = my_n > 1 ? 1 : 0;
  scan_items[e] = my_n;
  scan_slots[e] = split ? my_n : 0;
  scan_split[e] = split;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    const int a = e >= o ? scan_items[e - o] : 0, b = e >= o ? scan_slots[e - o] : 0, d = e >= o ? scan_split[e - o] : 0;
    __syncthreads();
    scan_items[e] += a; scan_slots[e] += b; scan_split[e] += d;
    __syncthreads();
  }
  if (e < E) {
    const int first = scan_items[e] - my_n, slot0 = scan_slots[e] - (split ? my_n : 0), sidx = scan_split[e] - split;
    const int row0 = offsets ? min(max(offsets[my_e], 0), P) : 0;
    // the host sizes the lists for the worst case; offsets that are not a monotone scan ending at P cannot overflow them
    const bool fits = slot0 + my_n <= it.max_slots && sidx < it.max_split;
    for (int j = 0; j < my_n && first + j < it.max_items; ++j) {
      it.expert[first + j] = my_e;
      it.k0[first + j] = row0 + (fits || !split ? j * chunk_rows : 0);
      it.k1[first + j] = fits || !split ? row0 + min(my_c, (j + 1) * chunk_rows) : (j == 0 ? row0 + my_c : row0);
      it.slot[first + j] = split && fits ? slot0 + j : (split && j > 0 ? -2 : -1);   // -2: nothing to do
    }
    if (split && fits) {
      it.split_expert[sidx] = my_e;
      it.split_slot0[sidx] = slot0;
      it.split_n[sidx] = my_n;
    }
  }
  if (e == 1023) {
    it.count[0] = min(scan_items[1023], it.max_items);
    it.count[1] = min(scan_split[1023], it.max_split);
  }
}
__global__ __launch_bounds__(1024) void build_wgrad_items_kernel(const int32_t* __restrict__ offsets, int E, int P,
                                                                  int chunk_rows, WgradItems it) {
  build_wgrad_items(offsets, E, P, chunk_rows, it);
}

// entries of padding behind the list of row tokens: the scalar loads that run one slab ahead never leave it
constexpr int kRowTokenPad = 256;

// Everything a pass needs before its first product, in one launch: block 0 builds the (expert, row tile)
// list, block 1 the weight-gradient work items (backward only), the remaining blocks expand pair_of_row into
// the token (and combine weight) of every expert-ordered row (gathered passes only).
struct ScheduleArgs {
  const int32_t* offsets; int E, P;
  int bm; RowTiles rt;
  int chunk_rows; WgradItems items;      // chunk_rows == 0: no weight-gradient items
  const int32_t* pair_of_row;            // null: no row lists
  const float* topk_w; int T, k;
  int32_t* row_token; float* row_w;      // row_w may be null
};
__global__ __launch_bounds__(1024) void build_schedules_kernel(ScheduleArgs a) {
  if (blockIdx.x == 0) {
    build_row_tiles(a.offsets, a.E, a.P, a.bm, a.rt);
  } else if (blockIdx.x == 1) {
    if (a.chunk_rows > 0) build_wgrad_items(a.offsets, a.E, a.P, a.chunk_rows, a.items);
  } else {
    const int r = (blockIdx.x - 2) * 1024 + threadIdx.x;
    if (r >= a.P + kRowTokenPad) return;
    if (r >= a.P) { a.row_token[r] = 0; return; }
    const int pair = min(max(a.pair_of_row[r], 0), a.P - 1);
    a.row_token[r] = min(pair / a.k, a.T - 1);
    if (a.row_w) a.row_w[r] = a.topk_w[pair];
  }
}
static void launch_schedules(const ScheduleArgs& a, hipStream_t s) {
  const int blocks = 2 + (a.pair_of_row ? ceil_div(a.P + kRowTokenPad, 1024) : 0);
  MOE_LAUNCH("build_schedules", build_schedules_kernel, dim3(blocks), dim3(1024), 0, s, a);
}

struct WgradArgs {
  const bf16_t* lhs; long ld_lhs; int M;
  const bf16_t* rhs; long ld_rhs; int N;
  int E; int P;
  WgradItems items;
  int tiles_m, tiles_n;
  bf16_t* out0; bf16_t* out1; int m_split;     // out1 rows are (m - m_split)
  float* partial;                              // [max_slots][M][N]
  const bf16_t* zeros;     // at least 16 zero bytes
  const int32_t* row_token;    // GATHER kernels: [P + padding], token of each expert-ordered row
  // a side job of the reduction launch that follows dW_down in the gathered backward (null: none): the partial dot
  // products of the combine-weight gradient, one per (column slot, row), are added in slot order and scattered to [T, k]
  const float* dw_partial; int dw_slots; const int32_t* pair_of_row; float* dtopk_w;
};

// Column tiles one workgroup of a weight-gradient product takes in turn (see the kernel).  Measured in the layer
// step: two for [dW_gate; dW_up] (7 % faster at 512 rows per expert, no change at 2560), one for dW_down (with two
// or all three of its column tiles per workgroup it is 15-40 % slower).
template <class T, int WHICH> constexpr int kWgradSpan = (T::kWaves == 8 && T::BM == 256 && WHICH == 1) ? 2 : 1;

// WHICH 0: dW_down, 1: [dW_gate; dW_up], 2: router (separate symbols so profiles tell them apart).
// GATHER: the operand that holds one row per token -- lhs for WHICH 0 (the output gradient), rhs for WHICH 1
// (the layer input) -- is the token-major matrix itself, and reduction row r reads its row row_token[r].
template <int WHICH, class T, bool GATHER = false>
__global__ __launch_bounds__(T::kThreads) __attribute__((amdgpu_waves_per_eu(T::kWavesPerSimd, T::kWavesPerSimd))) void wgrad_kernel(WgradArgs p) {
  static_assert(!GATHER || WHICH < 2, "the router's operands are token-major already");
  constexpr bool GA = GATHER && WHICH == 0, GB = GATHER && WHICH == 1;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int BM = T::BM, BN = T::BN, WM = T::WM, WN = T::WN, MI = T::MI, NI = T::NI;
  // A workgroup takes kWgradSpan<T, WHICH> column tiles of one (work item, row tile) in turn: they share the lhs
  // panel, and where the staging strips sit behind the first stage the first slab of the next tile is
  // already on its way while the epilogue of the current one runs.
  constexpr int SPAN = kWgradSpan<T, WHICH>;
  const int spans_n = (p.tiles_n + SPAN - 1) / SPAN;
  const int per_e = p.tiles_m * spans_n;
  const int n_items = p.items.count[0];
  // order of a work item's tiles: row tile fastest for [dW_gate; dW_up] (neighbouring workgroups share the rhs panel;
  // measured 6 % faster at 512 rows per expert), column span fastest for the others
  constexpr bool MT_FASTEST = WHICH == 1;
  // Work items come sorted by length, so consecutive stretches of the list differ in work: they are dealt to the
  // XCDs (workgroup b runs on XCD b % 8) in turn, in units of 1/g of an item's tiles -- whole items while there
  // are at least 8 per XCD, otherwise g runs of the slow tile index, so that under skewed routing every XCD still
  // gets several units of the few long items.  A unit's workgroups are consecutive on their XCD (shared panels).
  const int slow = MT_FASTEST ? spans_n : p.tiles_m;
  int g = 1;
  while (g < slow && (n_items * g < 8 * kXcds || slow % g != 0)) ++g;
  const int per_u = per_e / g;                          // g divides slow, so it divides per_e
  const int unit = (blockIdx.x / kXcds) / per_u * kXcds + blockIdx.x % kXcds;
  if (unit >= n_items * g) return;
  const int item = unit / g;
  const int vi = (unit % g) * per_u + (blockIdx.x / kXcds) % per_u;   // position among the item's tiles
  const int mt = MT_FASTEST ? vi % p.tiles_m : vi / spans_n;
  const int nt0 = (MT_FASTEST ? vi / p.tiles_m : vi % spans_n) * SPAN;
  const int e = p.items.expert[item];
  const int slot = p.items.slot[item];
  if (slot == -2) return;
  const int begin = p.items.k0[item], end = p.items.k1[item];
  const int m0 = mt * BM;
  const int mrows = min(BM, p.M - m0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / T::WGN, wn = wave % T::WGN;

  f32x16 acc[MI][NI];
  int a_row[MI], b_row[NI];
#pragma unroll
  for (int i = 0; i < MI; ++i) a_row[i] = wm * WM + i * 32;
#pragma unroll
  for (int i = 0; i < NI; ++i) b_row[i] = wn * WN + i * 32;
  Operand opA, opB;
  opA.ld = p.ld_lhs;
  opA.half[0] = p.lhs + (GA ? 0L : static_cast<long>(begin) * p.ld_lhs) + m0;
  opA.half[1] = opA.half[0] + BM / 2;
  opA.valid[0] = min(mrows, BM / 2);
  opA.valid[1] = max(mrows - BM / 2, 0);
  opA.gather = GA ? p.row_token : nullptr;
  opA.grow = begin;
  opB.ld = p.ld_rhs;
  opB.gather = GB ? p.row_token : nullptr;
  opB.grow = begin;
  auto point_b = [&](int nt) {                         // rhs columns of column tile nt
    const int n0 = nt * BN, ncols = min(BN, p.N - n0);
    opB.half[0] = p.rhs + (GB ? 0L : static_cast<long>(begin) * p.ld_rhs) + n0;
    opB.half[1] = opB.half[0] + BN / 2;
    opB.valid[0] = min(ncols, BN / 2);
    opB.valid[1] = max(ncols - BN / 2, 0);
  };
  MainLoop<T, true, true, GA, GB> ml;
  ml.prepare(end - begin, lds, p.zeros, a_row, b_row);
  point_b(nt0);
  ml.start(opA, opB);

  float* strip = reinterpret_cast<float*>(lds + T::kStripBase + wave * Strip<T>::kBytes);
  constexpr int LPR = WN / 8;
  constexpr int RPP = 64 / LPR;
  float* part = slot >= 0 ? p.partial + static_cast<long>(slot) * p.M * p.N : nullptr;
  constexpr int NP = 32 / RPP;                         // passes per strip; all their LDS reads are issued before the first is used
#pragma nounroll
  for (int t = 0; t < SPAN; ++t) {
    const int nt = nt0 + t;
    if (nt >= p.tiles_n) break;
    const int n0 = nt * BN, ncols = min(BN, p.N - n0);
    zero_acc<T>(acc);
    ml.go(true, acc);
    const bool more = t + 1 < SPAN && nt + 1 < p.tiles_n;
    if (more) point_b(nt + 1);
    const int el = not_before_here(lane);             // this lane, for the epilogue
    const int cl = wn * WN + (el % LPR) * 8;
    if (part) {                                        // chunk of a split expert: fp32 partial tile
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        park_strip<T>(acc[mi], strip, el);
        float v[NP][8];
#pragma unroll
        for (int pass = 0; pass < NP; ++pass)
          read8(strip + (pass * RPP + el / LPR) * Strip<T>::LD + (el % LPR) * 8, v[pass]);
#pragma unroll
        for (int pass = 0; pass < NP; ++pass) {
          const int rl = wm * WM + mi * 32 + pass * RPP + el / LPR;
          if (cl < ncols && rl < mrows) {
            float* o = part + static_cast<long>(m0 + rl) * p.N + n0 + cl;
            store16(o, v[pass][0], v[pass][1], v[pass][2], v[pass][3]);
            store16(o + 4, v[pass][4], v[pass][5], v[pass][6], v[pass][7]);
          }
        }
      }
    } else {                                           // whole expert: rounded once, staged as bf16
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        park_strip_bf16<T>(acc[mi], reinterpret_cast<char*>(strip), el);
        uint4 v[NP];
#pragma unroll
        for (int pass = 0; pass < NP; ++pass)
          v[pass] = read_strip_bf16<T>(reinterpret_cast<const char*>(strip), pass * RPP + el / LPR, el % LPR);
#pragma unroll
        for (int pass = 0; pass < NP; ++pass) {
          const int rl = wm * WM + mi * 32 + pass * RPP + el / LPR;
          if (cl < ncols && rl < mrows) {
            const int m = m0 + rl;
            bf16_t* out = m < p.m_split ? p.out0 + (static_cast<long>(e) * p.m_split + m) * p.N
                                        : p.out1 + (static_cast<long>(e) * (p.M - p.m_split) + (m - p.m_split)) * p.N;
            store16(out + n0 + cl, v[pass]);
          }
        }
      }
    }
    if (more) {
      __syncthreads();                                 // every wave is done with its strip: the rings may be refilled
      ml.start(opA, opB);
    }
  }
}

// out[e] = bf16( sum over the chunks of a split expert, in chunk order, of its fp32 partial tiles )
// (with balanced routing there are no split experts, and the launch is blocks that read one counter and leave)
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(WgradArgs p) {
  if (p.dw_partial) {                                  // dtopk_w[pair_of_row[r]] = sum over the column slots, in slot order
    for (int r = blockIdx.x * 256 + threadIdx.x; r < p.P; r += gridDim.x * 256) {
      float s = 0.0f;
      for (int j = 0; j < p.dw_slots; ++j) s += p.dw_partial[static_cast<long>(j) * p.P + r];
      p.dtopk_w[min(max(p.pair_of_row[r], 0), p.P - 1)] = s;
    }
  }
  // every (split expert, 8 outputs) pair is one unit of a single grid-strided loop: the launch is latency-bound (a unit is
  // one round of loads and one store), so the split experts are reduced side by side, not one after the other
  const int n_split = p.items.count[1];
  const long mn = static_cast<long>(p.M) * p.N, per = mn / 8;          // N is a multiple of 8: a unit lies in one row
  for (long unit = static_cast<long>(blockIdx.x) * 256 + threadIdx.x; unit < n_split * per; unit += static_cast<long>(gridDim.x) * 256) {
    const int s = static_cast<int>(unit / per);
    const long i = (unit - s * per) * 8;
    const int e = p.items.split_expert[s], n = p.items.split_n[s];
    const float* part = p.partial + static_cast<long>(p.items.split_slot0[s]) * mn;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < n; j += 4) {                       // four partial tiles requested together, added in slot order
      float v[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) read8(part + min(j + u, n - 1) * mn + i, v[u]);   // past the last slot: re-read it, not added
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (j + u < n) {
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[q] += v[u][q];
        }
      }
    }
    const int m = static_cast<int>(i / p.N), col = static_cast<int>(i % p.N);
    bf16_t* out = m < p.m_split ? p.out0 + (static_cast<long>(e) * p.m_split + m) * p.N
                                : p.out1 + (static_cast<long>(e) * (p.M - p.m_split) + (m - p.m_split)) * p.N;
    store16(out + col, pack8(acc));
  }
}

// ============================================================================================
// Host side
// ============================================================================================
// Tile shapes in use.
//   TileBig: 256 x 256 outputs, 64-wide slabs, one 8-wave workgroup per CU (2 x 4 wavefronts of 128 x 64), two
//     stages of 64 KiB.  A slab row is a whole 128-byte line: the fewest L2 requests per flop that fit the CU.
//   TileBigW16: the TileBig ring under 16 waves (4 x 4 of 64 x 64, four per SIMD, 128 VGPRs) for the weight
//     gradients: both their operands are read transposed (twice the LDS read instructions per MFMA), and four
//     waves per SIMD cover that better -- 3-5 % faster on dW_down at every size and on [dW_gate; dW_up] from
//     about 1000 rows per expert; the row products are 2-5 % slower with it and keep 8 waves.
//   TileRouter: 64 x 128 x 64 for the skinny products with N = E, two workgroups per CU.
typedef Tile<256, 256, 64, 2, 4, 2, 3> TileBig;
typedef Tile<256, 256, 64, 4, 4, 2, 3> TileBigW16;
typedef Tile<64, 128, 64, 2, 2, 3, 3> TileRouter;

static int row_bm() { return TileBig::BM; }
// bound used for workspace sizing: the smallest row tile gives the longest list
static int max_row_tiles(int P, int E) { return ceil_div(P, 128) + E; }

// Rows per reduction chunk of the weight gradients: long enough that the fp32 partial tiles stay a small
// part of the traffic, short enough that the largest work item is a small part of the launch.  At most
// 2 * ceil(P / chunk) <= 64 partial slots can ever be needed (an expert is split only if it has more than
// one chunk, and the chunks of split experts hold more than half their rows each but the last).  The floor of
// 2048 rows is the measured optimum when 16 experts share 16K rows with two thirds of them on one expert
// (1024: a third more partial traffic; 3072: too few work items per XCD).
static int wgrad_chunk_rows(int P) { return std::max(2048, static_cast<int>(align_up(static_cast<size_t>(ceil_div(P, 32)), 256))); }
static int wgrad_max_items(int P, int E, int chunk) { return E + ceil_div(P, chunk); }
static int wgrad_max_split(int P, int E, int chunk) { return std::max(1, std::min(E, ceil_div(P, chunk))); }
static int wgrad_max_slots(int P, int chunk) { return 2 * ceil_div(P, chunk); }
static int wgrad_max_items(int P, int E) { return wgrad_max_items(P, E, wgrad_chunk_rows(P)); }
static int wgrad_max_split(int P, int E) { return wgrad_max_split(P, E, wgrad_chunk_rows(P)); }
static int wgrad_max_slots(int P) { return wgrad_max_slots(P, wgrad_chunk_rows(P)); }
// The router's weight gradient has a single "expert" of all T rows and only E x d outputs: shorter chunks
// (at least 64 of them) so that the launch fills the chip.
static int router_chunk_rows(int T) { return std::max(256, static_cast<int>(align_up(static_cast<size_t>(ceil_div(T, 64)), 256))); }

struct WsLayout {
  size_t tiles_count, zeros, tiles_expert, tiles_row0, dgu, g, u, items, partial, total;
};
static WsLayout ws_layout(int P, int d, int f, int E, bool need_dgu, bool need_gu) {
  WsLayout w{};
  size_t off = 0;
  w.tiles_count = off; off += 256;
  w.zeros = off; off += 256;
  const size_t t = align_up(static_cast<size_t>(max_row_tiles(P, E)) * sizeof(int32_t), 256);
  w.tiles_expert = off; off += t;
  w.tiles_row0 = off; off += t;
  const size_t pf = align_up(static_cast<size_t>(P) * f * 2, 256);
  w.dgu = off; if (need_dgu) off += 2 * pf;
  w.g = off; if (need_gu) off += pf;
  w.u = off; if (need_gu) off += pf;
  w.items = off; w.partial = off;
  if (need_dgu) {                                      // backward only: weight-gradient schedule and partial tiles
    const size_t it = align_up(static_cast<size_t>(wgrad_max_items(P, E)) * sizeof(int32_t), 256);
    const size_t sp = align_up(static_cast<size_t>(wgrad_max_split(P, E)) * sizeof(int32_t), 256);
    off += 256 + 4 * it + 3 * sp;
    w.partial = off;
    off += align_up(static_cast<size_t>(wgrad_max_slots(P)) * 2 * f * d * sizeof(float), 256);
  }
  w.total = off + 256;
  return w;
}

size_t ffn_fwd_ws_bytes_bf16(int P, int d, int f, int E) { return ws_layout(P, d, f, E, false, false).total; }
size_t ffn_bwd_ws_bytes_bf16(int P, int d, int f, int E, int have_saved) {
  return ws_layout(P, d, f, E, true, !have_saved).total;
}

static RowTiles row_tiles_at(void* ws, const WsLayout& w, int P, int E) {
  char* b = static_cast<char*>(ws);
  RowTiles rt;
  rt.max_tiles = max_row_tiles(P, E);
  rt.count = reinterpret_cast<int32_t*>(b + w.tiles_count);
  rt.zeros = reinterpret_cast<uint32_t*>(b + w.zeros);
  rt.expert = reinterpret_cast<int32_t*>(b + w.tiles_expert);
  rt.row0 = reinterpret_cast<int32_t*>(b + w.tiles_row0);
  return rt;
}

static WgradItems wgrad_items_at(void* ws, const WsLayout& w, int P, int E) {
  char* b = static_cast<char*>(ws) + w.items;
  WgradItems it;
  it.max_items = wgrad_max_items(P, E);
  it.max_split = wgrad_max_split(P, E);
  it.max_slots = wgrad_max_slots(P);
  const size_t li = align_up(static_cast<size_t>(it.max_items) * sizeof(int32_t), 256);
  const size_t ls = align_up(static_cast<size_t>(it.max_split) * sizeof(int32_t), 256);
  it.count = reinterpret_cast<int32_t*>(b); b += 256;
  it.expert = reinterpret_cast<int32_t*>(b); b += li;
  it.k0 = reinterpret_cast<int32_t*>(b); b += li;
  it.k1 = reinterpret_cast<int32_t*>(b); b += li;
  it.slot = reinterpret_cast<int32_t*>(b); b += li;
  it.split_expert = reinterpret_cast<int32_t*>(b); b += ls;
  it.split_slot0 = reinterpret_cast<int32_t*>(b); b += ls;
  it.split_n = reinterpret_cast<int32_t*>(b);
  return it;
}

// A kernel that needs more than 64 KiB of dynamic LDS has to be granted it once per device.  Each kernel has its
// own set of flags (a static of its launcher's template instance); the status is kept, and a failure is reported
// through the call's launch status instead of surfacing later as an opaque launch error.
constexpr int kMaxDevices = 64;
struct LdsGrant { std::once_flag once[kMaxDevices]; hipError_t status[kMaxDevices] = {}; };
static bool allow_lds(LdsGrant& g, const void* kernel, int bytes, const char* name) {
  int dev = 0;
  hipError_t err = hipGetDevice(&dev);
  if (err == hipSuccess && (dev < 0 || dev >= kMaxDevices)) err = hipErrorInvalidDevice;
  if (err == hipSuccess) {
    std::call_once(g.once[dev], [&] { g.status[dev] = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); });
    err = g.status[dev];
  }
  if (err != hipSuccess) note_hip_failure(name, err);
  return err == hipSuccess;
}

static unsigned padded_grid(int tiles) { return static_cast<unsigned>(ceil_div(tiles < 1 ? 1 : tiles, kXcds) * kXcds); }

template <int KIND, class T, bool FUSED = false>
static void launch_row_t(RowArgs p, int P, int E, hipStream_t s) {
  static const char* const names[6] = {"ffn_gate_up", "ffn_down", "ffn_dact", "ffn_dx", "router_logits", "router_dx"};
  static LdsGrant grant;
  if (!allow_lds(grant, reinterpret_cast<const void*>(&row_grouped_kernel<KIND, T, FUSED>), T::kLdsAlloc, names[KIND])) return;
  p.n_tiles_n = ceil_div(p.N, KIND == kGateUp ? T::BN / 2 : T::BN);
  const unsigned grid = padded_grid((ceil_div(P, T::BM) + E) * p.n_tiles_n);
  MOE_LAUNCH(names[KIND], (row_grouped_kernel<KIND, T, FUSED>), dim3(grid), dim3(T::kThreads), T::kLdsAlloc, s, p);
}

template <int KIND, bool FUSED = false>
static void launch_row(const RowArgs& p, int P, int E, hipStream_t s) {
  launch_row_t<KIND, TileBig, FUSED>(p, P, E, s);
}

template <int WHICH, class T, bool GATHER = false>
static void launch_wgrad_t(WgradArgs p, hipStream_t s) {
  static LdsGrant grant;
  if (!allow_lds(grant, reinterpret_cast<const void*>(&wgrad_kernel<WHICH, T, GATHER>), T::kLdsAlloc, "wgrad")) return;
  p.tiles_m = ceil_div(p.M, T::BM);
  p.tiles_n = ceil_div(p.N, T::BN);
  // units are dealt to the XCDs in groups of 8, the last group may be partial: up to 8 more units than items
  const unsigned grid = padded_grid(p.tiles_m * ceil_div(p.tiles_n, kWgradSpan<T, WHICH>) * (p.items.max_items + kXcds));
  MOE_LAUNCH(WHICH == 0 ? "wgrad_down" : WHICH == 1 ? "wgrad_gate_up" : "wgrad_router", (wgrad_kernel<WHICH, T, GATHER>), dim3(grid),
             dim3(T::kThreads), T::kLdsAlloc, s, p);
  // the reduction loops are grid-strided: a launch with nothing to reduce (balanced routing) should cost as little as a launch can
  // (room for two split experts per pass of the loop; more only repeat it)
  const long rblocks = std::max(2 * ((static_cast<long>(p.M) * p.N + 2047) / 2048), p.dw_partial ? (static_cast<long>(p.P) + 255) / 256 : 1L);
  const dim3 rgrid(static_cast<unsigned>(std::min(rblocks, 2048L)));
  MOE_LAUNCH(WHICH == 0 ? "wgrad_down_reduce" : WHICH == 1 ? "wgrad_gate_up_reduce" : "wgrad_router_reduce", wgrad_reduce_kernel, rgrid,
             dim3(256), 0, s, p);
}

template <int WHICH, bool GATHER = false>
static void launch_wgrad(const WgradArgs& p, hipStream_t s) {
  // [dW_gate; dW_up] with short reductions is faster with TileBig's paired column tiles
  if (WHICH == 0 || (WHICH == 1 && p.P >= 1536L * p.E)) {
    if constexpr (WHICH < 2) launch_wgrad_t<WHICH, TileBigW16, GATHER>(p, s);
  } else {
    launch_wgrad_t<WHICH, TileBig, GATHER>(p, s);
  }
}

// row_token == null: xp is in expert order; else xp is the token-major input and rows are gathered from it
static void launch_gate_up(const void* xp, const void* wg, const void* wu, int P, int d, int f, int E,
                           const int32_t* offsets, const RowTiles& rt, void* G, void* U, void* act, hipStream_t s,
                           const int32_t* row_token = nullptr, const float* row_w = nullptr) {
  RowArgs p{};
  p.row_token = row_token;
  p.row_w = row_w;
  p.a = static_cast<const bf16_t*>(xp); p.lda = d;
  p.w0 = static_cast<const bf16_t*>(wg); p.w1 = static_cast<const bf16_t*>(wu);
  p.w_expert_stride = static_cast<long>(f) * d; p.ldw = d;
  p.K = d; p.N = f; p.offsets = offsets; p.P = P; p.rt = rt; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
  p.out0 = static_cast<bf16_t*>(G); p.out1 = static_cast<bf16_t*>(U); p.out2 = static_cast<bf16_t*>(act); p.ldo = f;
  if (row_token) launch_row<kGateUp, true>(p, P, E, s);
  else launch_row<kGateUp>(p, P, E, s);
}

static void launch_down(const void* act, const void* wd, int P, int d, int f, int E, const int32_t* offsets,
                        const RowTiles& rt, void* yp, hipStream_t s) {
  RowArgs p{};
  p.a = static_cast<const bf16_t*>(act); p.lda = f;
  p.w0 = static_cast<const bf16_t*>(wd); p.w_expert_stride = static_cast<long>(d) * f; p.ldw = f;
  p.K = f; p.N = d; p.offsets = offsets; p.P = P; p.rt = rt; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
  p.out0 = static_cast<bf16_t*>(yp); p.ldo = d;
  launch_row<kDown>(p, P, E, s);
}

static void launch_dx(const bf16_t* dgu, const void* wg, const void* wu, int P, int d, int f, int E, const int32_t* offsets,
                      const RowTiles& rt, void* dxp, hipStream_t s) {
  RowArgs p{};
  p.a = dgu; p.lda = 2L * f;
  p.w0 = static_cast<const bf16_t*>(wg); p.w1 = static_cast<const bf16_t*>(wu);
  p.w_expert_stride = static_cast<long>(f) * d; p.ldw = d;
  p.K = f; p.N = d; p.offsets = offsets; p.P = P; p.rt = rt; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
  p.out0 = static_cast<bf16_t*>(dxp); p.ldo = d;
  launch_row<kDX>(p, P, E, s);
}

void ffn_fwd_bf16(const FfnFwdArgs& a) {
  const WsLayout w = ws_layout(a.P, a.d, a.f, a.E, false, false);
  const RowTiles rt = row_tiles_at(a.ws, w, a.P, a.E);
  MOE_LAUNCH("build_row_tiles", build_row_tiles_kernel, dim3(1), dim3(1024), 0, a.stream, a.offsets, a.E, a.P, row_bm(), rt);
  launch_gate_up(a.xp, a.w_gate, a.w_up, a.P, a.d, a.f, a.E, a.offsets, rt, a.g_save, a.u_save, a.act, a.stream);
  launch_down(a.act, a.w_down, a.P, a.d, a.f, a.E, a.offsets, rt, a.yp, a.stream);
}

void ffn_bwd_bf16(const FfnBwdArgs& a) {
  const bool recompute = a.g_save == nullptr;
  const WsLayout w = ws_layout(a.P, a.d, a.f, a.E, true, recompute);
  const RowTiles rt = row_tiles_at(a.ws, w, a.P, a.E);
  char* base = static_cast<char*>(a.ws);
  bf16_t* dgu = reinterpret_cast<bf16_t*>(base + w.dgu);       // [P, 2f] = [dG | dU]
  const bf16_t* G = static_cast<const bf16_t*>(a.g_save);
  const bf16_t* U = static_cast<const bf16_t*>(a.u_save);
  const WgradItems items = wgrad_items_at(a.ws, w, a.P, a.E);
  {
    ScheduleArgs sa{};
    sa.offsets = a.offsets; sa.E = a.E; sa.P = a.P; sa.bm = row_bm(); sa.rt = rt;
    sa.chunk_rows = wgrad_chunk_rows(a.P); sa.items = items;
    launch_schedules(sa, a.stream);
  }
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
    p.K = a.d; p.N = a.f; p.offsets = a.offsets; p.P = a.P; p.rt = rt; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
    p.out0 = dgu; p.ldo = 2L * a.f; p.g = G; p.u = U;
    launch_row<kDAct>(p, a.P, a.E, a.stream);
  }
  launch_dx(dgu, a.w_gate, a.w_up, a.P, a.d, a.f, a.E, a.offsets, rt, a.dxp, a.stream);   // dxp = dG Wg + dU Wu
  float* partial = reinterpret_cast<float*>(base + w.partial);
  {  // dWd[e] = dyp^T act
    WgradArgs p{};
    p.lhs = static_cast<const bf16_t*>(a.dyp); p.ld_lhs = a.d; p.M = a.d;
    p.rhs = static_cast<const bf16_t*>(a.act); p.ld_rhs = a.f; p.N = a.f;
    p.E = a.E; p.P = a.P; p.items = items; p.partial = partial; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
    p.out0 = static_cast<bf16_t*>(a.dw_down); p.out1 = p.out0; p.m_split = a.d;
    launch_wgrad<0>(p, a.stream);
  }
  {  // [dWg[e]; dWu[e]] = [dG | dU]^T xp
    WgradArgs p{};
    p.lhs = dgu; p.ld_lhs = 2L * a.f; p.M = 2 * a.f;
    p.rhs = static_cast<const bf16_t*>(a.xp); p.ld_rhs = a.d; p.N = a.d;
    p.E = a.E; p.P = a.P; p.items = items; p.partial = partial; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
    p.out0 = static_cast<bf16_t*>(a.dw_gate); p.out1 = static_cast<bf16_t*>(a.dw_up); p.m_split = a.f;
    launch_wgrad<1>(p, a.stream);
  }
}

// ============================================================================================
// The same two passes without the expert-ordered copies of the layer input and of the output gradient
// (the dispatch / return of Sec. 3.2.3 folded into the products that consume the rows):
//   forward   G, U, act, yp as above, rows read as x[token(r)]                              (no xp)
//   backward  dA = w_r dy[token(r)] Wd,  dWd = dy[token]^T (w act),  d w = <dy[token] Wd, act>,
//             [dWg; dWu] = [dG | dU]^T x[token]                                             (no dyp, no yp)
// token(r) = pair_of_row[r] / k and w_r = topk_w[pair_of_row[r]] are expanded once per call into two
// row-indexed lists; the list of tokens is padded so that the scalar loads that run one slab ahead of the
// weight-gradient products never leave it.
// ============================================================================================

// column slots of the partial dot products: one per (column tile, wavefront column) of the dA product
static int dw_slots(int f) { return ceil_div(f, TileBig::BN) * TileBig::WGN; }

struct GatherWs { size_t row_token, row_w, act_w, dw_partial, total; };
static GatherWs gather_ws(const WsLayout& w, int P, int f, bool bwd) {
  GatherWs g{};
  size_t off = w.total;
  g.row_token = off; off += align_up(static_cast<size_t>(P + kRowTokenPad) * sizeof(int32_t), 256);
  g.row_w = off; off += align_up(static_cast<size_t>(P) * sizeof(float), 256);
  g.act_w = off; g.dw_partial = off;
  if (bwd) {
    g.act_w = off; off += align_up(static_cast<size_t>(P) * f * 2, 256);
    g.dw_partial = off; off += align_up(static_cast<size_t>(dw_slots(f)) * P * sizeof(float), 256);
  }
  g.total = off;
  return g;
}
size_t ffn_fwd_gather_ws_bytes_bf16(int P, int d, int f, int E) {
  return gather_ws(ws_layout(P, d, f, E, false, false), P, f, false).total;
}
size_t ffn_bwd_gather_ws_bytes_bf16(int P, int d, int f, int E, int have_saved) {
  return gather_ws(ws_layout(P, d, f, E, true, !have_saved), P, f, true).total;
}

void ffn_fwd_gather_bf16(const FfnFwdGatherArgs& a) {
  const WsLayout w = ws_layout(a.P, a.d, a.f, a.E, false, false);
  const GatherWs g = gather_ws(w, a.P, a.f, false);
  const RowTiles rt = row_tiles_at(a.ws, w, a.P, a.E);
  int32_t* row_token = reinterpret_cast<int32_t*>(static_cast<char*>(a.ws) + g.row_token);
  float* row_w = reinterpret_cast<float*>(static_cast<char*>(a.ws) + g.row_w);
  {
    ScheduleArgs sa{};
    sa.offsets = a.offsets; sa.E = a.E; sa.P = a.P; sa.bm = row_bm(); sa.rt = rt;
    sa.pair_of_row = a.pair_of_row; sa.T = a.T; sa.k = a.k; sa.row_token = row_token;
    if (a.topk_w) { sa.topk_w = a.topk_w; sa.row_w = row_w; }
    launch_schedules(sa, a.stream);
  }
  launch_gate_up(a.x, a.w_gate, a.w_up, a.P, a.d, a.f, a.E, a.offsets, rt, a.g_save, a.u_save, a.act, a.stream, row_token,
                 a.topk_w ? row_w : nullptr);
  launch_down(a.act, a.w_down, a.P, a.d, a.f, a.E, a.offsets, rt, a.yp, a.stream);
}

void ffn_bwd_gather_bf16(const FfnBwdGatherArgs& a) {
  const bool recompute = a.g_save == nullptr;
  const WsLayout w = ws_layout(a.P, a.d, a.f, a.E, true, recompute);
  const GatherWs gw = gather_ws(w, a.P, a.f, true);
  const RowTiles rt = row_tiles_at(a.ws, w, a.P, a.E);
  char* base = static_cast<char*>(a.ws);
  bf16_t* dgu = reinterpret_cast<bf16_t*>(base + w.dgu);       // [P, 2f] = [dG | dU]
  int32_t* row_token = reinterpret_cast<int32_t*>(base + gw.row_token);
  float* row_w = reinterpret_cast<float*>(base + gw.row_w);
  bf16_t* act_w_ws = reinterpret_cast<bf16_t*>(base + gw.act_w);
  const bf16_t* act_w = a.act_w ? static_cast<const bf16_t*>(a.act_w) : act_w_ws;
  float* dw_partial = reinterpret_cast<float*>(base + gw.dw_partial);
  const bf16_t* G = static_cast<const bf16_t*>(a.g_save);
  const bf16_t* U = static_cast<const bf16_t*>(a.u_save);
  const WgradItems items = wgrad_items_at(a.ws, w, a.P, a.E);
  {
    ScheduleArgs sa{};
    sa.offsets = a.offsets; sa.E = a.E; sa.P = a.P; sa.bm = row_bm(); sa.rt = rt;
    sa.chunk_rows = wgrad_chunk_rows(a.P); sa.items = items;
    sa.pair_of_row = a.pair_of_row; sa.topk_w = a.topk_w; sa.T = a.T; sa.k = a.k; sa.row_token = row_token; sa.row_w = row_w;
    launch_schedules(sa, a.stream);
  }
  if (recompute) {
    bf16_t* Gr = reinterpret_cast<bf16_t*>(base + w.g);
    bf16_t* Ur = reinterpret_cast<bf16_t*>(base + w.u);
    launch_gate_up(a.x, a.w_gate, a.w_up, a.P, a.d, a.f, a.E, a.offsets, rt, Gr, Ur, nullptr, a.stream, row_token);
    G = Gr; U = Ur;
  }
  {  // dA = w (dy[token] Wd) with the SwiGLU derivative, the weight gradient's dot products and w * act
    RowArgs p{};
    p.a = static_cast<const bf16_t*>(a.dy); p.lda = a.d;
    p.w0 = static_cast<const bf16_t*>(a.w_down); p.w_expert_stride = static_cast<long>(a.d) * a.f; p.ldw = a.f;
    p.K = a.d; p.N = a.f; p.offsets = a.offsets; p.P = a.P; p.rt = rt; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
    p.out0 = dgu; p.ldo = 2L * a.f; p.g = G; p.u = U;
    p.row_token = row_token; p.row_w = row_w; p.act_w = a.act_w ? nullptr : act_w_ws; p.dw_partial = dw_partial;
    launch_row<kDAct, true>(p, a.P, a.E, a.stream);
  }
  launch_dx(dgu, a.w_gate, a.w_up, a.P, a.d, a.f, a.E, a.offsets, rt, a.dxp, a.stream);
  float* partial = reinterpret_cast<float*>(base + w.partial);
  {  // dWd[e] = dy[token]^T (w act)
    WgradArgs p{};
    p.lhs = static_cast<const bf16_t*>(a.dy); p.ld_lhs = a.d; p.M = a.d;
    p.rhs = act_w; p.ld_rhs = a.f; p.N = a.f;
    p.E = a.E; p.P = a.P; p.items = items; p.partial = partial; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
    p.out0 = static_cast<bf16_t*>(a.dw_down); p.out1 = p.out0; p.m_split = a.d;
    p.row_token = row_token;
    p.dw_partial = dw_partial; p.dw_slots = dw_slots(a.f); p.pair_of_row = a.pair_of_row; p.dtopk_w = a.dtopk_w;   // rides in the reduction launch
    launch_wgrad<0, true>(p, a.stream);
  }
  {  // [dWg[e]; dWu[e]] = [dG | dU]^T x[token]
    WgradArgs p{};
    p.lhs = dgu; p.ld_lhs = 2L * a.f; p.M = 2 * a.f;
    p.rhs = static_cast<const bf16_t*>(a.x); p.ld_rhs = a.d; p.N = a.d;
    p.E = a.E; p.P = a.P; p.items = items; p.partial = partial; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
    p.out0 = static_cast<bf16_t*>(a.dw_gate); p.out1 = static_cast<bf16_t*>(a.dw_up); p.m_split = a.f;
    p.row_token = row_token;
    launch_wgrad<1, true>(p, a.stream);
  }
}

// ============================================================================================
// Router linear (the gate that produces the logits) and its backward, on the same skeleton:
//   logits[T, E] (fp32)  = x[T, d] * Wr[E, d]^T          one segment of T rows, fp32 epilogue
//   dx[T, d]   (+)=  bf16(dz)[T, E] * Wr[E, d]           reduction over E, optional read-modify-write
//   dWr[E, d]       =  bf16(dz)[T, E]^T * x[T, d]         reduction over the T rows, chunked like the others
// The fp32 logit gradient is rounded to bf16 once for the two backward products (bf16 operands,
// fp32 accumulation, like every other product here).
// ============================================================================================
__global__ __launch_bounds__(256) void cast_f32_bf16_kernel(const float* __restrict__ in, bf16_t* __restrict__ out, long n8) {
  const long i = static_cast<long>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n8) return;
  float v[8];
  read8(in + i * 8, v);
  store16(out + i * 8, pack8(v));
}

struct RouterWs { size_t tiles_count, zeros, tiles_expert, tiles_row0, dz, items, partial, total; };
static RouterWs router_ws(int T, int d, int E, bool bwd) {
  RouterWs w{};
  size_t off = 0;
  w.tiles_count = off; off += 256;
  w.zeros = off; off += 256;
  const size_t t = align_up(static_cast<size_t>(ceil_div(T, 64) + 1) * sizeof(int32_t), 256);   // row tiles of 64 or 128 rows
  w.tiles_expert = off; off += t;
  w.tiles_row0 = off; off += t;
  w.dz = off; w.items = off; w.partial = off;
  if (bwd) {
    off += align_up(static_cast<size_t>(T) * E * 2, 256);
    w.items = off;
    const int chunk = router_chunk_rows(T);
    const size_t it = align_up(static_cast<size_t>(wgrad_max_items(T, 1, chunk)) * sizeof(int32_t), 256);
    const size_t sp = align_up(static_cast<size_t>(wgrad_max_split(T, 1, chunk)) * sizeof(int32_t), 256);
    off += 256 + 4 * it + 3 * sp;
    w.partial = off;
    off += align_up(static_cast<size_t>(wgrad_max_slots(T, chunk)) * E * d * sizeof(float), 256);
  }
  w.total = off + 256;
  return w;
}
size_t router_fwd_ws_bytes_bf16(int T, int d, int E) { return router_ws(T, d, E, false).total; }
size_t router_bwd_ws_bytes_bf16(int T, int d, int E) { return router_ws(T, d, E, true).total; }

static RowTiles router_tiles_at(void* ws, const RouterWs& w, int T) {
  char* b = static_cast<char*>(ws);
  RowTiles rt;
  rt.max_tiles = ceil_div(T, 64) + 1;
  rt.count = reinterpret_cast<int32_t*>(b + w.tiles_count);
  rt.zeros = reinterpret_cast<uint32_t*>(b + w.zeros);
  rt.expert = reinterpret_cast<int32_t*>(b + w.tiles_expert);
  rt.row0 = reinterpret_cast<int32_t*>(b + w.tiles_row0);
  return rt;
}

void router_fwd_bf16(const RouterFwdArgs& a) {
  const RouterWs w = router_ws(a.T, a.d, a.E, false);
  const RowTiles rt = router_tiles_at(a.ws, w, a.T);
  MOE_LAUNCH("build_row_tiles", build_row_tiles_kernel, dim3(1), dim3(1024), 0, a.stream, static_cast<const int32_t*>(nullptr), 1, a.T,
             TileRouter::BM, rt);
  RowArgs p{};
  p.a = static_cast<const bf16_t*>(a.x); p.lda = a.d;
  p.w0 = static_cast<const bf16_t*>(a.w_router); p.w_expert_stride = 0; p.ldw = a.d;
  p.K = a.d; p.N = a.E; p.offsets = nullptr; p.P = a.T; p.rt = rt; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
  p.out_f32 = a.logits; p.ldo = a.E;
  launch_row_t<kRouterFwd, TileRouter>(p, a.T, 1, a.stream);
}

void router_bwd_bf16(const RouterBwdArgs& a) {
  const RouterWs w = router_ws(a.T, a.d, a.E, true);
  const RowTiles rt = router_tiles_at(a.ws, w, a.T);
  char* base = static_cast<char*>(a.ws);
  bf16_t* dz = reinterpret_cast<bf16_t*>(base + w.dz);
  const long n8 = static_cast<long>(a.T) * a.E / 8;
  MOE_LAUNCH("router_cast_dz", cast_f32_bf16_kernel, dim3(static_cast<unsigned>((n8 + 255) / 256)), dim3(256), 0, a.stream, a.dlogits, dz, n8);
  MOE_LAUNCH("build_row_tiles", build_row_tiles_kernel, dim3(1), dim3(1024), 0, a.stream, static_cast<const int32_t*>(nullptr), 1, a.T,
             row_bm(), rt);
  {  // dx (+)= dz * Wr
    RowArgs p{};
    p.a = dz; p.lda = a.E;
    p.w0 = static_cast<const bf16_t*>(a.w_router); p.w_expert_stride = 0; p.ldw = a.d;
    p.K = a.E; p.N = a.d; p.offsets = nullptr; p.P = a.T; p.rt = rt; p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
    p.out0 = static_cast<bf16_t*>(a.dx); p.ldo = a.d; p.accumulate = a.accumulate;
    launch_row<kRouterDx>(p, a.T, 1, a.stream);
  }
  {  // dWr = dz^T x
    WgradItems items;
    {
      char* b = base + w.items;
      items.max_items = wgrad_max_items(a.T, 1, router_chunk_rows(a.T));
      items.max_split = wgrad_max_split(a.T, 1, router_chunk_rows(a.T));
      items.max_slots = wgrad_max_slots(a.T, router_chunk_rows(a.T));
      const size_t li = align_up(static_cast<size_t>(items.max_items) * sizeof(int32_t), 256);
      const size_t ls = align_up(static_cast<size_t>(items.max_split) * sizeof(int32_t), 256);
      items.count = reinterpret_cast<int32_t*>(b); b += 256;
      items.expert = reinterpret_cast<int32_t*>(b); b += li;
      items.k0 = reinterpret_cast<int32_t*>(b); b += li;
      items.k1 = reinterpret_cast<int32_t*>(b); b += li;
      items.slot = reinterpret_cast<int32_t*>(b); b += li;
      items.split_expert = reinterpret_cast<int32_t*>(b); b += ls;
      items.split_slot0 = reinterpret_cast<int32_t*>(b); b += ls;
      items.split_n = reinterpret_cast<int32_t*>(b);
    }
    MOE_LAUNCH("build_wgrad_items", build_wgrad_items_kernel, dim3(1), dim3(1024), 0, a.stream, static_cast<const int32_t*>(nullptr), 1, a.T,
               router_chunk_rows(a.T), items);
    WgradArgs p{};
    p.lhs = dz; p.ld_lhs = a.E; p.M = a.E;
    p.rhs = static_cast<const bf16_t*>(a.x); p.ld_rhs = a.d; p.N = a.d;
    p.E = 1; p.P = a.T; p.items = items; p.partial = reinterpret_cast<float*>(base + w.partial);
    p.zeros = reinterpret_cast<const bf16_t*>(rt.zeros);
    p.out0 = static_cast<bf16_t*>(a.dw_router); p.out1 = p.out0; p.m_split = a.E;
    launch_wgrad<2>(p, a.stream);
  }
}

// ============================================================================================
// Forward products with 8-bit block-scaled operands (same tiles, loaders and staging strips)
// ============================================================================================
#include "gemm_mx8.inc"

}  // namespace moe
