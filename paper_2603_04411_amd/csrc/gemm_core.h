// MFMA macro-tile main loop shared by every contraction of the library (gfx950).
//
// All contractions (logits, logits recompute for dZ, dH, dW; the KV path's spectral projection,
// gate logits and ragged reconstruction) are brought to the same form
// C[m][n] = sum_k A[m][k] * B[n][k]  with both operands K-contiguous.
// A workgroup owns a BM x BN tile of C; each wavefront owns a (BM/WGM) x (BN/WGN)
// sub-tile built from 16x16 (bf16, e4m3) or 32x32 (fp32) MFMA blocks.
//
// Data movement: K is consumed 128 bytes per row per step (64 bf16 or 32 fp32), i.e. one
// full cache line per row: the vector L1 moves one 128-byte line per ~2 clocks whether or
// not all of it is used, so half-line steps would halve the load throughput.  Tiles go
// from global memory straight into LDS (buffer_load_dwordx4 ... lds, no register staging).
// LDS is a ring of five 32 KB slots, each holding one operand's tile for one K-step; the
// units A(0) B(0) A(1) B(1) ... (or B first) go round the ring, so besides the two units being
// multiplied, three are resident or in flight.  The hand-over barrier of K-step k (in the middle
// of the step for the two-sub-step loops, three quarters in for the four-sub-step loop) frees the
// slots of K-step k's two units, and a wave puts them to use straight away, so no slot is ever
// idle: the operand that leads the ring has one to one and a half K-steps to land before the
// barrier that hands it over, the other half a K-step to a whole one.  Loads go one behind every
// few MFMAs: the vector L1 then never sees a burst (a burst backs up the address queue and blocks
// the wave's in-order issue, MFMAs included).
// One workgroup barrier per K-step; a unit is complete when each wave's own vmcnt has
// drained past it (loads retire in order) and all waves have passed that barrier.
//
// LDS slot layout: 256 rows of 128 bytes (eight 16-byte chunks); chunk c of row r sits at chunk
// position c ^ swz(r) of its row, and the rows of the five slots are interleaved by groups of 8
// (see GSTR below).  A direct-to-LDS load writes lane L's 16 bytes at wave_base + 16 L, i.e. row
// L/8, position L%8 of an 8-row group, so lane L simply fetches the global chunk (L%8) ^ swz(row).
//
// Fragment layout used for both operands (what matters is only that A and B agree): the wave tile
// is cut into NB x NB MFMA blocks; lane l of a block holds row l % NB and, in K sub-step s, the
// 16-byte chunk (64 / NB) * s + l / NB of the row's 128-byte K slice.
//   bf16: NB = 16, v_mfma_f32_16x16x32_bf16, two sub-steps per K-step.  Per flop this form moves half
//         the accumulator data of the 32x32x16 form, and the part is power-limited: on static random
//         operands a bare loop of it sustains 2092 TFLOP/s against 1843 for 32x32x16 (2447 / 2482 on
//         zeros).  -DLMHEAD_BF16_BLOCK=32 builds the 32x32x16 form (four sub-steps) for comparison.
//   fp32: NB = 32, the chunk's four floats feed four v_mfma_f32_32x32x2_f32, four sub-steps.
//   e4m3: NB = 16, v_mfma_f32_16x16x128_f8f6f4: one MFMA takes the whole K-step of a block pair, two chunks per
//         lane (lane group g holds chunks 2g and 2g + 1).  Like the bf16 form it moves half the accumulator data
//         of its 32x32 counterpart (32x32x64) per flop; measured on the 32x8x2048 workload the forward gained 6 %
//         and the dZ kernel 5 % over a two-sub-step loop on 32x32x64.
// Fragments are double-buffered in registers (e4m3: one set, refilled behind its last reader) and the hand-over
// barrier is skewed so that the MFMAs after it overlap the first fragment reads of the next K-step and the
// issue of the next loads.
//
// Accumulator layout of a block (NB * NB / 64 floats per lane); a lane owns one column n = l % NB:
//   NB = 32: element v of lane l  <->  m = 8*(v/4) + 4*(l/32) + v%4   (16 values)
//   NB = 16: element v of lane l  <->  m = 4*(l/16) + v               (4 values)
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "tile_map.h"

namespace lmhead {

// Per-workgroup time stamps, compiled in only with -DLMHEAD_TRACE (a diagnostic build; nothing below costs an
// instruction otherwise).  Lane 0 of wave 0 of workgroup b < 2^19 writes stamp k into word 16 b + k of a buffer the
// host hands over with lmhead_debug_set_trace: trace_stamp the 100 MHz real-time counter, trace_cycles the shader
// clock counter into the second half of the buffer (word 16 (2^19 + b) + k), so that the pair gives the clock
// frequency over a section (words 11-13 there hold the hardware ids and the tile coordinates of a forward tile).
// One kernel records at a time (g_trace_kind); GemmTile::run() is told its caller's kind.  Each translation unit
// has its own copy of the two variables; only the one next to the LM-head kernels is ever set, the others stay
// null and record nothing.
#ifdef LMHEAD_TRACE
constexpr unsigned kTraceWorkgroups = 1u << 19;
static __device__ unsigned long long* g_trace;
static __device__ int g_trace_kind;      // which kernel records: 1 forward, 2 dZ, 3 dH, 4 dW
__device__ inline void trace_stamp(int k, int kind) {
  if (g_trace && g_trace_kind == kind && threadIdx.x == 0 && blockIdx.x < kTraceWorkgroups)
    g_trace[(size_t)blockIdx.x * 16 + k] = __builtin_amdgcn_s_memrealtime();
}
__device__ inline void trace_cycles(int k, int kind) {
  if (g_trace && g_trace_kind == kind && threadIdx.x == 0 && blockIdx.x < kTraceWorkgroups)
    g_trace[((size_t)kTraceWorkgroups + blockIdx.x) * 16 + k] = __builtin_readcyclecounter();
}
#else
__device__ inline void trace_stamp(int, int) {}
__device__ inline void trace_cycles(int, int) {}
#endif

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

typedef __attribute__((ext_vector_type(8))) int i32x8_t;

struct bf16_tag {};
struct f32_tag {};
struct fp8_tag {};   // OCP e4m3 operands (logits only), fp32 accumulation

template <typename E>
struct Elem;
#ifndef LMHEAD_BF16_BLOCK
#define LMHEAD_BF16_BLOCK 16
#endif
template <>
struct Elem<bf16_tag> {
  static constexpr int size = 2;
  static constexpr int dtype = 1;
  static constexpr int block = LMHEAD_BF16_BLOCK;   // MFMA block edge: 16 (16x16x32) or 32 (32x32x16)
  static constexpr int frag_chunks = 1;   // 16-byte chunks of K per lane and MFMA group
  static constexpr int mfma_per_block = 1;
  using acc_t = std::conditional<block == 16, f32x4_t, f32x16_t>::type;
  __device__ static inline void mma(f32x16_t& c, const u32x4_t (&a)[1], const u32x4_t (&b)[1]) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[0]),
                                                __builtin_bit_cast(bf16x8_t, b[0]), c, 0, 0, 0);
  }
  // Written as an asm statement with the accumulator tied to one AGPR tuple: with the builtin the
  // register allocator does not keep sixty-four 4-register accumulators in place across the loop
  // (hundreds of v_accvgpr moves per K-step, and spills).  The compiler then neither knows the
  // instruction's latency nor counts it as an MFMA for scheduling hints: the main loop for this
  // form spells out its interleave in program order, and run_rows() ends with the wait states
  // that reading a just-written accumulator needs.
  __device__ static inline void mma(f32x4_t& c, const u32x4_t (&a)[1], const u32x4_t (&b)[1]) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a[0]), "v"(b[0]));
  }
};
template <>
struct Elem<f32_tag> {
  static constexpr int size = 4;
  static constexpr int dtype = 0;
  static constexpr int block = 32;
  static constexpr int frag_chunks = 1;
  static constexpr int mfma_per_block = 4;
  using acc_t = f32x16_t;
  __device__ static inline void mma(f32x16_t& c, const u32x4_t (&a)[1], const u32x4_t (&b)[1]) {
    // whole-vector casts, then named components: element-wise bit casts of a[q] are avoided
    const f32x4_t fa = __builtin_bit_cast(f32x4_t, a[0]);
    const f32x4_t fb = __builtin_bit_cast(f32x4_t, b[0]);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.x, fb.x, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.y, fb.y, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.z, fb.z, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.w, fb.w, c, 0, 0, 0);
  }
};

template <>
struct Elem<fp8_tag> {
  static constexpr int size = 1;
  static constexpr int block = 16;
  static constexpr int frag_chunks = 2;   // 32 bytes = 32 e4m3 values of K per lane
  static constexpr int mfma_per_block = 1;
  using acc_t = f32x4_t;
  // v_mfma_f32_16x16x128_f8f6f4 with both formats e4m3 (format code 0, the default) and no block scaling:
  // one instruction consumes a whole 128-byte K-step of a 16-row block.  Lane l supplies row l % 16 and 32 of
  // the 128 K values; which 32 does not matter as long as both operands are cut the same way (here: the
  // 16-byte chunks 2 (l / 16) and 2 (l / 16) + 1 of the K-step).  An asm statement for the same reason as the
  // bf16 form above: sixty-four 4-register accumulators that must stay in their AGPR tuples.
  __device__ static inline void mma(f32x4_t& c, const i32x8_t& a, const i32x8_t& b) {
    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
  }
  // the same from two 16-byte chunks per operand (the form the generic fragment arrays hold)
  __device__ static inline void mma(f32x4_t& c, const u32x4_t (&a)[2], const u32x4_t (&b)[2]) {
    const i32x8_t va = {(int)a[0].x, (int)a[0].y, (int)a[0].z, (int)a[0].w, (int)a[1].x, (int)a[1].y, (int)a[1].z, (int)a[1].w};
    const i32x8_t vb = {(int)b[0].x, (int)b[0].y, (int)b[0].z, (int)b[0].w, (int)b[1].x, (int)b[1].y, (int)b[1].z, (int)b[1].w};
    mma(c, va, vb);
  }
};

// s_waitcnt immediates (gfx9 encoding): only the named counter is constrained.
constexpr int wait_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }
constexpr int kWaitVm0 = wait_vm(0);
constexpr int kWaitLgkm0 = 0xC07F;

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits until every global
// store issued before it has completed; the epilogues stage a tile through LDS in phases and
// stream it out with global stores that nothing in the workgroup reads back, so they keep those
// stores in flight across the barrier instead.
__device__ inline void lds_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
}

// kLeadB selects which operand goes first round the LDS ring (see run()).
// kMaskB: every B row has its own K extent (ragged rows); loads past it fetch zeros (see run()).
template <typename E, int BM_, int BN_, int WGM_, int WGN_, bool kLeadB = false, bool kMaskB = false>
struct GemmTile {
  static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
  static constexpr int NWAVES = WGM * WGN;
  static constexpr int NT = 64 * NWAVES;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int NB = Elem<E>::block;           // edge of an MFMA block
  static constexpr int LG = 64 / NB;                  // lane groups of a block (each holds other K chunks / rows)
  static constexpr int VB = NB * NB / 64;             // accumulator values per lane and block
  static constexpr int TM = WM / NB, TN = WN / NB;
  static constexpr int KB = 128;                      // bytes of K per row per step (a cache line)
  static constexpr int FC = Elem<E>::frag_chunks;     // 16-byte chunks per lane and fragment
  static constexpr int NSUB = KB / 16 / (LG * FC);    // K sub-steps (one fragment pair each)
  static constexpr int NSLOT = 5;                     // ring of operand-tile slots
  static constexpr int SLOT = (BM > BN ? BM : BN) * KB;
  static constexpr int LDS_BYTES = NSLOT * SLOT;
  // The slots are interleaved in LDS by groups of 8 rows (1 KB, what one load instruction writes):
  // group g of slot s sits at (g * NSLOT + s) KB.  A fragment's address is then a lane-dependent part
  // that does not depend on the slot plus s KB, which fits the DS instructions' immediate offset.
  static constexpr int SSTR = 8 * KB;                 // from a slot to the next, within a row group
  static constexpr int GSTR = NSLOT * SSTR;           // from a row group to the next
  __device__ static inline int row_off(int r) { return (r >> 3) * GSTR + (r & 7) * KB; }
  static constexpr int A_LD = BM / 8 / NWAVES;        // direct-to-LDS load instructions per wave
  static constexpr int B_LD = BN / 8 / NWAVES;        // per K-step (each moves 8 rows)
  static constexpr int LOADS_PER_STEP = A_LD + B_LD;
  static_assert(BM % (WGM * NB) == 0 && BN % (WGN * NB) == 0, "wave tiles are made of MFMA blocks");
  static_assert(NB == 32 || NB == 16, "block edge");
  static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "tile loads divide evenly");
  static_assert(NSUB == 1 || NSUB % 2 == 0, "fragment double-buffering assumes an even number of sub-steps");

  using Block = typename Elem<E>::acc_t;
  using Acc = Block[TM][TN];

  __device__ static inline int lane() { return threadIdx.x & 63; }
  __device__ static inline int wave() { return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }
  __device__ static inline int wave_m() { return wave() % WGM; }
  __device__ static inline int wave_n() { return wave() / WGM; }
  // Tile-relative coordinates of accumulator element v of block (i, j).
  __device__ static inline int m_of(int i, int v) { return m_base() + m_const(i, v); }
  // m_of split into its lane-dependent part and a compile-time constant, so that comparisons
  // against it can be written with immediates instead of one live register per (i, v)
  __device__ static inline int m_base() { return wave_m() * WM + 4 * (lane() / NB); }
  __device__ static constexpr int m_const(int i, int v) {
    return NB == 32 ? i * 32 + 8 * (v >> 2) + (v & 3) : i * 16 + v;
  }
  __device__ static inline int n_of(int j) { return wave_n() * WN + j * NB + (lane() % NB); }

  __device__ static inline int swz(int r) { return (r ^ (r >> 3)) & 7; }

  // Tile row that this lane fetches in the wave's q-th load of A (or B), and the byte offset
  // inside that row's 128-byte K slice that it must fetch to realise the swizzled layout.
  __device__ static inline int ldA_row(int q) { return (wave() * A_LD + q) * 8 + (lane() >> 3); }
  __device__ static inline int ldB_row(int q) { return (wave() * B_LD + q) * 8 + (lane() >> 3); }
  __device__ static inline int ld_byte(int row) { return ((lane() & 7) ^ swz(row)) << 4; }

  __device__ static inline void zero(Acc& acc) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < VB; ++v) acc[i][j][v] = 0.f;
  }

  // The asm-statement MFMAs are invisible to the compiler's hazard recognizer: it inserts no wait states
  // between an instruction that writes an accumulator register (the zero fill, which it is free to sink
  // right in front of the first use) and an MFMA that reads it as its addend.  Called once before the first
  // such MFMA: every accumulator is forced into its AGPR tuple here (asm statements keep their order), and
  // the wait states follow.
  __device__ static inline void settle(Acc& acc) {
    if constexpr (NB == 16) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) asm volatile("" : "+a"(acc[i][j]));
      asm volatile("s_nop 7");
    }
  }

  // acc += A_tile * B_tile^T over `ksteps` steps of 128 bytes.
  // A / B: uniform pointers to the tile's first row at K offset 0.  offA[q] / offB[q]: this
  // lane's byte offset from that pointer for its q-th load: (row, already clamped by the caller,
  // relative to the tile's first row) * pitch + ld_byte(row).
  // `lds` must provide LDS_BYTES bytes.  Returns with every wave past a barrier and no load
  // in flight, so LDS may be reused by the caller right away.
  // kLeadB selects which operand goes first round the ring, i.e. which one is loaded a full K-step
  // or more ahead (the other has half a K-step to a K-step): false = A, true = B.  Give the long
  // lead to the operand that misses L2 more often (the one fewer concurrent workgroups share).
  __device__ static inline void run(Acc& acc, const char* __restrict__ A, const uint32_t (&offA)[A_LD],
                                    const char* __restrict__ B, const uint32_t (&offB)[B_LD],
                                    int ksteps, char* lds, int trace_kind = 0) {
    static_assert(!kMaskB, "ragged rows need their limits");
    const int none[B_LD] = {};
    run_rows(acc, A, offA, B, offB, none, 0x7fffffffu, ksteps, lds, trace_kind);
  }

  // Same, with B given as one buffer of `bytesB` bytes (at most 2^31) that holds rows of differing
  // K extent: offB[q] is the byte offset of this lane's chunk of its row at K-step 0, and with
  // kMaskB the load of K-step ks is taken only while ks * KB < limB[q] (limB[q] = the row's extent
  // in bytes, a multiple of 16, minus the lane's byte position in the step); otherwise the lane
  // asks for an offset outside the buffer, which the hardware range check turns into zeros in
  // LDS without touching memory.
  __device__ static inline void run_rows(Acc& acc, const char* __restrict__ A, const uint32_t (&offA)[A_LD],
                                         const char* __restrict__ B, const uint32_t (&offB)[B_LD],
                                         const int (&limB)[B_LD], uint32_t bytesB, int ksteps, char* lds,
                                         int trace_kind = 0) {
    typedef __attribute__((address_space(3))) void* lptr_t;
    const int w = wave();
    const int l = lane();
    const int grp = l / NB;
    const int rA0 = wave_m() * WM + (l % NB);
    const int rB0 = wave_n() * WN + (l % NB);

    // Loads of one operand tile for K-step ks into ring slot `slot`; `part` selects which of
    // the NPART groups of this wave's load instructions to issue.
    constexpr int NPART = 2;
    static_assert(A_LD % NPART == 0 && B_LD % NPART == 0, "loads split evenly over the regions");
    // Raw buffer descriptors over each operand tile: base = the tile's first row, 2 GiB window,
    // so a load needs one 32-bit VGPR offset (row * pitch + byte) and a scalar K offset.
    // The tile pointers are wave-uniform by construction; saying so explicitly keeps the
    // descriptors in SGPRs (otherwise every load is wrapped in a readfirstlane loop).
    auto uniform_ptr = [](const char* p) {
      const uint64_t v = reinterpret_cast<uint64_t>(p);
      const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
      const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
      return reinterpret_cast<void*>(((uint64_t)hi << 32) | lo);
    };
    const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(A), 0, 0x7fffffff, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc(
        uniform_ptr(B), 0, (int)__builtin_amdgcn_readfirstlane(bytesB), 0x00020000);
    auto issue_a = [&](int ks, int slot, int part) {
      char* st = lds + slot * SSTR;
#pragma unroll
      for (int q = part * (A_LD / NPART); q < (part + 1) * (A_LD / NPART); ++q)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lptr_t)(st + (w * A_LD + q) * GSTR), 16, offA[q], ks * KB, 0, 0);
    };
    auto issue_b = [&](int ks, int slot, int part) {
      char* st = lds + slot * SSTR;
#pragma unroll
      for (int q = part * (B_LD / NPART); q < (part + 1) * (B_LD / NPART); ++q) {
        uint32_t vo = offB[q];
        if constexpr (kMaskB) vo = (ks * KB < limB[q]) ? vo : 0x80000000u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB, (lptr_t)(st + (w * B_LD + q) * GSTR), 16, vo, ks * KB, 0, 0);
      }
    };

    u32x4_t fa[2][TM][FC], fb[2][TN][FC];
    auto read_a = [&](const char* sa, int s, int buf) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int r = rA0 + i * NB;
#pragma unroll
        for (int c = 0; c < FC; ++c) {
          const int ch = (LG * s + grp) * FC + c;
          fa[buf][i][c] = *reinterpret_cast<const u32x4_t*>(sa + row_off(r) + ((ch ^ swz(r)) << 4));
        }
      }
    };
    auto read_b = [&](const char* sb, int s, int buf) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int r = rB0 + j * NB;
#pragma unroll
        for (int c = 0; c < FC; ++c) {
          const int ch = (LG * s + grp) * FC + c;
          fb[buf][j][c] = *reinterpret_cast<const u32x4_t*>(sb + row_off(r) + ((ch ^ swz(r)) << 4));
        }
      }
    };
    auto read_frags = [&](const char* sa, const char* sb, int s, int buf) {
      read_a(sa, s, buf);
      read_b(sb, s, buf);
    };
    // MFMAs of the row blocks [i0, i1) of the wave tile
    auto mma_rows = [&](int buf, int i0, int i1) {
#pragma unroll
      for (int i = i0; i < i1; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) Elem<E>::mma(acc[i][j], fa[buf][i], fb[buf][j]);
    };
    auto mma_all = [&](int buf) { mma_rows(buf, 0, TM); };

    // Scheduling hints: behind each MFMA of a region one fragment read, and behind every
    // (MMAS / loads)-th MFMA one global->LDS load, so that nothing leaves the matrix pipe idle.
    constexpr int kDsRead = 0x100, kVmem = 0x010, kMfma = 0x008;
    constexpr int MMAS = TM * TN * Elem<E>::mfma_per_block;
    constexpr int FR = TM + TN;
    constexpr int LD_REGION = A_LD / NPART;     // loads per region (A_LD == B_LD is not required
    constexpr int LD_REGION_B = B_LD / NPART;   // but both are spread the same way)
    static_assert(MMAS - (FR + 1) / 2 >= LD_REGION && MMAS - (FR + 1) / 2 >= LD_REGION_B, "region too short");
    // (program order is reads, loads, MFMAs; the loads must stay behind the reads because both
    // touch LDS, so the reads go two per MFMA up front and the loads are spread over the rest)
    auto sched_region = [&](int nloads) {
      constexpr int RD_SLOTS = (FR + 1) / 2;
#pragma unroll
      for (int i = 0; i < MMAS; ++i) {
        __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        if (i < RD_SLOTS) {
          if (i == RD_SLOTS - 1 && (FR & 1))
            __builtin_amdgcn_sched_group_barrier(kDsRead, 1, 0);
          else
            __builtin_amdgcn_sched_group_barrier(kDsRead, 2, 0);
        }
        if (nloads > 0 && i >= RD_SLOTS) {
          const int gap = (MMAS - RD_SLOTS) / nloads;
          const int j = i - RD_SLOTS + 1;
          if (j % gap == 0 && j / gap <= nloads) __builtin_amdgcn_sched_group_barrier(kVmem, 1, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    auto next_slot = [](int s, int by) { s += by; return s >= NSLOT ? s - NSLOT : s; };
    // X = the operand that leads the ring, Y = the other one
    static_assert(A_LD == B_LD, "the ring treats both operands' load counts alike");
    auto issue_x = [&](int ks, int slot, int part) {
      if constexpr (kLeadB) issue_b(ks, slot, part); else issue_a(ks, slot, part);
    };
    auto issue_y = [&](int ks, int slot, int part) {
      if constexpr (kLeadB) issue_a(ks, slot, part); else issue_b(ks, slot, part);
    };
    auto frags_xy = [&](const char* cx, const char* cy, int s, int buf) {
      if constexpr (kLeadB) read_frags(cy, cx, s, buf); else read_frags(cx, cy, s, buf);
    };

    if (ksteps <= 0) return;
    if constexpr (NSUB == 4) {
      // ring state: slots of X(ks) and Y(ks); unit u lives in slot u % NSLOT
      int sA = 0, sB = 1;
      issue_x(0, 0, 0); issue_x(0, 0, 1);
      issue_y(0, 1, 0); issue_y(0, 1, 1);
      if (ksteps > 1) {
        issue_x(1, 2, 0); issue_x(1, 2, 1);
        issue_y(1, 3, 0);
        __builtin_amdgcn_s_waitcnt(wait_vm(A_LD + A_LD / NPART));
      } else {
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
      }
      __builtin_amdgcn_s_barrier();
      frags_xy(lds + sA * SSTR, lds + sB * SSTR, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      int ks = 0;
      // Steady state.  Entering K-step ks: X(ks), Y(ks), X(ks+1) and the first half of Y(ks+1) are
      // resident or in flight; the slot of Y(ks-1) is free.  The barrier near the end of the step
      // frees the slots of X(ks) and Y(ks), and the first of them is put to use at once (Y(ks+2)),
      // so no slot is ever idle: Y has half a K-step to a whole one to land, X one to one and a half.
      for (; ks + 2 < ksteps; ++ks) {
        const char* ca = lds + sA * SSTR;
        const char* cb = lds + sB * SSTR;
        const int sB1 = next_slot(sB, 2);   // slot of Y(ks+1) == slot of X(ks-1)
        const int sA1 = next_slot(sA, 2);   // slot of X(ks+1)
        const int sA2 = next_slot(sA1, 2);  // slot of X(ks+2) == slot of Y(ks-1)
        // sub-step 0: second half of Y(ks+1)
        frags_xy(ca, cb, 1, 1);
        issue_y(ks + 1, sB1, 1);
        mma_all(0);
        sched_region(LD_REGION_B);
        // sub-steps 1 and 2: X(ks+2)
        frags_xy(ca, cb, 2, 0);
        issue_x(ks + 2, sA2, 0);
        mma_all(1);
        sched_region(LD_REGION);
        frags_xy(ca, cb, 3, 1);
        issue_x(ks + 2, sA2, 1);
        mma_all(0);
        sched_region(LD_REGION);
        // hand-over: everything but X(ks+2), this wave's youngest A_LD loads, has landed
        __builtin_amdgcn_s_waitcnt(wait_vm(A_LD));
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // sub-step 3 overlaps the first fragment reads of K-step ks+1 and the first half of Y(ks+2),
        // which goes into the slot of X(ks) that this barrier has just freed
        frags_xy(lds + sA1 * SSTR, lds + sB1 * SSTR, 0, 0);
        issue_y(ks + 2, sA, 0);
        mma_all(1);
        sched_region(LD_REGION_B);
        sA = sA1;
        sB = sB1;
      }
      // drain: the last two K-steps (the first half of Y(ks+1) is already under way)
      for (; ks < ksteps; ++ks) {
        const char* ca = lds + sA * SSTR;
        const char* cb = lds + sB * SSTR;
        const int sB1 = next_slot(sB, 2);
        const int sA1 = next_slot(sA, 2);
        const bool more = ks + 1 < ksteps;
        frags_xy(ca, cb, 1, 1);
        if (more) issue_y(ks + 1, sB1, 1);
        mma_all(0);
        __builtin_amdgcn_sched_barrier(0);
        frags_xy(ca, cb, 2, 0);
        mma_all(1);
        __builtin_amdgcn_sched_barrier(0);
        frags_xy(ca, cb, 3, 1);
        mma_all(0);
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
          __builtin_amdgcn_s_waitcnt(kWaitVm0);
          __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
          __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_sched_barrier(0);
          frags_xy(lds + sA1 * SSTR, lds + sB1 * SSTR, 0, 0);
        }
        mma_all(1);
        __builtin_amdgcn_sched_barrier(0);
        sA = sA1;
        sB = sB1;
      }
    } else if constexpr (NB == 16 && FC == 1) {
      // bf16 on 16x16x32 blocks: two sub-steps per K-step, four lane groups with one chunk each.  Same
      // ring and the same four regions per K-step as below (32 MFMAs, eight fragment reads, four loads
      // each; hand-over barrier in the middle of the K-step), but the MFMAs are asm statements, so
      // the interleave is written out: behind each of the first eight MFMAs of a region one fragment
      // read, then one load behind every sixth MFMA, each step pinned by a scheduling barrier (an MFMA
      // of this form issues every 16 cycles, which leaves room for about three other instructions).
      static_assert(NSUB == 2 && FC == 1 && TM == TN && TM % 2 == 0, "two regions per sub-step");
      constexpr int RMMAS = TM * TN / 2;     // MFMAs per region
      constexpr int RREADS = TM;             // fragment reads per region
      static_assert(RREADS + LD_REGION <= RMMAS, "region pattern");
      auto read_a1 = [&](const char* sa, int sub, int buf, int i) {
        const int r = rA0 + i * NB;
        fa[buf][i][0] = *reinterpret_cast<const u32x4_t*>(sa + row_off(r) + (((LG * sub + grp) ^ swz(r)) << 4));
      };
      auto read_b1 = [&](const char* sb, int sub, int buf, int j) {
        const int r = rB0 + j * NB;
        fb[buf][j][0] = *reinterpret_cast<const u32x4_t*>(sb + row_off(r) + (((LG * sub + grp) ^ swz(r)) << 4));
      };
      auto issue_a1 = [&](int ks, int slot, int q) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lptr_t)(lds + slot * SSTR + (w * A_LD + q) * GSTR), 16, offA[q],
                                                 ks * KB, 0, 0);
      };
      auto issue_b1 = [&](int ks, int slot, int q) {
        uint32_t vo = offB[q];
        if constexpr (kMaskB) vo = (ks * KB < limB[q]) ? vo : 0x80000000u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB, (lptr_t)(lds + slot * SSTR + (w * B_LD + q) * GSTR), 16, vo,
                                                 ks * KB, 0, 0);
      };
      // One region: the MFMAs of row blocks [i0, i0 + TM/2) on fragment set `buf`, with the reads of
      // operand `rx` (true: X) for (slot base `src`, sub-step `sub`) into set `rbuf`, and, when `ld`,
      // the loads [q0, q0 + LD_REGION) of operand `lx` for K-step `lks` into ring slot `lslot`.
      auto region = [&](int buf, int i0, bool rd, bool rx, const char* src, int sub, int rbuf, bool ld, bool lx, int lks,
                        int lslot, int q0) {
        constexpr int kGap = (RMMAS - RREADS) / LD_REGION;
#pragma unroll
        for (int idx = 0; idx < RMMAS; ++idx) {
          const int i = i0 + idx / TN, j = idx % TN;
          Elem<E>::mma(acc[i][j], fa[buf][i], fb[buf][j]);
          if (rd && idx < RREADS) {
            if (rx == !kLeadB) read_a1(src, sub, rbuf, idx); else read_b1(src, sub, rbuf, idx);
          }
          if (ld && idx >= RREADS && (idx - RREADS) % kGap == 0 && (idx - RREADS) / kGap < LD_REGION) {
            const int q = q0 + (idx - RREADS) / kGap;
            if (lx == !kLeadB) issue_a1(lks, lslot, q); else issue_b1(lks, lslot, q);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      int sX = 0, sY = 1;
      issue_x(0, 0, 0); issue_x(0, 0, 1);
      issue_y(0, 1, 0); issue_y(0, 1, 1);
      if (ksteps > 1) {
        issue_x(1, 2, 0); issue_x(1, 2, 1);
        issue_y(1, 3, 0); issue_y(1, 3, 1);
        __builtin_amdgcn_s_waitcnt(wait_vm(2 * A_LD));
      } else {
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
      }
      trace_stamp(4, trace_kind);
      __builtin_amdgcn_s_barrier();
      trace_stamp(5, trace_kind); trace_cycles(5, trace_kind);
      frags_xy(lds + sX * SSTR, lds + sY * SSTR, 0, 0);
      settle(acc);
      __builtin_amdgcn_sched_barrier(0);
      int ks = 0;
      // One steady-state K-step with X(ks), Y(ks) in slots sx, sy.  Entering it: X(ks), Y(ks) landed,
      // X(ks+1), Y(ks+1) resident or in flight; the slot of Y(ks-1) is free (the barrier in the middle
      // of K-step ks-1).
      auto kstep = [&](int ks_, int sx, int sy) {
        const char* cx = lds + sx * SSTR;
        const char* cy = lds + sy * SSTR;
        const int sX1 = next_slot(sx, 2), sY1 = next_slot(sy, 2);
        const int sX2 = next_slot(sX1, 2);   // slot of X(ks+2) == slot of Y(ks-1)
        const int sY2 = sx;                  // slot of Y(ks+2) == slot of X(ks)
        region(0, 0, true, true, cx, 1, 1, true, true, ks_ + 2, sX2, 0);
        region(0, TM / 2, true, false, cy, 1, 1, true, true, ks_ + 2, sX2, LD_REGION);
        // hand-over: everything but X(ks+2) has landed, i.e. X(ks+1) and Y(ks+1) are complete
        __builtin_amdgcn_s_waitcnt(wait_vm(A_LD));
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        region(1, 0, true, true, lds + sX1 * SSTR, 0, 0, true, false, ks_ + 2, sY2, 0);
        region(1, TM / 2, true, false, lds + sY1 * SSTR, 0, 0, true, false, ks_ + 2, sY2, LD_REGION);
      };
      // The ring returns to its starting state every NSLOT K-steps: unrolled by that many, every slot
      // number is a constant, and with the interleaved slot layout a fragment's LDS address is a
      // loop-invariant register plus an immediate (no address arithmetic left in the loop).
      static_assert(NSLOT == 5, "unrolled by the ring's period");
      for (; ks + 2 + (NSLOT - 1) < ksteps; ks += NSLOT) {
        kstep(ks, 0, 1);
        kstep(ks + 1, 2, 3);
        kstep(ks + 2, 4, 0);
        kstep(ks + 3, 1, 2);
        kstep(ks + 4, 3, 4);
        if (ks == 0) { trace_stamp(6, trace_kind); trace_cycles(6, trace_kind); }
        if (ks == 5) trace_stamp(7, trace_kind);
        if (ks == 10) { trace_stamp(8, trace_kind); trace_cycles(8, trace_kind); }
      }
      trace_stamp(9, trace_kind); trace_cycles(9, trace_kind);
      for (; ks + 2 < ksteps; ++ks) {
        kstep(ks, sX, sY);
        sX = next_slot(sX, 2);
        sY = next_slot(sY, 2);
      }
      // drain: the last two K-steps (their tiles were all requested above or in the prologue)
      for (; ks < ksteps; ++ks) {
        const char* cx = lds + sX * SSTR;
        const char* cy = lds + sY * SSTR;
        const int sX1 = next_slot(sX, 2), sY1 = next_slot(sY, 2);
        const bool more = ks + 1 < ksteps;
        region(0, 0, true, true, cx, 1, 1, false, false, 0, 0, 0);
        region(0, TM / 2, true, false, cy, 1, 1, false, false, 0, 0, 0);
        region(1, 0, false, false, cx, 0, 0, false, false, 0, 0, 0);
        if (more) {
          __builtin_amdgcn_s_waitcnt(kWaitVm0);
          __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
          __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_sched_barrier(0);
          frags_xy(lds + sX1 * SSTR, lds + sY1 * SSTR, 0, 0);
        }
        region(1, TM / 2, false, false, cx, 0, 0, false, false, 0, 0, 0);
        sX = sX1;
        sY = sY1;
      }
      // the asm MFMAs' results are read by ordinary instructions next: let the last ones retire
      asm volatile("s_nop 15\n\ts_nop 15");
      trace_stamp(10, trace_kind);
    } else if constexpr (NB == 16 && FC == 2) {
      // e4m3 on 16x16x128 blocks: ONE MFMA per block pair consumes the whole K-step (32 cycles each, 64 per
      // K-step).  A second set of fragments does not fit the register file (2 x 128 registers), so there is
      // one set, refilled behind the MFMAs that read it last.  The MFMAs of a K-step go over the column blocks
      // in two halves (j < 4 for all rows i, then j >= 4 for all rows), which spreads the refills over the
      // K-step (row-major order would pile all B refills up behind the last row: 2 KB of LDS reads per MFMA
      // and wave; measured 1-2.5 % slower):
      //   B[0..3] of K-step c + 1   during the second half of K-step c (their last readers end the first half)
      //   A[i], i < 7, of c + 1     behind the first MFMA of row i + 1 of the second half
      //   A[7], B[4..7] of c + 1    behind the first five MFMAs of K-step c + 1 itself
      // A refill is always placed behind the MFMA that FOLLOWS the register's last reader: when that one has
      // been accepted by the matrix pipe the reader has long fetched its operands.
      // Reads thus run up to one K-step ahead of the MFMAs.  The barrier of K-step c (behind its ninth MFMA, when
      // the last reads of the tiles of c have returned) publishes the tiles of c + 1 and frees the two slots of
      // c, which take Y(c + 2) and X(c + 3) at once: with X(c + 2) that is five units resident or in flight.
      static_assert(NSUB == 1 && TM == TN && TM == 8 && A_LD == B_LD, "64 MFMAs per K-step");
      i32x8_t ga[TM], gb[TN];
      auto read_frag = [&](const char* slot, int r) {
        const char* row = slot + row_off(r);
        const u32x4_t lo = *reinterpret_cast<const u32x4_t*>(row + (((2 * grp) ^ swz(r)) << 4));
        const u32x4_t hi = *reinterpret_cast<const u32x4_t*>(row + (((2 * grp + 1) ^ swz(r)) << 4));
        const i32x8_t f = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        return f;
      };
      // slot bases of the A and B tiles of a K-step whose X / Y units sit in slots sx / sy
      auto a_of = [&](int sx, int sy) { return lds + (kLeadB ? sy : sx) * SSTR; };
      auto b_of = [&](int sx, int sy) { return lds + (kLeadB ? sx : sy) * SSTR; };
      auto issue_a1 = [&](int ks, int slot, int q) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lptr_t)(lds + slot * SSTR + (w * A_LD + q) * GSTR), 16, offA[q],
                                                 ks * KB, 0, 0);
      };
      auto issue_b1 = [&](int ks, int slot, int q) {
        uint32_t vo = offB[q];
        if constexpr (kMaskB) vo = (ks * KB < limB[q]) ? vo : 0x80000000u;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB, (lptr_t)(lds + slot * SSTR + (w * B_LD + q) * GSTR), 16, vo,
                                                 ks * KB, 0, 0);
      };
      auto issue_x1 = [&](int ks, int slot, int q) {
        if constexpr (kLeadB) issue_b1(ks, slot, q); else issue_a1(ks, slot, q);
      };
      auto issue_y1 = [&](int ks, int slot, int q) {
        if constexpr (kLeadB) issue_a1(ks, slot, q); else issue_b1(ks, slot, q);
      };
      // K-step c with X(c), Y(c) in slots sx, sy.  next: there is a K-step c + 1 (barrier and refills);
      // ldy / ldx: Y(c + 2) / X(c + 3) exist and are requested; x2: X(c + 2) exists (it is then the only unit
      // that may still be in flight at the barrier).
      auto kstep = [&](int c, int sx, int sy, bool next, bool ldy, bool ldx, bool x2) {
        const int sx1 = next_slot(sx, 2), sy1 = next_slot(sy, 2);
        const char* a0 = a_of(sx, sy);
        const char* b0 = b_of(sx, sy);
        const char* a1 = a_of(sx1, sy1);
        const char* b1 = b_of(sx1, sy1);
        constexpr int kBar = 8;   // MFMA behind which the hand-over barrier sits
#pragma unroll
        for (int idx = 0; idx < TM * TN; ++idx) {
          const int h = idx / 32, r = idx % 32;
          const int i = r / 4, j = 4 * h + r % 4;
          Elem<E>::mma(acc[i][j], ga[i], gb[j]);
          __builtin_amdgcn_sched_barrier(0);   // what follows stays behind this MFMA (see the refill rule above)
          if (idx == 0) ga[TM - 1] = read_frag(a0, rA0 + (TM - 1) * NB);
          if (idx >= 1 && idx <= 4) gb[3 + idx] = read_frag(b0, rB0 + (3 + idx) * NB);
          if (idx == kBar && next) {
            if (x2) __builtin_amdgcn_s_waitcnt(wait_vm(A_LD)); else __builtin_amdgcn_s_waitcnt(kWaitVm0);
            __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
          }
          if (next) {
            if (idx == 33 || idx == 35 || idx == 37 || idx == 39) gb[(idx - 33) / 2] = read_frag(b1, rB0 + ((idx - 33) / 2) * NB);
            if (idx >= 36 && idx % 4 == 0) ga[(idx - 36) / 4] = read_frag(a1, rA0 + ((idx - 36) / 4) * NB);
            if (idx >= kBar && (idx - kBar) % 3 == 0 && (idx - kBar) / 3 < 2 * A_LD) {
              const int q = (idx - kBar) / 3;
              if (q < A_LD) {
                if (ldy) issue_y1(c + 2, sx, q);
              } else {
                if (ldx) issue_x1(c + 3, sy, q - A_LD);
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      // prologue: X(0) Y(0) X(1) Y(1) X(2); wait for K-step 0's pair
      issue_x(0, 0, 0); issue_x(0, 0, 1);
      issue_y(0, 1, 0); issue_y(0, 1, 1);
      if (ksteps > 1) {
        issue_x(1, 2, 0); issue_x(1, 2, 1);
        issue_y(1, 3, 0); issue_y(1, 3, 1);
      }
      if (ksteps > 2) {
        issue_x(2, 4, 0); issue_x(2, 4, 1);
        __builtin_amdgcn_s_waitcnt(wait_vm(3 * A_LD));
      } else if (ksteps > 1) {
        __builtin_amdgcn_s_waitcnt(wait_vm(2 * A_LD));
      } else {
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
      }
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i + 1 < TM; ++i) {
        ga[i] = read_frag(a_of(0, 1), rA0 + i * NB);
        if (i < TN / 2) gb[i] = read_frag(b_of(0, 1), rB0 + i * NB);
      }
      settle(acc);
      __builtin_amdgcn_sched_barrier(0);
      int ks = 0;
      // unrolled by the ring's period, so that every slot number is a constant (see the bf16 loop)
      static_assert(NSLOT == 5, "unrolled by the ring's period");
      for (; ks + 3 + (NSLOT - 1) < ksteps; ks += NSLOT) {
        kstep(ks, 0, 1, true, true, true, true);
        kstep(ks + 1, 2, 3, true, true, true, true);
        kstep(ks + 2, 4, 0, true, true, true, true);
        kstep(ks + 3, 1, 2, true, true, true, true);
        kstep(ks + 4, 3, 4, true, true, true, true);
      }
      int sX = 0, sY = 1;
      for (; ks + 3 < ksteps; ++ks) {
        kstep(ks, sX, sY, true, true, true, true);
        sX = next_slot(sX, 2);
        sY = next_slot(sY, 2);
      }
      // the last three K-steps: Y(ksteps - 1) is the last unit to request
      for (; ks < ksteps; ++ks) {
        kstep(ks, sX, sY, ks + 1 < ksteps, ks + 2 < ksteps, false, ks + 2 < ksteps);
        sX = next_slot(sX, 2);
        sY = next_slot(sY, 2);
      }
      // the asm MFMAs' results are read by ordinary instructions next: let the last ones retire
      asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15");
    } else {
      // Two sub-steps per K-step (32x32 blocks whose MFMA consumes half of the K-step).  Same ring, shifted by a quarter step so that the
      // work still falls into four equal regions of TM*TN/2 MFMAs, eight fragment reads and half a
      // tile of loads each: the hand-over barrier sits in the middle of the K-step; after it a wave
      // reads the first fragments of K-step ks+1 and issues Y(ks+2) into the slot of X(ks), which that
      // barrier has just freed; X(ks+2) follows in the first half of K-step ks+1.
      static_assert(NSUB == 2 && TM % 2 == 0, "two regions per sub-step");
      auto read_x = [&](const char* cx, int sub, int buf) {
        if constexpr (kLeadB) read_b(cx, sub, buf); else read_a(cx, sub, buf);
      };
      auto read_y = [&](const char* cy, int sub, int buf) {
        if constexpr (kLeadB) read_a(cy, sub, buf); else read_b(cy, sub, buf);
      };
      constexpr int RMMAS = TM * TN / 2;     // MFMAs per region
      constexpr int RREADS = TM * FC;        // fragment reads per region (TM == TN)
      static_assert(TM == TN && RREADS % 2 == 0 && RREADS / 2 + LD_REGION <= RMMAS, "region pattern");
      // behind each of the first MFMAs of a region two fragment reads, then one load behind every
      // kGap-th MFMA of the rest
      auto sched_half = [&](bool loads) {
        constexpr int kGap = (RMMAS - RREADS / 2) / LD_REGION;
#pragma unroll
        for (int i = 0; i < RMMAS; ++i) {
          __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
          if (i < RREADS / 2) __builtin_amdgcn_sched_group_barrier(kDsRead, 2, 0);
          if (loads && i >= RREADS / 2 && (i - RREADS / 2) % kGap == 0 && (i - RREADS / 2) / kGap < LD_REGION)
            __builtin_amdgcn_sched_group_barrier(kVmem, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      int sX = 0, sY = 1;
      issue_x(0, 0, 0); issue_x(0, 0, 1);
      issue_y(0, 1, 0); issue_y(0, 1, 1);
      if (ksteps > 1) {
        issue_x(1, 2, 0); issue_x(1, 2, 1);
        issue_y(1, 3, 0); issue_y(1, 3, 1);
        __builtin_amdgcn_s_waitcnt(wait_vm(2 * A_LD));
      } else {
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
      }
      __builtin_amdgcn_s_barrier();
      frags_xy(lds + sX * SSTR, lds + sY * SSTR, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      int ks = 0;
      // Entering K-step ks: X(ks), Y(ks) landed, X(ks+1), Y(ks+1) resident or in flight; the slot of
      // Y(ks-1) is free (the barrier in the middle of K-step ks-1).
      for (; ks + 2 < ksteps; ++ks) {
        const char* cx = lds + sX * SSTR;
        const char* cy = lds + sY * SSTR;
        const int sX1 = next_slot(sX, 2), sY1 = next_slot(sY, 2);
        const int sX2 = next_slot(sX1, 2);   // slot of X(ks+2) == slot of Y(ks-1)
        const int sY2 = sX;                  // slot of Y(ks+2) == slot of X(ks)
        read_x(cx, 1, 1);
        issue_x(ks + 2, sX2, 0);
        mma_rows(0, 0, TM / 2);
        sched_half(true);
        read_y(cy, 1, 1);
        issue_x(ks + 2, sX2, 1);
        mma_rows(0, TM / 2, TM);
        sched_half(true);
        // hand-over: everything but X(ks+2) has landed, i.e. X(ks+1) and Y(ks+1) are complete
        __builtin_amdgcn_s_waitcnt(wait_vm(A_LD));
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        read_x(lds + sX1 * SSTR, 0, 0);
        issue_y(ks + 2, sY2, 0);
        mma_rows(1, 0, TM / 2);
        sched_half(true);
        read_y(lds + sY1 * SSTR, 0, 0);
        issue_y(ks + 2, sY2, 1);
        mma_rows(1, TM / 2, TM);
        sched_half(true);
        sX = sX1;
        sY = sY1;
      }
      // drain: the last two K-steps (their tiles were all requested above or in the prologue)
      for (; ks < ksteps; ++ks) {
        const char* cx = lds + sX * SSTR;
        const char* cy = lds + sY * SSTR;
        const int sX1 = next_slot(sX, 2), sY1 = next_slot(sY, 2);
        const bool more = ks + 1 < ksteps;
        read_x(cx, 1, 1);
        mma_rows(0, 0, TM / 2);
        __builtin_amdgcn_sched_barrier(0);
        read_y(cy, 1, 1);
        mma_rows(0, TM / 2, TM);
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
          __builtin_amdgcn_s_waitcnt(kWaitVm0);
          __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
          __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_sched_barrier(0);
          frags_xy(lds + sX1 * SSTR, lds + sY1 * SSTR, 0, 0);
        }
        mma_rows(1, 0, TM);
        __builtin_amdgcn_sched_barrier(0);
        sX = sX1;
        sY = sY1;
      }
    }
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    __builtin_amdgcn_s_barrier();
  }
};

}  // namespace lmhead
