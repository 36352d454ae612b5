// MFMA macro-tile main loop shared by every contraction of the library (gfx950).
//
// All four contractions (logits, logits recompute for dZ, dH, dW) are brought to the
// same form  C[m][n] = sum_k A[m][k] * B[n][k]  with both operands K-contiguous.
// A workgroup owns a BM x BN tile of C; each wavefront owns a (BM/WGM) x (BN/WGN)
// sub-tile built from 32x32 MFMA blocks.
//
// Data movement: K is consumed 64 bytes per row per step (32 bf16 or 16 fp32).  Tiles go
// from global memory straight into LDS (global_load_lds_dwordx4, no register staging)
// through a ring of four stages, so three K-steps of loads are always in flight behind
// the one being multiplied.  One workgroup barrier per K-step; completion of a stage is
// tracked with the wave's own vmcnt (loads retire in order) followed by that barrier.
//
// LDS stage layout: A rows then B rows, 64 bytes (four 16-byte chunks) per row; chunk c
// of row r sits at chunk position c ^ swz(r).  A direct-to-LDS load writes lane L's 16
// bytes at wave_base + 16 L, i.e. row L/4, position L%4 of a 16-row group, so lane L
// simply fetches the global chunk (L%4) ^ swz(row).  swz is chosen so that the 128-bit
// fragment reads (32 consecutive rows, fixed chunk) are bank-conflict-free whether the
// hardware serves 8 lanes over 32 banks or 16 lanes over 64 banks per cycle.
//
// Fragment layout used for both operands (what matters is only that A and B agree):
// lane l of a 32-row block holds row l % 32 and the 16-byte chunk 2*s + l/32 of K
// sub-step s (two sub-steps per K-step).  For bf16 one v_mfma_f32_32x32x16_bf16 consumes
// the chunk; for fp32 the chunk's four floats feed four v_mfma_f32_32x32x2_f32.
// Fragments are double-buffered in registers and the pipeline is skewed so that the
// barrier falls between the two sub-steps: the MFMAs of sub-step 1 overlap the first
// fragment reads of the next stage.
//
// Accumulator layout of a 32x32 block (16 floats per lane):
//   element v of lane l  <->  m = 8*(v/4) + 4*(l/32) + v%4,  n = l % 32.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lmhead {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

struct bf16_tag {};
struct f32_tag {};

template <typename E>
struct Elem;
template <>
struct Elem<bf16_tag> {
  static constexpr int size = 2;
  static constexpr int dtype = 1;
  __device__ static inline void mma(f32x16_t& c, const u32x4_t& a, const u32x4_t& b) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};
template <>
struct Elem<f32_tag> {
  static constexpr int size = 4;
  static constexpr int dtype = 0;
  __device__ static inline void mma(f32x16_t& c, const u32x4_t& a, const u32x4_t& b) {
    // whole-vector casts, then named components: element-wise bit casts of a[q] are avoided
    const f32x4_t fa = __builtin_bit_cast(f32x4_t, a);
    const f32x4_t fb = __builtin_bit_cast(f32x4_t, b);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.x, fb.x, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.y, fb.y, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.z, fb.z, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.w, fb.w, c, 0, 0, 0);
  }
};

// s_waitcnt immediates (gfx9 encoding): only the named counter is constrained.
constexpr int kWaitVm0 = 0x0F70;
constexpr int kWaitVm16 = 0x4F70;
constexpr int kWaitLgkm0 = 0xC07F;

template <typename E, int BM_, int BN_, int WGM_, int WGN_>
struct GemmTile {
  static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
  static constexpr int NWAVES = WGM * WGN;
  static constexpr int NT = 64 * NWAVES;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int KB = 64;                       // bytes of K per row per step
  static constexpr int NSTAGE = 4;
  static constexpr int STAGE = (BM + BN) * KB;
  static constexpr int LDS_BYTES = NSTAGE * STAGE;
  static constexpr int A_LD = BM / 16 / NWAVES;       // direct-to-LDS load instructions per wave
  static constexpr int B_LD = BN / 16 / NWAVES;       // per K-step (each moves 16 rows)
  static constexpr int LOADS_PER_STEP = A_LD + B_LD;
  static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tiles are 32x32 blocks");
  static_assert(BM % (16 * NWAVES) == 0 && BN % (16 * NWAVES) == 0, "tile loads divide evenly");
  static_assert(LOADS_PER_STEP == 8, "kWaitVm16 assumes 8 loads per wave per K-step");

  using Acc = f32x16_t[TM][TN];

  __device__ static inline int lane() { return threadIdx.x & 63; }
  __device__ static inline int wave() { return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }
  __device__ static inline int wave_m() { return wave() % WGM; }
  __device__ static inline int wave_n() { return wave() / WGM; }
  // Tile-relative coordinates of accumulator element v of block (i, j).
  __device__ static inline int m_of(int i, int v) {
    return wave_m() * WM + i * 32 + 8 * (v >> 2) + 4 * (lane() >> 5) + (v & 3);
  }
  __device__ static inline int n_of(int j) { return wave_n() * WN + j * 32 + (lane() & 31); }

  __device__ static inline int swz(int r) { return ((r >> 1) ^ (r >> 3)) & 3; }

  // Tile row that this lane fetches in the wave's q-th load of A (or B), and the byte offset
  // inside that row's 64-byte K slice that it must fetch to realise the swizzled layout.
  __device__ static inline int ldA_row(int q) { return (wave() * A_LD + q) * 16 + (lane() >> 2); }
  __device__ static inline int ldB_row(int q) { return (wave() * B_LD + q) * 16 + (lane() >> 2); }
  __device__ static inline int ld_byte(int row) { return ((lane() & 3) ^ swz(row)) << 4; }

  __device__ static inline void zero(Acc& acc) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  }

  // acc += A_tile * B_tile^T over `ksteps` steps of 64 bytes.
  // A / B: uniform pointers to the tile's first row at K offset 0.  offA[q] / offB[q]: this
  // lane's byte offset from that pointer for its q-th load: (row, already clamped by the caller,
  // relative to the tile's first row) * pitch + ld_byte(row).
  // `lds` must provide LDS_BYTES bytes.  Returns with every wave past a barrier and no load
  // in flight, so LDS may be reused by the caller right away.
  __device__ static inline void run(Acc& acc, const char* __restrict__ A, const uint32_t (&offA)[A_LD],
                                    const char* __restrict__ B, const uint32_t (&offB)[B_LD],
                                    int ksteps, char* lds) {
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    const int w = wave();
    const int l = lane();
    const int half = l >> 5;
    const int rA0 = wave_m() * WM + (l & 31);
    const int rB0 = wave_n() * WN + (l & 31);

    auto issue = [&](int ks) {
      char* st = lds + (ks & (NSTAGE - 1)) * STAGE;
      const char* pa = A + (int64_t)ks * KB;
      const char* pb = B + (int64_t)ks * KB;
#pragma unroll
      for (int q = 0; q < A_LD; ++q)
        __builtin_amdgcn_global_load_lds((gptr_t)(pa + offA[q]), (lptr_t)(st + (w * A_LD + q) * 1024), 16, 0, 0);
#pragma unroll
      for (int q = 0; q < B_LD; ++q)
        __builtin_amdgcn_global_load_lds((gptr_t)(pb + offB[q]),
                                         (lptr_t)(st + BM * KB + (w * B_LD + q) * 1024), 16, 0, 0);
    };

    u32x4_t fa[2][TM], fb[2][TN];
    auto read_frags = [&](const char* stage, int s, int buf) {
      const int ch = 2 * s + half;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int r = rA0 + i * 32;
        fa[buf][i] = *reinterpret_cast<const u32x4_t*>(stage + r * KB + ((ch ^ swz(r)) << 4));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int r = rB0 + j * 32;
        fb[buf][j] = *reinterpret_cast<const u32x4_t*>(stage + BM * KB + r * KB + ((ch ^ swz(r)) << 4));
      }
    };
    auto mma_all = [&](int buf) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) Elem<E>::mma(acc[i][j], fa[buf][i], fb[buf][j]);
    };

    // Scheduling hints: interleave one LDS read (then one global->LDS load) with each MFMA so
    // that neither the fragment reads nor the load issue ever leave the matrix pipe idle.
    constexpr int kDsRead = 0x100, kVmem = 0x010;
    constexpr int MMAS = TM * TN * (Elem<E>::size == 2 ? 1 : 4);
    constexpr int FR = TM + TN;

    if (ksteps <= 0) return;
    const int pre = ksteps < NSTAGE - 1 ? ksteps : NSTAGE - 1;
    for (int ks = 0; ks < pre; ++ks) issue(ks);
    if (ksteps >= NSTAGE - 1)
      __builtin_amdgcn_s_waitcnt(kWaitVm16);
    else
      __builtin_amdgcn_s_waitcnt(kWaitVm0);
    __builtin_amdgcn_s_barrier();
    read_frags(lds, 0, 0);
    int ks = 0;
    // steady state: three K-steps of loads in flight, straight-line body
    for (; ks + NSTAGE - 1 < ksteps; ++ks) {
      read_frags(lds + (ks & (NSTAGE - 1)) * STAGE, 1, 1);
      issue(ks + NSTAGE - 1);   // refills the stage whose reads ended before the last barrier
      mma_all(0);
#pragma unroll
      for (int i = 0; i < FR; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(kDsRead, 1, 0);
      }
#pragma unroll
      for (int i = 0; i < LOADS_PER_STEP; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(kVmem, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, MMAS - FR - LOADS_PER_STEP, 0);
      __builtin_amdgcn_sched_barrier(0);        // nothing is scheduled across the stage hand-over
      __builtin_amdgcn_s_waitcnt(kWaitVm16);    // this wave's loads of K-step ks+1 have landed
      __builtin_amdgcn_s_waitcnt(kWaitLgkm0);   // and its reads of the current stage are complete
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      read_frags(lds + ((ks + 1) & (NSTAGE - 1)) * STAGE, 0, 0);
      mma_all(1);
#pragma unroll
      for (int i = 0; i < FR; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(kDsRead, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, MMAS - FR, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // drain: nothing left to issue
    for (; ks < ksteps; ++ks) {
      read_frags(lds + (ks & (NSTAGE - 1)) * STAGE, 1, 1);
      mma_all(0);
      if (ks + 1 < ksteps) {
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
        __builtin_amdgcn_s_barrier();
        read_frags(lds + ((ks + 1) & (NSTAGE - 1)) * STAGE, 0, 0);
      }
      mma_all(1);
    }
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    __builtin_amdgcn_s_barrier();
  }
};

}  // namespace lmhead
