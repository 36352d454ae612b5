// MFMA macro-tile main loop shared by every contraction of the library (gfx950).
//
// All four contractions (logits, logits recompute for dZ, dH, dW) are brought to the
// same form  C[m][n] = sum_k A[m][k] * B[n][k]  with both operands K-contiguous.
// A workgroup owns a BM x BN tile of C; each wavefront owns a (BM/WGM) x (BN/WGN)
// sub-tile built from 32x32 MFMA blocks.  K is consumed 128 bytes per row per step
// (64 bf16 or 32 fp32), staged through LDS in two alternating buffers while the next
// step's global loads are in flight in registers.
//
// LDS tile layout: row-major, 128 bytes (eight 16-byte chunks) per row, chunk c of
// row r stored at chunk position c ^ (r & 7) so that the eight lanes served together
// by a 128-bit LDS access touch all banks once, for the row-strided fragment reads as
// well as for the row-contiguous tile writes.
//
// Fragment layout used for both operands (what matters is only that A and B agree):
// lane l of a 32-row block holds row l % 32 and the 16-byte chunk 2*s + l/32 of K
// sub-step s.  For bf16 one v_mfma_f32_32x32x16_bf16 consumes the chunk; for fp32 the
// chunk's four floats feed four v_mfma_f32_32x32x2_f32.
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
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

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

template <typename E, int BM_, int BN_, int WGM_, int WGN_>
struct GemmTile {
  static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
  static constexpr int NT = 64 * WGM * WGN;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;  // 16-byte chunks per thread
  static constexpr int ROWS_PER_PASS = NT / 8;
  static constexpr int STAGE = (BM + BN) * 128;
  static constexpr int LDS_BYTES = 2 * STAGE;
  static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tiles are 32x32 blocks");
  static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "tile loads divide evenly");

  using Acc = f32x16_t[TM][TN];

  __device__ static inline int lane() { return threadIdx.x & 63; }
  __device__ static inline int wave_m() { return (threadIdx.x >> 6) % WGM; }
  __device__ static inline int wave_n() { return (threadIdx.x >> 6) / WGM; }
  // Tile-relative coordinates of accumulator element v of block (i, j).
  __device__ static inline int m_of(int i, int v) {
    return wave_m() * WM + i * 32 + 8 * (v >> 2) + 4 * (lane() >> 5) + (v & 3);
  }
  __device__ static inline int n_of(int j) { return wave_n() * WN + j * 32 + (lane() & 31); }

  // Row (within the tile) and chunk of this thread's p-th 16-byte piece of a tile load.
  __device__ static inline int ld_row(int p) { return (threadIdx.x >> 3) + p * ROWS_PER_PASS; }
  __device__ static inline int ld_chunk() { return threadIdx.x & 7; }

  __device__ static inline void zero(Acc& acc) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  }

  // acc += A_tile * B_tile^T over `ksteps` steps of 128 bytes.
  // offA[p] / offB[p]: byte offset (from A / B) of this thread's p-th piece at k-step 0, i.e.
  // row_index * pitch + ld_chunk() * 16, with the row index already clamped by the caller.
  // `lds` must provide LDS_BYTES bytes, 16-byte aligned.  Ends with all waves past a barrier,
  // so LDS may be reused by the caller right away.
  __device__ static inline void run(Acc& acc, const char* __restrict__ A, const int64_t (&offA)[A_CH],
                                    const char* __restrict__ B, const int64_t (&offB)[B_CH],
                                    int ksteps, char* lds) {
    u32x4_t ra[A_CH], rb[B_CH];
    const int c = ld_chunk();
    int wofsA[A_CH], wofsB[B_CH];
#pragma unroll
    for (int p = 0; p < A_CH; ++p) {
      const int r = ld_row(p);
      wofsA[p] = r * 128 + ((c ^ (r & 7)) << 4);
    }
#pragma unroll
    for (int p = 0; p < B_CH; ++p) {
      const int r = ld_row(p);
      wofsB[p] = BM * 128 + r * 128 + ((c ^ (r & 7)) << 4);
    }
    const int l = lane();
    const int half = l >> 5;
    const int rA0 = wave_m() * WM + (l & 31);
    const int rB0 = wave_n() * WN + (l & 31);

    auto gload = [&](int ks) {
      const int64_t kofs = (int64_t)ks * 128;
#pragma unroll
      for (int p = 0; p < A_CH; ++p) ra[p] = *reinterpret_cast<const u32x4_t*>(A + offA[p] + kofs);
#pragma unroll
      for (int p = 0; p < B_CH; ++p) rb[p] = *reinterpret_cast<const u32x4_t*>(B + offB[p] + kofs);
    };
    auto lstore = [&](char* stage) {
#pragma unroll
      for (int p = 0; p < A_CH; ++p) *reinterpret_cast<u32x4_t*>(stage + wofsA[p]) = ra[p];
#pragma unroll
      for (int p = 0; p < B_CH; ++p) *reinterpret_cast<u32x4_t*>(stage + wofsB[p]) = rb[p];
    };
    auto compute = [&](const char* stage) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        u32x4_t fa[TM], fb[TN];
        const int ch = 2 * s + half;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int r = rA0 + i * 32;
          fa[i] = *reinterpret_cast<const u32x4_t*>(stage + r * 128 + ((ch ^ (r & 7)) << 4));
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int r = rB0 + j * 32;
          fb[j] = *reinterpret_cast<const u32x4_t*>(stage + BM * 128 + r * 128 + ((ch ^ (r & 7)) << 4));
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) Elem<E>::mma(acc[i][j], fa[i], fb[j]);
      }
    };

    if (ksteps <= 0) return;
    gload(0);
    lstore(lds);
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
      char* cur = lds + (ks & 1) * STAGE;
      char* nxt = lds + ((ks & 1) ^ 1) * STAGE;
      const bool more = ks + 1 < ksteps;
      if (more) gload(ks + 1);
      compute(cur);
      if (more) lstore(nxt);
      __syncthreads();
    }
  }
};

}  // namespace lmhead
