// Matrix-core kernels of the KV-compression path, built on GemmTile (gemm_core.h):
//   mode 0  spectral projection     x~ = x U                      (Eq. 1); also the two token-major
//           products of the gate's backward pass, optionally added to what the output holds
//   mode 1  gate logits             x~ W          (fp32, bias added by the mask kernel; Eq. 5)
//   mode 2  dynamic low-rank reconstruction  x_bar = x^[0:k] U^-1[0:k, :]   (Eq. 3)
// All three are  out[row(n)][m] = sum_k A[m][k] Bop[n][k]  with the parameter matrix (transposed
// copy, K-contiguous) on the MFMA M axis and tokens on N, as in the LM-head kernels.  The
// parameter matrix (2 MB at d = 1024) stays in every XCD's L2; the token rows stream through once
// per XCD because an XCD runs all M tiles of a token tile together (tile_map.h).
//
// Mode 2 reads token rows of differing length straight from the packed store: row n of a tile is
// the segment of token order[n] (its byte offset and length come with it in pos_off / pos_len),
// loads beyond the segment's end fetch zeros (GemmTile's kMaskB), and the tile runs as many
// K-steps as its first token needs: `order` lists tokens by descending step count, so that is
// the tile's maximum and tiles of short tokens are short.
#include "dynakv_common.h"
#include "gemm_core.h"

#include <type_traits>

namespace lmhead {

namespace {

constexpr int kKvMapBx = 4, kKvMapBy = 4;

// Compute units of the current device (256 on MI355X); asked once.
int compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v >= kNumXcd)
      cus = v;
    else
      cus = 256;
  }
  return cus;
}

// Tile edge of the KV kernels.  256: one workgroup per compute unit (all of LDS).  128 (build with
// -DKV_TILE=128): half the LDS and a quarter of the accumulators per workgroup, so two workgroups
// share a compute unit and one can run its main loop while the other is in its prologue or
// epilogue, at twice the operand traffic per flop.  Measured on the 262144 x 1024 stream, 128 is
// 25-40 % slower (714 / 818 / 623 us against 562 / 570 / 500 us for the three kernels), so 256 it is.
#ifndef KV_TILE
#define KV_TILE 256
#endif
constexpr int kKvTileEdge = KV_TILE;
constexpr int kKvWgPerCu = kKvTileEdge == 256 ? 1 : 2;

typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;

template <typename E, bool kMask>
using KvTile = GemmTile<E, kKvTileEdge, kKvTileEdge, 2, 2, /*kLeadB=*/true, kMask>;

// One output tile; `wg` is the tile's position in the XCD-aware walk.
template <typename E, int Mode>
__device__ inline void kv_tile(const KvGemmArgs& a, int wg, char* smem) {
  using G = KvTile<E, Mode == 2>;
  constexpr int ESZ = Elem<E>::size;
  const int mtiles = (a.M + G::BM - 1) / G::BM;
  const int ntiles = (int)((a.Nn + G::BN - 1) / G::BN);
  int mt, nt;
  if (!xcd_tile_coords(wg, mtiles, ntiles, kKvMapBx, kKvMapBy, mt, nt)) return;
  const int64_t n0 = (int64_t)nt * G::BN;
  const int m0 = mt * G::BM;
  const int64_t pitchA = a.ldA * ESZ;

  uint32_t offA[G::A_LD], offB[G::B_LD];
  int limB[G::B_LD];
#pragma unroll
  for (int q = 0; q < G::A_LD; ++q) {
    const int row = G::ldA_row(q);
    offA[q] = (uint32_t)(row * pitchA) + G::ld_byte(row);
  }
  const char* Bbase;
  uint32_t bytesB;
  int ksteps;
  if constexpr (Mode == 2) {
#pragma unroll
    for (int q = 0; q < G::B_LD; ++q) {
      const int row = G::ldB_row(q);
      offB[q] = a.pos_off[n0 + row] + G::ld_byte(row);       // stays outside the buffer for padding rows
      limB[q] = a.pos_len[n0 + row] - G::ld_byte(row);
    }
    ksteps = (a.pos_len[n0] + G::KB - 1) / G::KB;
    Bbase = static_cast<const char*>(a.B);
    bytesB = (uint32_t)a.bytesB;
  } else {
    const int64_t pitchB = a.ldB * ESZ;
    const int last = (int)min((int64_t)G::BN - 1, a.Nn - 1 - n0);   // rows past the end re-read the last one
#pragma unroll
    for (int q = 0; q < G::B_LD; ++q) {
      const int row = G::ldB_row(q);
      offB[q] = (uint32_t)(min(row, last) * pitchB) + G::ld_byte(row);
      limB[q] = 0;
    }
    ksteps = a.K * ESZ / G::KB;
    Bbase = static_cast<const char*>(a.B) + n0 * pitchB;
    bytesB = 0x7fffffffu;
  }

  // output row of tile column threadIdx.x (fetched now, used after the main loop)
  int my_row = -1;
  if (threadIdx.x < G::BN) {
    if constexpr (Mode == 2)
      my_row = a.order[n0 + threadIdx.x];
    else
      my_row = n0 + threadIdx.x < a.Nn ? (int)(n0 + threadIdx.x) : -1;
  }

  typename G::Acc acc;
  G::zero(acc);
  G::run_rows(acc, static_cast<const char*>(a.A) + (int64_t)m0 * pitchA, offA, Bbase, offB, limB, bytesB, ksteps,
              smem);

  // The tile leaves through LDS as [n][m] rows of fp32 (as many tile columns per phase as fit) so that
  // each output row segment is written with 16 bytes per lane for fp32 and 8 for bf16, a whole
  // number of rows per wavefront instruction.
  constexpr int JG = G::LDS_BYTES >= G::BN * (G::BM * 4 + 16) + G::BN * 4 ? G::TN : G::TN / 2;   // blocks per wave and phase
  constexpr int NPH = G::TN / JG;                 // phases
  constexpr int NCOL = G::WGN * JG * G::NB;       // tile columns staged per phase
  constexpr int P = G::BM * 4 + 16;               // staging row pitch in bytes
  constexpr int CH = G::BM * 4 / 16;              // lanes per staged row
  constexpr int RPI = 64 / CH;                    // staged rows per wavefront instruction
  constexpr int RPW = NCOL / G::NWAVES;           // staged rows per wave and phase
  static_assert(NCOL * P + G::BN * 4 <= G::LDS_BYTES && G::TN % JG == 0, "staging fits in LDS");
  static_assert(64 % CH == 0 && RPW % RPI == 0 && RPW * NPH <= 64, "row mapping");
  int* rows_lds = reinterpret_cast<int*>(smem + NCOL * P);
  if (threadIdx.x < G::BN) rows_lds[threadIdx.x] = my_row;
  // staged row -> tile column
  auto tile_col = [&](int phase, int r) {
    return (r / (JG * G::NB)) * G::WN + phase * (JG * G::NB) + r % (JG * G::NB);
  };
  const int h = G::lane() / CH;                   // which of the instruction's rows this lane works on
  const int c = G::lane() % CH;                   // its 16-byte chunk of the row = 4 output columns
  const int m = m0 + c * 4;
  constexpr int IPW = RPW / RPI;                  // instructions per wave and phase
  using OldT = typename std::conditional<ESZ == 2, bf16x4_t, f32x4_t>::type;
  const bool accumulate = Mode != 2 && a.accumulate && m < a.M;
#pragma unroll
  for (int jg = 0; jg < NPH; ++jg) {
    // When the tile is added to what the output holds, the old values of all the rows this wave writes
    // in this phase are requested now, so that their latency runs under the staging of the tile and is
    // paid once per phase.  (Dense modes only: the output row of a staged row is n0 + its tile column.)
    OldT oldv[IPW];
    if constexpr (Mode != 2) {
      if (accumulate) {
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
          const int64_t row = n0 + tile_col(jg, (G::wave() + G::NWAVES * i) * RPI + h);
          oldv[i] = OldT{};
          if (row < a.Nn) oldv[i] = *reinterpret_cast<const OldT*>(static_cast<const char*>(a.out_e) + (row * a.ldo + m) * ESZ);
        }
      }
    }
#pragma unroll
    for (int jj = 0; jj < JG; ++jj) {
      const int j = jg * JG + jj;
      const int nl = G::wave_n() * (JG * G::NB) + jj * G::NB + (G::lane() % G::NB);
#pragma unroll
      for (int i = 0; i < G::TM; ++i)
#pragma unroll
        for (int q = 0; q < G::VB / 4; ++q) {
          const f32x4_t v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          *reinterpret_cast<f32x4_t*>(smem + nl * P + G::m_of(i, 4 * q) * 4) = v;
        }
    }
    lds_barrier();
    // Instruction i of a wave streams out the staged rows (wave + NWAVES i) RPI + h.  Their output row
    // indices are fetched once (lane RPW p + RPI i + h holds the one of phase p) and read back with
    // readlane, and the loop is unrolled in batches whose LDS reads are all issued before the first
    // store, so that a wave is not serialised on one LDS round trip per row.
    if (jg == 0) {
      const int l = G::lane();
      const int ph = l / RPW, idx = l % RPW;
      const int r = (G::wave() + G::NWAVES * (idx / RPI)) * RPI + idx % RPI;
      my_row = ph < NPH ? rows_lds[tile_col(ph, r)] : -1;
    }
    constexpr int RB = IPW < 8 ? IPW : 8;
#pragma unroll
    for (int i0 = 0; i0 < IPW; i0 += RB) {
      f32x4_t v[RB];
      int64_t orow[RB];
#pragma unroll
      for (int u = 0; u < RB; ++u)
        v[u] = *reinterpret_cast<const f32x4_t*>(smem + ((G::wave() + G::NWAVES * (i0 + u)) * RPI + h) * P + c * 16);
#pragma unroll
      for (int u = 0; u < RB; ++u) {
        int64_t row = __builtin_amdgcn_readlane(my_row, jg * RPW + (i0 + u) * RPI);
        if constexpr (RPI == 2) {
          const int r1 = __builtin_amdgcn_readlane(my_row, jg * RPW + (i0 + u) * RPI + 1);
          row = h ? r1 : row;
        }
        orow[u] = m < a.M ? row : -1;
      }
      if constexpr (Mode != 2) {
        if (accumulate) {
#pragma unroll
          for (int u = 0; u < RB; ++u) {
            const OldT o = oldv[i0 + u];
            v[u] += f32x4_t{(float)o.x, (float)o.y, (float)o.z, (float)o.w};
          }
        }
      }
#pragma unroll
      for (int u = 0; u < RB; ++u) {
        const int64_t row = orow[u];
        if (row < 0) continue;
        if (a.out_f) {
          *reinterpret_cast<f32x4_t*>(a.out_f + row * a.ldo + m) = v[u];
        } else if constexpr (ESZ == 4) {
          *reinterpret_cast<f32x4_t*>(static_cast<float*>(a.out_e) + row * a.ldo + m) = v[u];
        } else {
          const bf16x4_t hb = {(__bf16)v[u].x, (__bf16)v[u].y, (__bf16)v[u].z, (__bf16)v[u].w};
          *reinterpret_cast<bf16x4_t*>(static_cast<__bf16*>(a.out_e) + row * a.ldo + m) = hb;
        }
      }
    }
    lds_barrier();
  }
}

// Tiles here are short (d_kv / 64 K-steps or fewer), so the workgroups are persistent: as many as
// are resident at a time, each taking every gridDim.x-th tile of the walk, which saves a workgroup
// launch per tile.  gridDim.x is a multiple of 8, so a tile stays on the XCD that the walk meant it for.
template <typename E, int Mode>
__global__ __launch_bounds__(256) void kv_gemm_kernel(KvGemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  for (int wg = blockIdx.x; wg < a.walk_len; wg += gridDim.x) kv_tile<E, Mode>(a, wg, smem);
}

template <typename E, int Mode>
hipError_t launch_mode(const KvGemmArgs& a, hipStream_t s) {
  using G = KvTile<E, Mode == 2>;
  const int mtiles = (a.M + G::BM - 1) / G::BM;
  const int64_t ntiles = (a.Nn + G::BN - 1) / G::BN;
  if (a.accumulate && (Mode == 2 || a.out_f || !a.out_e)) return hipErrorInvalidValue;
  KvGemmArgs b = a;
  b.walk_len = (int)xcd_grid_size(mtiles, ntiles, kKvMapBy);
  const unsigned resident = (unsigned)compute_units() / kNumXcd * kNumXcd * kKvWgPerCu;   // LDS-bound
  const dim3 grid(b.walk_len < (int)resident ? (unsigned)b.walk_len : resident);
  hipError_t e = allow_lds<kv_gemm_kernel<E, Mode>>(G::LDS_BYTES);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((kv_gemm_kernel<E, Mode>), grid, dim3(G::NT), G::LDS_BYTES, s, b);
  return hipGetLastError();
}

template <typename E>
hipError_t launch_e(const KvGemmArgs& a, hipStream_t s) {
  switch (a.mode) {
    case 0: return launch_mode<E, 0>(a, s);
    case 1: return launch_mode<E, 1>(a, s);
    default: return launch_mode<E, 2>(a, s);
  }
}

}  // namespace

hipError_t launch_kv_gemm(int dtype, const KvGemmArgs& a, hipStream_t s) {
  return dtype == LMHEAD_BF16 ? launch_e<bf16_tag>(a, s) : launch_e<f32_tag>(a, s);
}

}  // namespace lmhead
