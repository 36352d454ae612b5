// The three MFMA kernels of the LM-head path, all built on GemmTile (gemm_core.h):
//   fwd_kernel    logits tile (vocabulary x tokens) -> max / sum-exp / sum-exp*z per token and tile,
//                 target-logit capture; nothing of the tile is stored           (log-softmax of L_CE, Eq. 9)
//   dz_kernel     logits tile recomputed -> dZ = g (onehot - softmax), stored in both orientations
//   gemm_t_kernel plain contraction with a transposed, row-mapped fp32 store    (dH and dW)
// fwd_kernel and dz_kernel also exist for 8-bit (e4m3) copies of their operands.
//
// Orientation: the vocabulary (or d) runs along the MFMA M axis and tokens (or vocabulary
// rows of dW) along N.  With the MFMA accumulator layouts (16x16 blocks for bf16 and e4m3, 32x32 for
// fp32) a lane then owns ONE token column per block and 4 (or 16) vocabulary entries of it, so
// the softmax statistics are reduced inside the lane and need two (or one) cross-lane steps per
// tile; and a lane's four consecutive M entries are contiguous in the row-major outputs (dZ row,
// dH row, dW row).
#include <atomic>
#include <type_traits>

#include "common.h"
#include "gemm_core.h"

namespace lmhead {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegInf = -__builtin_huge_valf();

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Which operand leads the LDS ring in each kernel (see GemmTile::run); true = the B side.
// Measured on the 32x8x2048 workload with the 16x16x32 main loop: the logits kernels do best with the
// hidden states leading (+2 % and +1 % over W leading), the two backward contractions with the dZ side
// leading (within 0.5 % either way).
constexpr bool kLeadFwd = true, kLeadDz = true, kLeadDh = true, kLeadDw = true;

// 256 x 256 workgroup tile, four wavefronts (2 x 2) of 128 x 128.
template <typename E, bool kLeadB = false>
using Tile = GemmTile<E, 256, 256, 2, 2, kLeadB>;

// Block shape of the XCD-local tile walk (see xcd_tile_coords): 4 x 4 work items.
constexpr int kMapBx = 4, kMapBy = 4;
// The forward does best with narrower, taller blocks (measured on the 32x8x2048 workload).
constexpr int kFwdMapBx = 2, kFwdMapBy = 8;

// Merge (m2, s2, t2) into (m, s, t): statistics of a union of disjoint logit sets.
__device__ inline void merge_stats(float& m, float& s, float& t, float m2, float s2, float t2) {
  const float mn = fmaxf(m, m2);
  const float ms = (mn == kNegInf) ? 0.f : mn;
  const float a = fast_exp2((m - ms) * kLog2e);
  const float b = fast_exp2((m2 - ms) * kLog2e);
  s = s * a + s2 * b;
  t = t * a + t2 * b;
  m = mn;
}

template <typename E>
__global__ __launch_bounds__(Tile<E>::NT) void fwd_kernel(FwdArgs a) {
  using G = Tile<E, kLeadFwd>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int nv = a.hdr->nv;
  const int nblk = (nv + G::BN - 1) / G::BN;
  // one vocabulary tile x one token block per workgroup: short-lived workgroups are dispatched in
  // tile-walk order, which keeps the ones that share operand slabs in step with each other
  // a launch may cover several weight matrices over the same hidden states: the walk's x axis then
  // runs over (policy, vocabulary tile), and neighbours in x still share the token block's rows of Hc
  int tx, nb;
  if (!xcd_tile_coords(blockIdx.x, a.ntiles * a.npol, nblk, kFwdMapBx, kFwdMapBy, tx, nb)) return;
  trace_stamp(0, 1);
  const int pol = tx / a.ntiles;
  const int tile = tx - pol * a.ntiles;
  const char* Wp = static_cast<const char*>(a.W[0]);
#pragma unroll
  for (int p = 1; p < kMaxPolicies; ++p) Wp = (pol == p) ? static_cast<const char*>(a.W[p]) : Wp;
  float* const zy = a.zy + (size_t)pol * a.Ncap;
  int32_t* const gid = a.gid + (size_t)pol * a.Ncap;
  float* const part = a.part + (size_t)pol * 3 * a.ntiles * a.Ncap;
  const int64_t n0 = (int64_t)nb * G::BN;
  const int m0 = tile * G::BM;
  const int ksteps = a.d * Elem<E>::size / G::KB;
  const int64_t pitchH = a.ldHc * Elem<E>::size;
  const int64_t pitchW = a.ldW * Elem<E>::size;

  uint32_t offA[G::A_LD], offB[G::B_LD];
#pragma unroll
  for (int q = 0; q < G::A_LD; ++q) {
    const int row = G::ldA_row(q);
    offA[q] = (uint32_t)((min(m0 + row, a.V - 1) - m0) * pitchW) + G::ld_byte(row);
  }
#pragma unroll
  for (int q = 0; q < G::B_LD; ++q) {
    const int row = G::ldB_row(q);
    offB[q] = (uint32_t)(row * pitchH) + G::ld_byte(row);
  }
  // target ids of this lane's token columns: fetched before the main loop so that their latency is hidden
  int tkj[G::TN];
#pragma unroll
  for (int j = 0; j < G::TN; ++j) tkj[j] = a.tok_c[n0 + G::n_of(j)];

  typename G::Acc acc;
  G::zero(acc);
  trace_stamp(1, 1);
  G::run(acc, Wp + (int64_t)m0 * pitchW, offA, static_cast<const char*>(a.Hc) + n0 * pitchH, offB, ksteps, smem, 1);
  trace_stamp(2, 1); trace_cycles(2, 1);

  float mr[G::TN], sr[G::TN], tr[G::TN];
#pragma unroll
  for (int j = 0; j < G::TN; ++j) {
    mr[j] = kNegInf;
    sr[j] = 0.f;
    tr[j] = 0.f;
  }

  // target-logit capture: only where some lane's target falls inside this tile
  {
    int relj[G::TN];
    bool hit = false;
#pragma unroll
    for (int j = 0; j < G::TN; ++j) {
      const int tk = tkj[j];
      hit |= (tk >= m0) & (tk < m0 + G::BM);
      relj[j] = tk - m0 - G::m_base();   // compared with compile-time constants
    }
    if (__any(hit)) {
#pragma unroll
      for (int j = 0; j < G::TN; ++j) {
        float zsel = 0.f;
        bool found = false;
#pragma unroll
        for (int i = 0; i < G::TM; ++i)
#pragma unroll
          for (int v = 0; v < G::VB; ++v) {
            const bool eq = relj[j] == G::m_const(i, v);
            zsel = eq ? acc[i][j][v] : zsel;
            found |= eq;
          }
        if (found) {
          zy[n0 + G::n_of(j)] = zsel * a.zscale;
          // vocabulary column of the accumulator element just selected (the compare above held for it)
          gid[n0 + G::n_of(j)] = m0 + G::m_base() + relj[j];
        }
      }
    }
  }

  trace_stamp(11, 1);
  // softmax statistics of this tile, inside the lane, 16 values of one token column at a time (one
  // 32x32 block or four 16x16 blocks); the scheduling barrier after each group keeps the
  // accumulator reads of later groups from being hoisted, so only 16 values are live in VGPRs at a time
  {
    const int vlim = a.V - m0 - G::m_base();   // vocabulary rows with m_const >= vlim are padding
    // logit = accumulator * zscale (zscale = 1 unless the operands are scaled 8-bit copies); the factor
    // is folded into the constants of the group instead of being applied per element
    const float zscale = a.zscale;
    const float kz = kLog2e * zscale;
    constexpr int BPC = 16 / G::VB;            // blocks per group of 16 values
    static_assert(G::TM % BPC == 0, "groups of 16 values");
    auto group_stats = [&](auto full_tag, auto ent_tag, int ic, int j, float& m_run, float& s_run, float& t_run) {
      constexpr bool kFull = decltype(full_tag)::value;
      constexpr bool kEnt = decltype(ent_tag)::value;   // the third accumulator (sum exp * z) feeds the entropy only
      float z[16];
      bool ok[16];
#pragma unroll
      for (int b = 0; b < BPC; ++b)
#pragma unroll
        for (int v = 0; v < G::VB; ++v) {
          ok[b * G::VB + v] = kFull || G::m_const(ic * BPC + b, v) < vlim;
          z[b * G::VB + v] = ok[b * G::VB + v] ? acc[ic * BPC + b][j][v] : kNegInf;
        }
      float tmax = fmaxf(z[0], z[1]);
#pragma unroll
      for (int v = 2; v < 16; v += 2) tmax = fmaxf(tmax, fmaxf(z[v], z[v + 1]));
      const float mn = fmaxf(m_run, tmax * zscale);
      const float ms = (mn == kNegInf) ? 0.f : mn;
      const float sc = fast_exp2((m_run - ms) * kLog2e);
      const float bias = -ms * kLog2e;
      float ss = 0.f, ts = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float e = fast_exp2(fmaf(z[v], kz, bias));   // exp2(-inf) = 0 on padding rows
        ss += e;
        if constexpr (kEnt) ts = fmaf(e, ok[v] ? z[v] : 0.f, ts);
      }
      s_run = fmaf(s_run, sc, ss);
      if constexpr (kEnt) t_run = fmaf(t_run, sc, ts * zscale);
      m_run = mn;
      __builtin_amdgcn_sched_barrier(0);
    };
    auto all_groups = [&](auto full_tag, auto ent_tag) {
#pragma unroll
      for (int j = 0; j < G::TN; ++j)
#pragma unroll
        for (int ic = 0; ic < G::TM / BPC; ++ic) group_stats(full_tag, ent_tag, ic, j, mr[j], sr[j], tr[j]);
    };
    const bool want_t = a.want_entropy && pol == 0;   // entropy is reported for the first weight matrix only
    if (m0 + G::BM <= a.V) {
      if (want_t) all_groups(std::true_type{}, std::true_type{}); else all_groups(std::true_type{}, std::false_type{});
    } else {
      if (want_t) all_groups(std::false_type{}, std::true_type{}); else all_groups(std::false_type{}, std::false_type{});
    }
  }

  trace_stamp(12, 1);
  // combine the lane groups of a block (same token, other vocabulary rows), then the WGM waves via LDS
  float* red = reinterpret_cast<float*>(smem);  // [WGM][BN][3]
#pragma unroll
  for (int j = 0; j < G::TN; ++j) {
#pragma unroll
    for (int o = 32; o >= G::NB; o >>= 1) {
      const float m2 = __shfl_xor(mr[j], o);
      const float s2 = __shfl_xor(sr[j], o);
      const float t2 = __shfl_xor(tr[j], o);
      merge_stats(mr[j], sr[j], tr[j], m2, s2, t2);
    }
    if (G::lane() < G::NB) {
      float* q = red + ((size_t)G::wave_m() * G::BN + G::n_of(j)) * 3;
      q[0] = mr[j];
      q[1] = sr[j];
      q[2] = tr[j];
    }
  }
  trace_stamp(13, 1);
  lds_barrier();
  for (int n = threadIdx.x; n < G::BN; n += G::NT) {
    float m = red[n * 3], s = red[n * 3 + 1], t = red[n * 3 + 2];
#pragma unroll
    for (int w = 1; w < G::WGM; ++w) {
      const float* q = red + ((size_t)w * G::BN + n) * 3;
      merge_stats(m, s, t, q[0], q[1], q[2]);
    }
    const size_t base = (size_t)tile * a.Ncap + n0 + n;
    const size_t plane = (size_t)a.ntiles * a.Ncap;
    part[base] = m;
    part[plane + base] = s;
    if (a.want_entropy && pol == 0) part[2 * plane + base] = t;
  }
#ifdef LMHEAD_TRACE
  trace_stamp(3, 1);
  trace_cycles(3, 1);
  if (g_trace && g_trace_kind == 1 && threadIdx.x == 0 && blockIdx.x < kTraceWorkgroups) {
    unsigned xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    unsigned long long* ids = g_trace + ((size_t)kTraceWorkgroups + blockIdx.x) * 16;   // next to the cycle counts
    ids[11] = __builtin_amdgcn_s_getreg(4 | (15 << 11));   // HW_ID, bits 15:0
    ids[12] = xcc;
    ids[13] = ((unsigned long long)tx << 32) | (unsigned)nb;
  }
#endif
}

template <typename E>
struct Store4;
template <>
struct Store4<bf16_tag> {
  __device__ static inline void row(void* p, float a, float b, float c, float d) {
    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
    bf16x4_t v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
    *reinterpret_cast<bf16x4_t*>(p) = v;
  }
  __device__ static inline void one(void* p, float a) { *reinterpret_cast<__bf16*>(p) = (__bf16)a; }
};
template <>
struct Store4<f32_tag> {
  __device__ static inline void row(void* p, float a, float b, float c, float d) {
    f32x4_t v = {a, b, c, d};
    *reinterpret_cast<f32x4_t*>(p) = v;
  }
  __device__ static inline void one(void* p, float a) { *reinterpret_cast<float*>(p) = a; }
};

// Row order of the W tile in LDS for the 16x16-block dZ kernel.  LDS row R = 128 w + 16 i + r feeds
// row r of MFMA block i of wave row w, and accumulator element v of lane group q belongs to block row
// r = 4 q + v.  Loading vocabulary row 128 w + 32 (i / 2) + 8 q + 4 (i % 2) + v there makes the eight
// values that a lane holds in blocks 2a and 2a + 1 the vocabulary rows 128 w + 32 a + 8 q + [0, 8) of its
// token: 16 bytes of a dZ row, stored straight from registers.
struct DzRows {
  __device__ static constexpr int tile_row_of_lds_row(int R) {
    return (R & ~127) + 32 * ((R >> 5) & 3) + 8 * ((R >> 2) & 3) + 4 * ((R >> 4) & 1) + (R & 3);
  }
  // compile-time part of the tile row of element v of block i (the rest depends on the lane only)
  __device__ static constexpr int offset(int i, int v) { return 32 * (i >> 1) + 4 * (i & 1) + v; }
};

// Epilogue of the dZ kernel on 16x16 blocks with bf16 output (bf16 or e4m3 operands; permuted W rows):
// dZ = g (onehot - p) in bf16;
//  - dZ [token][vocabulary] leaves straight from registers, 16 bytes per lane and block pair (a token's
//    64 contiguous bytes come from the four lane groups of one store);
//  - dZT [vocabulary][token] needs consecutive tokens, which sit in different lanes: the whole tile is
//    staged once in LDS as [vocabulary row][token] and streamed out with 16 bytes per lane on
//    line-contiguous rows.  One barrier per tile.
// (Also tried: returning the packed block pairs transposed from the matrix cores, by multiplying them with a
// 0/1 selection matrix, so that dZT leaves from registers too and LDS is not used at all.  It is exact, but
// its stores, like those of dZ here, put consecutive lanes on different rows, and with both orientations
// stored that way the kernel was 5 % slower than with this staging.)
template <typename G>
__device__ inline void dz_epilogue_direct(const DzArgs& a, typename G::Acc& acc, int m0, int mrel0, int64_t n0,
                                          char* smem) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  constexpr int P2 = G::BN * 2 + 16;             // pitch of a staged [vocabulary row] of BN tokens
  static_assert(G::BM * P2 <= G::LDS_BYTES && G::NB == 16 && G::VB == 4 && G::TM % 2 == 0, "staging fits in LDS");
  const int q = G::lane() / 16, nl = G::lane() % 16;
  const int mb = G::wave_m() * G::WM + 8 * q;    // lane part of the tile-relative vocabulary row
  const int vlim = a.V - m0 - mb;                // vocabulary rows with offset >= vlim are padding
  const float kz = kLog2e * a.zscale;            // logit = accumulator * zscale

  // per-token scalars of this lane's token columns, requested in one batch (one exposed round trip per
  // tile; requested before the main loop they do not fit next to its double-buffered fragments, and the
  // compiler then spills each one right after its load, which serialises the loads)
  float gj[G::TN], lsej[G::TN];
  int relj[G::TN];
  bool hit = false;
#pragma unroll
  for (int j = 0; j < G::TN; ++j) {
    const int64_t n = n0 + G::n_of(j);
    gj[j] = a.g_c[n];
    lsej[j] = a.lse_c[n];
    relj[j] = a.tok_c[n];
  }
#pragma unroll
  for (int j = 0; j < G::TN; ++j) {
    hit |= (relj[j] >= m0) & (relj[j] < m0 + G::BM);
    relj[j] -= m0 + mb;                          // compared with compile-time constants
  }
  trace_stamp(11, 2);
  // mode 0: no target of the wave's columns in this tile, no padding rows: dZ = -g p, with |g| folded into
  //         the exponent and the sign applied to the packed pair.
  // mode 1: a target somewhere in the tile: the one-hot term by a select (about a third of the tiles have
  //         such a wave at V = 152 k).   mode 2: the vocabulary's last tile (padding rows give 0).
  const int mode = (m0 + G::BM <= a.V) ? (__any(hit) ? 1 : 0) : 2;
  char* const dZ = static_cast<char*>(a.dZ);
  char* const dZT = static_cast<char*>(a.dZT);

#pragma unroll
  for (int j = 0; j < G::TN; ++j) {
    const float g = gj[j];
    const float bias = -lsej[j] * kLog2e;
    const int rel = relj[j];
    const int tl = G::n_of(j);                   // token within the tile
    // rows 8 apart (the four lane groups) would share LDS banks: the 32-byte token groups of a staged
    // row are permuted by (row / 8) % 4, which for this lane's rows is its lane group
    char* const srow = smem + mb * P2 + (((tl >> 4) ^ q) << 5) + nl * 2;
    char* const grow = dZ + ((size_t)(n0 + tl) * a.ldZ + mrel0 + mb) * 2;
    auto emit = [&](auto mode_tag) {
      constexpr int kMode = decltype(mode_tag)::value;
      const float bias0 = bias + __builtin_amdgcn_logf(fabsf(g));   // log2 |g|; -inf for g = 0 gives p = 0
      const uint32_t smask = g > 0.f ? 0x80008000u : 0u;
      const float ng = -g;
#pragma unroll
      for (int ap = 0; ap < G::TM / 2; ++ap) {
        u32x4_t pk;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float dz[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int i = 2 * ap + (w >> 1), v = 2 * (w & 1) + u;
            const float z = acc[i][j][v];
            if constexpr (kMode == 0) {
              dz[u] = fast_exp2(fmaf(z, kz, bias0));
            } else {
              const float p = fast_exp2(fmaf(z, kz, bias));
              const bool oh = DzRows::offset(i, v) == rel;
              if constexpr (kMode == 1)
                dz[u] = fmaf(ng, p, oh ? g : 0.f);
              else
                dz[u] = (DzRows::offset(i, v) < vlim) ? g * ((oh ? 1.f : 0.f) - p) : 0.f;
            }
          }
          const f32x2_t pair = {dz[0], dz[1]};
          uint32_t word = __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf16x2_t));
          if constexpr (kMode == 0) word ^= smask;
          pk[w] = word;
          const int mo = DzRows::offset(2 * ap + (w >> 1), 2 * (w & 1));
          *reinterpret_cast<uint16_t*>(srow + mo * P2) = (uint16_t)word;
          *reinterpret_cast<uint16_t*>(srow + (mo + 1) * P2) = (uint16_t)(word >> 16);
        }
        *reinterpret_cast<u32x4_t*>(grow + 64 * ap) = pk;
        __builtin_amdgcn_sched_barrier(0);        // one block pair's values live at a time
      }
    };
    if (mode == 0)
      emit(std::integral_constant<int, 0>{});
    else if (mode == 1)
      emit(std::integral_constant<int, 1>{});
    else
      emit(std::integral_constant<int, 2>{});
  }
  trace_stamp(12, 2);
  lds_barrier();
  trace_stamp(13, 2);
  // [vocabulary row][token] rows -> dZT
  constexpr int CPR = G::BN * 2 / 16;            // 16-byte chunks per staged row
  constexpr int RPP = G::NT / CPR;               // rows per pass
  static_assert(RPP == 8, "the rows of a pass share their bank permutation");
  const int c = threadIdx.x % CPR;
  const int rin = threadIdx.x / CPR;
#pragma unroll 8
  for (int r0 = 0; r0 < G::BM; r0 += RPP) {
    const int m = r0 + rin;
    const int f = (r0 >> 3) & 3;
    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(smem + m * P2 + ((((c >> 1) ^ f) << 5) | ((c & 1) << 4)));
    *reinterpret_cast<u32x4_t*>(dZT + ((size_t)(mrel0 + m) * a.ldZT + n0 + c * 8) * 2) = v;
  }
}

// E: type of the operands Hc and W (possibly e4m3 copies); EO: type of dZ / dZT.
template <typename E, typename EO>
__global__ __launch_bounds__(Tile<E>::NT) void dz_kernel(DzArgs a) {
  using G = Tile<E, kLeadDz>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int nv = a.hdr->nv;
  const int nblk = (nv + G::BN - 1) / G::BN;
  int mt, nb;
  if (!xcd_tile_coords(blockIdx.x, a.ntiles, nblk, kMapBx, kMapBy, mt, nb)) return;
  trace_stamp(0, 2);
  const int64_t n0 = (int64_t)nb * G::BN;
  const int mrel0 = mt * G::BM;  // within the chunk
  const int m0 = a.c0 + mrel0;
  const int ksteps = a.d * Elem<E>::size / G::KB;
  const int64_t pitchH = a.ldHc * Elem<E>::size;
  const int64_t pitchW = a.ldW * Elem<E>::size;

  // With 16x16 blocks and bf16 output the rows of the W tile enter LDS in a permuted order (DzRows), chosen so that a
  // lane's accumulators of two neighbouring blocks are EIGHT consecutive vocabulary entries of its token:
  // 16 bytes of a dZ row, stored straight from registers.
  constexpr bool kDirect = G::NB == 16 && std::is_same<EO, bf16_tag>::value;
  uint32_t offA[G::A_LD], offB[G::B_LD];
#pragma unroll
  for (int q = 0; q < G::A_LD; ++q) {
    const int row = G::ldA_row(q);
    const int vrow = kDirect ? DzRows::tile_row_of_lds_row(row) : row;
    offA[q] = (uint32_t)((min(m0 + vrow, a.V - 1) - m0) * pitchW) + G::ld_byte(row);
  }
#pragma unroll
  for (int q = 0; q < G::B_LD; ++q) {
    const int row = G::ldB_row(q);
    offB[q] = (uint32_t)(row * pitchH) + G::ld_byte(row);
  }

  typename G::Acc acc;
  G::zero(acc);
  trace_stamp(1, 2);
  G::run(acc, static_cast<const char*>(a.W) + (int64_t)m0 * pitchW, offA,
         static_cast<const char*>(a.Hc) + n0 * pitchH, offB, ksteps, smem, 2);
  trace_stamp(2, 2); trace_cycles(2, 2);
  if constexpr (kDirect) {
    dz_epilogue_direct<G>(a, acc, m0, mrel0, n0, smem);
    trace_stamp(3, 2); trace_cycles(3, 2);
    return;
  }

  // Per-token scalars of this lane's token columns, requested after the main loop in one batch (one
  // exposed round trip per tile).  Requested before it they do not fit the register file next to the
  // loop's double-buffered fragments: the compiler then spills each one right after its load, which
  // serialises the loads (measured: a dozen dependent round trips per tile).
  float gj[G::TN], lsej[G::TN];
  int tkj[G::TN];
#pragma unroll
  for (int j = 0; j < G::TN; ++j) {
    const int64_t n = n0 + G::n_of(j);
    gj[j] = a.g_c[n];
    lsej[j] = a.lse_c[n];
    tkj[j] = a.tok_c[n];
  }
  float biasj[G::TN];
  int relj[G::TN];
  bool hit = false;
#pragma unroll
  for (int j = 0; j < G::TN; ++j) {
    biasj[j] = -lsej[j] * kLog2e;
    hit |= (tkj[j] >= m0) & (tkj[j] < m0 + G::BM);
    relj[j] = tkj[j] - m0 - G::m_base();   // compared with compile-time constants
  }

  char* dZ = static_cast<char*>(a.dZ);
  char* dZT = static_cast<char*>(a.dZT);
  // The tile leaves through LDS so that both copies are written with full 16-byte-per-lane,
  // line-contiguous stores: registers hold 4 consecutive vocabulary entries of one token, which
  // is neither orientation's row.  JG of the wave's TN token blocks are staged per phase (as many
  // as fit next to each other in LDS in both orientations).
  constexpr int ESZ = Elem<EO>::size;
  constexpr int JG = (ESZ == 2 ? 64 : 32) / G::NB;   // token blocks per wave per phase
  constexpr int NTOK = G::WGN * JG * G::NB;       // tokens staged per phase
  constexpr int P1 = G::BM * ESZ + 16;            // pitch of the [token][vocab] staging rows
  constexpr int P2 = NTOK * ESZ + 16;             // pitch of the [vocab][token] staging rows
  constexpr int L2_OFF = NTOK * P1;
  static_assert(L2_OFF + G::BM * P2 <= G::LDS_BYTES, "both staging layouts fit in LDS");
  static_assert(G::TN % JG == 0, "phases cover the wave tile evenly");
  char* st1 = smem;
  char* st2 = smem + L2_OFF;
  const int vlim = a.V - m0 - G::m_base();
  const float kz = kLog2e * a.zscale;              // logit = accumulator * zscale
  // Which form of the element-wise work this wave needs (wave-uniform, see emit below).
  const int mode = (m0 + G::BM <= a.V) ? (__any(hit) ? 1 : 0) : 2;
#pragma unroll
  for (int jg = 0; jg < G::TN / JG; ++jg) {
#pragma unroll
    for (int jj = 0; jj < JG; ++jj) {
      const int j = jg * JG + jj;
      const float g = gj[j];
      const float bias = biasj[j];
      const int rel = relj[j];
      const int tl = G::wave_n() * (JG * G::NB) + jj * G::NB + (G::lane() % G::NB);   // token within the phase
      // mode 0: no target of the wave's columns in this tile, no padding rows: dZ = -g p.
      // mode 1: a target somewhere in the tile: the one-hot term by a select, still no tests around the
      //         exponential (about a third of the tiles have such a wave at V = 152 k).
      // mode 2: the vocabulary's last tile (padding rows give 0).
      auto emit = [&](auto mode_tag) {
        constexpr int kMode = decltype(mode_tag)::value;
        const float ng = -g;
#pragma unroll
        for (int i = 0; i < G::TM; ++i)
#pragma unroll
          for (int q = 0; q < G::VB / 4; ++q) {
            float dz[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float p = fast_exp2(fmaf(acc[i][j][4 * q + e], kz, bias));
              if constexpr (kMode == 0) {
                dz[e] = ng * p;
              } else if constexpr (kMode == 1) {
                dz[e] = fmaf(ng, p, (G::m_const(i, 4 * q + e) == rel) ? g : 0.f);
              } else {
                const float oh = (G::m_const(i, 4 * q + e) == rel) ? 1.f : 0.f;
                dz[e] = (G::m_const(i, 4 * q + e) < vlim) ? g * (oh - p) : 0.f;
              }
            }
            const int mt = G::m_of(i, 4 * q);   // tile-relative vocabulary row, multiple of 4
            Store4<EO>::row(st1 + tl * P1 + mt * ESZ, dz[0], dz[1], dz[2], dz[3]);
#pragma unroll
            for (int e = 0; e < 4; ++e) Store4<EO>::one(st2 + (mt + e) * P2 + tl * ESZ, dz[e]);
          }
      };
      if (mode == 0)
        emit(std::integral_constant<int, 0>{});
      else if (mode == 1)
        emit(std::integral_constant<int, 1>{});
      else
        emit(std::integral_constant<int, 2>{});
    }
    lds_barrier();
    // [token][vocab] rows -> dZ: one staged row is BM*ESZ contiguous bytes of a dZ row
    {
      constexpr int CPR = G::BM * ESZ / 16;   // 16-byte chunks per row
      constexpr int RPP = G::NT / CPR;        // rows per pass
      const int c = threadIdx.x % CPR;
#pragma unroll
      for (int r0 = 0; r0 < NTOK; r0 += RPP) {
        const int tl = r0 + threadIdx.x / CPR;
        const int nl = (tl / (JG * G::NB)) * G::WN + jg * (JG * G::NB) + tl % (JG * G::NB);   // token within the tile
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(st1 + tl * P1 + c * 16);
        *reinterpret_cast<u32x4_t*>(dZ + ((size_t)(n0 + nl) * a.ldZ + mrel0) * ESZ + c * 16) = v;
      }
    }
    // [vocab][token] rows -> dZT: a staged row holds WGN runs of JG*32 consecutive tokens
    {
      constexpr int CPR = NTOK * ESZ / 16;
      constexpr int RPP = G::NT / CPR;
      constexpr int TPC = 16 / ESZ;           // tokens per 16-byte chunk
      const int c = threadIdx.x % CPR;
      const int tl = c * TPC;
      const int nl = (tl / (JG * G::NB)) * G::WN + jg * (JG * G::NB) + tl % (JG * G::NB);
#pragma unroll
      for (int r0 = 0; r0 < G::BM; r0 += RPP) {
        const int m = r0 + threadIdx.x / CPR;
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(st2 + m * P2 + c * 16);
        *reinterpret_cast<u32x4_t*>(dZT + ((size_t)(mrel0 + m) * a.ldZT + n0 + nl) * ESZ) = v;
      }
    }
    if (jg + 1 < G::TN / JG) lds_barrier();
  }
}

// Role: 0 = dH (contracts over a vocabulary chunk), 1 = dW (contracts over the valid tokens), 2 = a
// parameter gradient of the KV gate (contracts over the tokens of a stream).  The code is the same; the
// parameter only gives the uses distinct kernel names in profiles (and picks the lead operand).
template <typename E, int Role>
__global__ __launch_bounds__(Tile<E>::NT) void gemm_t_kernel(GemmTArgs a) {
  using G = Tile<E, (Role == 0 ? kLeadDh : kLeadDw)>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int nv = a.hdr->nv;
  const int64_t n_lim = a.n_from_nv ? (int64_t)nv : a.n_limit;
  // the walk's y axis runs over (slice of the contraction, n tile): neighbours share the slice's K range
  const int ntiles = (int)((n_lim + G::BN - 1) / G::BN);
  int mt, ny;
  if (!xcd_tile_coords(blockIdx.x, (a.M + G::BM - 1) / G::BM, ntiles * a.ksplit, kMapBx, kMapBy, mt, ny)) return;
  const int slice = ny / ntiles;
  const int nt = ny - slice * ntiles;
  const int64_t n0 = (int64_t)nt * G::BN;
  const int m0 = mt * G::BM;
  const int64_t kel = a.k_from_nv ? (int64_t)nv : a.K;
  const int ksteps_all = (int)((kel * Elem<E>::size + G::KB - 1) / G::KB);
  const int per_slice = (ksteps_all + a.ksplit - 1) / a.ksplit;
  const int k_first = slice * per_slice;
  const int ksteps = max(0, min(per_slice, ksteps_all - k_first));
  const int64_t pitchA = a.ldA * Elem<E>::size;
  const int64_t pitchB = a.ldB * Elem<E>::size;

  uint32_t offA[G::A_LD], offB[G::B_LD];
#pragma unroll
  for (int q = 0; q < G::A_LD; ++q) {
    const int row = G::ldA_row(q);
    offA[q] = (uint32_t)(row * pitchA) + G::ld_byte(row);
  }
#pragma unroll
  for (int q = 0; q < G::B_LD; ++q) {
    const int row = G::ldB_row(q);
    offB[q] = (uint32_t)(row * pitchB) + G::ld_byte(row);
  }

  // The wave streams out tile columns (output rows) wave, wave + 4, ... of each phase of the epilogue.
  // Lane 32 p + i fetches the output row of iteration i of phase p now; the epilogue reads it with
  // readlane instead of one dependent global load per row.
  constexpr int JG = 64 / G::NB;                  // column blocks per wave per phase (64 columns)
  constexpr int NCOL = G::WGN * JG * G::NB;       // tile columns (n) staged per phase
  constexpr int ROWS_PER_WAVE = NCOL / G::NWAVES; // per phase
  static_assert(ROWS_PER_WAVE * (G::TN / JG) == 64, "one output row index per lane");
  int my_row;
  {
    const int p = G::lane() / ROWS_PER_WAVE, i = G::lane() % ROWS_PER_WAVE;
    const int r = G::wave() + G::NWAVES * i;
    const int64_t n = n0 + (r / (JG * G::NB)) * G::WN + p * (JG * G::NB) + r % (JG * G::NB);
    int64_t row = -1;
    if (n < n_lim) row = a.part ? n : (a.rowmap ? (int64_t)a.rowmap[n] : a.row_base + n);
    my_row = (int)row;
  }
  float* const outp = a.part ? a.part + (size_t)slice * a.part_slice : a.out;
  const int64_t ldo = a.part ? a.part_ld : a.ldo;
  const bool accumulate = a.part ? a.part_accumulate : a.accumulate;

  typename G::Acc acc;
  G::zero(acc);
  G::run(acc, static_cast<const char*>(a.A) + (int64_t)m0 * pitchA + (int64_t)k_first * G::KB, offA,
         static_cast<const char*>(a.B) + n0 * pitchB + (int64_t)k_first * G::KB, offB, ksteps, smem, Role == 0 ? 3 : (Role == 1 ? 4 : 0));

  // The fp32 tile leaves through LDS as [n][m] rows, so that each output row segment (BM floats
  // = 1 KB) is read-modify-written by one wavefront instruction with 16 bytes per lane.  Rows go in
  // batches: the LDS reads and the loads of the old values of a whole batch are issued before its
  // first store, so the wave (alone on its SIMD) does not sit out one memory round trip per row.
  constexpr int P = G::BM * 4 + 16;               // staging row pitch in bytes
  static_assert(NCOL * P <= G::LDS_BYTES && G::TN % JG == 0, "staging fits in LDS");
  static_assert(G::BM * 4 / 16 == 64, "one staged row is one wavefront store");
  const int c = G::lane();                        // 16-byte chunk of the row = 4 output columns
  const int m = m0 + c * 4;
  const bool m_ok = m < a.M;
#pragma unroll
  for (int jg = 0; jg < G::TN / JG; ++jg) {
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
    constexpr int RB = 8;
#pragma unroll
    for (int i0 = 0; i0 < ROWS_PER_WAVE; i0 += RB) {
      f32x4_t v[RB], old[RB];
      f32x4_t* dst[RB];
#pragma unroll
      for (int u = 0; u < RB; ++u) {
        const int64_t row = __builtin_amdgcn_readlane(my_row, jg * ROWS_PER_WAVE + i0 + u);
        dst[u] = (row >= 0 && m_ok) ? reinterpret_cast<f32x4_t*>(outp + row * ldo + m) : nullptr;
        v[u] = *reinterpret_cast<const f32x4_t*>(smem + (G::wave() + G::NWAVES * (i0 + u)) * P + c * 16);
      }
      if (accumulate) {
#pragma unroll
        for (int u = 0; u < RB; ++u) old[u] = dst[u] ? *dst[u] : f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < RB; ++u) v[u] += old[u];
      }
#pragma unroll
      for (int u = 0; u < RB; ++u)
        if (dst[u]) *dst[u] = v[u];
    }
    if (jg + 1 < G::TN / JG) lds_barrier();
  }
}

}  // namespace

template <typename E>
static hipError_t launch_fwd_e(const FwdArgs& a, hipStream_t s) {
  using G = Tile<E>;
  const dim3 grid(xcd_grid_size(a.ntiles * a.npol, a.Ncap / kTile, kFwdMapBy));
  hipError_t e = allow_lds<fwd_kernel<E>>(G::LDS_BYTES);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fwd_kernel<E>, grid, dim3(G::NT), G::LDS_BYTES, s, a);
  return hipGetLastError();
}

hipError_t launch_fwd(int dtype, const FwdArgs& a, hipStream_t s) {
  if (dtype == kDtypeFp8) return launch_fwd_e<fp8_tag>(a, s);
  return dtype == LMHEAD_BF16 ? launch_fwd_e<bf16_tag>(a, s) : launch_fwd_e<f32_tag>(a, s);
}

template <typename E, typename EO>
static hipError_t launch_dz_e(const DzArgs& a, hipStream_t s) {
  using G = Tile<E>;
  const dim3 grid(xcd_grid_size(a.ntiles, a.Ncap / kTile, kMapBy));
  hipError_t e = allow_lds<dz_kernel<E, EO>>(G::LDS_BYTES);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((dz_kernel<E, EO>), grid, dim3(G::NT), G::LDS_BYTES, s, a);
  return hipGetLastError();
}

hipError_t launch_dz(int op_dtype, int out_dtype, const DzArgs& a, hipStream_t s) {
  if (op_dtype == kDtypeFp8)
    return out_dtype == LMHEAD_BF16 ? launch_dz_e<fp8_tag, bf16_tag>(a, s) : launch_dz_e<fp8_tag, f32_tag>(a, s);
  return op_dtype == LMHEAD_BF16 ? launch_dz_e<bf16_tag, bf16_tag>(a, s) : launch_dz_e<f32_tag, f32_tag>(a, s);
}

template <typename E, int Role>
static hipError_t launch_gemm_t_impl(const GemmTArgs& a, hipStream_t s) {
  using G = Tile<E>;
  const dim3 grid(xcd_grid_size((a.M + kTile - 1) / kTile, a.n_tiles_cap * a.ksplit, kMapBy));
  hipError_t e = allow_lds<gemm_t_kernel<E, Role>>(G::LDS_BYTES);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((gemm_t_kernel<E, Role>), grid, dim3(G::NT), G::LDS_BYTES, s, a);
  return hipGetLastError();
}

hipError_t launch_gemm_t(int dtype, const GemmTArgs& a, hipStream_t s, int role) {
  const bool dw = a.k_from_nv;
  if (role == 2)
    return dtype == LMHEAD_BF16 ? launch_gemm_t_impl<bf16_tag, 2>(a, s) : launch_gemm_t_impl<f32_tag, 2>(a, s);
  if (dtype == LMHEAD_BF16)
    return dw ? launch_gemm_t_impl<bf16_tag, 1>(a, s) : launch_gemm_t_impl<bf16_tag, 0>(a, s);
  return dw ? launch_gemm_t_impl<f32_tag, 1>(a, s) : launch_gemm_t_impl<f32_tag, 0>(a, s);
}

}  // namespace lmhead

#ifdef LMHEAD_TRACE
// Diagnostic build only (not part of the boundary): hands the kernel of the given kind (1 forward, 2 dZ, 3 dH,
// 4 dW) a device buffer of 2 x 2^19 x 16 64-bit words for its time stamps (see trace_stamp in gemm_core.h); NULL
// switches them off.
extern "C" __attribute__((visibility("default"))) int lmhead_debug_set_trace(void* dev_buf, int kind) {
  unsigned long long* p = static_cast<unsigned long long*>(dev_buf);
  hipError_t e = hipMemcpyToSymbol(HIP_SYMBOL(lmhead::g_trace_kind), &kind, sizeof(kind));
  if (e != hipSuccess) return (int)e;
  return (int)hipMemcpyToSymbol(HIP_SYMBOL(lmhead::g_trace), &p, sizeof(p));
}
#endif
