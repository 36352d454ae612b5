// Shared internal declarations of the lmhead library: workspace layout, launcher
// prototypes and small device helpers.  Nothing here is part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/lmhead.h"

namespace lmhead {

// Macro-tile of every contraction: 256 x 256 outputs.
constexpr int kTile = 256;

// Internal operand-type code of the logits kernels when LMHEAD_FLAG_FP8_LOGITS is set (the public
// dtype codes are LMHEAD_F32 = 0 and LMHEAD_BF16 = 1).
constexpr int kDtypeFp8 = 2;

// Sticky error bits written by kernels into WsHeader::err.
constexpr int kErrLen = 1;  // a length outside [0, T]
constexpr int kErrTok = 2;  // a token id outside [0, V) on a valid slot

struct WsHeader {
  int32_t err;  // sticky error bits
  int32_t nv;   // number of valid slots N_v (written by the index kernel)
  int32_t pad[62];
};
static_assert(sizeof(WsHeader) == 256, "header is one 256-byte line");

static inline size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

// Byte offsets of every workspace region for one descriptor.  All regions are
// 256-byte aligned.  "cap" sizes are worst cases (every slot valid) because
// N_v lives on the device.
struct WsLayout {
  int esz;          // element size of H/W in bytes
  int64_t N, R;     // slots, responses
  int64_t Ncap;     // N rounded up to the tile
  int64_t Vp;       // V rounded up to the tile
  int64_t dp;       // d rounded up to the tile
  int64_t Vc;       // vocabulary chunk of the backward (multiple of the tile)
  int64_t nchunks;  // number of vocabulary chunks
  int64_t ntiles;   // vocabulary tiles = planes of per-tile softmax statistics per row
  // Row pitches (elements) of the workspace matrices.  Each is its logical width plus one
  // 128-byte line: a power-of-two pitch would put every row of a tile on the same L2
  // channel and set (the token-major operands have a pitch of Ncap elements, often 2^k).
  int64_t ldHc, ldHcT, ldWT, ldZ, ldZT;
  int64_t ld8;      // pitch (bytes) of the e4m3 operand copies: d + one 128-byte line
  int ksplit;       // dH: slices of the contraction per output tile (> 1 only when the tile grid
                    // alone would leave most of the chip idle); partial tiles go to dHpart
  size_t dHpart;
  size_t dWpart;        // partial tiles of the dW launches that split a remainder of vocabulary tiles
  size_t dWpart_bytes;
  size_t hdr, cu_len, row_slot, tok_c, gid, g_c, lse_c, zy, part, Hc, HcT, WT, dZ, dZT, Hc8, W8, total;
};

// Default backward chunk: as wide as keeps the two dZ copies (worst case: every slot valid)
// within about 48 GB, at most 262144 columns (small problems take the whole vocabulary in one
// chunk).  Wider chunks mean fewer read-modify-write passes over dH and longer contractions per
// launch.
static inline int64_t default_vocab_chunk(const lmhead_desc* d) {
  const int64_t esz = d->dtype == LMHEAD_BF16 ? 2 : 4;
  const int64_t N = (int64_t)d->P * d->G * d->T;
  int64_t vc = (48ll << 30) / (2 * esz * (N > 0 ? N : 1));
  vc = vc / kTile * kTile;
  if (vc > 262144) vc = 262144;
  if (vc < 4 * kTile) vc = 4 * kTile;
  return vc;
}


// Weight matrices one forward launch can evaluate over the same hidden states.
constexpr int kMaxPolicies = 4;

// npol: number of weight matrices of a multi-policy forward (each has its own target-logit vector
// and planes of per-tile softmax statistics).
static inline WsLayout make_layout(const lmhead_desc* d, int npol = 1) {
  WsLayout L{};
  L.esz = d->dtype == LMHEAD_BF16 ? 2 : 4;
  L.R = (int64_t)d->P * d->G;
  L.N = L.R * d->T;
  L.Ncap = (int64_t)round_up((size_t)L.N, kTile);
  L.Vp = (int64_t)round_up((size_t)d->V, kTile);
  L.dp = (int64_t)round_up((size_t)d->d, kTile);
  int64_t vc = d->vocab_chunk > 0 ? d->vocab_chunk : default_vocab_chunk(d);
  vc = (int64_t)round_up((size_t)vc, kTile);
  if (vc > L.Vp) vc = L.Vp;
  L.Vc = vc;
  L.nchunks = (L.Vp + vc - 1) / vc;
  L.ntiles = L.Vp / kTile;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += round_up(bytes, 256);
    return o;
  };
  L.hdr = take(sizeof(WsHeader));
  L.cu_len = take((size_t)(L.R + 1) * 4);
  L.row_slot = take((size_t)L.Ncap * 4);
  L.tok_c = take((size_t)L.Ncap * 4);
  L.gid = take((size_t)npol * L.Ncap * 4);
  L.g_c = take((size_t)L.Ncap * 4);
  L.lse_c = take((size_t)L.Ncap * 4);
  L.zy = take((size_t)npol * L.Ncap * 4);
  L.part = take((size_t)npol * 3 * L.ntiles * L.Ncap * 4);
  const int64_t pad = 128 / L.esz;
  L.ldHc = d->d + pad;
  L.ldHcT = L.Ncap + pad;
  L.ldWT = L.Vp + pad;
  L.ldZ = L.Vc + pad;
  L.ldZT = L.Ncap + pad;
  L.Hc = take((size_t)L.Ncap * L.ldHc * L.esz);
  L.HcT = take((size_t)L.dp * L.ldHcT * L.esz);
  L.WT = take((size_t)L.dp * L.ldWT * L.esz);
  L.dZ = take((size_t)L.Ncap * L.ldZ * L.esz);
  L.dZT = take((size_t)L.Vc * L.ldZT * L.esz);
  // dH has (d / 256) x (tokens / 256) output tiles.  Below about four per compute unit the last
  // round of workgroups is mostly empty, so the contraction of each tile is cut into ksplit slices
  // that run as separate workgroups and are summed afterwards in a fixed order.
  {
    const int64_t tiles = (L.dp / kTile) * (L.Ncap / kTile);
    int64_t ks = tiles >= 1024 ? 1 : (1536 + tiles - 1) / tiles;
    if (ks > 8) ks = 8;
    L.ksplit = (int)ks;
    // a bf16 dH is accumulated in these fp32 buffers too and rounded once at the end
    const bool need = ks > 1 || (d->flags & LMHEAD_FLAG_DH_BF16) != 0;
    L.dHpart = take(need ? (size_t)ks * L.Ncap * L.dp * 4 : 0);
  }
  // dW: the vocabulary tiles of a chunk that would start a mostly empty round of workgroups are contracted
  // in slices instead (see lmhead_logprob_bwd); slices x rows x d of them never exceed compute units x 64 Ki floats
  L.dWpart_bytes = (size_t)128 << 20;
  if ((size_t)L.Vc * L.dp * 4 * 8 < L.dWpart_bytes) L.dWpart_bytes = (size_t)L.Vc * L.dp * 4 * 8;
  L.dWpart = take(L.dWpart_bytes);
  L.ld8 = d->d + 128;
  const bool fp8 = (d->flags & LMHEAD_FLAG_FP8_LOGITS) != 0;
  L.Hc8 = take(fp8 ? (size_t)L.Ncap * L.ld8 : 0);
  L.W8 = take(fp8 ? (size_t)npol * L.Vp * L.ld8 : 0);
  L.total = off;
  return L;
}

// ---- launchers (each enqueues on `s` and returns hipGetLastError()) --------------------

// lens -> cu_len, header.nv, mask, row_slot (padded with -1 up to the next tile multiple).
hipError_t launch_index(const int32_t* len, int R, int T, WsHeader* hdr, int32_t* cu_ws,
                        int32_t* row_slot, uint8_t* mask_out, int32_t* cu_out, hipStream_t s);

// Gathers the valid rows of H into the dense, zero-padded Hc[Ncap x d]; also compacts tok
// (range-checked), and optionally g_logp and lse.  The npol vectors zy[p * Ncap + .] are cleared and
// the npol vectors gid[p * Ncap + .] set to -1.
hipError_t launch_compact(int dtype, const void* H, int64_t ldH, int d, int V, const int32_t* tok,
                          const float* g, const float* lse, int64_t N, WsHeader* hdr,
                          const int32_t* row_slot, void* Hc, int64_t ldHc, int32_t* tok_c, float* g_c,
                          float* lse_c, float* zy, int32_t* gid, int npol, int64_t Ncap, hipStream_t s);

// out[c][r] = in[r][c] for r < rows (rows read from the header when rows_from_nv), zero padding
// up to out's extent [cols_p x rows_p] (pitch ld_out >= rows_p).
hipError_t launch_transpose(int dtype, const void* in, int64_t ld_in, int64_t rows_cap, int cols,
                            bool rows_from_nv, const WsHeader* hdr, void* out, int64_t ld_out,
                            int64_t rows_p, int64_t cols_p, hipStream_t s);

struct FwdArgs {
  const void* Hc;      // [Ncap x d], pitch ldHc
  int64_t ldHc;
  const void* W[kMaxPolicies];   // npol matrices [V x d], stride ldW (same hidden states for all)
  int npol;
  int64_t ldW;
  int d, V;
  int64_t Ncap;
  int ntiles;          // vocabulary tiles (one per workgroup and policy)
  const int32_t* tok_c;
  const WsHeader* hdr;
  float* part;         // [npol][3][ntiles][Ncap]: per-tile (max, sum exp, sum exp*z) of each row
  bool want_entropy;   // false: sum exp*z is not accumulated (its plane holds zeros)
  float* zy;           // [npol][Ncap]
  int32_t* gid;        // [npol][Ncap]: vocabulary column whose logit was captured as the target's
  float zscale;        // logits = accumulator * zscale (1, or 2^-(e_H + e_W) for e4m3 operands)
};
hipError_t launch_fwd(int dtype, const FwdArgs& a, hipStream_t s);

// Merges the per-tile partials and scatters logp / lse / entropy to slot order (0 on padding).
hipError_t launch_finalize(const float* part, const float* zy, int ntiles, int64_t Ncap,
                           const int32_t* len, const int32_t* cu_len, int R, int T, float* logp,
                           float* lse, float* entropy, hipStream_t s);

struct DzArgs {
  const void* Hc;
  int64_t ldHc;
  const void* W;
  int64_t ldW;
  int d, V;
  int64_t Ncap;
  int64_t ldZ;    // pitch of dZ (elements)
  int64_t ldZT;   // pitch of dZT (elements)
  int c0;         // first vocabulary id of the chunk
  int ntiles;     // vocabulary tiles in this chunk
  const int32_t* tok_c;
  const float* g_c;
  const float* lse_c;
  const WsHeader* hdr;
  void* dZ;       // [Ncap x chunk], pitch ldZ
  void* dZT;      // [chunk x Ncap], pitch ldZT
  float zscale;   // as in FwdArgs
};
// op_dtype: type of Hc / W as given in the arguments (LMHEAD_F32, LMHEAD_BF16 or kDtypeFp8);
// out_dtype: type of dZ / dZT (LMHEAD_F32 or LMHEAD_BF16; equal to op_dtype unless that is e4m3).
hipError_t launch_dz(int op_dtype, int out_dtype, const DzArgs& a, hipStream_t s);

// out[r][c] = e4m3(in[r][c] * 2^exp2) (clamped to +-448, round to nearest even) for r < rows, 0 for the
// padding rows up to rows_p; rows = header.nv when rows_from_nv (then only rows below the next tile
// multiple are written).  cols is a multiple of 8; ld_out in bytes.
hipError_t launch_quantize_e4m3(int dtype, const void* in, int64_t ld_in, int64_t rows_fixed, bool rows_from_nv,
                                const WsHeader* hdr, int cols, int exp2, void* out, int64_t ld_out, int64_t rows_p,
                                hipStream_t s);

// Generic C^T-store contraction: for m < M, n < Nn: out[rowmap(n)][m] (+)= sum_k A[m][k] B[n][k].
struct GemmTArgs {
  const void* A;       // [Mp x K], pitch ldA elements
  int64_t ldA;
  const void* B;       // [Np x K], pitch ldB elements
  int64_t ldB;
  int M;               // valid output columns (d)
  int64_t n_limit;     // valid n (ignored when n_from_nv)
  bool n_from_nv;      // n extent = header.nv (dH); else n_limit (dW)
  bool k_from_nv;      // K extent = header.nv rounded up (dW); else K
  int64_t K;           // contraction length in elements (multiple of 128/esz)
  const int32_t* rowmap;  // output row of n, or NULL for identity + row_base
  int64_t row_base;
  float* out;          // dense rows of M floats
  int64_t ldo;
  bool accumulate;
  int64_t n_tiles_cap; // grid extent over n
  const WsHeader* hdr;
  int ksplit;          // slices of the contraction per output tile (>= 1)
  float* part;         // non-null: slice s writes (part_accumulate: adds) its tile to part[s][n][m], dense
  int64_t part_ld;     // rows of part_ld floats without the row map, and launch_splitk_reduce forms out
  int64_t part_slice;  // from the slices.  part_slice = floats per slice.  Required when ksplit > 1.
  bool part_accumulate;
};

// out[row(n)][m] (+)= sum_s part[s][n][m] for n < n_valid, m < M, slices summed in order.  With a row map:
// row(n) = rowmap[n] and n_valid = header.nv; without: row(n) = row_base + n and n_valid = n_cap.
// out is float, or bf16 when out_bf16 (then accumulate must be false).
hipError_t launch_splitk_reduce(const float* part, int ksplit, int64_t part_slice, int64_t part_ld, int M,
                                const int32_t* rowmap, const WsHeader* hdr, int64_t n_cap, void* out, int64_t ldo,
                                bool accumulate, bool out_bf16, hipStream_t s, int64_t row_base = 0);
// Compute units of the current device (asked of the runtime once per device; 256 if it cannot be asked).
int device_compute_units();
// role: -1 = by use (dW when k_from_nv, else dH); 2 = parameter gradient of the KV gate (distinct kernel name).
hipError_t launch_gemm_t(int dtype, const GemmTArgs& a, hipStream_t s, int role = -1);

// Rows of dH that belong to padded slots are set to 0.
hipError_t launch_zero_padded_rows(void* dH, bool bf16, int d, const int32_t* len, int R, int T,
                                   hipStream_t s);

hipError_t launch_group_advantage(const float* reward, int P, int G, float eps, int ddof,
                                  float* adv, hipStream_t s);
hipError_t launch_grpo(const float* lp, const float* lo, const float* lr, const float* adv,
                       const int32_t* len, int P, int G, int T, float clip_lo, float clip_hi,
                       float kl, int agg, float* loss, float* g, float* stats, float* ws,
                       hipStream_t s);
hipError_t launch_ce(const float* lp, const int32_t* len, int R, int T, float* loss, float* g, float* ws,
                     hipStream_t s);
hipError_t launch_flowrl(const float* lp, const float* lr, const float* reward, const float* logZ,
                         const int32_t* len, int P, int G, int T, float beta, float* loss,
                         float* g, float* gz, float* resid, float* ws, hipStream_t s);

// Bare matrix-core loop on register operands (measurement aid): `workgroups` x 4 wavefronts, `iters` x 2^20
// flop each; operands: 256 bytes per thread, sink: one float per thread.
hipError_t launch_mfma_probe(const void* operands, float* sink, int workgroups, int iters, hipStream_t s);

constexpr int kLossSlotsPerBlock = 2048;

// grpo_loss_noalloc keeps its block partials (four floats per block of kLossSlotsPerBlock slots of one
// response) in a device array of the library image: at most this many blocks, 1 MiB.
constexpr int kStaticLossParts = 65536;
// Device address of that array on the current device (no allocation; resolved once per device).
hipError_t static_scratch(float** out);

// ---- optional per-kernel timing -------------------------------------------------------
// When enabled, each MFMA kernel launch is bracketed by two HIP events recorded on the launch
// stream.  The pool is fixed-size; launches beyond it are simply not timed.
// Kinds: 0 logits fwd, 1 dZ recompute, 2 dH, 3 dW, 4 spectral projection, 5 gate logits,
// 6 truncation mask, 7 low-rank reconstruction; gate backward: 8 mask backward, 9 g_x~ product, 10 dx
// product, 11 dW, 12 dU, 13 operand transposes.
constexpr int kTimingKinds = 14;
constexpr int kTimingPool = 8192;
struct TimingState {
  bool on = false;
  int used = 0;
  hipEvent_t start[kTimingPool];
  hipEvent_t stop[kTimingPool];
  int kind[kTimingPool];
  int created = 0;
};
extern TimingState g_timing;

struct TimedLaunch {
  hipStream_t s;
  int slot = -1;
  TimedLaunch(int kind, hipStream_t stream) : s(stream) {
    if (!g_timing.on || g_timing.used >= g_timing.created) return;
    slot = g_timing.used++;
    g_timing.kind[slot] = kind;
    (void)hipEventRecord(g_timing.start[slot], s);
  }
  ~TimedLaunch() {
    if (slot >= 0) (void)hipEventRecord(g_timing.stop[slot], s);
  }
};

#define LM_TRY(expr)                               \
  do {                                             \
    if ((expr) != hipSuccess) return LMHEAD_E_HIP; \
  } while (0)

// Raises a kernel's dynamic LDS limit to at least `bytes`.  The runtime is asked only when a launch needs more
// than what it has already granted this kernel on the current device (the kernel is a template argument, so
// each instantiation keeps its own record).
template <auto kernel>
inline hipError_t allow_lds(int bytes) {
  constexpr int kMaxDev = 64;
  static std::atomic<int> granted[kMaxDev];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < kMaxDev;
  if (tracked && granted[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && tracked) {
    int seen = granted[dev].load(std::memory_order_relaxed);
    while (seen < bytes && !granted[dev].compare_exchange_weak(seen, bytes, std::memory_order_release)) {
    }
  }
  return e;
}

}  // namespace lmhead
