// Internal declarations of the KV-compression path: workspace layout and launcher prototypes.
#pragma once

#include "../../include/dynakv.h"
#include "common.h"

namespace lmhead {

constexpr int kKvMaxD = 8192;
constexpr int kKvScanBlock = 1024;   // tokens per block of the offset scan

// Sticky error bits of this path (same header word as the LM-head path).
constexpr int kErrKvCount = 4;       // a k outside [0, d]
constexpr int kErrKvCapacity = 8;    // a segment beyond the capacity of the store

struct KvLayout {
  int esz;
  int64_t n, d;
  int64_t ncap;      // n rounded up to the tile
  int64_t dp;        // d rounded up to the tile
  int64_t ldT;       // pitch (elements) of the transposed parameter copies: d + one 128-byte line
  int nbuckets;      // K-steps a token can need, plus one: d * esz / 128 + 1
  size_t hdr, UT, WT, UiT, logits, order, pos_off, pos_len, hist, blocksum, red, total;
};

static inline KvLayout make_kv_layout(const dynakv_desc* d) {
  KvLayout L{};
  L.esz = d->dtype == LMHEAD_BF16 ? 2 : 4;
  L.n = d->n;
  L.d = d->d;
  L.ncap = (int64_t)round_up((size_t)L.n, kTile);
  L.dp = (int64_t)round_up((size_t)L.d, kTile);
  L.ldT = L.d + 128 / L.esz;
  L.nbuckets = (int)(L.d * L.esz / 128) + 1;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += round_up(bytes, 256);
    return o;
  };
  L.hdr = take(sizeof(WsHeader));
  L.UT = take((size_t)L.dp * L.ldT * L.esz);
  L.WT = take((size_t)L.dp * L.ldT * L.esz);
  L.UiT = take((size_t)L.dp * L.ldT * L.esz);
  L.logits = take((size_t)L.ncap * L.d * 4);
  L.order = take((size_t)L.ncap * 4);
  L.pos_off = take((size_t)L.ncap * 4);
  L.pos_len = take((size_t)L.ncap * 4);
  L.hist = take((size_t)L.nbuckets * 3 * 4);          // counts, start positions, cursors
  L.blocksum = take((size_t)(L.ncap / kKvScanBlock + 2) * 8);
  L.red = take((size_t)(L.ncap / 256 + 2) * 2 * 8);   // per-block partial sums of the retain rate
  L.total = off;
  return L;
}

// Workspace of the gate's backward pass (dynakv_gate_bwd).  The two token-major gradients g_l and
// g_xt are kept in the storage type; T1 / T2 hold the token-contiguous (transposed) operand copies of
// one parameter-gradient contraction at a time.
struct KvBwdLayout {
  int esz;
  int64_t n, d, ncap, dp, ldT;
  int64_t ldK;       // pitch (elements) of the token-contiguous copies: ncap + one 128-byte line
  int ksplit;        // slices of the contraction over tokens per output tile of dW / dU
  int nblk;          // workgroups of the mask backward kernel = rows of the db partial sums
  size_t hdr, Wp, Up, WT, logits, gl, gxt, T1, T2, part, dbpart, total;
};

// Workgroups of the mask backward kernel: four 256-thread workgroups fit a compute unit (128 VGPRs),
// so 1024 is one resident round on 256 compute units; each wavefront loops over its share of tokens.
constexpr int kKvBwdMaxBlocks = 1024;

static inline KvBwdLayout make_kv_bwd_layout(const dynakv_desc* d) {
  KvBwdLayout L{};
  L.esz = d->dtype == LMHEAD_BF16 ? 2 : 4;
  L.n = d->n;
  L.d = d->d;
  L.ncap = (int64_t)round_up((size_t)L.n, kTile);
  L.dp = (int64_t)round_up((size_t)L.d, kTile);
  L.ldT = L.d + 128 / L.esz;
  L.ldK = L.ncap + 128 / L.esz;
  {
    // (d / 256)^2 output tiles; the contraction over the tokens is cut so that about one workgroup
    // per compute unit runs, each slice keeping at least 8 K-steps
    const int64_t tiles = (L.dp / kTile) * (L.dp / kTile);
    const int64_t ksteps = L.ncap * L.esz / 128;
    int64_t ks = (256 + tiles - 1) / tiles;
    if (ks > ksteps / 8) ks = ksteps / 8;
    if (ks < 1) ks = 1;
    L.ksplit = (int)ks;
  }
  {
    const int64_t blocks = (L.n + 3) / 4;
    L.nblk = (int)(blocks < kKvBwdMaxBlocks ? blocks : kKvBwdMaxBlocks);
  }
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += round_up(bytes, 256);
    return o;
  };
  L.hdr = take(sizeof(WsHeader));
  L.Wp = take((size_t)L.dp * L.ldT * L.esz);
  L.Up = take((size_t)L.dp * L.ldT * L.esz);
  L.WT = take((size_t)L.dp * L.ldT * L.esz);
  L.logits = take((size_t)L.ncap * L.d * 4);
  L.gl = take((size_t)L.ncap * L.d * L.esz);
  L.gxt = take((size_t)L.ncap * L.d * L.esz);
  L.T1 = take((size_t)L.dp * L.ldK * L.esz);
  L.T2 = take((size_t)L.dp * L.ldK * L.esz);
  L.part = take((size_t)L.ksplit * L.d * L.d * 4);
  L.dbpart = take((size_t)L.nblk * L.d * 4);
  L.total = off;
  return L;
}

// Plain contraction on the MFMA tile core with a transposed store:
//   out[row(n)][m] = sum_k A[m][k] * Bop[n][k],  m < M, n < Nn.
// mode 0/1: Bop rows are dense rows of B (pitch ldB), row(n) = n.  The output is the storage type
//           (out_e) or fp32 (out_f), whichever is non-null.
// mode 2:   ragged rows: Bop[n] = the pos_len[n] bytes of the packed store at byte offset pos_off[n],
//           zero beyond; row(n) = order[n] (< 0: no token); the tile's step count follows its
//           first row, the longest (the three arrays are written by launch_kv_order).
struct KvGemmArgs {
  int mode;
  const void* A;        // [dp x K] transposed parameter copy, pitch ldA
  int64_t ldA;
  const void* B;        // dense rows (mode 0/1) or the packed store (mode 2)
  int64_t ldB;
  int64_t bytesB;       // mode 2: bytes readable at B
  int M;                // output columns (d)
  int64_t Nn;           // tokens
  int K;                // contraction length in elements (d)
  const int32_t* order;     // mode 2
  const uint32_t* pos_off;  // mode 2
  const int32_t* pos_len;   // mode 2
  void* out_e;
  float* out_f;
  int64_t ldo;
  bool accumulate;      // mode 0/1: the tile is added to what the output holds (rounded once more for bf16)
  WsHeader* hdr;
  int walk_len;         // set by the launcher: length of the tile walk (tile_map.h)
};
hipError_t launch_kv_gemm(int dtype, const KvGemmArgs& a, hipStream_t s);

// Softmax over the gate logits (+ bias), the cumulative mask, the threshold count and the
// optional training outputs.
hipError_t launch_kv_mask(int dtype, const float* logits, const float* b, const void* xt, int64_t n, int d,
                          float tau, bool literal, int32_t* k, float* m, void* xhat, hipStream_t s);

// off = off_base + exclusive prefix sum of roundup(k, 8); then the segments are copied.
hipError_t launch_kv_store(int dtype, const void* xt, const int32_t* k, int64_t n, int d, int64_t off_base,
                           int64_t* off, void* packed, int64_t capacity, int64_t* blocksum, WsHeader* hdr,
                           hipStream_t s);

// order = tokens sorted by descending number of K-steps (ceil(k * esz / 128)), padded with -1 up to
// ncap; pos_off / pos_len = byte offset and byte length (k rounded up to the granule) of each sorted
// position's segment in a store of `bytes` readable bytes (0x80000000 / 0 for padding and for
// segments that do not lie inside it, which also set the error word).  hist holds 3 * nbuckets ints
// of scratch.
hipError_t launch_kv_order(int dtype, const int32_t* k, const int64_t* off, int64_t bytes, int64_t n, int64_t ncap,
                           int d, int nbuckets, int32_t* hist, int32_t* order, uint32_t* pos_off, int32_t* pos_len,
                           WsHeader* hdr, hipStream_t s);

hipError_t launch_kv_retain(const int32_t* k, const float* m, int64_t n, int d, float alpha, float* out,
                            float* g_m, double* red, hipStream_t s);

// Backward of softmax + cumulative mask + soft gating for every token (one wavefront per token):
//   q = g_xhat * xt + g_m + g_m_const;  r = inclusive prefix sums of q;  g_l = p * (r - sum p r);
//   a = g_xhat * m.
// g_l goes to gl (gate column order) and a to a_out, both [n x d] in the storage type; dbpart
// receives one row of column sums of g_l per workgroup (nblk rows, launch grid = nblk).
hipError_t launch_kv_mask_bwd(int dtype, const float* logits, const float* b, const void* xt, const void* g_xhat,
                              const float* g_m, float g_m_const, int64_t n, int d, bool literal, void* gl,
                              void* a_out, float* dbpart, int nblk, hipStream_t s);

// out[j] (+)= sum_r part[r][j] for j < len (rows of pitch row_pitch floats), in a fixed order.
hipError_t launch_kv_sum_rows(const float* part, int rows, int64_t row_pitch, int64_t len, float* out,
                              bool accumulate, hipStream_t s);

// out[r][c] = in[r][c] for r < rows, c < cols; zero up to [rows_p x ld_out].
hipError_t launch_kv_pad_copy(int dtype, const void* in, int64_t ld_in, int rows, int cols, void* out,
                              int64_t ld_out, int rows_p, hipStream_t s);

// out[c][r] = in[r][c] for r < rows, c < cols; zero up to [cols_p x rows_p] (pitch ld_out).  Rows of both
// sides 16-byte aligned; cols, cols_p, rows_p multiples of 64.
hipError_t launch_kv_transpose(int dtype, const void* in, int64_t ld_in, int64_t rows, int cols, void* out,
                               int64_t ld_out, int64_t rows_p, int cols_p, hipStream_t s);

hipError_t launch_kv_clear_header(WsHeader* hdr, hipStream_t s);

}  // namespace lmhead
