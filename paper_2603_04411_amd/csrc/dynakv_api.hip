// extern "C" entry points of the KV-compression path: host-side validation, workspace carving and
// kernel sequencing.  Every argument error is returned before anything is enqueued.
#include "dynakv_common.h"

using namespace lmhead;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

int validate(const dynakv_desc* d) {
  if (!d) return LMHEAD_E_NULL;
  if (d->n <= 0 || d->d <= 0 || d->d > kKvMaxD || d->d % 64 != 0) return LMHEAD_E_SHAPE;
  if (d->dtype != LMHEAD_F32 && d->dtype != LMHEAD_BF16) return LMHEAD_E_DTYPE;
  if (d->flags & ~(uint32_t)(DYNAKV_FLAG_LITERAL_FLIP | DYNAKV_FLAG_ACCUM_GRAD)) return LMHEAD_E_DTYPE;
  if (d->reserved != 0 || d->ldx < d->d) return LMHEAD_E_SHAPE;
  const int64_t esz = d->dtype == LMHEAD_BF16 ? 2 : 4;
  if ((int64_t)d->n * d->d * esz > ((int64_t)1 << 31) - ((int64_t)1 << 20)) return LMHEAD_E_SHAPE;
  if ((int64_t)d->n > (int64_t)INT32_MAX - 2 * kTile) return LMHEAD_E_SHAPE;
  if ((d->ldx * esz) % 16 != 0) return LMHEAD_E_ALIGN;
  return LMHEAD_OK;
}

struct Ws {
  KvLayout L;
  char* base;
  template <typename T>
  T* at(size_t off) const { return reinterpret_cast<T*>(base + off); }
};

// common prologue of the compute entry points
int open_ws(const dynakv_desc* desc, void* ws, size_t ws_bytes, Ws& w) {
  const int rc = validate(desc);
  if (rc != LMHEAD_OK) return rc;
  if (!ws) return LMHEAD_E_NULL;
  if (!aligned256(ws)) return LMHEAD_E_ALIGN;
  w.L = make_kv_layout(desc);
  w.base = static_cast<char*>(ws);
  if (ws_bytes < w.L.total) return LMHEAD_E_WORKSPACE;
  return LMHEAD_OK;
}

}  // namespace

extern "C" {

int dynakv_validate_desc(const dynakv_desc* desc) { return validate(desc); }

size_t dynakv_workspace_bytes(const dynakv_desc* desc) {
  if (validate(desc) != LMHEAD_OK) return 0;
  return make_kv_layout(desc).total;
}

int dynakv_gate(const dynakv_desc* desc, const void* x, const void* U, const void* W, const float* b, float tau,
                void* xt, int32_t* k, float* m, void* xhat, void* ws, size_t ws_bytes, void* stream) {
  Ws w;
  const int rc = open_ws(desc, ws, ws_bytes, w);
  if (rc != LMHEAD_OK) return rc;
  if (!x || !U || !W || !b || !xt || !k) return LMHEAD_E_NULL;
  if (!aligned16(x) || !aligned16(U) || !aligned16(W) || !aligned16(b) || !aligned16(xt) ||
      (m && !aligned16(m)) || (xhat && !aligned16(xhat)))
    return LMHEAD_E_ALIGN;
  const KvLayout& L = w.L;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WsHeader* hdr = w.at<WsHeader>(L.hdr);
  const int dt = desc->dtype;
  const int d = desc->d;

  LM_TRY(launch_kv_clear_header(hdr, s));
  // K-contiguous copies of the two parameter matrices: UT[j][k] = U[k][j], WT likewise
  LM_TRY(launch_transpose(dt, U, d, d, d, false, hdr, w.at<void>(L.UT), L.ldT, d, L.dp, s));
  LM_TRY(launch_transpose(dt, W, d, d, d, false, hdr, w.at<void>(L.WT), L.ldT, d, L.dp, s));

  KvGemmArgs ga{};
  ga.mode = 0;
  ga.A = w.at<void>(L.UT);
  ga.ldA = L.ldT;
  ga.B = x;
  ga.ldB = desc->ldx;
  ga.M = d;
  ga.Nn = L.n;
  ga.K = d;
  ga.out_e = xt;
  ga.ldo = d;
  ga.hdr = hdr;
  {
    TimedLaunch tl(4, s);
    LM_TRY(launch_kv_gemm(dt, ga, s));
  }
  ga.mode = 1;
  ga.A = w.at<void>(L.WT);
  ga.B = xt;
  ga.ldB = d;
  ga.out_e = nullptr;
  ga.out_f = w.at<float>(L.logits);
  {
    TimedLaunch tl(5, s);
    LM_TRY(launch_kv_gemm(dt, ga, s));
  }
  {
    TimedLaunch tl(6, s);
    LM_TRY(launch_kv_mask(dt, w.at<float>(L.logits), b, xt, L.n, d, tau,
                          (desc->flags & DYNAKV_FLAG_LITERAL_FLIP) != 0, k, m, xhat, s));
  }
  return LMHEAD_OK;
}

int dynakv_store(const dynakv_desc* desc, const void* xt, const int32_t* k, int64_t off_base, int64_t* off,
                 void* packed, int64_t capacity, void* ws, size_t ws_bytes, void* stream) {
  Ws w;
  const int rc = open_ws(desc, ws, ws_bytes, w);
  if (rc != LMHEAD_OK) return rc;
  if (!xt || !k || !off || !packed) return LMHEAD_E_NULL;
  if (capacity < 0 || off_base < 0 || off_base % DYNAKV_GRANULE != 0) return LMHEAD_E_SHAPE;
  if (!aligned16(xt) || !aligned16(packed) || (reinterpret_cast<uintptr_t>(off) & 7u)) return LMHEAD_E_ALIGN;
  const KvLayout& L = w.L;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WsHeader* hdr = w.at<WsHeader>(L.hdr);
  LM_TRY(launch_kv_clear_header(hdr, s));
  LM_TRY(launch_kv_store(desc->dtype, xt, k, L.n, desc->d, off_base, off, packed, capacity,
                         w.at<int64_t>(L.blocksum), hdr, s));
  return LMHEAD_OK;
}

int dynakv_reconstruct(const dynakv_desc* desc, const void* packed, int64_t packed_elems, const int64_t* off,
                       const int32_t* k, const void* U_inv, void* xbar, void* ws, size_t ws_bytes, void* stream) {
  Ws w;
  const int rc = open_ws(desc, ws, ws_bytes, w);
  if (rc != LMHEAD_OK) return rc;
  if (!packed || !off || !k || !U_inv || !xbar) return LMHEAD_E_NULL;
  const KvLayout& L = w.L;
  if (packed_elems < 0 || packed_elems * L.esz > ((int64_t)1 << 31) - 256) return LMHEAD_E_SHAPE;
  if (!aligned16(packed) || !aligned16(U_inv) || !aligned16(xbar) || (reinterpret_cast<uintptr_t>(off) & 7u))
    return LMHEAD_E_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WsHeader* hdr = w.at<WsHeader>(L.hdr);
  const int dt = desc->dtype;
  const int d = desc->d;

  LM_TRY(launch_kv_clear_header(hdr, s));
  // A[j][kk] = U_inv[kk][j]: row j of the copy is output column j, contiguous over the retained index
  LM_TRY(launch_transpose(dt, U_inv, d, d, d, false, hdr, w.at<void>(L.UiT), L.ldT, d, L.dp, s));
  LM_TRY(launch_kv_order(dt, k, off, packed_elems * L.esz, L.n, L.ncap, d, L.nbuckets, w.at<int32_t>(L.hist),
                         w.at<int32_t>(L.order), w.at<uint32_t>(L.pos_off), w.at<int32_t>(L.pos_len), hdr, s));

  KvGemmArgs ga{};
  ga.mode = 2;
  ga.A = w.at<void>(L.UiT);
  ga.ldA = L.ldT;
  ga.B = packed;
  ga.bytesB = packed_elems * L.esz;
  ga.M = d;
  ga.Nn = L.n;
  ga.K = d;
  ga.order = w.at<int32_t>(L.order);
  ga.pos_off = w.at<uint32_t>(L.pos_off);
  ga.pos_len = w.at<int32_t>(L.pos_len);
  ga.out_e = xbar;
  ga.ldo = d;
  ga.hdr = hdr;
  {
    TimedLaunch tl(7, s);
    LM_TRY(launch_kv_gemm(dt, ga, s));
  }
  return LMHEAD_OK;
}

int dynakv_retain(const dynakv_desc* desc, const int32_t* k, const float* m, float alpha, float* out, float* g_m,
                  void* ws, size_t ws_bytes, void* stream) {
  Ws w;
  const int rc = open_ws(desc, ws, ws_bytes, w);
  if (rc != LMHEAD_OK) return rc;
  if (!out) return LMHEAD_E_NULL;
  if ((m && !aligned16(m)) || (g_m && !aligned16(g_m))) return LMHEAD_E_ALIGN;
  const KvLayout& L = w.L;
  hipStream_t s = static_cast<hipStream_t>(stream);
  LM_TRY(launch_kv_clear_header(w.at<WsHeader>(L.hdr), s));
  LM_TRY(launch_kv_retain(k, m, L.n, desc->d, alpha, out, g_m, w.at<double>(L.red), s));
  return LMHEAD_OK;
}

size_t dynakv_bwd_workspace_bytes(const dynakv_desc* desc) {
  if (validate(desc) != LMHEAD_OK) return 0;
  return make_kv_bwd_layout(desc).total;
}

int dynakv_gate_bwd(const dynakv_desc* desc, const void* x, const void* U, const void* W, const float* b,
                    const void* xt, const void* g_xhat, const float* g_m, float g_m_const, void* dx, float* dU,
                    float* dW, float* db, void* ws, size_t ws_bytes, void* stream) {
  const int rc = validate(desc);
  if (rc != LMHEAD_OK) return rc;
  if (!ws || !x || !U || !W || !b || !xt || !g_xhat || !dx || !dU || !dW || !db) return LMHEAD_E_NULL;
  if (!aligned256(ws)) return LMHEAD_E_ALIGN;
  if (!aligned16(x) || !aligned16(U) || !aligned16(W) || !aligned16(b) || !aligned16(xt) || !aligned16(g_xhat) ||
      (g_m && !aligned16(g_m)) || !aligned16(dx) || !aligned16(dU) || !aligned16(dW) || !aligned16(db))
    return LMHEAD_E_ALIGN;
  const KvBwdLayout L = make_kv_bwd_layout(desc);
  if (ws_bytes < L.total) return LMHEAD_E_WORKSPACE;
  char* const base = static_cast<char*>(ws);
  auto at = [&](size_t off) { return static_cast<void*>(base + off); };
  hipStream_t s = static_cast<hipStream_t>(stream);
  WsHeader* hdr = static_cast<WsHeader*>(at(L.hdr));
  const int dt = desc->dtype;
  const int d = desc->d;
  const bool literal = (desc->flags & DYNAKV_FLAG_LITERAL_FLIP) != 0;
  const bool accum = (desc->flags & DYNAKV_FLAG_ACCUM_GRAD) != 0;

  LM_TRY(launch_kv_clear_header(hdr, s));
  // parameter operands of the three token-major products: W^T (K-contiguous copy) for the logits, and
  // row-padded copies of W and U, which are K-contiguous as they are for g_l W^T and g_x~ U^T
  LM_TRY(launch_transpose(dt, W, d, d, d, false, hdr, at(L.WT), L.ldT, d, L.dp, s));
  LM_TRY(launch_kv_pad_copy(dt, W, d, d, d, at(L.Wp), L.ldT, (int)L.dp, s));
  LM_TRY(launch_kv_pad_copy(dt, U, d, d, d, at(L.Up), L.ldT, (int)L.dp, s));

  KvGemmArgs ga{};
  ga.mode = 1;
  ga.A = at(L.WT);
  ga.ldA = L.ldT;
  ga.B = xt;
  ga.ldB = d;
  ga.M = d;
  ga.Nn = L.n;
  ga.K = d;
  ga.out_f = static_cast<float*>(at(L.logits));
  ga.ldo = d;
  ga.hdr = hdr;
  {
    TimedLaunch tl(5, s);
    LM_TRY(launch_kv_gemm(dt, ga, s));
  }
  {
    // g_l, and the direct part g_xhat * m of dL/dx~ (into the buffer that the next product adds to)
    TimedLaunch tl(8, s);
    LM_TRY(launch_kv_mask_bwd(dt, static_cast<const float*>(at(L.logits)), b, xt, g_xhat, g_m, g_m_const, L.n, d,
                              literal, at(L.gl), at(L.gxt), static_cast<float*>(at(L.dbpart)), L.nblk, s));
  }
  LM_TRY(launch_kv_sum_rows(static_cast<const float*>(at(L.dbpart)), L.nblk, d, d, db, accum, s));

  // g_x~ += g_l W^T
  ga.mode = 0;
  ga.A = at(L.Wp);
  ga.B = at(L.gl);
  ga.out_f = nullptr;
  ga.out_e = at(L.gxt);
  ga.accumulate = true;
  {
    TimedLaunch tl(9, s);
    LM_TRY(launch_kv_gemm(dt, ga, s));
  }
  // dx = g_x~ U^T
  ga.A = at(L.Up);
  ga.B = at(L.gxt);
  ga.out_e = dx;
  ga.accumulate = false;
  {
    TimedLaunch tl(10, s);
    LM_TRY(launch_kv_gemm(dt, ga, s));
  }

  // Parameter gradients: contractions over the tokens, out[row][col] = sum_t B[row][t] A[col][t] with
  // token-contiguous copies of both operands, cut into ksplit slices of the token range.
  auto param_grad = [&](const void* rows_src, int64_t ld_rows, const void* cols_src, int kind, float* out) -> int {
    {
      TimedLaunch tl(13, s);
      LM_TRY(launch_kv_transpose(dt, rows_src, ld_rows, L.n, d, at(L.T1), L.ldK, L.ncap, (int)L.dp, s));
      LM_TRY(launch_kv_transpose(dt, cols_src, d, L.n, d, at(L.T2), L.ldK, L.ncap, (int)L.dp, s));
    }
    GemmTArgs ta{};
    ta.A = at(L.T2);
    ta.ldA = L.ldK;
    ta.B = at(L.T1);
    ta.ldB = L.ldK;
    ta.M = d;
    ta.n_limit = d;
    ta.K = L.ncap;
    ta.n_tiles_cap = L.dp / kTile;
    ta.hdr = hdr;
    ta.ksplit = L.ksplit;
    ta.part = static_cast<float*>(at(L.part));
    ta.part_ld = d;
    ta.part_slice = (int64_t)d * d;
    {
      TimedLaunch tl(kind, s);
      LM_TRY(launch_gemm_t(dt, ta, s, 2));
    }
    LM_TRY(launch_kv_sum_rows(ta.part, L.ksplit, ta.part_slice, ta.part_slice, out, accum, s));
    return LMHEAD_OK;
  };
  // dW[k][j] = sum_t x~[t][k] g_l[t][j];  dU[i][k] = sum_t x[t][i] g_x~[t][k]
  int prc = param_grad(xt, d, at(L.gl), 11, dW);
  if (prc != LMHEAD_OK) return prc;
  prc = param_grad(x, desc->ldx, at(L.gxt), 12, dU);
  if (prc != LMHEAD_OK) return prc;
  return LMHEAD_OK;
}

int dynakv_check(void* ws, void* stream) { return lmhead_check(ws, stream); }

}  // extern "C"
