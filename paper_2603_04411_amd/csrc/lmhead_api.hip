// extern "C" entry points: host-side validation, workspace carving and kernel sequencing.
// Every argument error is returned before anything is enqueued.
#include <math.h>

#include "common.h"

using namespace lmhead;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate(const lmhead_desc* d) {
  if (!d) return LMHEAD_E_NULL;
  if (d->P <= 0 || d->G <= 0 || d->T <= 0 || d->d <= 0 || d->V <= 0) return LMHEAD_E_SHAPE;
  if (d->dtype != LMHEAD_F32 && d->dtype != LMHEAD_BF16) return LMHEAD_E_DTYPE;
  if (d->flags & ~(uint32_t)(LMHEAD_FLAG_ACCUM_DW | LMHEAD_FLAG_FP8_LOGITS | LMHEAD_FLAG_DH_BF16)) return LMHEAD_E_DTYPE;
  if (d->vocab_chunk < 0) return LMHEAD_E_SHAPE;
  // one K-step of the matrix-core loops is a 128-byte line of a row: 64 bf16 or 32 fp32 values
  if (d->d % (d->dtype == LMHEAD_BF16 ? 64 : 32) != 0) return LMHEAD_E_SHAPE;
  if (d->flags & LMHEAD_FLAG_FP8_LOGITS) {
    // one K-step of the 8-bit kernels is 128 values; exponents beyond +-60 cannot be meant
    if (d->d % 128 != 0 || d->fp8_exp_h < -60 || d->fp8_exp_h > 60 || d->fp8_exp_w < -60 || d->fp8_exp_w > 60)
      return LMHEAD_E_SHAPE;
  } else if (d->fp8_exp_h != 0 || d->fp8_exp_w != 0) {
    return LMHEAD_E_SHAPE;
  }
  if (d->ldH < d->d || d->ldW < d->d) return LMHEAD_E_SHAPE;
  const int64_t R = (int64_t)d->P * d->G;
  const int64_t N = R * d->T;
  if (R > INT32_MAX || N > (int64_t)INT32_MAX - 2 * kTile) return LMHEAD_E_SHAPE;
  if ((int64_t)d->V > (int64_t)INT32_MAX - 2 * kTile) return LMHEAD_E_SHAPE;
  const int esz = d->dtype == LMHEAD_BF16 ? 2 : 4;
  if ((d->ldH * esz) % 16 != 0 || (d->ldW * esz) % 16 != 0) return LMHEAD_E_ALIGN;
  // The matrix-core kernels address an operand tile through one buffer descriptor with 32-bit byte
  // offsets inside a 2 GiB window: the last row of a 256-row tile plus the contraction's extent must
  // stay below 2^31.  The widest rows are the token-major operand copies of the backward (N slots wide).
  {
    const WsLayout L = make_layout(d, kMaxPolicies);
    int64_t pitch = d->ldW;
    for (int64_t p : {L.ldHc, L.ldHcT, L.ldWT, L.ldZ, L.ldZT}) pitch = p > pitch ? p : pitch;
    if ((int64_t)kTile * pitch * esz >= (1ll << 31)) return LMHEAD_E_SHAPE;
    // 1-D launch grids (tiles of the largest kernel, rounded up by the tile walk) must fit HIP's limit
    const int64_t tok_tiles = L.Ncap / kTile + 8 * 16, voc_tiles = L.Vp / kTile, d_tiles = L.dp / kTile;
    const int64_t widest = voc_tiles * kMaxPolicies > d_tiles * 8 ? voc_tiles * kMaxPolicies : d_tiles * 8;
    if (widest * tok_tiles > INT32_MAX || d_tiles * (voc_tiles + 8 * 16) > INT32_MAX) return LMHEAD_E_SHAPE;
  }
  return LMHEAD_OK;
}

struct Ws {
  WsLayout L;
  char* base;
  template <typename T>
  T* at(size_t off) const { return reinterpret_cast<T*>(base + off); }
};

size_t loss_ws_bytes(int64_t P, int64_t G, int64_t T) {
  const int64_t R = P * G;
  const int64_t nb = (T + kLossSlotsPerBlock - 1) / kLossSlotsPerBlock;
  return (size_t)(R * nb * 4 + R) * sizeof(float) + 256;
}

int validate_pgt(int32_t P, int32_t G, int32_t T) {
  if (P <= 0 || G <= 0 || T <= 0) return LMHEAD_E_SHAPE;
  const int64_t R = (int64_t)P * G;
  if (R > 65535 || R * T > INT32_MAX) return LMHEAD_E_SHAPE;  // R is a grid y-extent
  return LMHEAD_OK;
}

}  // namespace

namespace lmhead {
TimingState g_timing;
}

extern "C" {

int lmhead_abi_version(void) { return 2; }

int lmhead_validate_desc(const lmhead_desc* desc) { return validate(desc); }

size_t lmhead_workspace_bytes(const lmhead_desc* desc) {
  if (validate(desc) != LMHEAD_OK) return 0;
  return make_layout(desc).total;
}

int lmhead_workspace_region(const lmhead_desc* desc, int32_t npol, int32_t which, size_t* offset, size_t* bytes) {
  const int rc = validate(desc);
  if (rc != LMHEAD_OK) return rc;
  if (npol < 1 || npol > kMaxPolicies || which < 0 || which > LMHEAD_WS_GATHERED_ID) return LMHEAD_E_SHAPE;
  if (!offset || !bytes) return LMHEAD_E_NULL;
  const WsLayout L = make_layout(desc, npol);
  switch (which) {
    case LMHEAD_WS_NV: *offset = L.hdr + offsetof(WsHeader, nv); *bytes = 4; break;
    case LMHEAD_WS_ROW_SLOT: *offset = L.row_slot; *bytes = (size_t)L.Ncap * 4; break;
    case LMHEAD_WS_TOK_C: *offset = L.tok_c; *bytes = (size_t)L.Ncap * 4; break;
    default: *offset = L.gid; *bytes = (size_t)npol * L.Ncap * 4; break;
  }
  return LMHEAD_OK;
}

// Shared body of the two forward entry points: index, compaction, one logits launch over all
// npol weight matrices, then one merge of the per-tile statistics per matrix.
static int forward(const lmhead_desc* desc, const void* H, const void* const* W, int npol, const int32_t* tok,
                   const int32_t* len, float* const* logp, float* lse, float* entropy, uint8_t* mask,
                   int32_t* cu_len, void* ws, size_t ws_bytes, void* stream) {
  Ws w{make_layout(desc, npol), static_cast<char*>(ws)};
  if (ws_bytes < w.L.total) return LMHEAD_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const WsLayout& L = w.L;
  WsHeader* hdr = w.at<WsHeader>(L.hdr);

  LM_TRY(launch_index(len, (int)L.R, desc->T, hdr, w.at<int32_t>(L.cu_len), w.at<int32_t>(L.row_slot),
                      mask, cu_len, s));
  LM_TRY(launch_compact(desc->dtype, H, desc->ldH, desc->d, desc->V, tok, nullptr, nullptr, L.N, hdr,
                        w.at<int32_t>(L.row_slot), w.at<void>(L.Hc), L.ldHc, w.at<int32_t>(L.tok_c), nullptr,
                        nullptr, w.at<float>(L.zy), w.at<int32_t>(L.gid), npol, L.Ncap, s));
  const bool fp8 = (desc->flags & LMHEAD_FLAG_FP8_LOGITS) != 0;
  FwdArgs fa{};
  fa.zscale = 1.0f;
  if (fp8) {
    // 8-bit copies of the gathered hidden states and of every weight matrix
    LM_TRY(launch_quantize_e4m3(desc->dtype, w.at<void>(L.Hc), L.ldHc, 0, true, hdr, desc->d, desc->fp8_exp_h,
                                w.at<void>(L.Hc8), L.ld8, L.Ncap, s));
    for (int p = 0; p < npol; ++p) {
      char* w8 = w.at<char>(L.W8) + (size_t)p * L.Vp * L.ld8;
      LM_TRY(launch_quantize_e4m3(desc->dtype, W[p], desc->ldW, desc->V, false, hdr, desc->d, desc->fp8_exp_w, w8,
                                  L.ld8, L.Vp, s));
      fa.W[p] = w8;
    }
    for (int p = npol; p < kMaxPolicies; ++p) fa.W[p] = fa.W[0];
    fa.Hc = w.at<void>(L.Hc8);
    fa.ldHc = L.ld8;
    fa.ldW = L.ld8;
    fa.zscale = ldexpf(1.0f, -(desc->fp8_exp_h + desc->fp8_exp_w));
  } else {
    fa.Hc = w.at<void>(L.Hc);
    fa.ldHc = L.ldHc;
    for (int p = 0; p < kMaxPolicies; ++p) fa.W[p] = W[p < npol ? p : 0];
    fa.ldW = desc->ldW;
  }
  fa.npol = npol;
  fa.d = desc->d;
  fa.V = desc->V;
  fa.Ncap = L.Ncap;
  fa.ntiles = (int)L.ntiles;
  fa.tok_c = w.at<int32_t>(L.tok_c);
  fa.hdr = hdr;
  fa.part = w.at<float>(L.part);
  fa.want_entropy = entropy != nullptr;
  fa.zy = w.at<float>(L.zy);
  fa.gid = w.at<int32_t>(L.gid);
  {
    TimedLaunch tl(0, s);
    LM_TRY(launch_fwd(fp8 ? kDtypeFp8 : desc->dtype, fa, s));
  }
  for (int p = 0; p < npol; ++p)
    LM_TRY(launch_finalize(w.at<float>(L.part) + (size_t)p * 3 * L.ntiles * L.Ncap,
                           w.at<float>(L.zy) + (size_t)p * L.Ncap, (int)L.ntiles, L.Ncap, len,
                           w.at<int32_t>(L.cu_len), (int)L.R, desc->T, logp[p], p == 0 ? lse : nullptr,
                           p == 0 ? entropy : nullptr, s));
  return LMHEAD_OK;
}

int lmhead_logprob_fwd(const lmhead_desc* desc, const void* H, const void* W, const int32_t* tok,
                       const int32_t* len, float* logp, float* lse, float* entropy, uint8_t* mask,
                       int32_t* cu_len, void* ws, size_t ws_bytes, void* stream) {
  const int rc = validate(desc);
  if (rc != LMHEAD_OK) return rc;
  if (!H || !W || !tok || !len || !logp || !ws) return LMHEAD_E_NULL;
  if (!aligned16(H) || !aligned16(W) || (reinterpret_cast<uintptr_t>(ws) & 255u)) return LMHEAD_E_ALIGN;
  return forward(desc, H, &W, 1, tok, len, &logp, lse, entropy, mask, cu_len, ws, ws_bytes, stream);
}

size_t lmhead_multi_workspace_bytes(const lmhead_desc* desc, int32_t npol) {
  if (validate(desc) != LMHEAD_OK || npol < 1 || npol > kMaxPolicies) return 0;
  const size_t fwd = make_layout(desc, npol).total, base = make_layout(desc).total;
  return fwd > base ? fwd : base;
}

int lmhead_logprob_fwd_multi(const lmhead_desc* desc, const void* H, const void* const* W, int32_t npol,
                             const int32_t* tok, const int32_t* len, float* const* logp, float* lse,
                             float* entropy, uint8_t* mask, int32_t* cu_len, void* ws, size_t ws_bytes,
                             void* stream) {
  const int rc = validate(desc);
  if (rc != LMHEAD_OK) return rc;
  if (npol < 1 || npol > kMaxPolicies) return LMHEAD_E_SHAPE;
  if (!H || !W || !tok || !len || !logp || !ws) return LMHEAD_E_NULL;
  for (int p = 0; p < npol; ++p) {
    if (!W[p] || !logp[p]) return LMHEAD_E_NULL;
    if (!aligned16(W[p])) return LMHEAD_E_ALIGN;
  }
  if (!aligned16(H) || (reinterpret_cast<uintptr_t>(ws) & 255u)) return LMHEAD_E_ALIGN;
  return forward(desc, H, W, npol, tok, len, logp, lse, entropy, mask, cu_len, ws, ws_bytes, stream);
}

int lmhead_logprob_bwd(const lmhead_desc* desc, const void* H, const void* W, const int32_t* tok,
                       const int32_t* len, const float* lse, const float* g_logp, void* dH, float* dW,
                       void* ws, size_t ws_bytes, void* stream) {
  const int rc = validate(desc);
  if (rc != LMHEAD_OK) return rc;
  if (!H || !W || !tok || !len || !lse || !g_logp || !dH || !dW || !ws) return LMHEAD_E_NULL;
  if (!aligned16(H) || !aligned16(W) || !aligned16(dH) || !aligned16(dW) ||
      (reinterpret_cast<uintptr_t>(ws) & 255u))
    return LMHEAD_E_ALIGN;
  Ws w{make_layout(desc), static_cast<char*>(ws)};
  if (ws_bytes < w.L.total) return LMHEAD_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const WsLayout& L = w.L;
  WsHeader* hdr = w.at<WsHeader>(L.hdr);
  const int dt = desc->dtype;

  LM_TRY(launch_index(len, (int)L.R, desc->T, hdr, w.at<int32_t>(L.cu_len), w.at<int32_t>(L.row_slot),
                      nullptr, nullptr, s));
  LM_TRY(launch_compact(dt, H, desc->ldH, desc->d, desc->V, tok, g_logp, lse, L.N, hdr,
                        w.at<int32_t>(L.row_slot), w.at<void>(L.Hc), L.ldHc, w.at<int32_t>(L.tok_c),
                        w.at<float>(L.g_c), w.at<float>(L.lse_c), w.at<float>(L.zy), w.at<int32_t>(L.gid), 1, L.Ncap, s));
  // K-contiguous copies of the two operands that the backward contracts along their rows
  LM_TRY(launch_transpose(dt, w.at<void>(L.Hc), L.ldHc, L.Ncap, desc->d, true, hdr, w.at<void>(L.HcT),
                          L.ldHcT, L.Ncap, L.dp, s));
  LM_TRY(launch_transpose(dt, W, desc->ldW, desc->V, desc->d, false, hdr, w.at<void>(L.WT), L.ldWT, L.Vp,
                          L.dp, s));
  const bool dh16 = (desc->flags & LMHEAD_FLAG_DH_BF16) != 0;
  LM_TRY(launch_zero_padded_rows(dH, dh16, desc->d, len, (int)L.R, desc->T, s));
  const bool fp8 = (desc->flags & LMHEAD_FLAG_FP8_LOGITS) != 0;
  if (fp8) {
    // the recompute must see the logits the forward saw: same 8-bit copies
    LM_TRY(launch_quantize_e4m3(dt, w.at<void>(L.Hc), L.ldHc, 0, true, hdr, desc->d, desc->fp8_exp_h,
                                w.at<void>(L.Hc8), L.ld8, L.Ncap, s));
    LM_TRY(launch_quantize_e4m3(dt, W, desc->ldW, desc->V, false, hdr, desc->d, desc->fp8_exp_w, w.at<void>(L.W8),
                                L.ld8, L.Vp, s));
  }

  const int total_tiles = (int)(L.Vp / kTile);
  const int tiles_per_chunk = (int)(L.Vc / kTile);
  for (int c = 0; c < (int)L.nchunks; ++c) {
    const int t_lo = c * tiles_per_chunk;
    const int ntiles = (total_tiles - t_lo < tiles_per_chunk) ? total_tiles - t_lo : tiles_per_chunk;
    const int c0 = t_lo * kTile;
    DzArgs za{};
    za.Hc = fp8 ? w.at<void>(L.Hc8) : w.at<void>(L.Hc);
    za.ldHc = fp8 ? L.ld8 : L.ldHc;
    za.W = fp8 ? w.at<void>(L.W8) : W;
    za.ldW = fp8 ? L.ld8 : desc->ldW;
    za.zscale = fp8 ? ldexpf(1.0f, -(desc->fp8_exp_h + desc->fp8_exp_w)) : 1.0f;
    za.d = desc->d;
    za.V = desc->V;
    za.Ncap = L.Ncap;
    za.ldZ = L.ldZ;
    za.ldZT = L.ldZT;
    za.c0 = c0;
    za.ntiles = ntiles;
    za.tok_c = w.at<int32_t>(L.tok_c);
    za.g_c = w.at<float>(L.g_c);
    za.lse_c = w.at<float>(L.lse_c);
    za.hdr = hdr;
    za.dZ = w.at<void>(L.dZ);
    za.dZT = w.at<void>(L.dZT);
    {
      TimedLaunch tl(1, s);
      LM_TRY(launch_dz(fp8 ? kDtypeFp8 : dt, dt, za, s));
    }

    // dH[slot(n)][m] (+)= sum_v W^T[m][c0 + v] dZ[n][v]
    GemmTArgs ha{};
    ha.A = w.at<char>(L.WT) + (size_t)c0 * L.esz;
    ha.ldA = L.ldWT;
    ha.B = w.at<void>(L.dZ);
    ha.ldB = L.ldZ;
    ha.M = desc->d;
    ha.n_from_nv = true;
    ha.k_from_nv = false;
    ha.K = (int64_t)ntiles * kTile;
    ha.rowmap = w.at<int32_t>(L.row_slot);
    ha.out = static_cast<float*>(dH);   // unused when the tiles go to the fp32 scratch slices
    ha.ldo = desc->d;
    ha.accumulate = c > 0;
    ha.n_tiles_cap = L.Ncap / kTile;
    ha.hdr = hdr;
    ha.ksplit = L.ksplit;
    ha.part = (L.ksplit > 1 || dh16) ? w.at<float>(L.dHpart) : nullptr;
    ha.part_ld = L.dp;
    ha.part_slice = L.Ncap * L.dp;
    ha.part_accumulate = dh16 && c > 0;   // a bf16 dH is summed over the chunks in the scratch slices
    {
      TimedLaunch tl(2, s);
      LM_TRY(launch_gemm_t(dt, ha, s));
      if (dh16) {
        if (c + 1 == (int)L.nchunks)
          LM_TRY(launch_splitk_reduce(ha.part, L.ksplit, ha.part_slice, ha.part_ld, desc->d, ha.rowmap, hdr,
                                      L.Ncap, dH, desc->d, false, true, s));
      } else if (L.ksplit > 1) {
        LM_TRY(launch_splitk_reduce(ha.part, L.ksplit, ha.part_slice, ha.part_ld, desc->d, ha.rowmap, hdr, L.Ncap,
                                    dH, desc->d, c > 0, false, s));
      }
    }

    // dW[c0 + n][m] = sum_i Hc^T[m][i] dZ^T[n][i]
    GemmTArgs wa{};
    wa.A = w.at<void>(L.HcT);
    wa.ldA = L.ldHcT;
    wa.B = w.at<void>(L.dZT);
    wa.ldB = L.ldZT;
    wa.M = desc->d;
    wa.n_limit = (desc->V - c0 < ntiles * kTile) ? desc->V - c0 : ntiles * kTile;
    wa.n_from_nv = false;
    wa.k_from_nv = true;
    wa.rowmap = nullptr;
    wa.row_base = c0;
    wa.out = dW;
    wa.ldo = desc->d;
    wa.accumulate = (desc->flags & LMHEAD_FLAG_ACCUM_DW) != 0;
    wa.hdr = hdr;
    // Every output tile is one workgroup and the compute units take them a round at a time.  The vocabulary
    // tiles of this chunk that would start a mostly empty last round (with d / 256 tiles along d, 16 of them
    // fill the 256 compute units at d = 4096; a chunk of 18 leaves 2) are launched apart, their contraction
    // over the tokens cut into as many slices as make that round full; the slices are summed in a fixed order.
    const int m_tiles = (int)(L.dp / kTile), cus = device_compute_units();
    int t_rem = 0, ks = 1;
    if (m_tiles <= cus && cus % m_tiles == 0) {
      t_rem = ntiles % (cus / m_tiles);
      ks = t_rem > 0 ? cus / (t_rem * m_tiles) : 1;
      if (ks > 8) ks = 8;
      if (ks < 2 || (size_t)ks * t_rem * kTile * L.dp * 4 > L.dWpart_bytes) t_rem = 0;
    }
    const int t_main = ntiles - t_rem;
    {
      TimedLaunch tl(3, s);
      if (t_main > 0) {
        GemmTArgs m = wa;
        m.n_limit = wa.n_limit < (int64_t)t_main * kTile ? wa.n_limit : (int64_t)t_main * kTile;
        m.n_tiles_cap = t_main;
        m.ksplit = 1;
        m.part = nullptr;
        LM_TRY(launch_gemm_t(dt, m, s));
      }
      if (t_rem > 0) {
        GemmTArgs r = wa;
        r.B = w.at<char>(L.dZT) + (size_t)t_main * kTile * L.ldZT * L.esz;
        r.n_limit = wa.n_limit - (int64_t)t_main * kTile;
        r.n_tiles_cap = t_rem;
        r.ksplit = ks;
        r.part = w.at<float>(L.dWpart);
        r.part_ld = L.dp;
        r.part_slice = (int64_t)t_rem * kTile * L.dp;
        r.part_accumulate = false;
        if (r.n_limit > 0) {
          LM_TRY(launch_gemm_t(dt, r, s));
          LM_TRY(launch_splitk_reduce(r.part, ks, r.part_slice, r.part_ld, desc->d, nullptr, hdr, r.n_limit, dW,
                                      desc->d, wa.accumulate, false, s, c0 + (int64_t)t_main * kTile));
        }
      }
    }
  }
  return LMHEAD_OK;
}

int group_advantage(const float* reward, int32_t P, int32_t G, float eps, int32_t ddof, float* adv,
                    void* stream) {
  if (P <= 0 || G <= 0 || (int64_t)P * G > INT32_MAX) return LMHEAD_E_SHAPE;
  if (ddof != 0 && ddof != 1) return LMHEAD_E_SHAPE;
  if (!reward || !adv) return LMHEAD_E_NULL;
  LM_TRY(launch_group_advantage(reward, P, G, eps, ddof, adv, static_cast<hipStream_t>(stream)));
  return LMHEAD_OK;
}

size_t lmhead_loss_workspace_bytes(int32_t P, int32_t G, int32_t T) {
  if (validate_pgt(P, G, T) != LMHEAD_OK) return 0;
  return loss_ws_bytes(P, G, T);
}

int grpo_loss(const float* logp, const float* logp_old, const float* logp_ref, const float* adv,
              const int32_t* len, int32_t P, int32_t G, int32_t T, float clip_lo, float clip_hi,
              float kl_coef, int32_t agg_mode, float* loss, float* g_logp, float* stats, void* ws,
              size_t ws_bytes, void* stream) {
  const int rc = validate_pgt(P, G, T);
  if (rc != LMHEAD_OK) return rc;
  if (agg_mode != 0 && agg_mode != 1) return LMHEAD_E_SHAPE;
  if (!logp || !logp_old || !adv || !len || !loss || !ws) return LMHEAD_E_NULL;
  if (ws_bytes < loss_ws_bytes(P, G, T)) return LMHEAD_E_WORKSPACE;
  LM_TRY(launch_grpo(logp, logp_old, logp_ref, adv, len, P, G, T, clip_lo, clip_hi, kl_coef, agg_mode,
                     loss, g_logp, stats, static_cast<float*>(ws), static_cast<hipStream_t>(stream)));
  return LMHEAD_OK;
}

int grpo_loss_noalloc(const float* logp, const float* logp_old, const float* logp_ref, const float* adv,
                      const int32_t* len, int32_t P, int32_t G, int32_t T, float clip_lo, float clip_hi,
                      float kl_coef, int32_t agg_mode, float* loss, float* g_logp, float* stats, void* stream) {
  const int rc = validate_pgt(P, G, T);
  if (rc != LMHEAD_OK) return rc;
  if (agg_mode != 0 && agg_mode != 1) return LMHEAD_E_SHAPE;
  if (!logp || !logp_old || !adv || !len || !loss) return LMHEAD_E_NULL;
  const int64_t nb = ((int64_t)T + kLossSlotsPerBlock - 1) / kLossSlotsPerBlock;
  if ((int64_t)P * G * nb > kStaticLossParts) return LMHEAD_E_WORKSPACE;   // beyond the static scratch
  float* scratch_dev = nullptr;
  LM_TRY(static_scratch(&scratch_dev));
  // every partial the final kernel reads is written by the first kernel of this call: nothing to clear
  LM_TRY(launch_grpo(logp, logp_old, logp_ref, adv, len, P, G, T, clip_lo, clip_hi, kl_coef, agg_mode, loss,
                     g_logp, stats, scratch_dev, static_cast<hipStream_t>(stream)));
  return LMHEAD_OK;
}

int ce_loss(const float* logp, const int32_t* len, int32_t R, int32_t T, float* loss, float* g_logp,
            void* ws, size_t ws_bytes, void* stream) {
  const int rc = validate_pgt(R, 1, T);
  if (rc != LMHEAD_OK) return rc;
  if (!logp || !len || !loss || !ws) return LMHEAD_E_NULL;
  if (ws_bytes < loss_ws_bytes(R, 1, T)) return LMHEAD_E_WORKSPACE;
  LM_TRY(launch_ce(logp, len, R, T, loss, g_logp, static_cast<float*>(ws), static_cast<hipStream_t>(stream)));
  return LMHEAD_OK;
}

int flowrl_tb_loss(const float* logp, const float* logp_ref, const float* reward, const float* logZ,
                   const int32_t* len, int32_t P, int32_t G, int32_t T, float beta, float* loss,
                   float* g_logp, float* g_logZ, float* resid, void* ws, size_t ws_bytes, void* stream) {
  const int rc = validate_pgt(P, G, T);
  if (rc != LMHEAD_OK) return rc;
  if (!logp || !logp_ref || !reward || !logZ || !len || !loss || !ws) return LMHEAD_E_NULL;
  if (ws_bytes < loss_ws_bytes(P, G, T)) return LMHEAD_E_WORKSPACE;
  LM_TRY(launch_flowrl(logp, logp_ref, reward, logZ, len, P, G, T, beta, loss, g_logp, g_logZ, resid,
                       static_cast<float*>(ws), static_cast<hipStream_t>(stream)));
  return LMHEAD_OK;
}

int lmhead_check(void* ws, void* stream) {
  if (!ws) return LMHEAD_E_NULL;
  WsHeader h;
  if (hipMemcpyAsync(&h, ws, sizeof(int32_t) * 2, hipMemcpyDeviceToHost,
                     static_cast<hipStream_t>(stream)) != hipSuccess)
    return LMHEAD_E_HIP;
  if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return LMHEAD_E_HIP;
  return h.err != 0 ? LMHEAD_E_RANGE : LMHEAD_OK;
}

int lmhead_probe_mfma(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes,
                      int32_t workgroups, int32_t iters, void* stream) {
  if (!operands || !sink) return LMHEAD_E_NULL;
  if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0) return LMHEAD_E_SHAPE;
  if (!aligned16(operands)) return LMHEAD_E_ALIGN;
  const size_t threads = (size_t)workgroups * 256;
  if (operand_bytes < threads * 256 || sink_bytes < threads * 4) return LMHEAD_E_WORKSPACE;
  LM_TRY(launch_mfma_probe(operands, sink, workgroups, iters, static_cast<hipStream_t>(stream)));
  return LMHEAD_OK;
}

int lmhead_timing_enable(int on) {
  if (on && g_timing.created == 0) {
    for (int i = 0; i < kTimingPool; ++i) {
      if (hipEventCreate(&g_timing.start[i]) != hipSuccess) return LMHEAD_E_HIP;
      if (hipEventCreate(&g_timing.stop[i]) != hipSuccess) return LMHEAD_E_HIP;
      g_timing.created = i + 1;
    }
  }
  g_timing.on = on != 0;
  g_timing.used = 0;
  return LMHEAD_OK;
}

int lmhead_timing_read(int kind, double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) return LMHEAD_E_NULL;
  if (kind < 0 || kind >= kTimingKinds) return LMHEAD_E_SHAPE;
  double tot = 0.0;
  int64_t cnt = 0;
  for (int i = 0; i < g_timing.used; ++i) {
    if (g_timing.kind[i] != kind) continue;
    if (hipEventSynchronize(g_timing.stop[i]) != hipSuccess) return LMHEAD_E_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_timing.start[i], g_timing.stop[i]) != hipSuccess) return LMHEAD_E_HIP;
    tot += ms;
    ++cnt;
  }
  *total_ms = tot;
  *launches = cnt;
  return LMHEAD_OK;
}

}  // extern "C"
