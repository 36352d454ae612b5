/*
 * dynakv.h - C ABI of the token-adaptive KV-cache compression path for AMD MI355X (gfx950):
 * spectral projection, differentiable truncation gate, ragged store and low-rank
 * reconstruction (Sec. 3 "Dynamic Compressing" of the paper, Eqs. 1-8) and the retain-rate
 * regulariser of the training objective (Sec. 3.3, Eq. 9).
 *
 * Notation (the paper's): a token's pre-RoPE key or value state is the row vector x with
 * d = d_kv entries; U [d x d] is the spectral basis, W [d x d] and b [d] the gate layer,
 * tau the threshold.  Keys and values have separate parameters: one call handles one stream.
 *
 * Conventions
 *  - Every pointer is DEVICE memory owned by the caller, except the descriptor (host).  The
 *    library allocates nothing and keeps no state between calls; `ws` is scratch whose
 *    contents are undefined after a call, except the error word read by dynakv_check().
 *  - Matrices are row-major.  x has row stride ldx; every other matrix is dense (row stride d).
 *    Matrix pointers must be 16-byte aligned, `ws` 256-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream); calls enqueue work
 *    and return without synchronising.
 *  - Return value: LMHEAD_OK or a negative LMHEAD_E_* code (lmhead.h).  Argument errors are
 *    found on the host before anything is launched and leave all outputs untouched.
 *  - Results are bit-reproducible from run to run: no floating-point atomics are used.
 *
 * Readings of the paper taken by this library (also listed in the design notes):
 *  - Eq. 6 is evaluated as the reverse cumulative sum m_i = sum_{j >= i} p_j, which is the mask
 *    its text describes (1 before the predicted cut-off, 0 after it).  The formula as printed,
 *    Flip(cumsum(p))_i = sum_{j <= d-1-i} p_j, is selected by DYNAKV_FLAG_LITERAL_FLIP; the two
 *    differ by relabelling the gate's output columns j <-> d-1-j.
 *  - The spectral state x~ is rounded to the storage type before it enters the gate layer and
 *    the cache.  Logits, softmax and the mask are fp32; Eq. 8 compares fp32 values.
 *  - The store keeps x~[0:k] of token i at element offset off[i], a multiple of 8 elements
 *    (16 bytes for bf16); the unused tail of the last 8-element granule is written as 0.
 *  - U^-1 of Eq. 3 is an input (U^T for an orthogonal U); the library inverts nothing.
 */
#ifndef DYNAKV_H_
#define DYNAKV_H_

#include <stddef.h>
#include <stdint.h>

#include "lmhead.h"

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DYNAKV_FLAG_LITERAL_FLIP = 1u << 0, /* Eq. 6 as printed instead of the reverse cumulative sum */
  DYNAKV_FLAG_ACCUM_GRAD = 1u << 1    /* dynakv_gate_bwd adds to dU, dW, db instead of overwriting them
                                         (the other calls ignore it) */
};

enum { DYNAKV_GRANULE = 8 }; /* elements; segment offsets in the store are multiples of this */

/* Problem descriptor (host memory). */
typedef struct dynakv_desc {
  int32_t n;        /* tokens in this call (> 0)                                              */
  int32_t d;        /* d_kv: a multiple of 64, at most 8192                                   */
  int32_t dtype;    /* LMHEAD_F32 or LMHEAD_BF16: storage type of x, U, W, U_inv, x~, the      */
                    /* store and x_bar.  n * d * sizeof(type) must not exceed 2^31 - 2^20.     */
  uint32_t flags;   /* DYNAKV_FLAG_*                                                           */
  int64_t ldx;      /* row stride of x in elements (>= d, ldx * sizeof(type) % 16 == 0)        */
  int64_t reserved; /* must be 0                                                               */
} dynakv_desc;

/* Scratch bytes needed by any of the calls below for this descriptor; 0 if it is invalid.
 * Host-only. */
LMHEAD_API size_t dynakv_workspace_bytes(const dynakv_desc* desc);

/* LMHEAD_OK or the code the compute entry points would return for this descriptor. Host-only. */
LMHEAD_API int dynakv_validate_desc(const dynakv_desc* desc);

/*
 * The gate (Eqs. 1, 5, 6, 7, 8).  Per token (row) i:
 *     x~   = x U                         rounded to the storage type           (Eq. 1)
 *     p    = Softmax(x~ W + b)           fp32                                   (Eq. 5)
 *     m_j  = sum_{l >= j} p_l            soft mask, non-increasing, m_0 = 1     (Eq. 6)
 *     x^   = x~ * m                      element-wise, storage type             (Eq. 7)
 *     k    = #{ j : m_j > tau }          retained leading components            (Eq. 8)
 *   x     [n x d] row stride ldx  (in)     U, W  [d x d]  (in)     b  float[d]  (in)
 *   xt    [n x d] storage type    (out)    x~
 *   k     int32[n]                (out)    the hard mask of token i is 1 on [0, k[i]) and 0 after
 *   m     float[n x d] or NULL    (out)    soft mask (training)
 *   xhat  [n x d] storage type or NULL (out)  softly gated state (training)
 */
LMHEAD_API int dynakv_gate(const dynakv_desc* desc, const void* x, const void* U, const void* W,
                           const float* b, float tau, void* xt, int32_t* k, float* m, void* xhat,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * The ragged store (the components that Eq. 2 leaves and that are "explicitly persisted").
 *     off[0] = off_base,  off[i+1] = off[i] + roundup(k[i], 8)
 *     packed[off[i] + j] = xt[i][j]  for j < k[i],   0 for k[i] <= j < roundup(k[i], 8)
 *   xt       [n x d] storage type (in)      k  int32[n], each in [0, d]  (in)
 *   off_base first element offset to use: 0 for a new store; to append the tokens of a decoding step
 *            to a cache, pass the cache's current end (its off[n_prev]) with `off` pointing at that
 *            entry of the cache's offset array and `packed` at the cache's base.  A multiple of 8, >= 0.
 *   off      int64[n+1]           (out)
 *   packed   storage type, `capacity` elements counted from `packed` (out); 16-byte aligned
 * A k[i] outside [0, d] is clamped into it, and a token whose segment would end beyond
 * `capacity` is not written; either sets the error word (dynakv_check -> LMHEAD_E_RANGE).
 * off_base + n * d elements always suffice.
 */
LMHEAD_API int dynakv_store(const dynakv_desc* desc, const void* xt, const int32_t* k, int64_t off_base,
                            int64_t* off, void* packed, int64_t capacity, void* ws, size_t ws_bytes,
                            void* stream);

/*
 * Dynamic low-rank reconstruction (Eq. 3): x_bar_i = x^_i[0:k_i] U^-1[0:k_i, :], a product whose
 * contraction length differs from token to token.  Tokens are grouped by length on the device so
 * that each matrix-core tile only runs as many steps as its longest token needs.
 *   packed, off, k   as written by dynakv_store; `packed_elems` = elements readable at `packed`
 *                    (at least off[n], at most 2^31 bytes worth)
 *   U_inv   [d x d] storage type (in)
 *   xbar    [n x d] storage type (out)
 * Offsets or counts that point outside `packed_elems` read as zeros and set the error word.
 */
LMHEAD_API int dynakv_reconstruct(const dynakv_desc* desc, const void* packed, int64_t packed_elems,
                                  const int64_t* off, const int32_t* k, const void* U_inv, void* xbar,
                                  void* ws, size_t ws_bytes, void* stream);

/*
 * Retain rate (Eq. 4) and the regulariser of the training objective (Eq. 9).
 *     R_hard = mean_i k[i] / d                         (k may be NULL: reported as 0)
 *     R_soft = mean_{i,j} m[i][j]                      (m may be NULL: reported as 0)
 *     penalty = alpha * R_soft^2,   g_m[i][j] = d penalty / d m[i][j] = 2 alpha R_soft / (n d)
 *   out   float[3] = { R_hard, R_soft, penalty }   (device)
 *   g_m   float[n x d] or NULL                      (device)
 * The sums are taken in a fixed order (deterministic tree), in fp32 with fp64 block totals.
 */
LMHEAD_API int dynakv_retain(const dynakv_desc* desc, const int32_t* k, const float* m, float alpha,
                             float* out, float* g_m, void* ws, size_t ws_bytes, void* stream);

/*
 * Backward of the training-time gate: the chain rule through Eqs. 1, 5, 6 and 7 (the paper trains U, W
 * and b through this "differentiable gate" with the objective of Eq. 9 and states the forward pass only).
 * Given g_xhat = dL/dx^ and, optionally, a direct gradient on the soft mask (the regulariser's is the
 * constant 2 alpha R / (n d): pass it as g_m_const), per token, with p and m recomputed from x~:
 *     q    = dL/dm      = g_xhat * x~ + g_m + g_m_const
 *     r_j  = dL/dp_j    = sum_{i <= j} q_i             (p_j feeds m_0 .. m_j;
 *                                                       sum_{i <= d-1-j} q_i with DYNAKV_FLAG_LITERAL_FLIP)
 *     g_l  = dL/dlogits = p * (r - sum_j p_j r_j)       fp32, then rounded to the storage type
 *     g_x~ = dL/dx~     = g_xhat * m + g_l W^T          storage type (the rounding of x~ is passed
 *                                                       straight through)
 *     dx = g_x~ U^T,    dU = x^T g_x~,    dW = x~^T g_l,    db = sum over tokens of g_l.
 *   x      [n x d] row stride ldx (in)     U, W [d x d] (in)     b float[d] (in)
 *   xt     [n x d] storage type   (in)     x~ as written by dynakv_gate for the same x, U
 *   g_xhat [n x d] storage type   (in)
 *   g_m    float[n x d] or NULL   (in)     g_m_const: added to every element of dL/dm
 *   dx     [n x d] storage type, dense (out)
 *   dU, dW float[d x d]; db float[d]  (out; added to with DYNAKV_FLAG_ACCUM_GRAD)
 *   ws     dynakv_bwd_workspace_bytes(desc) bytes (larger than the forward's: it holds the logits, the
 *          two token-major gradients and token-contiguous copies of the operands of dW and dU)
 * The contractions over the tokens accumulate in fp32, in slices summed in a fixed order.
 */
LMHEAD_API size_t dynakv_bwd_workspace_bytes(const dynakv_desc* desc);
LMHEAD_API int dynakv_gate_bwd(const dynakv_desc* desc, const void* x, const void* U, const void* W,
                               const float* b, const void* xt, const void* g_xhat, const float* g_m,
                               float g_m_const, void* dx, float* dU, float* dW, float* db, void* ws,
                               size_t ws_bytes, void* stream);

/* Synchronises `stream` and returns LMHEAD_E_RANGE if the most recent dynakv_* call that used
 * `ws` met a device-side range fault (see dynakv_store / dynakv_reconstruct), else LMHEAD_OK
 * (every call clears the word when it starts). */
LMHEAD_API int dynakv_check(void* ws, void* stream);

#ifdef __cplusplus
}
#endif

#endif /* DYNAKV_H_ */
