/*
 * lmhead.h - C ABI of the fused LM-head token log-probability objective for AMD MI355X (gfx950).
 *
 * The library evaluates, forward and backward, the token log-probabilities
 *     logp_i = z[i, y_i] - logsumexp_v z[i, v],      z = H W^T,
 * i.e. (minus) the per-token terms of the standard cross-entropy L_CE in the
 * paper's training objective (Sec. 3.3, Eq. 9), over the full vocabulary in
 * vocabulary chunks and without ever storing the N x V logits, plus the
 * policy-optimisation losses that the benchmark's problem statement puts on
 * top of those log-probabilities (group-relative advantages, the clipped
 * importance-ratio surrogate with a k3 KL term, the trajectory-balance
 * residual).  The paper itself states only L_CE; the other formulas are given
 * in full in the comments below.
 *
 * Conventions shared by all entry points
 * --------------------------------------
 *  - P prompts, G responses per prompt, T slots per response; R = P*G, N = R*T.
 *    Slot i = r*T + t belongs to response r = p*G + g and is VALID iff t < len[r]
 *    (right padding).  N_v = sum_r len[r].
 *  - Every pointer is DEVICE memory owned by the caller unless it is the
 *    descriptor (host memory).  The library allocates and frees nothing and keeps
 *    no state between calls (the one exception is the optional benchmark
 *    instrumentation lmhead_timing_*, which is process-wide).  `ws` is scratch: its
 *    contents are undefined after a call, except the sticky error word read by
 *    lmhead_check() and the integer index regions named by lmhead_workspace_region().
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *    work is enqueued on it; calls return without synchronising.  Scalar results
 *    (`loss`) are device scalars.
 *  - Return value: LMHEAD_OK or a negative LMHEAD_E_* code.  Argument errors are
 *    detected on the host before anything is launched and leave all outputs
 *    untouched.  Data errors that only the device can see (a length outside
 *    [0, T], a token id outside [0, V) on a valid slot) set a sticky word in the
 *    workspace; lengths are then clamped into [0, T] and the offending token
 *    contributes as if it were never sampled (no target logit), and
 *    lmhead_check() reports LMHEAD_E_RANGE.
 *  - Outputs on padded slots are exactly 0 (logp, lse, entropy, g_logp, rows of
 *    dH); token ids on padded slots are ignored.
 *  - Results are bit-reproducible from run to run for a fixed descriptor: no
 *    floating-point atomics are used.
 */
#ifndef LMHEAD_H_
#define LMHEAD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LMHEAD_API __attribute__((visibility("default")))

enum {
  LMHEAD_OK = 0,
  LMHEAD_E_NULL = -1,      /* a required pointer is NULL                              */
  LMHEAD_E_SHAPE = -2,     /* P,G,T,d,V <= 0; ld < d; d not a multiple of one 128-byte K-step (64 for bf16, 32 for  */
                           /* fp32, 128 with 8-bit logits); a size beyond the limits given at lmhead_desc; bad exponent */
  LMHEAD_E_DTYPE = -3,     /* dtype not LMHEAD_F32 / LMHEAD_BF16, or unknown flag bits  */
  LMHEAD_E_ALIGN = -4,     /* a matrix pointer is not 16-byte aligned, or ld*elem % 16  */
  LMHEAD_E_WORKSPACE = -5, /* ws_bytes smaller than lmhead_workspace_bytes()           */
  LMHEAD_E_RANGE = -6,     /* device-side range fault, reported by lmhead_check()      */
  LMHEAD_E_HIP = -7        /* a HIP launch or runtime call failed                      */
};

enum { LMHEAD_F32 = 0, LMHEAD_BF16 = 1 };

enum {
  LMHEAD_FLAG_ACCUM_DW = 1u << 1,   /* lmhead_logprob_bwd adds into dW instead of overwriting it */
  LMHEAD_FLAG_DH_BF16 = 1u << 3,    /* lmhead_logprob_bwd writes dH as bf16 [N x d] (accumulated in fp32 */
                                    /* scratch over the vocabulary chunks, rounded once at the end)       */
  LMHEAD_FLAG_FP8_LOGITS = 1u << 2  /* logits (forward and the backward's recompute) from 8-bit copies */
                                    /* of H and W: OCP e4m3, x * 2^fp8_exp rounded to nearest even and  */
                                    /* clamped to +-448, fp32 accumulation; dH and dW still contract    */
                                    /* with H and W as given.  Needs d % 128 == 0.  Not the default:    */
                                    /* it changes the logits by up to ~6 % of their spread.             */
};

/* Problem descriptor (host memory).
 * Size limits: the matrix-core kernels consume K in steps of one 128-byte line per row, so d must be a
 * multiple of 64 (bf16) or 32 (fp32) - the caller's W cannot be padded by the library, and a partial
 * last step would read the next row's values.  Operand tiles are addressed with 32-bit byte offsets
 * inside a 2 GiB window, which bounds every row pitch to 8 MiB: N + 320, V + 320 and ldH, ldW must each
 * stay below 4 Mi elements for bf16 (2 Mi for fp32); LMHEAD_E_SHAPE otherwise.  Split larger batches
 * by prompt (dW accumulates with LMHEAD_FLAG_ACCUM_DW). */
typedef struct lmhead_desc {
  int32_t P, G, T;     /* R = P*G responses, N = R*T token slots                          */
  int32_t d, V;        /* hidden size (multiple of 64; 32 for fp32) and vocabulary size   */
  int32_t dtype;       /* LMHEAD_F32 or LMHEAD_BF16: storage type of H and W              */
  int32_t vocab_chunk; /* vocabulary chunk of the backward (columns of dZ held at once);  */
                       /* 0 = library default (as wide as ~48 GB of scratch allows, at    */
                       /* most 262144, so small problems take the vocabulary in one       */
                       /* chunk).  Rounded up to a multiple of the 256-wide tile.         */
  int32_t fp8_exp_h;   /* with LMHEAD_FLAG_FP8_LOGITS: H is scaled by 2^fp8_exp_h before rounding  */
                       /* (choose it so that max|H| * 2^e <= 448); otherwise must be 0            */
  int64_t ldH, ldW;    /* row strides of H and W in elements (>= d)                       */
  uint32_t flags;      /* LMHEAD_FLAG_*                                                    */
  int32_t fp8_exp_w;   /* likewise for W (every W of a multi-policy forward)                       */
} lmhead_desc;

/* Scratch bytes that lmhead_logprob_fwd / lmhead_logprob_bwd need for this descriptor
 * (the larger of the two).  Returns 0 if the descriptor is invalid.  Host-only; no GPU needed. */
LMHEAD_API size_t lmhead_workspace_bytes(const lmhead_desc* desc);

/* Validates a descriptor on the host.  Returns LMHEAD_OK or the LMHEAD_E_* code that
 * the compute entry points would return for it. */
LMHEAD_API int lmhead_validate_desc(const lmhead_desc* desc);

/*
 * Where a forward call leaves its integer indexing in the workspace (host-only query; for tests and
 * diagnostics - the benchmark's problem statement asks for these integers to be checked bit for bit).
 * Valid after lmhead_logprob_fwd / _fwd_multi on `ws` until `ws` is passed to another call.
 *   LMHEAD_WS_NV           int32        N_v = number of valid slots
 *   LMHEAD_WS_ROW_SLOT     int32[Ncap]  compaction map: entry k < N_v is the slot of the k-th valid token
 *                                       (slot order); -1 from N_v up to the next multiple of 256
 *   LMHEAD_WS_TOK_C        int32[Ncap]  tok[row_slot[k]] (-1 for an id outside [0, V) and on the padding)
 *   LMHEAD_WS_GATHERED_ID  int32[npol][Ncap]  vocabulary column whose logit the logits kernel captured
 *                                       as the target logit of compact row k (-1: none captured)
 * Ncap = N rounded up to a multiple of 256.  npol = 1 for lmhead_logprob_fwd.
 * *offset = byte offset of the region from `ws`, *bytes = its size.
 */
enum { LMHEAD_WS_NV = 0, LMHEAD_WS_ROW_SLOT = 1, LMHEAD_WS_TOK_C = 2, LMHEAD_WS_GATHERED_ID = 3 };
LMHEAD_API int lmhead_workspace_region(const lmhead_desc* desc, int32_t npol, int32_t which,
                                       size_t* offset, size_t* bytes);

/*
 * Forward (the log-softmax inside L_CE, Eq. 9).  For every valid slot i:
 *     z_v   = sum_k H[i,k] W[v,k]                 (fp32 accumulation, never stored)
 *     lse_i = log sum_v exp(z_v)                  (online max/sum over vocabulary tiles)
 *     logp_i = z[y_i] - lse_i,   y_i = tok[i]
 *     entropy_i = lse_i - sum_v softmax(z)_v z_v  (optional)
 * Also emits the integer indexing of the batch.
 *   H      [N x d], row stride ldH, dtype per desc      (in)
 *   W      [V x d], row stride ldW, row v = output embedding of token v   (in)
 *   tok    int32[N]                                      (in)
 *   len    int32[R]                                      (in)
 *   logp, lse   float[N]                                 (out; lse may be NULL)
 *   entropy     float[N] or NULL                         (out)
 *   mask        uint8[N] or NULL:  1 on valid slots      (out)
 *   cu_len      int32[R+1] or NULL: exclusive prefix sum of len   (out)
 */
LMHEAD_API int lmhead_logprob_fwd(const lmhead_desc* desc, const void* H, const void* W,
                       const int32_t* tok, const int32_t* len,
                       float* logp, float* lse, float* entropy,
                       uint8_t* mask, int32_t* cu_len,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * The same forward for several weight matrices over ONE set of hidden states, in a single pass:
 * the indexing and the gather of the valid rows are done once and one matrix-core launch covers
 * every (matrix, vocabulary tile) pair.  This is the step of a policy-optimisation iteration that
 * evaluates the current, the sampling ("old") and the reference policy on the same hidden states.
 *   W      host array of npol device pointers, each [V x d] with row stride ldW (1 <= npol <= 4)
 *   logp   host array of npol device pointers, each float[N]                         (out)
 *   lse, entropy   of the FIRST matrix only (NULL to skip)                            (out)
 * Needs lmhead_multi_workspace_bytes(desc, npol) bytes of scratch (0 if the arguments are invalid);
 * everything else as for lmhead_logprob_fwd, whose results it reproduces bit for bit.
 */
LMHEAD_API size_t lmhead_multi_workspace_bytes(const lmhead_desc* desc, int32_t npol);
LMHEAD_API int lmhead_logprob_fwd_multi(const lmhead_desc* desc, const void* H, const void* const* W,
                             int32_t npol, const int32_t* tok, const int32_t* len,
                             float* const* logp, float* lse, float* entropy,
                             uint8_t* mask, int32_t* cu_len,
                             void* ws, size_t ws_bytes, void* stream);

/*
 * Backward through the same chunked softmax.  Given g_logp[i] = dL/dlogp_i (0 on
 * padding) and the lse saved by the forward:
 *     dZ[i,v] = g_i (1[v == y_i] - exp(z[i,v] - lse_i))     (recomputed per vocabulary chunk)
 *     dH[i,:] = sum_v dZ[i,v] W[v,:]         float[N x d] (bf16 with LMHEAD_FLAG_DH_BF16), dense row stride d;
 *                                            padded rows = 0
 *     dW[v,:] = sum_i dZ[i,v] H[i,:]         float[V x d], dense row stride d
 * With LMHEAD_FLAG_ACCUM_DW the result is added to the contents of dW.
 */
LMHEAD_API int lmhead_logprob_bwd(const lmhead_desc* desc, const void* H, const void* W,
                       const int32_t* tok, const int32_t* len,
                       const float* lse, const float* g_logp,
                       void* dH, float* dW,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * Group-relative advantages (problem statement):
 *     A[p,g] = (r[p,g] - mean_g r[p,:]) / (std_g r[p,:] + eps)
 * ddof = 0: population standard deviation; ddof = 1: sample standard deviation
 * (taken as 0 when G = 1).  A group with all rewards equal gives A = 0.
 *   reward float[P*G] (in), adv float[P*G] (out).
 */
LMHEAD_API int group_advantage(const float* reward, int32_t P, int32_t G, float eps, int32_t ddof,
                    float* adv, void* stream);

/* Scratch bytes needed by grpo_loss / flowrl_tb_loss (host-only). */
LMHEAD_API size_t lmhead_loss_workspace_bytes(int32_t P, int32_t G, int32_t T);

/*
 * Clipped importance-ratio surrogate with a k3 KL penalty (problem statement).
 * Per valid slot i of response r, A = adv[r]:
 *     rho   = exp(logp_i - logp_old_i)
 *     surr  = min(rho A, clip(rho, 1 - clip_lo, 1 + clip_hi) A)
 *     delta = logp_ref_i - logp_i,   k3 = exp(delta) - delta - 1
 *     l_i   = -surr + kl_coef k3                         (no KL term if logp_ref == NULL)
 *     loss  = sum_i w_i l_i
 *     g_logp_i = w_i ( -A rho sel_i + kl_coef (1 - exp(delta)) ),
 *     sel_i = (A >= 0 and rho <= 1 + clip_hi) or (A < 0 and rho >= 1 - clip_lo)
 * agg_mode 0: w_i = 1/(R len_r) (mean over responses of the token mean);
 * agg_mode 1: w_i = 1/N_v (global token mean).
 * stats (optional, float[4]): fraction of valid tokens on the clipped branch,
 * token-mean k3, token-mean rho, N_v.
 *   logp, logp_old, logp_ref float[N]; adv float[R]; len int32[R];
 *   loss float[1] (out); g_logp float[N] or NULL (out).
 */
LMHEAD_API int grpo_loss(const float* logp, const float* logp_old, const float* logp_ref,
              const float* adv, const int32_t* len, int32_t P, int32_t G, int32_t T,
              float clip_lo, float clip_hi, float kl_coef, int32_t agg_mode,
              float* loss, float* g_logp, float* stats,
              void* ws, size_t ws_bytes, void* stream);

/*
 * grpo_loss for callers that cannot allocate or carry a workspace: code under HIP graph capture, tight
 * serving / training loops, harnesses that forbid hipMalloc.  Same arguments, results and error codes as
 * grpo_loss (bit-identical outputs: the same kernels run), without `ws`: the block partials live in a
 * 1 MiB device array that is part of the library image (one copy per GPU the library runs on, held until
 * the process ends).  The call allocates and frees nothing.
 *   Limit: P * G * ceil(T / 2048) <= 65536 blocks; beyond it LMHEAD_E_WORKSPACE, before any launch.
 *   The array's device address is looked up on the first call on each device (a symbol lookup, no
 *   allocation); make that first call outside graph capture.
 *   Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (different
 *   streams or threads) race; calls on one stream are ordered and safe.  Nothing needs clearing between
 *   calls: each call writes every partial it later reads.
 */
LMHEAD_API int grpo_loss_noalloc(const float* logp, const float* logp_old, const float* logp_ref,
              const float* adv, const int32_t* len, int32_t P, int32_t G, int32_t T,
              float clip_lo, float clip_hi, float kl_coef, int32_t agg_mode,
              float* loss, float* g_logp, float* stats, void* stream);

/*
 * Cross-entropy over the target tokens: the L_CE term of the paper's training objective
 * L = L_CE + alpha R^2 (Sec. 3.3, Eq. 9), evaluated from the forward's log-probabilities:
 *     loss = -(1/N_v) sum_{valid i} logp_i,      g_logp_i = -1/N_v on valid slots, 0 on padding.
 * Feeding g_logp to lmhead_logprob_bwd gives dL_CE/dH and dL_CE/dW.
 *   logp float[R*T]; len int32[R]; loss float[1] (out); g_logp float[R*T] or NULL (out).
 * Scratch: lmhead_loss_workspace_bytes(R, 1, T).
 */
LMHEAD_API int ce_loss(const float* logp, const int32_t* len, int32_t R, int32_t T,
                       float* loss, float* g_logp, void* ws, size_t ws_bytes, void* stream);

/*
 * Trajectory-balance residual (problem statement).  For response r of prompt p = r / G:
 *     sbar_theta = (1/len_r) sum_{t < len_r} logp[r,t],   sbar_ref likewise (0 if len_r = 0)
 *     delta_r = logZ[p] + sbar_theta - beta reward[r] - sbar_ref
 *     loss    = (1/R) sum_r delta_r^2
 *     g_logp[r,t] = 2 delta_r / (R len_r)  (valid slots),   g_logZ[p] = (2/R) sum_g delta_{pG+g}
 *   logp, logp_ref float[N]; reward float[R]; logZ float[P]; len int32[R];
 *   loss float[1]; g_logp float[N] or NULL; g_logZ float[P] or NULL; resid float[R] or NULL.
 */
LMHEAD_API int flowrl_tb_loss(const float* logp, const float* logp_ref, const float* reward,
                   const float* logZ, const int32_t* len, int32_t P, int32_t G, int32_t T,
                   float beta,
                   float* loss, float* g_logp, float* g_logZ, float* resid,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * Synchronises `stream` and returns LMHEAD_OK, LMHEAD_E_RANGE if the last
 * lmhead_logprob_fwd/bwd call that used `ws` saw an out-of-range length or token
 * id, or LMHEAD_E_HIP if the stream reports an error.  `ws` must be a workspace
 * that has been passed to one of those calls.
 */
LMHEAD_API int lmhead_check(void* ws, void* stream);

/*
 * Optional instrumentation for benchmarks.  This is the only process-wide mutable state of the
 * library and it is NOT thread-safe: enable, run and read from one thread, with no other thread
 * inside a library call meanwhile.  lmhead_timing_enable(1) makes lmhead_logprob_fwd/bwd and the dynakv_* calls
 * (dynakv.h) bracket each of their main kernel launches with two HIP events on the launch stream (a fixed pool of 8192
 * pairs; launches beyond it are not timed) and clears earlier records; (0) turns it off.
 * lmhead_timing_read waits for the recorded events and returns, for one kernel kind
 * (0 = logits forward, 1 = dZ recompute, 2 = dH contraction, 3 = dW contraction, 4 = spectral
 * projection, 5 = gate logits, 6 = truncation mask, 7 = low-rank reconstruction; of dynakv_gate_bwd:
 * 8 = mask backward, 9 = g_x~ product, 10 = dx product, 11 = dW, 12 = dU, 13 = operand transposes), the summed
 * elapsed milliseconds and the number of launches since the last enable call.
 */
LMHEAD_API int lmhead_timing_enable(int on);
LMHEAD_API int lmhead_timing_read(int kind, double* total_ms, int64_t* launches);

/*
 * Measurement aid (not part of the path): enqueues a bare loop of the matrix-core instruction behind the bf16
 * contractions, v_mfma_f32_16x16x32_bf16, on operands that each thread loads once into registers:
 * `workgroups` x 4 wavefronts, each doing `iters` x 64 MFMAs = iters x 2^20 flop, so the launch does
 * workgroups * 4 * iters * 2^20 flop and moves no data meanwhile.  Timed by the caller (events on `stream`),
 * it gives the rate the matrix cores sustain under the part's power management for the operand content
 * given: the benchmark reports it for zeros and for random bf16 values next to the nominal peak.
 *   operands  device, 256 bytes per thread (workgroups * 256 threads), any bf16 content        (in)
 *   sink      device, one float per thread                                                     (out)
 * LMHEAD_E_WORKSPACE if a buffer is smaller than that; LMHEAD_E_SHAPE for workgroups or iters <= 0.
 */
LMHEAD_API int lmhead_probe_mfma(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes,
                                 int32_t workgroups, int32_t iters, void* stream);

/* Version of this ABI (bumped on any incompatible change). */
LMHEAD_API int lmhead_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LMHEAD_H_ */
