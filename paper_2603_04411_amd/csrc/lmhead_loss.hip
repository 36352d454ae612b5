// Loss kernels on top of the token log-probabilities: group-relative advantages, the clipped
// importance-ratio surrogate with k3 KL, and the trajectory-balance residual.  All are O(N)
// and HBM-bound: coalesced fp32 streams, wavefront shuffles for reductions, and fixed-order
// two-level sums (per block, then one block over the partials) so results are reproducible.
#include <atomic>

#include "common.h"

// Block partials of grpo_loss_noalloc: device memory that belongs to the library image instead of the
// caller (each GPU the library runs on holds its own copy until the process ends).  Host code never
// uses the array's name as an address: static_scratch() resolves the device address once per device.
static __device__ __align__(256) float scratch[lmhead::kStaticLossParts * 4];

namespace lmhead {

namespace {

__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// Sum over a 256-thread block; result valid in every thread.
__device__ inline float block_sum_256(float x, float* sh /*[4]*/) {
  x = wave_sum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = x;
  __syncthreads();
  return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

__device__ inline int block_sum_256_int(int x, int* sh /*[4]*/) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = x;
  __syncthreads();
  return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// One wavefront per prompt.
__global__ __launch_bounds__(64) void advantage_kernel(const float* __restrict__ reward, int G, float eps,
                                                       int ddof, float* __restrict__ adv) {
  const int p = blockIdx.x, lane = threadIdx.x;
  const float* r = reward + (size_t)p * G;
  float s = 0.f;
  for (int g = lane; g < G; g += 64) s += r[g];
  const float mu = wave_sum(s) / (float)G;
  float q = 0.f;
  for (int g = lane; g < G; g += 64) {
    const float dv = r[g] - mu;
    q = fmaf(dv, dv, q);
  }
  q = wave_sum(q);
  const int denom = G - ddof;
  const float var = denom > 0 ? q / (float)denom : 0.f;
  const float inv = 1.f / (sqrtf(var) + eps);
  for (int g = lane; g < G; g += 64) adv[(size_t)p * G + g] = (r[g] - mu) * inv;
}

// grid (blocks over T, R).  Partials: ws[(r * nb + b) * 4 + {loss, clipped, k3, rho}].
__global__ __launch_bounds__(256) void grpo_kernel(const float* __restrict__ lp, const float* __restrict__ lo,
                                                   const float* __restrict__ lr, const float* __restrict__ adv,
                                                   const int32_t* __restrict__ len, int R, int T,
                                                   float one_lo, float one_hi, float kl, int agg,
                                                   float* __restrict__ g_out, float* __restrict__ ws) {
  __shared__ float sh[4];
  __shared__ int nv_s;
  const int r = blockIdx.y, b = blockIdx.x, nb = gridDim.x;
  const int n = min(max(len[r], 0), T);
  float w;
  if (agg == 0) {
    w = n > 0 ? 1.f / ((float)R * (float)n) : 0.f;
  } else {
    // global token mean: every block re-derives N_v from the (short) length vector
    int acc = 0;
    for (int q = threadIdx.x; q < R; q += 256) acc += min(max(len[q], 0), T);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (threadIdx.x == 0) nv_s = 0;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) atomicAdd(&nv_s, acc);
    __syncthreads();
    w = nv_s > 0 ? 1.f / (float)nv_s : 0.f;
  }
  const float A = adv[r];
  float s_loss = 0.f, s_clip = 0.f, s_k3 = 0.f, s_rho = 0.f;
  const int t0 = b * kLossSlotsPerBlock;
  for (int t = t0 + threadIdx.x; t < min(t0 + kLossSlotsPerBlock, T); t += 256) {
    const size_t i = (size_t)r * T + t;
    float g = 0.f;
    if (t < n) {
      const float x = lp[i];
      const float rho = expf(x - lo[i]);
      const float clipped = fminf(fmaxf(rho, one_lo), one_hi);
      const float surr = fminf(rho * A, clipped * A);
      const bool sel = (A >= 0.f) ? (rho <= one_hi) : (rho >= one_lo);
      float k3 = 0.f, dk3 = 0.f;
      if (lr) {
        const float dl = lr[i] - x;
        const float e = expf(dl);
        k3 = e - dl - 1.f;
        dk3 = 1.f - e;
      }
      s_loss += w * (-surr + kl * k3);
      s_clip += sel ? 0.f : 1.f;
      s_k3 += k3;
      s_rho += rho;
      g = w * ((sel ? -A * rho : 0.f) + kl * dk3);
    }
    if (g_out) g_out[i] = g;
  }
  s_loss = block_sum_256(s_loss, sh);
  s_clip = block_sum_256(s_clip, sh);
  s_k3 = block_sum_256(s_k3, sh);
  s_rho = block_sum_256(s_rho, sh);
  if (threadIdx.x == 0) {
    float* q = ws + ((size_t)r * nb + b) * 4;
    q[0] = s_loss;
    q[1] = s_clip;
    q[2] = s_k3;
    q[3] = s_rho;
  }
}

__global__ __launch_bounds__(256) void grpo_final_kernel(const float* __restrict__ ws, int nparts,
                                                         const int32_t* __restrict__ len, int R, int T,
                                                         float* __restrict__ loss, float* __restrict__ stats) {
  __shared__ float sh[4];
  __shared__ int shi[4];
  float a[4] = {0.f, 0.f, 0.f, 0.f};
  for (int q = threadIdx.x; q < nparts; q += 256)
#pragma unroll
    for (int c = 0; c < 4; ++c) a[c] += ws[(size_t)q * 4 + c];
  // N_v is counted in integers (exact for any N) and converted once
  int nvi = 0;
  for (int q = threadIdx.x; q < R; q += 256) nvi += min(max(len[q], 0), T);
#pragma unroll
  for (int c = 0; c < 4; ++c) a[c] = block_sum_256(a[c], sh);
  const int nv = block_sum_256_int(nvi, shi);
  if (threadIdx.x == 0) {
    loss[0] = a[0];
    if (stats) {
      const float nvf = (float)nv;
      const float inv = nv > 0 ? 1.f / nvf : 0.f;
      stats[0] = a[1] * inv;
      stats[1] = a[2] * inv;
      stats[2] = a[3] * inv;
      stats[3] = nvf;
    }
  }
}

// Cross-entropy over the valid targets: partial sums of logp per (response, block); the gradient
// -1/N_v is written in the same pass (every block re-derives N_v from the short length vector).
__global__ __launch_bounds__(256) void ce_kernel(const float* __restrict__ lp, const int32_t* __restrict__ len,
                                                 int R, int T, float* __restrict__ g_out,
                                                 float* __restrict__ ws) {
  __shared__ float sh[4];
  __shared__ int nv_s;
  const int r = blockIdx.y, b = blockIdx.x, nb = gridDim.x;
  const int n = min(max(len[r], 0), T);
  int acc = 0;
  for (int q = threadIdx.x; q < R; q += 256) acc += min(max(len[q], 0), T);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if (threadIdx.x == 0) nv_s = 0;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) atomicAdd(&nv_s, acc);
  __syncthreads();
  const float gv = nv_s > 0 ? -1.f / (float)nv_s : 0.f;
  float a = 0.f;
  const int t0 = b * kLossSlotsPerBlock;
  for (int t = t0 + threadIdx.x; t < min(t0 + kLossSlotsPerBlock, T); t += 256) {
    const size_t i = (size_t)r * T + t;
    if (t < n) a += lp[i];
    if (g_out) g_out[i] = t < n ? gv : 0.f;
  }
  a = block_sum_256(a, sh);
  if (threadIdx.x == 0) ws[(size_t)r * nb + b] = a;
}

__global__ __launch_bounds__(256) void ce_final_kernel(const float* __restrict__ ws, int nparts,
                                                       const int32_t* __restrict__ len, int R, int T,
                                                       float* __restrict__ loss) {
  __shared__ float sh[4];
  __shared__ int shi[4];
  float a = 0.f;
  int nvi = 0;
  for (int q = threadIdx.x; q < nparts; q += 256) a += ws[q];
  for (int q = threadIdx.x; q < R; q += 256) nvi += min(max(len[q], 0), T);
  a = block_sum_256(a, sh);
  const int nv = block_sum_256_int(nvi, shi);
  if (threadIdx.x == 0) loss[0] = nv > 0 ? -a / (float)nv : 0.f;
}

// Trajectory balance, pass 1: per (response, block) sums of logp and logp_ref over valid slots.
__global__ __launch_bounds__(256) void tb_sum_kernel(const float* __restrict__ lp, const float* __restrict__ lr,
                                                     const int32_t* __restrict__ len, int T,
                                                     float* __restrict__ ws) {
  __shared__ float sh[4];
  const int r = blockIdx.y, b = blockIdx.x, nb = gridDim.x;
  const int n = min(max(len[r], 0), T);
  float a = 0.f, c = 0.f;
  const int t0 = b * kLossSlotsPerBlock;
  for (int t = t0 + threadIdx.x; t < min(t0 + kLossSlotsPerBlock, n); t += 256) {
    const size_t i = (size_t)r * T + t;
    a += lp[i];
    c += lr[i];
  }
  a = block_sum_256(a, sh);
  c = block_sum_256(c, sh);
  if (threadIdx.x == 0) {
    ws[((size_t)r * nb + b) * 2] = a;
    ws[((size_t)r * nb + b) * 2 + 1] = c;
  }
}

// Pass 2 (one block): residuals, loss, dL/dlogZ.  delta_r is left in dl[r] for pass 3.
__global__ __launch_bounds__(256) void tb_resid_kernel(const float* __restrict__ ws, int nb,
                                                       const float* __restrict__ reward,
                                                       const float* __restrict__ logZ,
                                                       const int32_t* __restrict__ len, int P, int G, int T,
                                                       float beta, float* __restrict__ dl,
                                                       float* __restrict__ loss, float* __restrict__ gz,
                                                       float* __restrict__ resid) {
  __shared__ float sh[4];
  const int R = P * G;
  float sq = 0.f;
  for (int r = threadIdx.x; r < R; r += 256) {
    float a = 0.f, c = 0.f;
    for (int b = 0; b < nb; ++b) {
      a += ws[((size_t)r * nb + b) * 2];
      c += ws[((size_t)r * nb + b) * 2 + 1];
    }
    const int n = min(max(len[r], 0), T);
    const float inv = n > 0 ? 1.f / (float)n : 0.f;
    const float dv = logZ[r / G] + a * inv - beta * reward[r] - c * inv;
    dl[r] = dv;
    if (resid) resid[r] = dv;
    sq = fmaf(dv, dv, sq);
  }
  sq = block_sum_256(sq, sh);  // (contains the barrier that makes dl[] visible below)
  if (threadIdx.x == 0) loss[0] = sq / (float)R;
  if (gz) {
    __threadfence_block();
    __syncthreads();
    for (int p = threadIdx.x; p < P; p += 256) {
      float a = 0.f;
      for (int g = 0; g < G; ++g) a += dl[(size_t)p * G + g];
      gz[p] = 2.f * a / (float)R;
    }
  }
}

__global__ __launch_bounds__(256) void tb_grad_kernel(const float* __restrict__ dl,
                                                      const int32_t* __restrict__ len, int R, int T,
                                                      float* __restrict__ g_out) {
  const int r = blockIdx.y;
  const int n = min(max(len[r], 0), T);
  const float gv = n > 0 ? 2.f * dl[r] / ((float)R * (float)n) : 0.f;
  const int t0 = blockIdx.x * kLossSlotsPerBlock;
  for (int t = t0 + threadIdx.x; t < min(t0 + kLossSlotsPerBlock, T); t += 256)
    g_out[(size_t)r * T + t] = t < n ? gv : 0.f;
}

}  // namespace

hipError_t launch_group_advantage(const float* reward, int P, int G, float eps, int ddof, float* adv,
                                  hipStream_t s) {
  hipLaunchKernelGGL(advantage_kernel, dim3(P), dim3(64), 0, s, reward, G, eps, ddof, adv);
  return hipGetLastError();
}

hipError_t launch_grpo(const float* lp, const float* lo, const float* lr, const float* adv,
                       const int32_t* len, int P, int G, int T, float clip_lo, float clip_hi, float kl,
                       int agg, float* loss, float* g, float* stats, float* ws, hipStream_t s) {
  const int R = P * G;
  const int nb = (T + kLossSlotsPerBlock - 1) / kLossSlotsPerBlock;
  hipLaunchKernelGGL(grpo_kernel, dim3(nb, R), dim3(256), 0, s, lp, lo, lr, adv, len, R, T,
                     1.f - clip_lo, 1.f + clip_hi, kl, agg, g, ws);
  hipLaunchKernelGGL(grpo_final_kernel, dim3(1), dim3(256), 0, s, ws, R * nb, len, R, T, loss, stats);
  return hipGetLastError();
}

// Device address of `scratch` on the current device (resolved on the first call per device, with that
// device current; later calls read the kept pointer).
hipError_t static_scratch(float** out) {
  constexpr int kMaxDev = 64;
  static std::atomic<float*> ptr[kMaxDev];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
  float* p = ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!sym) return hipErrorInvalidSymbol;
    p = static_cast<float*>(sym);
    ptr[dev].store(p, std::memory_order_release);   // racing threads resolve the same address
  }
  *out = p;
  return hipSuccess;
}

hipError_t launch_ce(const float* lp, const int32_t* len, int R, int T, float* loss, float* g, float* ws,
                     hipStream_t s) {
  const int nb = (T + kLossSlotsPerBlock - 1) / kLossSlotsPerBlock;
  hipLaunchKernelGGL(ce_kernel, dim3(nb, R), dim3(256), 0, s, lp, len, R, T, g, ws);
  hipLaunchKernelGGL(ce_final_kernel, dim3(1), dim3(256), 0, s, ws, R * nb, len, R, T, loss);
  return hipGetLastError();
}

hipError_t launch_flowrl(const float* lp, const float* lr, const float* reward, const float* logZ,
                         const int32_t* len, int P, int G, int T, float beta, float* loss, float* g,
                         float* gz, float* resid, float* ws, hipStream_t s) {
  const int R = P * G;
  const int nb = (T + kLossSlotsPerBlock - 1) / kLossSlotsPerBlock;
  float* dl = ws + (size_t)R * nb * 2;
  hipLaunchKernelGGL(tb_sum_kernel, dim3(nb, R), dim3(256), 0, s, lp, lr, len, T, ws);
  hipLaunchKernelGGL(tb_resid_kernel, dim3(1), dim3(256), 0, s, ws, nb, reward, logZ, len, P, G, T, beta,
                     dl, loss, gz, resid);
  if (g) hipLaunchKernelGGL(tb_grad_kernel, dim3(nb, R), dim3(256), 0, s, dl, len, R, T, g);
  return hipGetLastError();
}

}  // namespace lmhead
