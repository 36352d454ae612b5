// Bandwidth-bound kernels of the KV-compression path: the truncation mask (softmax, cumulative
// sum, threshold; Eqs. 5-8), the ragged store (offset scan + segment copy), the grouping of
// tokens by contraction length for the reconstruction, and the retain rate (Eqs. 4 and 9).
// Rows are handled one wavefront per token with 16-byte accesses.
#include "dynakv_common.h"

namespace lmhead {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ inline int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <typename T>
struct Store4;
template <>
struct Store4<float> {
  __device__ static inline void load(const float* p, float (&v)[4]) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  __device__ static inline void store(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <>
struct Store4<__bf16> {
  typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
  __device__ static inline void load(const __bf16* p, float (&v)[4]) {
    const bf16x4_t t = *reinterpret_cast<const bf16x4_t*>(p);
    v[0] = (float)t.x; v[1] = (float)t.y; v[2] = (float)t.z; v[3] = (float)t.w;
  }
  __device__ static inline void store(__bf16* p, const float (&v)[4]) {
    const bf16x4_t t = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
    *reinterpret_cast<bf16x4_t*>(p) = t;
  }
};

// ---- truncation mask -----------------------------------------------------------------------
//
// One wavefront per token.  Mask position i belongs to gate column j(i) = i (reverse cumulative
// sum) or j(i) = d-1-i (Eq. 6 as printed: Flip(cumsum(p))_i = sum_{i' >= i} p_{d-1-i'}), so both
// readings are the same suffix sum over positions.  Positions are walked in groups of 256 (four
// per lane, contiguous), last group first, carrying the running suffix.
// NG > 0: the row has NG groups (d <= 256 NG) and is held in registers: one pass over memory.
// NG == 0: any d; the row of logits is read three times (max, sum, suffix), the second and third
// time from L1/L2.
template <typename T, int NG>
__global__ __launch_bounds__(256) void kv_mask_kernel(const float* __restrict__ logits,
                                                      const float* __restrict__ bias,
                                                      const T* __restrict__ xt, int64_t n, int d, float tau,
                                                      int literal, int32_t* __restrict__ k_out,
                                                      float* __restrict__ m_out, T* __restrict__ xhat) {
  const int lane = threadIdx.x & 63;
  const int64_t tok = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tok >= n) return;
  const float* z = logits + tok * d;
  const int ngroups = NG > 0 ? NG : (d + 255) / 256;

  // logits (+ bias) of the four positions that start at i0, in position order
  auto load4 = [&](int i0, float (&v)[4]) {
    if (!literal) {
      const float4 a = *reinterpret_cast<const float4*>(z + i0);
      const float4 b = *reinterpret_cast<const float4*>(bias + i0);
      v[0] = a.x + b.x; v[1] = a.y + b.y; v[2] = a.z + b.z; v[3] = a.w + b.w;
    } else {
      const int j0 = d - 4 - i0;   // columns j0 .. j0+3 are positions i0+3 .. i0
      const float4 a = *reinterpret_cast<const float4*>(z + j0);
      const float4 b = *reinterpret_cast<const float4*>(bias + j0);
      v[0] = a.w + b.w; v[1] = a.z + b.z; v[2] = a.y + b.y; v[3] = a.x + b.x;
    }
  };

  constexpr int NR = NG > 0 ? NG : 1;
  float row[NR][4];
  float mx = -__builtin_huge_valf();
  float sum = 0.f;
  if constexpr (NG > 0) {
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int i0 = g * 256 + lane * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) row[g][e] = -__builtin_huge_valf();
      if (i0 < d) load4(i0, row[g]);
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) mx = fmaxf(fmaxf(mx, fmaxf(row[g][0], row[g][1])), fmaxf(row[g][2], row[g][3]));
    mx = wave_max(mx);
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        row[g][e] = __builtin_amdgcn_exp2f((row[g][e] - mx) * kLog2e);   // exp(-inf) = 0 beyond d
        sum += row[g][e];
      }
  } else {
    for (int g = 0; g < ngroups; ++g) {
      const int i0 = g * 256 + lane * 4;
      if (i0 < d) {
        float v[4];
        load4(i0, v);
        mx = fmaxf(fmaxf(mx, fmaxf(v[0], v[1])), fmaxf(v[2], v[3]));
      }
    }
    mx = wave_max(mx);
    for (int g = 0; g < ngroups; ++g) {
      const int i0 = g * 256 + lane * 4;
      if (i0 < d) {
        float v[4];
        load4(i0, v);
#pragma unroll
        for (int e = 0; e < 4; ++e) sum += __builtin_amdgcn_exp2f((v[e] - mx) * kLog2e);
      }
    }
  }
  sum = wave_sum(sum);
  const float inv = 1.0f / sum;

  float carry = 0.f;   // sum of exp over all positions after the current group
  int count = 0;
  // one group: s[] = the lane's four exponentials in position order
  auto group = [&](int g, float (&s)[4]) {
    const int i0 = g * 256 + lane * 4;
    const bool on = i0 < d;
    s[2] += s[3];
    s[1] += s[2];
    s[0] += s[1];
    // inclusive suffix sum of the lanes' totals (this lane and the lanes above it)
    float incl = s[0];
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const float y = __shfl_down(incl, o);
      if (lane + o < 64) incl += y;
    }
    const float above = carry + (incl - s[0]);
    carry += __shfl(incl, 0);
    if (on) {
      float mk[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        mk[e] = (above + s[e]) * inv;
        count += mk[e] > tau ? 1 : 0;
      }
      if (m_out) Store4<float>::store(m_out + tok * d + i0, mk);
      if (xhat) {
        float xv[4];
        Store4<T>::load(xt + tok * d + i0, xv);
#pragma unroll
        for (int e = 0; e < 4; ++e) xv[e] *= mk[e];
        Store4<T>::store(xhat + tok * d + i0, xv);
      }
    }
  };
  if constexpr (NG > 0) {
#pragma unroll
    for (int g = NG - 1; g >= 0; --g) group(g, row[g]);
  } else {
    for (int g = ngroups - 1; g >= 0; --g) {
      const int i0 = g * 256 + lane * 4;
      float s[4] = {0.f, 0.f, 0.f, 0.f};
      if (i0 < d) {
        float v[4];
        load4(i0, v);
#pragma unroll
        for (int e = 0; e < 4; ++e) s[e] = __builtin_amdgcn_exp2f((v[e] - mx) * kLog2e);
      }
      group(g, s);
    }
  }
  count = wave_sum_i(count);
  if (lane == 0) k_out[tok] = count;
}

// ---- backward of the truncation mask ---------------------------------------------------------
//
// Chain rule through Eqs. 5-7 for one token, in the position order of kv_mask_kernel (position i =
// component i of x~, x^ and m; gate column j(i) = i, or d-1-i for Eq. 6 as printed):
//   p_i = softmax of the logits (+ bias),   m_i = sum_{i' >= i} p_i'          (recomputed)
//   q_i = dL/dm_i  = g_xhat_i * x~_i + g_m_i + g_m_const
//   r_i = dL/dp_i  = sum_{i' <= i} q_i'                (p_i feeds m_0 .. m_i)
//   g_l = dL/dlogit at column j(i) = p_i * (r_i - sum_i' p_i' r_i')             (softmax Jacobian)
//   a_i = g_xhat_i * m_i                               (the direct part of dL/dx~)
// One wavefront per token, looping over tokens with the grid's stride.  Each wavefront adds its g_l
// rows into its own strip of LDS (a lane always owns the same positions, so no atomics and a fixed
// order); the workgroup's four strips are summed at the end into one row of dbpart.
// NG as in kv_mask_kernel: NG > 0 keeps the row and q (then r) in registers; NG == 0 re-reads.
// Up to d = 1024 the kernel is held to 128 VGPRs so that four workgroups share a compute unit.
template <typename T, int NG>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NG > 0 && NG <= 4 ? 4 : 2)))
void kv_mask_bwd_kernel(const float* __restrict__ logits, const float* __restrict__ bias, const T* __restrict__ xt,
                        const T* __restrict__ gxh, const float* __restrict__ gm, float gmc, int64_t n, int d,
                        int literal, T* __restrict__ gl, T* __restrict__ a_out, float* __restrict__ dbpart) {
  extern __shared__ float colsum[];   // [4][d], position order
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  float* const acc = colsum + wave * d;
  const int ngroups = NG > 0 ? NG : (d + 255) / 256;
  for (int g = 0; g < ngroups; ++g) {
    const int i0 = g * 256 + lane * 4;
    if (i0 < d) *reinterpret_cast<float4*>(acc + i0) = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  constexpr int NR = NG > 0 ? NG : 1;

  for (int64_t tok = (int64_t)blockIdx.x * 4 + wave; tok < n; tok += (int64_t)gridDim.x * 4) {
    const float* z = logits + tok * d;
    auto load4 = [&](int i0, float (&v)[4]) {
      if (!literal) {
        const float4 a = *reinterpret_cast<const float4*>(z + i0);
        const float4 b = *reinterpret_cast<const float4*>(bias + i0);
        v[0] = a.x + b.x; v[1] = a.y + b.y; v[2] = a.z + b.z; v[3] = a.w + b.w;
      } else {
        const int j0 = d - 4 - i0;
        const float4 a = *reinterpret_cast<const float4*>(z + j0);
        const float4 b = *reinterpret_cast<const float4*>(bias + j0);
        v[0] = a.w + b.w; v[1] = a.z + b.z; v[2] = a.y + b.y; v[3] = a.x + b.x;
      }
    };

    // softmax statistics, as in the forward kernel
    float row[NR][4];
    float mx = -__builtin_huge_valf();
    float sum = 0.f;
    if constexpr (NG > 0) {
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int i0 = g * 256 + lane * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) row[g][e] = -__builtin_huge_valf();
        if (i0 < d) load4(i0, row[g]);
      }
#pragma unroll
      for (int g = 0; g < NG; ++g) mx = fmaxf(fmaxf(mx, fmaxf(row[g][0], row[g][1])), fmaxf(row[g][2], row[g][3]));
      mx = wave_max(mx);
#pragma unroll
      for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          row[g][e] = __builtin_amdgcn_exp2f((row[g][e] - mx) * kLog2e);
          sum += row[g][e];
        }
    } else {
      for (int g = 0; g < ngroups; ++g) {
        const int i0 = g * 256 + lane * 4;
        if (i0 < d) {
          float v[4];
          load4(i0, v);
          mx = fmaxf(fmaxf(mx, fmaxf(v[0], v[1])), fmaxf(v[2], v[3]));
        }
      }
      mx = wave_max(mx);
      for (int g = 0; g < ngroups; ++g) {
        const int i0 = g * 256 + lane * 4;
        if (i0 < d) {
          float v[4];
          load4(i0, v);
#pragma unroll
          for (int e = 0; e < 4; ++e) sum += __builtin_amdgcn_exp2f((v[e] - mx) * kLog2e);
        }
      }
    }
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;

    // the lane's four exponentials of group g (0 beyond d)
    auto expo = [&](int g, float (&s)[4]) {
      if constexpr (NG > 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) s[e] = row[g][e];
      } else {
        const int i0 = g * 256 + lane * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) s[e] = 0.f;
        if (i0 < d) {
          float v[4];
          load4(i0, v);
#pragma unroll
          for (int e = 0; e < 4; ++e) s[e] = __builtin_amdgcn_exp2f((v[e] - mx) * kLog2e);
        }
      }
    };
    // q of group g (0 beyond d) and the g_xhat values it was formed from
    auto load_q = [&](int g, float (&q)[4], float (&gx)[4]) {
      const int i0 = g * 256 + lane * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) q[e] = gx[e] = 0.f;
      if (i0 < d) {
        float xv[4];
        Store4<T>::load(xt + tok * d + i0, xv);
        Store4<T>::load(gxh + tok * d + i0, gx);
#pragma unroll
        for (int e = 0; e < 4; ++e) q[e] = gx[e] * xv[e] + gmc;
        if (gm) {
          const float4 t = *reinterpret_cast<const float4*>(gm + tok * d + i0);
          q[0] += t.x; q[1] += t.y; q[2] += t.z; q[3] += t.w;
        }
      }
    };
    // q of one group turned, in place, into r: the inclusive prefix sums over all positions up to each one
    auto scan_prefix = [&](float& carry, float (&r)[4]) {
      r[1] += r[0];
      r[2] += r[1];
      r[3] += r[2];
      float incl = r[3];
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const float y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
      }
      const float below = carry + (incl - r[3]);
      carry += __shfl(incl, 63);
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] += below;
    };

    // m (suffix sums, last group first), a = g_xhat * m, and q (kept when the row is held in registers)
    float qk[NR][4];
    {
      float carry = 0.f;
      auto step = [&](int g, float (&q)[4]) {
        const int i0 = g * 256 + lane * 4;
        float sfx[4];
        expo(g, sfx);
        sfx[2] += sfx[3];
        sfx[1] += sfx[2];
        sfx[0] += sfx[1];
        float incl = sfx[0];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const float y = __shfl_down(incl, o);
          if (lane + o < 64) incl += y;
        }
        const float above = carry + (incl - sfx[0]);
        carry += __shfl(incl, 0);
        float gx[4];
        load_q(g, q, gx);
        if (i0 < d) {
#pragma unroll
          for (int e = 0; e < 4; ++e) gx[e] *= (above + sfx[e]) * inv;
          Store4<T>::store(a_out + tok * d + i0, gx);
        }
      };
      if constexpr (NG > 0) {
#pragma unroll
        for (int g = NG - 1; g >= 0; --g) step(g, qk[g]);
      } else {
        for (int g = ngroups - 1; g >= 0; --g) step(g, qk[0]);
      }
    }

    // r (in place of q) and s = sum_i p_i r_i
    float s = 0.f;
    {
      float carry = 0.f;
      auto step = [&](int g, float (&r)[4]) {
        if constexpr (NG == 0) {
          float gx[4];
          load_q(g, r, gx);
        }
        scan_prefix(carry, r);
        float ex[4];
        expo(g, ex);
#pragma unroll
        for (int e = 0; e < 4; ++e) s += ex[e] * r[e];
      };
      if constexpr (NG > 0) {
#pragma unroll
        for (int g = 0; g < NG; ++g) step(g, qk[g]);
      } else {
        for (int g = 0; g < ngroups; ++g) step(g, qk[0]);
      }
    }
    s = wave_sum(s) * inv;

    // g_l = p (r - s), stored in gate column order and added to the wavefront's column sums
    {
      float carry = 0.f;
      auto step = [&](int g, float (&r)[4]) {
        const int i0 = g * 256 + lane * 4;
        if constexpr (NG == 0) {
          float gx[4];
          load_q(g, r, gx);
          scan_prefix(carry, r);
        }
        float ex[4];
        expo(g, ex);
        if (i0 < d) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = ex[e] * inv * (r[e] - s);
          float4 t = *reinterpret_cast<const float4*>(acc + i0);
          t.x += v[0]; t.y += v[1]; t.z += v[2]; t.w += v[3];
          *reinterpret_cast<float4*>(acc + i0) = t;
          if (!literal) {
            Store4<T>::store(gl + tok * d + i0, v);
          } else {
            const float w[4] = {v[3], v[2], v[1], v[0]};
            Store4<T>::store(gl + tok * d + (d - 4 - i0), w);
          }
        }
      };
      if constexpr (NG > 0) {
#pragma unroll
        for (int g = 0; g < NG; ++g) step(g, qk[g]);
      } else {
        for (int g = 0; g < ngroups; ++g) step(g, qk[0]);
      }
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += 256) {
    const float t = ((colsum[c] + colsum[d + c]) + colsum[2 * d + c]) + colsum[3 * d + c];
    dbpart[(int64_t)blockIdx.x * d + (literal ? d - 1 - c : c)] = t;
  }
}

// out[j] (+)= sum over the rows of part.  A workgroup owns 64 columns; its four wavefronts each sum
// every fourth row (four independent running sums each), and the partial sums are combined in a fixed
// order, so the result does not depend on the launch.
__global__ __launch_bounds__(256) void kv_sum_rows_kernel(const float* __restrict__ part, int rows, int64_t row_pitch,
                                                          int64_t len, float* __restrict__ out, int accumulate) {
  __shared__ float sm[4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int64_t j = (int64_t)blockIdx.x * 64 + cl;
  float t[4] = {0.f, 0.f, 0.f, 0.f};
  if (j < len) {
    int r = rl;
    for (; r + 12 < rows; r += 16) {
#pragma unroll
      for (int u = 0; u < 4; ++u) t[u] += part[(int64_t)(r + 4 * u) * row_pitch + j];
    }
    for (; r < rows; r += 4) t[0] += part[(int64_t)r * row_pitch + j];
  }
  sm[rl][cl] = (t[0] + t[1]) + (t[2] + t[3]);
  __syncthreads();
  if (rl == 0 && j < len) {
    const float v = (sm[0][cl] + sm[1][cl]) + (sm[2][cl] + sm[3][cl]);
    out[j] = accumulate ? out[j] + v : v;
  }
}

// Row-padded copy of a parameter matrix: 16 bytes per thread, zero beyond the source's extent.
__global__ __launch_bounds__(256) void kv_pad_copy_kernel(const char* __restrict__ in, int64_t in_pitch, int rows,
                                                          int row_bytes, char* __restrict__ out, int64_t out_pitch,
                                                          int rows_p) {
  const int chunks = (int)(out_pitch / 16);
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t r = id / chunks;
  const int c = (int)(id % chunks) * 16;
  if (r >= rows_p) return;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (r < rows && c < row_bytes) v = *reinterpret_cast<const uint4*>(in + r * in_pitch + c);
  *reinterpret_cast<uint4*>(out + r * out_pitch + c) = v;
}

// ---- ragged store ---------------------------------------------------------------------------

__device__ inline int seg_len(int k, int d, int& bad) {
  if (k < 0 || k > d) {
    bad = 1;
    k = k < 0 ? 0 : d;
  }
  return (k + DYNAKV_GRANULE - 1) / DYNAKV_GRANULE * DYNAKV_GRANULE;
}

// Block totals of the segment lengths (kKvScanBlock tokens per block).
__global__ __launch_bounds__(256) void kv_scan_totals_kernel(const int32_t* __restrict__ k, int64_t n, int d,
                                                             int64_t* __restrict__ blocksum, WsHeader* hdr) {
  __shared__ int wsum[4];
  const int64_t base = (int64_t)blockIdx.x * kKvScanBlock;
  int bad = 0, tot = 0;
  for (int i = threadIdx.x; i < kKvScanBlock; i += 256)
    if (base + i < n) tot += seg_len(k[base + i], d, bad);
  tot = wave_sum_i(tot);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = tot;
  if (bad) atomicOr(&hdr->err, kErrKvCount);
  __syncthreads();
  if (threadIdx.x == 0) blocksum[blockIdx.x] = (int64_t)wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

// One workgroup: blocksum <- its exclusive prefix sum; blocksum[nblocks] = grand total.
__global__ __launch_bounds__(1024) void kv_scan_blocks_kernel(int64_t* __restrict__ blocksum, int nblocks) {
  __shared__ int64_t buf[1024];
  __shared__ int64_t carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int base = 0; base < nblocks; base += 1024) {
    const int i = base + threadIdx.x;
    const int64_t x = i < nblocks ? blocksum[i] : 0;
    buf[threadIdx.x] = x;
    __syncthreads();
    for (unsigned o = 1; o < 1024; o <<= 1) {
      const int64_t y = threadIdx.x >= o ? buf[threadIdx.x - o] : 0;
      __syncthreads();
      buf[threadIdx.x] += y;
      __syncthreads();
    }
    const int64_t carry = carry_s;
    if (i < nblocks) blocksum[i] = carry + buf[threadIdx.x] - x;
    __syncthreads();
    if (threadIdx.x == 1023) carry_s = carry + buf[1023];
    __syncthreads();
  }
  if (threadIdx.x == 0) blocksum[nblocks] = carry_s;
}

// off[i] = prefix of the block + exclusive prefix inside the block; off[n] = grand total.
__global__ __launch_bounds__(1024) void kv_scan_offsets_kernel(const int32_t* __restrict__ k, int64_t n, int d,
                                                               const int64_t* __restrict__ blocksum,
                                                               int nblocks, int64_t off_base,
                                                               int64_t* __restrict__ off) {
  __shared__ int buf[1024];
  const int64_t i = (int64_t)blockIdx.x * kKvScanBlock + threadIdx.x;
  int bad = 0;
  const int x = i < n ? seg_len(k[i], d, bad) : 0;
  buf[threadIdx.x] = x;
  __syncthreads();
  for (unsigned o = 1; o < 1024; o <<= 1) {
    const int y = threadIdx.x >= o ? buf[threadIdx.x - o] : 0;
    __syncthreads();
    buf[threadIdx.x] += y;
    __syncthreads();
  }
  if (i < n) off[i] = off_base + blocksum[blockIdx.x] + buf[threadIdx.x] - x;
  if (i == n - 1) off[n] = off_base + blocksum[nblocks];
}
static_assert(kKvScanBlock == 1024, "the offset kernel scans one token per thread");

// One wavefront per token: copy the segment, zero the tail of its last granule.
template <typename T>
__global__ __launch_bounds__(256) void kv_pack_kernel(const T* __restrict__ xt, const int32_t* __restrict__ k,
                                                      const int64_t* __restrict__ off, int64_t n, int d,
                                                      T* __restrict__ packed, int64_t capacity, WsHeader* hdr) {
  constexpr int EPC = 16 / (int)sizeof(T);   // elements per 16-byte chunk
  const int lane = threadIdx.x & 63;
  const int64_t tok = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tok >= n) return;
  int bad = 0;
  const int kk = min(max(k[tok], 0), d);
  const int seg = seg_len(kk, d, bad);
  const int64_t o = off[tok];
  if (o + seg > capacity) {
    if (lane == 0) atomicOr(&hdr->err, kErrKvCapacity);
    return;
  }
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  for (int c = lane; c * EPC < seg; c += 64) {
    u32x4 v = *reinterpret_cast<const u32x4*>(xt + tok * d + c * EPC);
    if ((c + 1) * EPC > kk) {
      T e[EPC];
      __builtin_memcpy(e, &v, 16);
#pragma unroll
      for (int j = 0; j < EPC; ++j)
        if (c * EPC + j >= kk) e[j] = (T)0.0f;
      __builtin_memcpy(&v, e, 16);
    }
    *reinterpret_cast<u32x4*>(packed + o + c * EPC) = v;
  }
}

// ---- grouping by contraction length --------------------------------------------------------

__global__ __launch_bounds__(256) void kv_fill_i32_kernel(int32_t* __restrict__ p, int64_t count, int32_t v) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < count) p[i] = v;
}

__device__ inline int bucket_of(int k, int d, int esz) {
  k = min(max(k, 0), d);
  return (k * esz + 127) / 128;
}

__global__ __launch_bounds__(256) void kv_hist_kernel(const int32_t* __restrict__ k, int64_t n, int d, int esz,
                                                      int nbuckets, int32_t* __restrict__ hist) {
  extern __shared__ int32_t h[];
  for (int i = threadIdx.x; i < nbuckets; i += 256) h[i] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * 4096;
  for (int i = threadIdx.x; i < 4096; i += 256)
    if (base + i < n) atomicAdd(&h[bucket_of(k[base + i], d, esz)], 1);
  __syncthreads();
  for (int i = threadIdx.x; i < nbuckets; i += 256)
    if (h[i]) atomicAdd(&hist[i], h[i]);
}

// start[b] = number of tokens in longer buckets (descending order of step count)
__global__ void kv_bucket_start_kernel(int32_t* __restrict__ hist, int nbuckets) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int32_t run = 0;
  for (int b = nbuckets - 1; b >= 0; --b) {
    hist[nbuckets + b] = run;
    run += hist[b];
  }
}

// The position inside a bucket comes from integer atomics (a rank inside the workgroup's 4096 tokens
// from LDS, one global reservation per workgroup and bucket), so `order` may differ from run to run
// within a bucket; the reconstruction's results do not depend on it (a token's output only involves
// its own row, and extra K-steps of a tile add exact zeros).
// Besides the token, each sorted position gets the byte offset and byte length of the token's
// segment in the store (validated here against the readable extent), so that the reconstruction
// reads three contiguous arrays instead of chasing order -> off, k.
__global__ __launch_bounds__(256) void kv_scatter_kernel(const int32_t* __restrict__ k,
                                                         const int64_t* __restrict__ off, int64_t n, int d, int esz,
                                                         int64_t bytes, int nbuckets, int32_t* __restrict__ hist,
                                                         int32_t* __restrict__ order, uint32_t* __restrict__ pos_off,
                                                         int32_t* __restrict__ pos_len, WsHeader* hdr) {
  extern __shared__ int32_t h[];   // [nbuckets] counts, then [nbuckets] bases
  constexpr int PER = 16;          // tokens per thread
  for (int i = threadIdx.x; i < nbuckets; i += 256) h[i] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * (256 * PER);
  int bk[PER], rank[PER];
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int64_t i = base + j * 256 + threadIdx.x;
    bk[j] = -1;
    if (i < n) {
      bk[j] = bucket_of(k[i], d, esz);
      rank[j] = atomicAdd(&h[bk[j]], 1);
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < nbuckets; b += 256)
    h[nbuckets + b] = hist[nbuckets + b] + (h[b] ? atomicAdd(&hist[2 * nbuckets + b], h[b]) : 0);
  __syncthreads();
  int bad = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    if (bk[j] < 0) continue;
    const int64_t i = base + j * 256 + threadIdx.x;
    const int pos = h[nbuckets + bk[j]] + rank[j];
    const int64_t o = off[i];
    int dummy = 0;
    const int seg = seg_len(k[i], d, dummy);
    order[pos] = (int32_t)i;
    pos_len[pos] = seg * esz;
    if (o < 0 || (o & (DYNAKV_GRANULE - 1)) || (o + seg) * esz > bytes)
      bad = 1;                     // pos_off keeps its fill value: every load of the row is out of range -> zeros
    else
      pos_off[pos] = (uint32_t)(o * esz);
  }
  if (bad) atomicOr(&hdr->err, kErrKvCapacity);
}

// ---- retain rate ----------------------------------------------------------------------------

// red[2*b] = sum of k over the block's 256 tokens, red[2*b+1] = sum of m over their rows.
__global__ __launch_bounds__(256) void kv_retain_partial_kernel(const int32_t* __restrict__ k,
                                                                const float* __restrict__ m, int64_t n, int d,
                                                                double* __restrict__ red) {
  __shared__ double sk[4], sm[4];
  const int64_t t0 = (int64_t)blockIdx.x * 256;
  const int64_t tn = min((int64_t)256, n - t0);
  int ks = 0;
  if (k && threadIdx.x < tn) ks = min(max(k[t0 + threadIdx.x], 0), d);
  float ms = 0.f;
  if (m) {
    const int64_t cnt4 = tn * d / 4;
    const float4* p = reinterpret_cast<const float4*>(m + t0 * d);
    for (int64_t i = threadIdx.x; i < cnt4; i += 256) {
      const float4 v = p[i];
      ms += (v.x + v.y) + (v.z + v.w);
    }
  }
  ks = wave_sum_i(ks);
  ms = wave_sum(ms);
  if ((threadIdx.x & 63) == 0) {
    sk[threadIdx.x >> 6] = ks;
    sm[threadIdx.x >> 6] = ms;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    red[2 * blockIdx.x] = (sk[0] + sk[1]) + (sk[2] + sk[3]);
    red[2 * blockIdx.x + 1] = (sm[0] + sm[1]) + (sm[2] + sm[3]);
  }
}

__global__ __launch_bounds__(256) void kv_retain_final_kernel(const double* __restrict__ red, int nblocks,
                                                              int64_t n, int d, float alpha, int have_k,
                                                              int have_m, float* __restrict__ out) {
  __shared__ double sk[256], sm[256];
  double a = 0.0, b = 0.0;
  for (int i = threadIdx.x; i < nblocks; i += 256) {
    a += red[2 * i];
    b += red[2 * i + 1];
  }
  sk[threadIdx.x] = a;
  sm[threadIdx.x] = b;
  __syncthreads();
  for (unsigned o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) {
      sk[threadIdx.x] += sk[threadIdx.x + o];
      sm[threadIdx.x] += sm[threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double nd = (double)n * d;
    const double rh = have_k ? sk[0] / nd : 0.0;
    const double rs = have_m ? sm[0] / nd : 0.0;
    out[0] = (float)rh;
    out[1] = (float)rs;
    out[2] = (float)(alpha * rs * rs);
  }
}

__global__ __launch_bounds__(256) void kv_retain_grad_kernel(const float* __restrict__ out, float alpha,
                                                             int64_t count4, double nd, float* __restrict__ g) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count4) return;
  const float v = (float)(2.0 * alpha * (double)out[1] / nd);
  reinterpret_cast<float4*>(g)[i] = make_float4(v, v, v, v);
}

__global__ void kv_clear_header_kernel(WsHeader* hdr) {
  if (threadIdx.x == 0) {
    hdr->err = 0;
    hdr->nv = 0;
  }
}

}  // namespace

hipError_t launch_kv_clear_header(WsHeader* hdr, hipStream_t s) {
  hipLaunchKernelGGL(kv_clear_header_kernel, dim3(1), dim3(64), 0, s, hdr);
  return hipGetLastError();
}

template <typename T>
static void launch_mask_t(const float* logits, const float* b, const void* xt, int64_t n, int d, float tau,
                          bool literal, int32_t* k, float* m, void* xhat, hipStream_t s) {
  const dim3 grid((unsigned)((n + 3) / 4));
  const T* x = static_cast<const T*>(xt);
  T* xh = static_cast<T*>(xhat);
  const int lit = literal ? 1 : 0;
  const int ng = (d + 255) / 256;
#define KV_MASK(NG) hipLaunchKernelGGL((kv_mask_kernel<T, NG>), grid, dim3(256), 0, s, logits, b, x, n, d, tau, lit, k, m, xh)
  switch (ng) {
    case 1: KV_MASK(1); break;
    case 2: KV_MASK(2); break;
    case 3: KV_MASK(3); break;
    case 4: KV_MASK(4); break;
    case 5: case 6: KV_MASK(6); break;
    case 7: case 8: KV_MASK(8); break;
    default: KV_MASK(0); break;
  }
#undef KV_MASK
}

hipError_t launch_kv_mask(int dtype, const float* logits, const float* b, const void* xt, int64_t n, int d,
                          float tau, bool literal, int32_t* k, float* m, void* xhat, hipStream_t s) {
  if (dtype == LMHEAD_BF16)
    launch_mask_t<__bf16>(logits, b, xt, n, d, tau, literal, k, m, xhat, s);
  else
    launch_mask_t<float>(logits, b, xt, n, d, tau, literal, k, m, xhat, s);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_mask_bwd_t(const float* logits, const float* b, const void* xt, const void* g_xhat,
                                    const float* g_m, float g_m_const, int64_t n, int d, bool literal, void* gl,
                                    void* a_out, float* dbpart, int nblk, hipStream_t s) {
  const dim3 grid((unsigned)nblk);
  const size_t lds = (size_t)4 * d * sizeof(float);
  const T* x = static_cast<const T*>(xt);
  const T* gx = static_cast<const T*>(g_xhat);
  T* g1 = static_cast<T*>(gl);
  T* a1 = static_cast<T*>(a_out);
  const int lit = literal ? 1 : 0;
  const int ng = (d + 255) / 256;
#define KV_MASK_BWD(NG)                                                                                          \
  do {                                                                                                           \
    hipError_t e = allow_lds<kv_mask_bwd_kernel<T, NG>>((int)lds);                                               \
    if (e != hipSuccess) return e;                                                                               \
    hipLaunchKernelGGL((kv_mask_bwd_kernel<T, NG>), grid, dim3(256), lds, s, logits, b, x, gx, g_m, g_m_const, n, \
                       d, lit, g1, a1, dbpart);                                                                  \
  } while (0)
  switch (ng) {
    case 1: KV_MASK_BWD(1); break;
    case 2: KV_MASK_BWD(2); break;
    case 3: KV_MASK_BWD(3); break;
    case 4: KV_MASK_BWD(4); break;
    case 5: case 6: KV_MASK_BWD(6); break;
    case 7: case 8: KV_MASK_BWD(8); break;
    default: KV_MASK_BWD(0); break;
  }
#undef KV_MASK_BWD
  return hipGetLastError();
}

hipError_t launch_kv_mask_bwd(int dtype, const float* logits, const float* b, const void* xt, const void* g_xhat,
                              const float* g_m, float g_m_const, int64_t n, int d, bool literal, void* gl,
                              void* a_out, float* dbpart, int nblk, hipStream_t s) {
  if (dtype == LMHEAD_BF16)
    return launch_mask_bwd_t<__bf16>(logits, b, xt, g_xhat, g_m, g_m_const, n, d, literal, gl, a_out, dbpart, nblk, s);
  return launch_mask_bwd_t<float>(logits, b, xt, g_xhat, g_m, g_m_const, n, d, literal, gl, a_out, dbpart, nblk, s);
}

hipError_t launch_kv_sum_rows(const float* part, int rows, int64_t row_pitch, int64_t len, float* out,
                              bool accumulate, hipStream_t s) {
  hipLaunchKernelGGL(kv_sum_rows_kernel, dim3((unsigned)((len + 63) / 64)), dim3(256), 0, s, part, rows, row_pitch,
                     len, out, accumulate ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_kv_pad_copy(int dtype, const void* in, int64_t ld_in, int rows, int cols, void* out,
                              int64_t ld_out, int rows_p, hipStream_t s) {
  const int esz = dtype == LMHEAD_BF16 ? 2 : 4;
  const int64_t threads = (int64_t)rows_p * (ld_out * esz / 16);
  hipLaunchKernelGGL(kv_pad_copy_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                     static_cast<const char*>(in), ld_in * esz, rows, cols * esz, static_cast<char*>(out),
                     ld_out * esz, rows_p);
  return hipGetLastError();
}

hipError_t launch_kv_transpose(int dtype, const void* in, int64_t ld_in, int64_t rows, int cols, void* out,
                               int64_t ld_out, int64_t rows_p, int cols_p, hipStream_t s) {
  // rows 16-byte aligned and extents multiples of 64 here: takes the 16-byte-access kernel
  return launch_transpose(dtype, in, ld_in, rows, cols, false, nullptr, out, ld_out, rows_p, cols_p, s);
}

hipError_t launch_kv_store(int dtype, const void* xt, const int32_t* k, int64_t n, int d, int64_t off_base,
                           int64_t* off, void* packed, int64_t capacity, int64_t* blocksum, WsHeader* hdr,
                           hipStream_t s) {
  const int nblocks = (int)((n + kKvScanBlock - 1) / kKvScanBlock);
  hipLaunchKernelGGL(kv_scan_totals_kernel, dim3(nblocks), dim3(256), 0, s, k, n, d, blocksum, hdr);
  hipLaunchKernelGGL(kv_scan_blocks_kernel, dim3(1), dim3(1024), 0, s, blocksum, nblocks);
  hipLaunchKernelGGL(kv_scan_offsets_kernel, dim3(nblocks), dim3(1024), 0, s, k, n, d, blocksum, nblocks, off_base,
                     off);
  const dim3 grid((unsigned)((n + 3) / 4));
  if (dtype == LMHEAD_BF16)
    hipLaunchKernelGGL(kv_pack_kernel<__bf16>, grid, dim3(256), 0, s, static_cast<const __bf16*>(xt), k, off, n, d,
                       static_cast<__bf16*>(packed), capacity, hdr);
  else
    hipLaunchKernelGGL(kv_pack_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(xt), k, off, n, d,
                       static_cast<float*>(packed), capacity, hdr);
  return hipGetLastError();
}

hipError_t launch_kv_order(int dtype, const int32_t* k, const int64_t* off, int64_t bytes, int64_t n, int64_t ncap,
                           int d, int nbuckets, int32_t* hist, int32_t* order, uint32_t* pos_off, int32_t* pos_len,
                           WsHeader* hdr, hipStream_t s) {
  const int esz = dtype == LMHEAD_BF16 ? 2 : 4;
  const unsigned fill_blocks = (unsigned)((ncap + 255) / 256);
  hipLaunchKernelGGL(kv_fill_i32_kernel, dim3((unsigned)((3 * nbuckets + 255) / 256)), dim3(256), 0, s, hist,
                     (int64_t)3 * nbuckets, 0);
  hipLaunchKernelGGL(kv_fill_i32_kernel, dim3(fill_blocks), dim3(256), 0, s, order, ncap, -1);
  hipLaunchKernelGGL(kv_fill_i32_kernel, dim3(fill_blocks), dim3(256), 0, s, reinterpret_cast<int32_t*>(pos_off),
                     ncap, (int32_t)0x80000000u);
  hipLaunchKernelGGL(kv_fill_i32_kernel, dim3(fill_blocks), dim3(256), 0, s, pos_len, ncap, 0);
  hipLaunchKernelGGL(kv_hist_kernel, dim3((unsigned)((n + 4095) / 4096)), dim3(256), nbuckets * sizeof(int32_t), s,
                     k, n, d, esz, nbuckets, hist);
  hipLaunchKernelGGL(kv_bucket_start_kernel, dim3(1), dim3(64), 0, s, hist, nbuckets);
  hipLaunchKernelGGL(kv_scatter_kernel, dim3((unsigned)((n + 4095) / 4096)), dim3(256),
                     2 * nbuckets * sizeof(int32_t), s, k, off, n, d, esz, bytes, nbuckets, hist, order, pos_off,
                     pos_len, hdr);
  return hipGetLastError();
}

hipError_t launch_kv_retain(const int32_t* k, const float* m, int64_t n, int d, float alpha, float* out,
                            float* g_m, double* red, hipStream_t s) {
  const int nblocks = (int)((n + 255) / 256);
  hipLaunchKernelGGL(kv_retain_partial_kernel, dim3(nblocks), dim3(256), 0, s, k, m, n, d, red);
  hipLaunchKernelGGL(kv_retain_final_kernel, dim3(1), dim3(256), 0, s, red, nblocks, n, d, alpha, k ? 1 : 0,
                     m ? 1 : 0, out);
  if (g_m) {
    const int64_t count4 = n * d / 4;
    hipLaunchKernelGGL(kv_retain_grad_kernel, dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0, s, out, alpha,
                       count4, (double)n * d, g_m);
  }
  return hipGetLastError();
}

}  // namespace lmhead
