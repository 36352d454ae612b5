// Bandwidth-bound helper kernels around the MFMA kernels: batch indexing (mask, prefix
// sums, compaction map), row gather of H, operand transposes, 8-bit operand copies, the merge of
// the per-tile softmax statistics, the sum of split dH contractions, and zero-filling of padded dH rows.  All accesses are coalesced
// (16-byte vectors where rows allow); none of these kernels is more than a few passes
// over O(N d + V d) bytes.
#include <math.h>

#include <atomic>

#include "common.h"

namespace lmhead {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ---- indexing --------------------------------------------------------------------------

// One workgroup: exclusive prefix sum of the (clamped) lengths.
__global__ __launch_bounds__(1024) void scan_len_kernel(const int32_t* __restrict__ len, int R, int T,
                                                        WsHeader* hdr, int32_t* __restrict__ cu_ws,
                                                        int32_t* __restrict__ cu_out) {
  __shared__ int32_t wsum[16];
  __shared__ int32_t carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) {
    carry_s = 0;
    hdr->err = 0;  // this kernel is the first of every call: reset the sticky word here
  }
  int bad = 0;
  __syncthreads();
  for (int base = 0; base < R; base += 1024) {
    const int r = base + tid;
    int x = 0;
    if (r < R) {
      x = len[r];
      if (x < 0 || x > T) {
        bad = 1;
        x = x < 0 ? 0 : T;
      }
    }
    int incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(incl, o);
      if (lane >= o) incl += y;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int woff = 0;
    for (int w = 0; w < wave; ++w) woff += wsum[w];
    const int carry = carry_s;
    const int excl = carry + woff + incl - x;
    if (r < R) {
      cu_ws[r] = excl;
      if (cu_out) cu_out[r] = excl;
    }
    __syncthreads();
    if (tid == 1023) carry_s = excl + x;
    __syncthreads();
  }
  if (bad) atomicOr(&hdr->err, kErrLen);
  if (tid == 0) {
    const int total = carry_s;
    cu_ws[R] = total;
    if (cu_out) cu_out[R] = total;
    hdr->nv = total;
  }
}

// One thread per slot (plus one tile of tail threads that pad row_slot with -1).
__global__ __launch_bounds__(256) void fill_index_kernel(const int32_t* __restrict__ len, int R, int T,
                                                         const int32_t* __restrict__ cu,
                                                         int32_t* __restrict__ row_slot,
                                                         uint8_t* __restrict__ mask) {
  const int64_t N = (int64_t)R * T;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < N) {
    const int r = (int)(i / T);
    const int t = (int)(i - (int64_t)r * T);
    const int n = min(max(len[r], 0), T);
    const bool valid = t < n;
    if (mask) mask[i] = valid ? 1 : 0;
    if (valid) row_slot[cu[r] + t] = (int32_t)i;
  } else {
    const int64_t nv = cu[R];
    const int64_t k = nv + (i - N);
    const int64_t cap = (N + kTile - 1) / kTile * kTile;
    if (i - N < kTile && k < cap) row_slot[k] = -1;
  }
}

// ---- gather of valid rows ------------------------------------------------------------

// One wavefront per compact row k: copies H[row_slot[k], :] (16 bytes per lane per step) or
// zero-fills the rows between N_v and the next tile multiple.
__global__ __launch_bounds__(256) void compact_kernel(const char* __restrict__ H, int64_t pitchH,
                                                      int row_bytes, int64_t pitchHc, int V,
                                                      const int32_t* __restrict__ tok,
                                                      const float* __restrict__ g,
                                                      const float* __restrict__ lse, WsHeader* hdr,
                                                      const int32_t* __restrict__ row_slot,
                                                      char* __restrict__ Hc, int32_t* __restrict__ tok_c,
                                                      float* __restrict__ g_c, float* __restrict__ lse_c,
                                                      float* __restrict__ zy, int32_t* __restrict__ gid,
                                                      int npol, int64_t Ncap) {
  const int nv = hdr->nv;
  const int64_t nvp = ((int64_t)nv + kTile - 1) / kTile * kTile;
  const int64_t k = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (k >= nvp) return;
  const int lane = threadIdx.x & 63;
  typedef __attribute__((ext_vector_type(4))) uint32_t u4;
  u4* dst = reinterpret_cast<u4*>(Hc + k * pitchHc);
  const int nvec = row_bytes / 16;
  if (k < nv) {
    const int64_t slot = row_slot[k];
    const u4* src = reinterpret_cast<const u4*>(H + slot * pitchH);
    for (int c = lane; c < nvec; c += 64) dst[c] = src[c];
    if (lane == 0) {
      int tk = tok[slot];
      if (tk < 0 || tk >= V) {
        atomicOr(&hdr->err, kErrTok);
        tk = -1;
      }
      tok_c[k] = tk;
      if (g_c) g_c[k] = g[slot];
      if (lse_c) lse_c[k] = lse[slot];
      for (int p = 0; p < npol; ++p) {
        zy[p * Ncap + k] = 0.f;
        gid[p * Ncap + k] = -1;
      }
    }
  } else {
    const u4 z = {0, 0, 0, 0};
    for (int c = lane; c < nvec; c += 64) dst[c] = z;
    if (lane == 0) {
      tok_c[k] = -1;
      if (g_c) g_c[k] = 0.f;
      if (lse_c) lse_c[k] = 0.f;
      for (int p = 0; p < npol; ++p) {
        zy[p * Ncap + k] = 0.f;
        gid[p * Ncap + k] = -1;
      }
    }
  }
}

// ---- transpose -------------------------------------------------------------------------

// out[c][r] = in[r][c] through a 64x64 LDS tile; rows >= `rows` and columns >= `cols` of the
// source read as zero, so the padded extent of `out` is zero-filled.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, int64_t ld_in,
                                                        int64_t rows_fixed, int cols, int rows_from_nv,
                                                        const WsHeader* __restrict__ hdr,
                                                        T* __restrict__ out, int64_t ld_out,
                                                        int64_t rows_p, int64_t cols_p) {
  __shared__ T tile[64][65];
  const int64_t rows = rows_from_nv ? (int64_t)hdr->nv : rows_fixed;
  const int64_t r0 = (int64_t)blockIdx.x * 64;
  const int64_t c0 = (int64_t)blockIdx.y * 64;
  if (rows_from_nv) {
    // nothing beyond the tile-padded valid extent is ever read by the contractions
    const int64_t rp = (rows + kTile - 1) / kTile * kTile;
    if (r0 >= rp) return;
  }
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int rr = ty; rr < 64; rr += 4) {
    const int64_t r = r0 + rr, c = c0 + tx;
    tile[rr][tx] = (r < rows && c < cols) ? in[r * ld_in + c] : T(0);
  }
  __syncthreads();
  for (int cc = ty; cc < 64; cc += 4) {
    const int64_t c = c0 + cc, r = r0 + tx;
    if (c < cols_p && r < rows_p) out[c * ld_out + r] = tile[tx][cc];
  }
}

// The same transposition for the common case of 16-byte aligned rows on both sides and extents that are
// multiples of 64: 64 x 64 tiles with 16-byte global accesses on both sides (the element-wise kernel above
// moves 2 or 4 bytes per lane and runs at about half the rate).  Rows of the source go to LDS as they are
// (padded pitch); each thread then gathers the 16 bytes of one output chunk (consecutive r of one column).
template <typename T>
__global__ __launch_bounds__(256) void transpose16_kernel(const T* __restrict__ in, int64_t ld_in, int64_t rows_fixed,
                                                          int cols, int rows_from_nv, const WsHeader* __restrict__ hdr,
                                                          T* __restrict__ out, int64_t ld_out) {
  constexpr int VEC = 16 / sizeof(T);         // elements per 16-byte chunk
  constexpr int CPR = 64 / VEC;               // chunks per tile row
  constexpr int PITCH = 64 + 4 / sizeof(T);   // elements; keeps rows 4-byte aligned and the gather conflict-free
  __shared__ __attribute__((aligned(16))) T tile[64 * PITCH];
  const int64_t rows = rows_from_nv ? (int64_t)hdr->nv : rows_fixed;
  const int64_t r0 = (int64_t)blockIdx.x * 64;
  const int c0 = blockIdx.y * 64;
  // nothing beyond the tile-padded valid extent is ever read by the contractions
  if (rows_from_nv && r0 >= (rows + kTile - 1) / kTile * kTile) return;
#pragma unroll
  for (int pass = 0; pass < 64 * CPR / 256; ++pass) {
    const int id = pass * 256 + threadIdx.x;
    const int rr = id / CPR, cc = id % CPR;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r0 + rr < rows && c0 < cols) v = *reinterpret_cast<const uint4*>(in + (r0 + rr) * ld_in + c0 + cc * VEC);
    uint32_t* dst = reinterpret_cast<uint32_t*>(tile + rr * PITCH + cc * VEC);
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 64 * CPR / 256; ++pass) {
    const int id = pass * 256 + threadIdx.x;
    const int c = id / CPR, rc = id % CPR;
    T e[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) e[i] = tile[(rc * VEC + i) * PITCH + c];
    uint4 v;
    if constexpr (sizeof(T) == 2) {
      v.x = (uint32_t)e[0] | ((uint32_t)e[1] << 16);
      v.y = (uint32_t)e[2] | ((uint32_t)e[3] << 16);
      v.z = (uint32_t)e[4] | ((uint32_t)e[5] << 16);
      v.w = (uint32_t)e[6] | ((uint32_t)e[7] << 16);
    } else {
      v = make_uint4(e[0], e[1], e[2], e[3]);
    }
    *reinterpret_cast<uint4*>(out + (int64_t)(c0 + c) * ld_out + r0 + rc * VEC) = v;
  }
}

// ---- 8-bit operand copies ---------------------------------------------------------------

// One wavefront per row: out = e4m3(in * scale), eight values per lane and pass.  The hardware
// conversion rounds to nearest even but turns magnitudes beyond the format's range into NaN, so
// values are clamped to +-448 (the largest e4m3 number) first.
template <typename T>
__global__ __launch_bounds__(256) void quantize_e4m3_kernel(const T* __restrict__ in, int64_t ld_in,
                                                            int64_t rows_fixed, int rows_from_nv,
                                                            const WsHeader* __restrict__ hdr, int cols,
                                                            float scale, uint8_t* __restrict__ out,
                                                            int64_t ld_out, int64_t rows_p) {
  const int64_t rows = rows_from_nv ? (int64_t)hdr->nv : rows_fixed;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows_p) return;
  if (rows_from_nv && r >= (rows + kTile - 1) / kTile * kTile) return;
  const int lane = threadIdx.x & 63;
  for (int c = lane * 8; c < cols; c += 512) {
    uint2 packed = make_uint2(0u, 0u);
    if (r < rows) {
      float v[8];
      if constexpr (sizeof(T) == 2) {
        typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
        const bf16x8 t = *reinterpret_cast<const bf16x8*>(in + r * ld_in + c);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (float)t[e];
      } else {
        const float4 t0 = *reinterpret_cast<const float4*>(in + r * ld_in + c);
        const float4 t1 = *reinterpret_cast<const float4*>(in + r * ld_in + c + 4);
        v[0] = t0.x; v[1] = t0.y; v[2] = t0.z; v[3] = t0.w;
        v[4] = t1.x; v[5] = t1.y; v[6] = t1.z; v[7] = t1.w;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = fminf(fmaxf(v[e] * scale, -448.f), 448.f);
      int lo = 0, hi = 0;
      lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], lo, false);
      lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], lo, true);
      hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[4], v[5], hi, false);
      hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[6], v[7], hi, true);
      packed = make_uint2((unsigned)lo, (unsigned)hi);
    }
    *reinterpret_cast<uint2*>(out + r * ld_out + c) = packed;
  }
}

// ---- merge of per-chunk softmax statistics -------------------------------------------

__global__ __launch_bounds__(256) void finalize_kernel(const float* __restrict__ part,
                                                       const float* __restrict__ zy, int nchunks,
                                                       int64_t Ncap, const int32_t* __restrict__ len,
                                                       const int32_t* __restrict__ cu, int R, int T,
                                                       float* __restrict__ logp, float* __restrict__ lse,
                                                       float* __restrict__ ent) {
  const int64_t N = (int64_t)R * T;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= N) return;
  const int r = (int)(i / T);
  const int t = (int)(i - (int64_t)r * T);
  const int n = min(max(len[r], 0), T);
  float o_lp = 0.f, o_lse = 0.f, o_ent = 0.f;
  if (t < n) {
    const int64_t k = cu[r] + t;
    const size_t plane = (size_t)nchunks * Ncap;
    float m = -__builtin_huge_valf();
    for (int c = 0; c < nchunks; ++c) m = fmaxf(m, part[(size_t)c * Ncap + k]);
    float s = 0.f, tt = 0.f;
    for (int c = 0; c < nchunks; ++c) {
      const size_t idx = (size_t)c * Ncap + k;
      const float mc = part[idx];
      if (mc == -__builtin_huge_valf()) continue;
      const float w = __builtin_amdgcn_exp2f((mc - m) * kLog2e);
      s = fmaf(part[plane + idx], w, s);
      if (ent) tt = fmaf(part[2 * plane + idx], w, tt);
    }
    o_lse = m + __builtin_amdgcn_logf(s) * kLn2;
    o_lp = zy[k] - o_lse;
    o_ent = o_lse - tt / s;
  }
  logp[i] = o_lp;
  if (lse) lse[i] = o_lse;
  if (ent) ent[i] = o_ent;
}

// ---- sum of split contractions -----------------------------------------------------------

// One wavefront per valid row n: out[rowmap(n)][:] (+)= part[0][n][:] + part[1][n][:] + ... (in this order).
template <typename TO>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, int ksplit,
                                                            int64_t part_slice, int64_t part_ld, int M,
                                                            const int32_t* __restrict__ rowmap,
                                                            const WsHeader* __restrict__ hdr, int64_t n_cap,
                                                            int64_t row_base, TO* __restrict__ out, int64_t ldo,
                                                            int accumulate) {
  const int64_t n = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= (rowmap ? (int64_t)hdr->nv : n_cap)) return;
  const int64_t row = rowmap ? (int64_t)rowmap[n] : row_base + n;
  if (row < 0) return;
  const int lane = threadIdx.x & 63;
  for (int m = lane * 4; m < M; m += 256) {
    float4 v = *reinterpret_cast<const float4*>(part + n * part_ld + m);
    for (int s = 1; s < ksplit; ++s) {
      const float4 p = *reinterpret_cast<const float4*>(part + (size_t)s * part_slice + n * part_ld + m);
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    if constexpr (sizeof(TO) == 4) {
      float4* dst = reinterpret_cast<float4*>(out + row * ldo + m);
      if (accumulate) {
        const float4 o = *dst;
        v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
      }
      *dst = v;
    } else {
      typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
      const bf16x4_t h = {(__bf16)v.x, (__bf16)v.y, (__bf16)v.z, (__bf16)v.w};
      *reinterpret_cast<bf16x4_t*>(out + row * ldo + m) = h;
    }
  }
}

// ---- padded rows of dH -------------------------------------------------------------------

// One wavefront per slot; only padded slots write.
template <typename TO>
__global__ __launch_bounds__(256) void zero_rows_kernel(TO* __restrict__ dH, int d,
                                                        const int32_t* __restrict__ len, int R, int T) {
  const int64_t N = (int64_t)R * T;
  const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= N) return;
  const int r = (int)(i / T);
  const int t = (int)(i - (int64_t)r * T);
  if (t < min(max(len[r], 0), T)) return;
  typedef __attribute__((ext_vector_type(4))) float f4;    // 16 bytes of zeros, whatever the element type
  f4* row = reinterpret_cast<f4*>(dH + i * (int64_t)d);
  const f4 z = {0.f, 0.f, 0.f, 0.f};
  for (int c = threadIdx.x & 63; c < d * (int)sizeof(TO) / 16; c += 64) row[c] = z;
}

}  // namespace

hipError_t launch_index(const int32_t* len, int R, int T, WsHeader* hdr, int32_t* cu_ws,
                        int32_t* row_slot, uint8_t* mask_out, int32_t* cu_out, hipStream_t s) {
  hipLaunchKernelGGL(scan_len_kernel, dim3(1), dim3(1024), 0, s, len, R, T, hdr, cu_ws, cu_out);
  const int64_t N = (int64_t)R * T;
  const unsigned blocks = (unsigned)((N + kTile + 255) / 256);
  hipLaunchKernelGGL(fill_index_kernel, dim3(blocks), dim3(256), 0, s, len, R, T, cu_ws, row_slot, mask_out);
  return hipGetLastError();
}

hipError_t launch_compact(int dtype, const void* H, int64_t ldH, int d, int V, const int32_t* tok,
                          const float* g, const float* lse, int64_t N, WsHeader* hdr,
                          const int32_t* row_slot, void* Hc, int64_t ldHc, int32_t* tok_c, float* g_c,
                          float* lse_c, float* zy, int32_t* gid, int npol, int64_t Ncap, hipStream_t s) {
  const int esz = dtype == LMHEAD_BF16 ? 2 : 4;
  const int64_t cap = (N + kTile - 1) / kTile * kTile;
  hipLaunchKernelGGL(compact_kernel, dim3((unsigned)(cap / 4)), dim3(256), 0, s,
                     static_cast<const char*>(H), ldH * esz, d * esz, ldHc * esz, V, tok, g, lse, hdr, row_slot,
                     static_cast<char*>(Hc), tok_c, g ? g_c : nullptr, lse ? lse_c : nullptr, zy, gid, npol, Ncap);
  return hipGetLastError();
}

hipError_t launch_transpose(int dtype, const void* in, int64_t ld_in, int64_t rows_cap, int cols,
                            bool rows_from_nv, const WsHeader* hdr, void* out, int64_t ld_out,
                            int64_t rows_p, int64_t cols_p, hipStream_t s) {
  const dim3 grid((unsigned)((rows_p + 63) / 64), (unsigned)((cols_p + 63) / 64));
  const int esz = dtype == LMHEAD_BF16 ? 2 : 4;
  const bool wide = cols % 64 == 0 && cols_p % 64 == 0 && rows_p % 64 == 0 && (ld_in * esz) % 16 == 0 &&
                    (ld_out * esz) % 16 == 0 && (reinterpret_cast<uintptr_t>(in) & 15u) == 0 &&
                    (reinterpret_cast<uintptr_t>(out) & 15u) == 0;
  if (wide) {
    if (dtype == LMHEAD_BF16)
      hipLaunchKernelGGL(transpose16_kernel<uint16_t>, grid, dim3(256), 0, s, static_cast<const uint16_t*>(in), ld_in,
                         rows_cap, cols, rows_from_nv ? 1 : 0, hdr, static_cast<uint16_t*>(out), ld_out);
    else
      hipLaunchKernelGGL(transpose16_kernel<uint32_t>, grid, dim3(256), 0, s, static_cast<const uint32_t*>(in), ld_in,
                         rows_cap, cols, rows_from_nv ? 1 : 0, hdr, static_cast<uint32_t*>(out), ld_out);
    return hipGetLastError();
  }
  if (dtype == LMHEAD_BF16) {
    hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, s,
                       static_cast<const uint16_t*>(in), ld_in, rows_cap, cols, rows_from_nv ? 1 : 0,
                       hdr, static_cast<uint16_t*>(out), ld_out, rows_p, cols_p);
  } else {
    hipLaunchKernelGGL(transpose_kernel<uint32_t>, grid, dim3(256), 0, s,
                       static_cast<const uint32_t*>(in), ld_in, rows_cap, cols, rows_from_nv ? 1 : 0,
                       hdr, static_cast<uint32_t*>(out), ld_out, rows_p, cols_p);
  }
  return hipGetLastError();
}

hipError_t launch_quantize_e4m3(int dtype, const void* in, int64_t ld_in, int64_t rows_fixed, bool rows_from_nv,
                                const WsHeader* hdr, int cols, int exp2, void* out, int64_t ld_out, int64_t rows_p,
                                hipStream_t s) {
  const dim3 grid((unsigned)((rows_p + 3) / 4));
  const float scale = ldexpf(1.0f, exp2);
  if (dtype == LMHEAD_BF16)
    hipLaunchKernelGGL(quantize_e4m3_kernel<__bf16>, grid, dim3(256), 0, s, static_cast<const __bf16*>(in), ld_in,
                       rows_fixed, rows_from_nv ? 1 : 0, hdr, cols, scale, static_cast<uint8_t*>(out), ld_out, rows_p);
  else
    hipLaunchKernelGGL(quantize_e4m3_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(in), ld_in,
                       rows_fixed, rows_from_nv ? 1 : 0, hdr, cols, scale, static_cast<uint8_t*>(out), ld_out, rows_p);
  return hipGetLastError();
}

hipError_t launch_splitk_reduce(const float* part, int ksplit, int64_t part_slice, int64_t part_ld, int M,
                                const int32_t* rowmap, const WsHeader* hdr, int64_t n_cap, void* out, int64_t ldo,
                                bool accumulate, bool out_bf16, hipStream_t s, int64_t row_base) {
  const dim3 grid((unsigned)((n_cap + 3) / 4));
  if (out_bf16)
    hipLaunchKernelGGL(splitk_reduce_kernel<__bf16>, grid, dim3(256), 0, s, part, ksplit, part_slice, part_ld, M,
                       rowmap, hdr, n_cap, row_base, static_cast<__bf16*>(out), ldo, 0);
  else
    hipLaunchKernelGGL(splitk_reduce_kernel<float>, grid, dim3(256), 0, s, part, ksplit, part_slice, part_ld, M,
                       rowmap, hdr, n_cap, row_base, static_cast<float*>(out), ldo, accumulate ? 1 : 0);
  return hipGetLastError();
}

int device_compute_units() {
  constexpr int kMaxDev = 64;
  static std::atomic<int> cus[kMaxDev];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return 256;
  int n = cus[dev].load(std::memory_order_acquire);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cus[dev].store(n, std::memory_order_release);
  }
  return n;
}

hipError_t launch_finalize(const float* part, const float* zy, int nchunks, int64_t Ncap,
                           const int32_t* len, const int32_t* cu_len, int R, int T, float* logp,
                           float* lse, float* entropy, hipStream_t s) {
  const int64_t N = (int64_t)R * T;
  hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, part, zy,
                     nchunks, Ncap, len, cu_len, R, T, logp, lse, entropy);
  return hipGetLastError();
}

hipError_t launch_zero_padded_rows(void* dH, bool bf16, int d, const int32_t* len, int R, int T, hipStream_t s) {
  const int64_t N = (int64_t)R * T;
  const dim3 grid((unsigned)((N + 3) / 4));
  if (bf16)
    hipLaunchKernelGGL(zero_rows_kernel<__bf16>, grid, dim3(256), 0, s, static_cast<__bf16*>(dH), d, len, R, T);
  else
    hipLaunchKernelGGL(zero_rows_kernel<float>, grid, dim3(256), 0, s, static_cast<float*>(dH), d, len, R, T);
  return hipGetLastError();
}

}  // namespace lmhead
