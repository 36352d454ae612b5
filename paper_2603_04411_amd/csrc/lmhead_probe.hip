// Measurement aid, not part of the hot path: a bare loop of the matrix-core instruction that the bf16
// contractions are built on (v_mfma_f32_16x16x32_bf16), fed from registers that are loaded once.  It moves
// no data during the loop, so its rate is what the matrix cores of the part sustain under its power
// management for a given operand content: the practical ceiling that the fused kernels are compared with
// next to the nominal 2.5 PFLOP/s.
#include "common.h"
#include "gemm_core.h"

namespace lmhead {

namespace {

// One wavefront = a 128 x 128 output tile (8 x 8 blocks of 16 x 16), as in the contractions; one
// iteration = 64 MFMAs = 2^20 flop per wavefront.  The sums keep the loop from being optimised away.
__global__ __launch_bounds__(256) void mfma_probe_kernel(const u32x4_t* __restrict__ operands,
                                                         float* __restrict__ sink, int iters) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  u32x4_t fa[8], fb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    fa[i] = operands[t * 16 + i];
    fb[i] = operands[t * 16 + 8 + i];
  }
  f32x4_t acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, fa[i]),
                                                            __builtin_bit_cast(bf16x8_t, fb[j]), acc[i][j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[i][j].x + acc[i][j].y + acc[i][j].z + acc[i][j].w;
  sink[t] = s;
}

}  // namespace

hipError_t launch_mfma_probe(const void* operands, float* sink, int workgroups, int iters, hipStream_t s) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(256), 0, s, static_cast<const u32x4_t*>(operands),
                     sink, iters);
  return hipGetLastError();
}

}  // namespace lmhead
