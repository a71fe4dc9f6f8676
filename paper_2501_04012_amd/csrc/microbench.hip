// Microbenchmarks of the matrix pipe and the vector pipe of a compute unit, as the
// attention and GEMM kernels of a step load them: independent v_mfma_f32_32x32x16_bf16
// chains, v_exp_f32 streams, and the two together (in one wave, or in different waves of a
// workgroup).  They give the rates the step's kernels are to be read against on the part at
// hand (sustained clock under matrix load included) and are not part of a step.
#include "common.h"

namespace fc {

// mode bits: 1 = this wave issues MFMAs, 2 = this wave issues exponentials.
// split != 0: waves 0..3 of the workgroup take `mode_a`, waves 4..7 take `mode_b`.
// clocks[2 * wave_global] = shader-clock cycles of the loop, [2 * wave_global + 1] = the same
// interval on the constant-rate counter (100 MHz): their ratio is the shader clock.
template <int EXP_PER_MFMA>
__global__ __launch_bounds__(512, 1) void k_pipe_rates(const bf16_t* __restrict__ operands, int iters, int mode_a,
                                                       int mode_b, float* __restrict__ sink,
                                                       long long* __restrict__ clocks) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int mode = wave < 4 ? mode_a : mode_b;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    a[j] = *(const bf16x8*)(operands + ((size_t)(2 * j) * 64 + lane) * 8);
    b[j] = *(const bf16x8*)(operands + ((size_t)(2 * j + 1) * 64 + lane) * 8);
  }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
  float e[4 * EXP_PER_MFMA];
#pragma unroll
  for (int i = 0; i < 4 * EXP_PER_MFMA; ++i) e[i] = 0.01f * (float)(lane + i);

  const long long c0 = clock64(), w0 = wall_clock64();
  if (mode == 1) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], acc[j], 0, 0, 0);
    }
  } else if (mode == 2) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 4 * EXP_PER_MFMA; ++i) e[i] = __builtin_amdgcn_exp2f(-e[i]);
    }
  } else if (mode == 3) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], acc[j], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < EXP_PER_MFMA; ++i) e[j * EXP_PER_MFMA + i] = __builtin_amdgcn_exp2f(-e[j * EXP_PER_MFMA + i]);
      }
    }
  }
  const long long c1 = clock64(), w1 = wall_clock64();

  float s = 0.0f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
#pragma unroll
  for (int i = 0; i < 4 * EXP_PER_MFMA; ++i) s += e[i];
  const size_t wg = (size_t)blockIdx.x * 8 + wave;
  sink[wg * 64 + lane] = s;
  if (lane == 0) { clocks[2 * wg] = c1 - c0; clocks[2 * wg + 1] = w1 - w0; }
}

// operands: 8 x 64 x 8 bf16 (8 KB); sink: blocks * 512 floats; clocks: blocks * 8 * 2 int64.
hipError_t launch_pipe_rates(const void* operands, int iters, int mode_a, int mode_b, int blocks, float* sink,
                             long long* clocks, hipStream_t s) {
  if (blocks <= 0 || iters <= 0) return hipSuccess;
  k_pipe_rates<2><<<blocks, 512, 0, s>>>((const bf16_t*)operands, iters, mode_a, mode_b, sink, clocks);
  return hipGetLastError();
}

}  // namespace fc
