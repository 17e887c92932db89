// Measurement aid: a loop of v_mfma_f32_32x32x16_bf16 on register operands, one workgroup of
// four waves per launch slot, nothing else.  Timing it on all CUs gives the MFMA rate this
// machine sustains under its power limit -- the yardstick the attention kernels' TFLOP/s are
// compared with besides the published peak.  With random operands every mantissa bit toggles,
// which costs more power (a lower clock) than small-integer operands.
#include "winattn_common.hpp"
#include "winattn_launch.hpp"

namespace aeris {

__global__ __launch_bounds__(kThreads) void mfma_loop_kernel(float* __restrict__ sink, int iters,
                                                             int random_operands) {
  f32x16 acc[4];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[m][i] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    unsigned h = (threadIdx.x * 8 + i + blockIdx.x * 2048) * 2654435761u;
    h ^= h >> 15;
    h *= 2246822519u;
    h ^= h >> 13;
    const float ra = (h & 0xffff) / 32768.0f - 1.0f, rb = (h >> 16) / 32768.0f - 1.0f;
    a[i] = random_operands ? (bf16_t)ra : (bf16_t)(float)((int)((threadIdx.x * 7 + i) % 5) - 2);
    b[i] = random_operands ? (bf16_t)rb : (bf16_t)(0.25f * ((threadIdx.x + i) % 7));
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 8; ++m) acc[m % 4] = mfma32(a, b, acc[m % 4]);
  }
  float s = 0.f;
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[m][i];
  sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

int launch_mfma_loop(int blocks, int iters, bool random_operands, float* sink, hipStream_t stream) {
  return launch_kernel(mfma_loop_kernel, dim3(blocks), dim3(kThreads), 0, stream, sink, iters,
                       random_operands ? 1 : 0);
}

}  // namespace aeris
