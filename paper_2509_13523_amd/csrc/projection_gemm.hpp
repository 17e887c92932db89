// The bf16 GEMM of the projections, y = x W^T with both operands contiguous along the
// contraction (norm_linear.hip), as the other source files of the library launch it.
#pragma once
#include <hip/hip_runtime.h>

#include "winattn_common.hpp"

namespace aeris {

struct GemmParams {
  const bf16_t* x;             // [n_rows, K]
  const bf16_t* w;             // [F, K], or per sample [n_samples][F, K]
  long long w_sample_stride;   // elements between the samples' matrices (0: one for all)
  const float* r;              // [n_rows] row scale, or null
  const float* bias;           // [n_samples][F], or null
  bf16_t* y;                   // [n_rows, F]: the projection (plain), or uv (SwiGLU, may be null)
  bf16_t* g;                   // SwiGLU: [n_rows, F / 2]
  long long rows_per_sample;
  int m_tiles_per_sample;      // filled in by the launch
  int m_tiles;                 // n_samples * tiles per sample
  int n_tiles;
  int K, F;
  int swiglu;
};

// Shape limits of the kernel itself (K % 64, F % 8, 32-bit offsets inside a tile, grid size):
// 0 if (n_rows, rows_per_sample, K, F) can be launched, else an AERIS_ERR_ code.
int projection_gemm_check(long long n_rows, long long rows_per_sample, int K, int F);
// 0 on success, -1 if the launch failed.
int launch_projection_gemm(GemmParams p, hipStream_t stream);

}  // namespace aeris
