// Element-wise operations around the window attention of an AERIS transformer layer
// (paper, Model Architecture section: pre-RMSNorm, adaptive-layer-norm values alpha, beta,
// gamma, SwiGLU); formulas and argument contracts in include/aeris_layer_ops.h.
//
// All of them are bound by HBM traffic: every activation is read once and every result written
// once, 16 bytes per lane and access (non-temporal: nothing is reused), with fp32 arithmetic in
// between.  Row operations give a
// wavefront one token row at a time (lane l holds the 8-channel vectors l, l + 64, ...), so the
// row statistics need one cross-lane reduction and no barrier.  A workgroup works on a
// contiguous chunk of the rows of ONE sample, so the sample's modulation vectors are loaded
// once per workgroup (into LDS, or registers for the gate), and the sums over tokens
// (d gamma, d beta, d alpha, d w) are accumulated per lane in registers, combined over the four
// waves through LDS in a fixed order, written as one partial row per workgroup and summed by a
// small second kernel: no atomics, bitwise reproducible.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "aeris_layer_ops.h"
#include "aeris_winattn.h"
#include "winattn_common.hpp"
#include "winattn_launch.hpp"

namespace aeris {
namespace {

constexpr int kRowThreads = 256;
constexpr int kRowWaves = 4;
constexpr int kTargetChunks = 2048;   // workgroups per launch: eight per CU

// Workgroups (row chunks) per sample: about kTargetChunks in total, at least 4 rows each.
inline int chunks_per_sample(int64_t n_rows, int64_t rows_per_sample) {
  const int64_t n_samples = n_rows / rows_per_sample;
  int64_t cps = (kTargetChunks + n_samples - 1) / n_samples;
  const int64_t most = (rows_per_sample + kRowWaves - 1) / kRowWaves;
  if (cps > most) cps = most;
  if (cps < 1) cps = 1;
  return static_cast<int>(cps);
}

struct RowWork {
  int64_t rows_per_sample;
  int cps;      // chunks per sample
  int C;        // channels
};

// Rows [r0, r1) of this workgroup and its sample.
__device__ __forceinline__ void chunk_rows(const RowWork& rw, int64_t& r0, int64_t& r1, int& smp) {
  smp = blockIdx.x / rw.cps;
  const int k = blockIdx.x - smp * rw.cps;
  const int64_t base = static_cast<int64_t>(smp) * rw.rows_per_sample;
  r0 = base + rw.rows_per_sample * k / rw.cps;
  r1 = base + rw.rows_per_sample * (k + 1) / rw.cps;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

__device__ __forceinline__ void unpack8(const u32x4& raw, float (&f)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(raw[i] << 16);
    f[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ u32x4 pack8(const float (&f)[8]) {
  u32x4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = pack_bf16(f[2 * i], f[2 * i + 1]);
  return r;
}

// ---------------------------------------------------------------------------------------
// RMSNorm with adaptive modulation, forward.  K = vectors of 8 channels per lane.
// LDS: s[C] = w (1 + gamma_b), beta_b[C].
// ---------------------------------------------------------------------------------------
template <int K>
__global__ __launch_bounds__(kRowThreads) void rmsnorm_adaln_fwd_kernel(
    RowWork rw, const bf16_t* __restrict__ x, const float* __restrict__ w,
    const float* __restrict__ gamma, const float* __restrict__ beta, float eps,
    bf16_t* __restrict__ h, float* __restrict__ rstd) {
  extern __shared__ __align__(16) float lds_f[];
  float* s_lds = lds_f;
  float* b_lds = lds_f + rw.C;
  int64_t r0, r1;
  int smp;
  chunk_rows(rw, r0, r1, smp);
  const int C = rw.C;
  for (int c = threadIdx.x; c < C; c += kRowThreads) {
    s_lds[c] = w[c] * (1.f + gamma[(int64_t)smp * C + c]);
    b_lds[c] = beta[(int64_t)smp * C + c];
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float inv_c = 1.f / (float)C;
  for (int64_t row = r0 + wave; row < r1; row += kRowWaves) {
    const u32x4* src = reinterpret_cast<const u32x4*>(x + row * C);
    u32x4 raw[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int v = k * 64 + lane;
      raw[k] = (v * 8 < C) ? __builtin_nontemporal_load(&src[v]) : u32x4{0, 0, 0, 0};
    }
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      float f[8];
      unpack8(raw[k], f);
#pragma unroll
      for (int i = 0; i < 8; ++i) ss = __builtin_fmaf(f[i], f[i], ss);
    }
    ss = wave_sum(ss);
    const float r = 1.f / __builtin_sqrtf(ss * inv_c + eps);
    if (rstd != nullptr && lane == 0) rstd[row] = r;
    u32x4* dst = reinterpret_cast<u32x4*>(h + row * C);
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int v = k * 64 + lane;
      if (v * 8 < C) {
        float f[8], o[8];
        unpack8(raw[k], f);
        const f32x4 s0 = *reinterpret_cast<const f32x4*>(s_lds + v * 8);
        const f32x4 s1 = *reinterpret_cast<const f32x4*>(s_lds + v * 8 + 4);
        const f32x4 b0 = *reinterpret_cast<const f32x4*>(b_lds + v * 8);
        const f32x4 b1 = *reinterpret_cast<const f32x4*>(b_lds + v * 8 + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          o[i] = __builtin_fmaf(f[i] * r, s0[i], b0[i]);
          o[4 + i] = __builtin_fmaf(f[4 + i] * r, s1[i], b1[i]);
        }
        __builtin_nontemporal_store(pack8(o), &dst[v]);
      }
    }
  }
}

// Sum the four waves' per-lane column accumulators acc[A][K][8] through LDS in wave order and
// write them as this workgroup's partial row(s): partial[(block * A + a) * C + c].
template <int A, int K>
__device__ __forceinline__ void write_partials(float (&acc)[A][K][8], float* lds, int C,
                                               float* __restrict__ partial) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int turn = 0; turn < kRowWaves; ++turn) {
    if (wave == turn) {
#pragma unroll
      for (int a = 0; a < A; ++a)
#pragma unroll
        for (int k = 0; k < K; ++k) {
          const int v = k * 64 + lane;
          if (v * 8 < C) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              float* slot = lds + a * C + v * 8 + i;
              *slot = turn == 0 ? acc[a][k][i] : *slot + acc[a][k][i];
            }
          }
        }
    }
    __syncthreads();
  }
  float* out = partial + (int64_t)blockIdx.x * A * C;
  for (int c = threadIdx.x; c < A * C; c += kRowThreads) out[c] = lds[c];
}

// ---------------------------------------------------------------------------------------
// RMSNorm with adaptive modulation, backward.  LDS: s[C], then 2 x C for the partial sums.
// Partial rows: [sum dh * n | sum dh].
// ---------------------------------------------------------------------------------------
template <int K>
__global__ __launch_bounds__(kRowThreads) void rmsnorm_adaln_bwd_kernel(
    RowWork rw, const bf16_t* __restrict__ x, const float* __restrict__ w,
    const float* __restrict__ gamma, const float* __restrict__ rstd,
    const bf16_t* __restrict__ dh, const bf16_t* __restrict__ dres, bf16_t* __restrict__ dx,
    float* __restrict__ partial) {
  extern __shared__ __align__(16) float lds_f[];
  float* s_lds = lds_f;
  float* red = lds_f + rw.C;
  int64_t r0, r1;
  int smp;
  chunk_rows(rw, r0, r1, smp);
  const int C = rw.C;
  for (int c = threadIdx.x; c < C; c += kRowThreads)
    s_lds[c] = w[c] * (1.f + gamma[(int64_t)smp * C + c]);
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float inv_c = 1.f / (float)C;
  float acc[2][K][8];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[a][k][i] = 0.f;

  for (int64_t row = r0 + wave; row < r1; row += kRowWaves) {
    const u32x4* xs = reinterpret_cast<const u32x4*>(x + row * C);
    const u32x4* gs = reinterpret_cast<const u32x4*>(dh + row * C);
    u32x4 xr[K], gr[K], rr[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int v = k * 64 + lane;
      const bool in = v * 8 < C;
      xr[k] = in ? __builtin_nontemporal_load(&xs[v]) : u32x4{0, 0, 0, 0};
      gr[k] = in ? __builtin_nontemporal_load(&gs[v]) : u32x4{0, 0, 0, 0};
      // the gradient that reaches x along the residual path, added before the one rounding
      rr[k] = (in && dres) ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(dres + row * C) + v)
                           : u32x4{0, 0, 0, 0};
    }
    const float r = rstd[row];
    float dot = 0.f;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int v = k * 64 + lane;
      float xf[8], gf[8];
      unpack8(xr[k], xf);
      unpack8(gr[k], gf);
      f32x4 s0 = {0, 0, 0, 0}, s1 = {0, 0, 0, 0};
      if (v * 8 < C) {
        s0 = *reinterpret_cast<const f32x4*>(s_lds + v * 8);
        s1 = *reinterpret_cast<const f32x4*>(s_lds + v * 8 + 4);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float n = xf[i] * r;
        const float gn = gf[i] * n;
        dot = __builtin_fmaf(gn, i < 4 ? s0[i & 3] : s1[i & 3], dot);   // dn * n
        acc[0][k][i] += gn;
        acc[1][k][i] += gf[i];
      }
    }
    const float m = wave_sum(dot) * inv_c;
    u32x4* dst = reinterpret_cast<u32x4*>(dx + row * C);
    // second pass over the row in registers: n and dn are recomputed rather than kept
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int v = k * 64 + lane;
      if (v * 8 < C) {
        float xf[8], gf[8], rf[8], o[8];
        unpack8(xr[k], xf);
        unpack8(gr[k], gf);
        unpack8(rr[k], rf);
        const f32x4 s0 = *reinterpret_cast<const f32x4*>(s_lds + v * 8);
        const f32x4 s1 = *reinterpret_cast<const f32x4*>(s_lds + v * 8 + 4);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float n = xf[i] * r;
          const float dn = gf[i] * (i < 4 ? s0[i & 3] : s1[i & 3]);
          o[i] = __builtin_fmaf(r, __builtin_fmaf(-n, m, dn), rf[i]);
        }
        __builtin_nontemporal_store(pack8(o), &dst[v]);
      }
    }
  }
  write_partials<2, K>(acc, red, C, partial);
}

// Second stage of the sums over tokens.  One workgroup per 64 channels; thread (c, part) adds
// the partial rows part, part + 4, ... of a sample, the four parts are added in order.
// mode 0 (RMSNorm backward, A = 2): dbeta = sum B, dgamma = w sum A, dw = sum_b (1+gamma_b) sum A.
// mode 1 (gate backward, A = 1):    dalpha = sum A.
__global__ __launch_bounds__(256) void column_sums_finish_kernel(
    const float* __restrict__ partial, int n_samples, int cps, int C, int mode,
    const float* __restrict__ w, const float* __restrict__ gamma, float* __restrict__ out0,
    float* __restrict__ out1, float* __restrict__ out_w) {
  __shared__ float red[2][4][64];
  const int cx = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cx;
  const int A = mode == 0 ? 2 : 1;
  float dw_acc = 0.f;
  for (int b = 0; b < n_samples; ++b) {
    float a0 = 0.f, a1 = 0.f;
    if (c < C) {
      for (int k = part; k < cps; k += 4) {
        const float* row = partial + ((int64_t)(b * cps + k) * A) * C;
        a0 += row[c];
        if (A == 2) a1 += row[C + c];
      }
    }
    red[0][part][cx] = a0;
    red[1][part][cx] = a1;
    __syncthreads();
    if (part == 0 && c < C) {
      const float s0 = ((red[0][0][cx] + red[0][1][cx]) + red[0][2][cx]) + red[0][3][cx];
      const float s1 = ((red[1][0][cx] + red[1][1][cx]) + red[1][2][cx]) + red[1][3][cx];
      if (mode == 0) {
        if (out1 != nullptr) out1[(int64_t)b * C + c] = s1;                 // dbeta
        if (out0 != nullptr) out0[(int64_t)b * C + c] = w[c] * s0;          // dgamma
        dw_acc = __builtin_fmaf(1.f + gamma[(int64_t)b * C + c], s0, dw_acc);
      } else if (out0 != nullptr) {
        out0[(int64_t)b * C + c] = s0;                                      // dalpha
      }
    }
    __syncthreads();
  }
  if (mode == 0 && part == 0 && c < C && out_w != nullptr) out_w[c] = dw_acc;
}

// ---------------------------------------------------------------------------------------
// Gated residual.  The sample's alpha stays in registers.
// ---------------------------------------------------------------------------------------
template <int K>
__global__ __launch_bounds__(kRowThreads) void gate_residual_fwd_kernel(
    RowWork rw, const bf16_t* x, const bf16_t* y, const float* __restrict__ alpha, bf16_t* out) {
  int64_t r0, r1;
  int smp;
  chunk_rows(rw, r0, r1, smp);
  const int C = rw.C;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float a[K][8];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int v = k * 64 + lane;
#pragma unroll
    for (int i = 0; i < 8; ++i) a[k][i] = (v * 8 < C) ? alpha[(int64_t)smp * C + v * 8 + i] : 0.f;
  }
  for (int64_t row = r0 + wave; row < r1; row += kRowWaves) {
    const u32x4* xs = reinterpret_cast<const u32x4*>(x + row * C);
    const u32x4* ys = reinterpret_cast<const u32x4*>(y + row * C);
    u32x4* dst = reinterpret_cast<u32x4*>(out + row * C);
    u32x4 xr[K], yr[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int v = k * 64 + lane;
      if (v * 8 < C) {
        xr[k] = __builtin_nontemporal_load(&xs[v]);
        yr[k] = __builtin_nontemporal_load(&ys[v]);
      }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int v = k * 64 + lane;
      if (v * 8 < C) {
        float xf[8], yf[8], o[8];
        unpack8(xr[k], xf);
        unpack8(yr[k], yf);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = __builtin_fmaf(a[k][i], yf[i], xf[i]);
        __builtin_nontemporal_store(pack8(o), &dst[v]);
      }
    }
  }
}

template <int K>
__global__ __launch_bounds__(kRowThreads) void gate_residual_bwd_kernel(
    RowWork rw, const bf16_t* __restrict__ y, const float* __restrict__ alpha, const bf16_t* dout,
    bf16_t* dy, float* __restrict__ partial) {
  extern __shared__ __align__(16) float lds_f[];
  int64_t r0, r1;
  int smp;
  chunk_rows(rw, r0, r1, smp);
  const int C = rw.C;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float a[K][8], acc[1][K][8];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int v = k * 64 + lane;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[k][i] = (v * 8 < C) ? alpha[(int64_t)smp * C + v * 8 + i] : 0.f;
      acc[0][k][i] = 0.f;
    }
  }
  for (int64_t row = r0 + wave; row < r1; row += kRowWaves) {
    const u32x4* ys = reinterpret_cast<const u32x4*>(y + row * C);
    const u32x4* gs = reinterpret_cast<const u32x4*>(dout + row * C);
    u32x4* dst = reinterpret_cast<u32x4*>(dy + row * C);
    u32x4 yr[K], gr[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int v = k * 64 + lane;
      const bool in = v * 8 < C;
      yr[k] = in ? __builtin_nontemporal_load(&ys[v]) : u32x4{0, 0, 0, 0};
      gr[k] = in ? __builtin_nontemporal_load(&gs[v]) : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int v = k * 64 + lane;
      float yf[8], gf[8], o[8];
      unpack8(yr[k], yf);
      unpack8(gr[k], gf);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        o[i] = a[k][i] * gf[i];
        acc[0][k][i] = __builtin_fmaf(gf[i], yf[i], acc[0][k][i]);
      }
      if (v * 8 < C) __builtin_nontemporal_store(pack8(o), &dst[v]);
    }
  }
  write_partials<1, K>(acc, lds_f, C, partial);
}

// ---------------------------------------------------------------------------------------
// SwiGLU gate.  A workgroup takes a contiguous chunk of rows; its threads run over the
// 8-element vectors of a row.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float logistic(float u) {
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-u * kLog2e));
}

__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const bf16_t* __restrict__ uv,
                                                         int64_t n_rows, int F,
                                                         bf16_t* __restrict__ g) {
  const int fv = F / 8;
  const int64_t r0 = n_rows * blockIdx.x / gridDim.x, r1 = n_rows * (blockIdx.x + 1) / gridDim.x;
  for (int64_t row = r0; row < r1; ++row) {
    const u32x4* us = reinterpret_cast<const u32x4*>(uv + row * 2 * F);
    const u32x4* vs = us + fv;
    u32x4* dst = reinterpret_cast<u32x4*>(g + row * F);
    for (int j = threadIdx.x; j < fv; j += 256) {
      float u[8], v[8], o[8];
      unpack8(__builtin_nontemporal_load(&us[j]), u);
      unpack8(__builtin_nontemporal_load(&vs[j]), v);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = u[i] * logistic(u[i]) * v[i];
      __builtin_nontemporal_store(pack8(o), &dst[j]);
    }
  }
}

__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const bf16_t* uv,
                                                         const bf16_t* __restrict__ dg,
                                                         int64_t n_rows, int F, bf16_t* duv) {
  const int fv = F / 8;
  const int64_t r0 = n_rows * blockIdx.x / gridDim.x, r1 = n_rows * (blockIdx.x + 1) / gridDim.x;
  for (int64_t row = r0; row < r1; ++row) {
    const u32x4* us = reinterpret_cast<const u32x4*>(uv + row * 2 * F);
    const u32x4* vs = us + fv;
    const u32x4* gs = reinterpret_cast<const u32x4*>(dg + row * F);
    u32x4* du = reinterpret_cast<u32x4*>(duv + row * 2 * F);
    u32x4* dv = du + fv;
    for (int j = threadIdx.x; j < fv; j += 256) {
      float u[8], v[8], d[8], ou[8], ov[8];
      unpack8(__builtin_nontemporal_load(&us[j]), u);
      unpack8(__builtin_nontemporal_load(&vs[j]), v);
      unpack8(__builtin_nontemporal_load(&gs[j]), d);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float s = logistic(u[i]);
        ou[i] = d[i] * v[i] * s * __builtin_fmaf(u[i], 1.f - s, 1.f);
        ov[i] = d[i] * u[i] * s;
      }
      __builtin_nontemporal_store(pack8(ou), &du[j]);
      __builtin_nontemporal_store(pack8(ov), &dv[j]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------
bool bad_ptr(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

int check_rows(int64_t n_rows, int64_t rows_per_sample, int32_t channels) {
  if (n_rows <= 0 || rows_per_sample <= 0 || channels < 8 || channels > AERIS_MAX_CHANNELS)
    return AERIS_ERR_INVALID_SHAPE;
  if (channels % 8 != 0 || n_rows % rows_per_sample != 0) return AERIS_ERR_NOT_DIVISIBLE;
  if (n_rows / rows_per_sample > (1 << 20)) return AERIS_ERR_INVALID_SHAPE;
  return AERIS_OK;
}

int vectors_per_lane(int channels) {
  const int v = (channels / 8 + 63) / 64;
  return v <= 1 ? 1 : v <= 2 ? 2 : v <= 4 ? 4 : 8;
}

int status(int launch_rc) { return launch_rc == 0 ? AERIS_OK : AERIS_ERR_HIP_LAUNCH; }

// Calls f(Const<K>) for the K that fits `channels`.
template <typename F>
void with_k(int channels, F&& f) {
  switch (vectors_per_lane(channels)) {
    case 1: f(Const<1>{}); break;
    case 2: f(Const<2>{}); break;
    case 4: f(Const<4>{}); break;
    default: f(Const<8>{}); break;
  }
}

}  // namespace
}  // namespace aeris

using namespace aeris;

extern "C" int aeris_rmsnorm_adaln_fwd(const void* x, const float* w, const float* gamma,
                                       const float* beta, float eps, int64_t n_rows,
                                       int64_t rows_per_sample, int32_t channels, void* h,
                                       float* r, void* hip_stream) {
  if (!x || !w || !gamma || !beta || !h) return AERIS_ERR_NULL_POINTER;
  if (const int rc = check_rows(n_rows, rows_per_sample, channels)) return rc;
  if (!(eps >= 0.f)) return AERIS_ERR_INVALID_SHAPE;
  if (bad_ptr(x) || bad_ptr(h) || bad_ptr(w) || bad_ptr(gamma) || bad_ptr(beta) ||
      (reinterpret_cast<uintptr_t>(r) & 3))
    return AERIS_ERR_MISALIGNED;
  const int cps = chunks_per_sample(n_rows, rows_per_sample);
  const RowWork rw{rows_per_sample, cps, channels};
  const dim3 grid(static_cast<unsigned>(n_rows / rows_per_sample * cps));
  const size_t smem = 2 * sizeof(float) * channels;
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int rc = -1;
  with_k(channels, [&](auto kc) {
    rc = launch_kernel(rmsnorm_adaln_fwd_kernel<decltype(kc)::value>, grid, dim3(kRowThreads),
                       smem, st, rw, static_cast<const bf16_t*>(x), w, gamma, beta, eps,
                       static_cast<bf16_t*>(h), r);
  });
  return status(rc);
}

extern "C" size_t aeris_rmsnorm_adaln_bwd_workspace_bytes(int64_t n_rows, int64_t rows_per_sample,
                                                          int32_t channels) {
  if (check_rows(n_rows, rows_per_sample, channels) != AERIS_OK) return 0;
  const int64_t chunks = n_rows / rows_per_sample * chunks_per_sample(n_rows, rows_per_sample);
  return static_cast<size_t>(chunks) * 2 * channels * sizeof(float);
}

extern "C" int aeris_rmsnorm_adaln_bwd(const void* x, const float* w, const float* gamma,
                                       const float* r, const void* dh, int64_t n_rows,
                                       int64_t rows_per_sample, int32_t channels, void* dx,
                                       float* dw, float* dgamma, float* dbeta, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  return aeris_rmsnorm_adaln_bwd_residual(x, w, gamma, r, dh, nullptr, n_rows, rows_per_sample,
                                          channels, dx, dw, dgamma, dbeta, workspace,
                                          workspace_bytes, hip_stream);
}

extern "C" int aeris_rmsnorm_adaln_bwd_residual(const void* x, const float* w, const float* gamma,
                                                const float* r, const void* dh, const void* dres,
                                                int64_t n_rows, int64_t rows_per_sample,
                                                int32_t channels, void* dx, float* dw,
                                                float* dgamma, float* dbeta, void* workspace,
                                                size_t workspace_bytes, void* hip_stream) {
  if (!x || !w || !gamma || !r || !dh || !dx || !workspace) return AERIS_ERR_NULL_POINTER;
  if (const int rc = check_rows(n_rows, rows_per_sample, channels)) return rc;
  if (bad_ptr(x) || bad_ptr(dh) || bad_ptr(dres) || bad_ptr(dx) || bad_ptr(w) || bad_ptr(gamma) ||
      bad_ptr(workspace) || (reinterpret_cast<uintptr_t>(r) & 3) ||
      (reinterpret_cast<uintptr_t>(dw) & 3) || (reinterpret_cast<uintptr_t>(dgamma) & 3) ||
      (reinterpret_cast<uintptr_t>(dbeta) & 3))
    return AERIS_ERR_MISALIGNED;
  if (workspace_bytes < aeris_rmsnorm_adaln_bwd_workspace_bytes(n_rows, rows_per_sample, channels))
    return AERIS_ERR_WORKSPACE_TOO_SMALL;
  const int cps = chunks_per_sample(n_rows, rows_per_sample);
  const int n_samples = static_cast<int>(n_rows / rows_per_sample);
  const RowWork rw{rows_per_sample, cps, channels};
  const dim3 grid(static_cast<unsigned>(n_samples * cps));
  const size_t smem = 3 * sizeof(float) * channels;
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* partial = static_cast<float*>(workspace);
  int rc = -1;
  with_k(channels, [&](auto kc) {
    rc = launch_kernel(rmsnorm_adaln_bwd_kernel<decltype(kc)::value>, grid, dim3(kRowThreads),
                       smem, st, rw, static_cast<const bf16_t*>(x), w, gamma, r,
                       static_cast<const bf16_t*>(dh), static_cast<const bf16_t*>(dres),
                       static_cast<bf16_t*>(dx), partial);
  });
  if (rc != 0) return AERIS_ERR_HIP_LAUNCH;
  if (dw || dgamma || dbeta) {
    return status(launch_kernel(column_sums_finish_kernel, dim3((channels + 63) / 64), dim3(256), 0,
                                st, partial, n_samples, cps, channels, 0, w, gamma, dgamma, dbeta,
                                dw));
  }
  return AERIS_OK;
}

extern "C" int aeris_gate_residual_fwd(const void* x, const void* y, const float* alpha,
                                       int64_t n_rows, int64_t rows_per_sample, int32_t channels,
                                       void* out, void* hip_stream) {
  if (!x || !y || !alpha || !out) return AERIS_ERR_NULL_POINTER;
  if (const int rc = check_rows(n_rows, rows_per_sample, channels)) return rc;
  if (bad_ptr(x) || bad_ptr(y) || bad_ptr(out) || bad_ptr(alpha)) return AERIS_ERR_MISALIGNED;
  const int cps = chunks_per_sample(n_rows, rows_per_sample);
  const RowWork rw{rows_per_sample, cps, channels};
  const dim3 grid(static_cast<unsigned>(n_rows / rows_per_sample * cps));
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int rc = -1;
  with_k(channels, [&](auto kc) {
    rc = launch_kernel(gate_residual_fwd_kernel<decltype(kc)::value>, grid, dim3(kRowThreads),
                       0, st, rw, static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(y),
                       alpha, static_cast<bf16_t*>(out));
  });
  return status(rc);
}

extern "C" size_t aeris_gate_residual_bwd_workspace_bytes(int64_t n_rows, int64_t rows_per_sample,
                                                          int32_t channels) {
  if (check_rows(n_rows, rows_per_sample, channels) != AERIS_OK) return 0;
  const int64_t chunks = n_rows / rows_per_sample * chunks_per_sample(n_rows, rows_per_sample);
  return static_cast<size_t>(chunks) * channels * sizeof(float);
}

extern "C" int aeris_gate_residual_bwd(const void* y, const float* alpha, const void* dout,
                                       int64_t n_rows, int64_t rows_per_sample, int32_t channels,
                                       void* dy, float* dalpha, void* workspace,
                                       size_t workspace_bytes, void* hip_stream) {
  if (!y || !alpha || !dout || !dy || !workspace) return AERIS_ERR_NULL_POINTER;
  if (const int rc = check_rows(n_rows, rows_per_sample, channels)) return rc;
  if (bad_ptr(y) || bad_ptr(dout) || bad_ptr(dy) || bad_ptr(alpha) || bad_ptr(workspace) ||
      (reinterpret_cast<uintptr_t>(dalpha) & 3))
    return AERIS_ERR_MISALIGNED;
  if (workspace_bytes < aeris_gate_residual_bwd_workspace_bytes(n_rows, rows_per_sample, channels))
    return AERIS_ERR_WORKSPACE_TOO_SMALL;
  const int cps = chunks_per_sample(n_rows, rows_per_sample);
  const int n_samples = static_cast<int>(n_rows / rows_per_sample);
  const RowWork rw{rows_per_sample, cps, channels};
  const dim3 grid(static_cast<unsigned>(n_samples * cps));
  const size_t smem = sizeof(float) * channels;
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* partial = static_cast<float*>(workspace);
  int rc = -1;
  with_k(channels, [&](auto kc) {
    rc = launch_kernel(gate_residual_bwd_kernel<decltype(kc)::value>, grid, dim3(kRowThreads),
                       smem, st, rw, static_cast<const bf16_t*>(y), alpha,
                       static_cast<const bf16_t*>(dout), static_cast<bf16_t*>(dy), partial);
  });
  if (rc != 0) return AERIS_ERR_HIP_LAUNCH;
  if (dalpha) {
    return status(launch_kernel(column_sums_finish_kernel, dim3((channels + 63) / 64), dim3(256), 0,
                                st, partial, n_samples, cps, channels, 1, nullptr, nullptr, dalpha,
                                nullptr, nullptr));
  }
  return AERIS_OK;
}

namespace {
int check_swiglu(const void* a, const void* b, const void* c, int64_t n_rows, int32_t hidden) {
  if (!a || !b || !c) return AERIS_ERR_NULL_POINTER;
  if (n_rows <= 0 || hidden < 8) return AERIS_ERR_INVALID_SHAPE;
  if (hidden % 8 != 0) return AERIS_ERR_NOT_DIVISIBLE;
  if (bad_ptr(a) || bad_ptr(b) || bad_ptr(c)) return AERIS_ERR_MISALIGNED;
  return AERIS_OK;
}
unsigned swiglu_grid(int64_t n_rows) {
  return static_cast<unsigned>(n_rows < 4 * kTargetChunks ? n_rows : 4 * kTargetChunks);
}
}  // namespace

extern "C" int aeris_swiglu_fwd(const void* uv, int64_t n_rows, int32_t hidden, void* g,
                                void* hip_stream) {
  if (const int rc = check_swiglu(uv, g, g, n_rows, hidden)) return rc;
  return status(launch_kernel(swiglu_fwd_kernel, dim3(swiglu_grid(n_rows)), dim3(256), 0,
                              static_cast<hipStream_t>(hip_stream),
                              static_cast<const bf16_t*>(uv), n_rows, hidden,
                              static_cast<bf16_t*>(g)));
}

extern "C" int aeris_swiglu_bwd(const void* uv, const void* dg, int64_t n_rows, int32_t hidden,
                                void* duv, void* hip_stream) {
  if (const int rc = check_swiglu(uv, dg, duv, n_rows, hidden)) return rc;
  return status(launch_kernel(swiglu_bwd_kernel, dim3(swiglu_grid(n_rows)), dim3(256), 0,
                              static_cast<hipStream_t>(hip_stream),
                              static_cast<const bf16_t*>(uv), static_cast<const bf16_t*>(dg),
                              n_rows, hidden, static_cast<bf16_t*>(duv)));
}
