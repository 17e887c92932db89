// Input projections of an AERIS transformer layer with the pre-RMSNorm and the adaptive
// modulation folded in (paper, Model Architecture section: RMSNorm and the adaptive-layer-norm
// values precede the projection of queries, keys and values and the SwiGLU feed-forward part);
// argument contracts in include/aeris_layer_ops.h.
//
// The normalised, modulated row h_c = x_c r w_c (1 + gamma_bc) + beta_bc is never written:
//     y_f = sum_c h_c W_fc = r * sum_c x_c (W_fc w_c (1 + gamma_bc)) + sum_c beta_bc W_fc,
// so the projection is a plain bf16 GEMM of the raw rows x with a per-sample folded weight
//     Wf_b = W diag(w (1 + gamma_b))        (bf16, built by a small kernel per call)
// followed, in the epilogue, by the row's reciprocal RMS r (from a row pass over x) and a
// per-sample bias beta_b W^T.  The SwiGLU gate is a second epilogue: a workgroup's tile holds
// matching u and v columns, so g = silu(u) v is formed on the accumulators.
//
// GEMM kernel: one workgroup of eight wavefronts per 256 x 256 output tile, 64 channels per
// step, both operands K-contiguous ("NT").  Operand tiles go global -> LDS directly
// (global_load_lds_dwordx4), two stages of 64 KB, 16-byte chunks XOR-swizzled so that the
// row-major ds_read_b128 operand fetches are conflict free; v_mfma_f32_32x32x16_bf16 with the
// weight rows as the A operand and the token rows as the B operand, so that a lane owns one
// token row of the output: the row scale is a per-lane scalar.  Results are staged through the
// LDS and leave in 16-byte pieces, eight lanes per 128-byte row segment.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "aeris_layer_ops.h"
#include "aeris_winattn.h"
#include "projection_gemm.hpp"
#include "winattn_common.hpp"
#include "winattn_launch.hpp"

namespace aeris {
namespace {

constexpr int kBM = 256;                 // token rows per workgroup tile
constexpr int kBN = 256;                 // weight rows (output features) per workgroup tile
constexpr int kBK = 64;                  // channels per step
constexpr int kGemmWaves = 8;
constexpr int kPartBytes = kBN * kBK * 2;            // 32 KB: weight rows, then token rows
constexpr int kStageBytes = 2 * kPartBytes;
using Sub = Tile<64, kGemmWaves>;        // 64 rows x 64 channels, swizzled chunks

// Workgroup id -> (token tile, feature tile).  Consecutive ids go to the eight XCDs in turn;
// the 32 workgroups an XCD runs at a time are 8 token tiles x 4 feature tiles, so every
// operand tile that arrives in that XCD's L2 serves 4 or 8 workgroups.
__device__ __forceinline__ bool gemm_tile(const GemmParams& p, int& mt, int& nt) {
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int per_group = 8 * p.n_tiles;
  const int group = slot / per_group, rem = slot - group * per_group;
  nt = rem >> 3;
  mt = ((group * 8 + (rem & 7)) << 3) + xcd;
  return mt < p.m_tiles;
}
inline unsigned gemm_grid(const GemmParams& p) {
  return 8u * (unsigned)((p.m_tiles + 63) / 64) * 8u * (unsigned)p.n_tiles;
}

__device__ __forceinline__ float silu(float u) {
  return u * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-u * kLog2e));
}

__global__ __launch_bounds__(kGemmWaves * 64, 1) void norm_linear_gemm_kernel(GemmParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  int mt, nt;
  if (!gemm_tile(p, mt, nt)) return;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;          // 2 x 4 waves: 128 token rows x 64 features
  const int li = lane & 31, g = lane >> 5;

  const int sample = mt / p.m_tiles_per_sample;
  const int tile_in_sample = mt - sample * p.m_tiles_per_sample;
  const long long row0 = (long long)sample * p.rows_per_sample + (long long)tile_in_sample * kBM;
  const long long rows_left = p.rows_per_sample - (long long)tile_in_sample * kBM;
  const int valid_rows = rows_left < kBM ? (int)rows_left : kBM;
  const int hidden = p.F >> 1;

  // Feature (weight row) of tile row R.  SwiGLU tiles pair 128 u-features with their
  // v-features: wave column wn holds u rows in its first 32 tile rows, v rows in the next 32.
  auto feature = [&](int R) __attribute__((always_inline)) {
    if (p.swiglu) {
      int j = nt * (kBN / 2) + (R >> 6) * 32 + (R & 31);
      j = j < hidden ? j : hidden - 1;
      return ((R >> 5) & 1) ? hidden + j : j;
    }
    const int f = nt * kBN + R;
    return f < p.F ? f : p.F - 1;
  };

  // ---- copies: instruction j (0..63) moves rows 8j..8j+7 of the stage; wave w issues
  // j = w + 8i.  i < 4: weight rows, i >= 4: token rows.  Rows past the end repeat the last
  // valid row (never stored).  Lane: row j*8 + lane/8, LDS chunk position lane%8.
  const bf16_t* wmat = p.w + (long long)sample * p.w_sample_stride;
  const unsigned long long wbase = reinterpret_cast<unsigned long long>(wmat);
  const unsigned long long xbase = reinterpret_cast<unsigned long long>(p.x + row0 * p.K);
  uint32_t voff[8];
  {
    const int r_in = lane >> 3;
    const int r_sub = ((wave & 1) << 3) | r_in;                  // row within a 64-row sub-tile, mod 16
    const int chunk = (lane & 7) ^ Sub::swz(r_sub);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int R = ((wave + 8 * i) << 3) + r_in;               // 0..511
      if (i < 4) {
        voff[i] = (uint32_t)((long long)feature(R) * p.K * 2 + chunk * 16);
      } else {
        int m = R - kBN;
        m = m < valid_rows ? m : valid_rows - 1;
        voff[i] = (uint32_t)((long long)m * p.K * 2 + chunk * 16);
      }
    }
  }
  const uint32_t lds0 = lds_address(smem);
  auto copy_piece = [&](int i, uint32_t stage, int k0, uint32_t enable) __attribute__((always_inline)) {
    async_copy16_off(voff[i], (i < 4 ? wbase : xbase) + (unsigned long long)k0 * 2,
                     stage + (uint32_t)((wave + 8 * i) << 10), enable);
  };

  // ---- operand reads: per lane four chunk offsets (one per 16-channel block of a step)
  uint32_t va[4], vb[4];
  {
    const int s = Sub::swz(li);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const uint32_t off = li * 128 + (((2 * kk + g) ^ s) << 4);
      va[kk] = lds0 + wn * 8192 + off;
      vb[kk] = lds0 + kPartBytes + wm * 16384 + off;
    }
  }

  f32x16 acc[2][4];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  const int k_steps = p.K / kBK;
#pragma unroll
  for (int i = 0; i < 8; ++i) copy_piece(i, lds0, 0, 1);

  bf16x8 ao[2][2], bo[2][4];
  auto fetch = [&](int set, int kk, uint32_t stage_off) __attribute__((always_inline)) {
#pragma unroll
    for (int a = 0; a < 2; ++a) ao[set][a] = Sub::read_rm(va[kk] + stage_off + a * 4096);
#pragma unroll
    for (int b = 0; b < 4; ++b) bo[set][b] = Sub::read_rm(vb[kk] + stage_off + b * 4096);
  };

  for (int ks = 0; ks < k_steps; ++ks) {
    const uint32_t stage_off = (ks & 1) * kStageBytes;
    wait_async_loads();
    __syncthreads();               // this stage has landed; every reader of the other one is done
    const uint32_t more = ks + 1 < k_steps;
    const uint32_t next_stage = lds0 + (kStageBytes - stage_off);
    fetch(0, 0, stage_off);
    sched_fence();
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk < 3) fetch((kk + 1) & 1, kk + 1, stage_off);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          acc[a][b] = mfma32(ao[kk & 1][a], bo[kk & 1][b], acc[a][b]);
          // the next stage's copies ride in the first half of the step, one per two products,
          // so that they have the second half to land before the wait that opens the next step
          if (kk < 2 && (b & 1)) copy_piece(4 * kk + 2 * a + (b >> 1), next_stage, (ks + 1) * kBK, more);
        }
      sched_fence();
    }
  }

  // ---- epilogue: row scale, bias, (gate); results pass through the LDS so that they leave in
  // 16-byte pieces, eight lanes per 128-byte row segment.  Each wave stages its 128 x 64 part
  // in a region of its own (row pitch 144 bytes: 16-byte aligned, rows on different banks).
  constexpr int kPitch = 144;
  __syncthreads();                                   // every wave is done with the operand stages
  const float* bias = p.bias ? p.bias + (long long)sample * p.F : nullptr;
  const uint32_t stage_w = lds0 + wave * (128 * kPitch);

  // writes the wave's staged [128][64] bf16 block (8 chunks per row) to `dst` (row pitch ld):
  // chunk c of a row goes to column col_of(c)
  auto flush = [&](bf16_t* dst, long long ld, int chunks, auto col_of, int limit)
      __attribute__((always_inline)) {
    const int rows_per_inst = 64 / chunks;
    const int r_in = lane / chunks, c = lane % chunks;
    const int col = col_of(c);
    for (int t = 0; t < 128 / rows_per_inst; ++t) {
      const int ml = t * rows_per_inst + r_in;
      const int m = wm * 128 + ml;
      const u32x4 v = *reinterpret_cast<const AERIS_LDS u32x4*>(stage_w + ml * kPitch + c * 16);
      if (m < valid_rows && col < limit)
        *reinterpret_cast<u32x4*>(dst + (row0 + m) * ld + col) = v;
    }
  };

  float rs[4];
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    int m = wm * 128 + b * 32 + li;
    m = m < valid_rows ? m : valid_rows - 1;
    rs[b] = p.r ? p.r[row0 + m] : 1.f;
  }
  auto stage_store = [&](int b, int col, float o0, float o1, float o2, float o3)
      __attribute__((always_inline)) {
    u32x2 v = {pack_bf16(o0, o1), pack_bf16(o2, o3)};
    *reinterpret_cast<AERIS_LDS u32x2*>(stage_w + (b * 32 + li) * kPitch + col * 2) = v;
  };

  if (p.swiglu) {
    const int jw = nt * (kBN / 2) + wn * 32;         // first gate column of this wave
    f32x4 bu[4], bv[4];
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      int j = jw + 8 * vq + 4 * g;
      j = j < hidden ? j : hidden - 4;
      bu[vq] = bias ? *reinterpret_cast<const f32x4*>(bias + j) : f32x4{0.f, 0.f, 0.f, 0.f};
      bv[vq] = bias ? *reinterpret_cast<const f32x4*>(bias + hidden + j) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // u and v (kept in registers), staged as [u 32 | v 32] for the optional uv output
    float uu[4][16], vv[4][16];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        uu[b][i] = __builtin_fmaf(acc[0][b][i], rs[b], bu[i >> 2][i & 3]);
        vv[b][i] = __builtin_fmaf(acc[1][b][i], rs[b], bv[i >> 2][i & 3]);
      }
    if (p.y) {
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          stage_store(b, 8 * vq + 4 * g, uu[b][4 * vq], uu[b][4 * vq + 1], uu[b][4 * vq + 2],
                      uu[b][4 * vq + 3]);
          stage_store(b, 32 + 8 * vq + 4 * g, vv[b][4 * vq], vv[b][4 * vq + 1], vv[b][4 * vq + 2],
                      vv[b][4 * vq + 3]);
        }
      // chunk c: c < 4 -> u columns jw + 8c, else v columns hidden + jw + 8(c - 4); a column
      // past `hidden` (ragged last tile) is marked by F, which the limit rejects
      flush(p.y, p.F, 8, [&](int c) {
        const int j = jw + 8 * (c & 3);
        return j < hidden ? (c < 4 ? j : hidden + j) : p.F;
      }, p.F);
    }
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq)
        stage_store(b, 8 * vq + 4 * g, silu(uu[b][4 * vq]) * vv[b][4 * vq],
                    silu(uu[b][4 * vq + 1]) * vv[b][4 * vq + 1],
                    silu(uu[b][4 * vq + 2]) * vv[b][4 * vq + 2],
                    silu(uu[b][4 * vq + 3]) * vv[b][4 * vq + 3]);
    flush(p.g, hidden, 4, [&](int c) { return jw + 8 * c; }, hidden);
  } else {
    const int fw = nt * kBN + wn * 64;               // first feature of this wave
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        int f = fw + a * 32 + 8 * vq + 4 * g;
        f = f < p.F ? f : p.F - 4;
        const f32x4 b4 = bias ? *reinterpret_cast<const f32x4*>(bias + f) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int b = 0; b < 4; ++b)
          stage_store(b, a * 32 + 8 * vq + 4 * g,
                      __builtin_fmaf(acc[a][b][4 * vq], rs[b], b4[0]),
                      __builtin_fmaf(acc[a][b][4 * vq + 1], rs[b], b4[1]),
                      __builtin_fmaf(acc[a][b][4 * vq + 2], rs[b], b4[2]),
                      __builtin_fmaf(acc[a][b][4 * vq + 3], rs[b], b4[3]));
      }
    flush(p.y, p.F, 8, [&](int c) { return fw + 8 * c; }, p.F);
  }
}

// r_i = (mean_c x_ic^2 + eps)^(-1/2): one wavefront per row, 16 bytes per lane and access.
__global__ __launch_bounds__(256) void rms_rows_kernel(const bf16_t* __restrict__ x, long long n_rows,
                                                       int channels, float eps, float* __restrict__ r) {
  const int lane = threadIdx.x & 63;
  const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long long n_waves = (long long)gridDim.x * 4;
  for (long long row = wave; row < n_rows; row += n_waves) {
    const bf16_t* xr = x + row * channels;
    float s = 0.f;
    for (int c = lane * 8; c < channels; c += 512) {
      const bf16x8 v = *reinterpret_cast<const bf16x8*>(xr + c);
#pragma unroll
      for (int e = 0; e < 8; ++e) s = __builtin_fmaf((float)v[e], (float)v[e], s);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d);
    if (lane == 0) r[row] = 1.f / sqrtf(s / (float)channels + eps);
  }
}

// Wf_b[f][c] = bf16(W[f][c] w[c] (1 + gamma_b[c])),  bias_b[f] = sum_c beta_b[c] W[f][c].
// One workgroup per (feature, sample); the bias sum is taken in a fixed order.
__global__ __launch_bounds__(256) void fold_weights_kernel(const bf16_t* __restrict__ w_in,
                                                           const float* __restrict__ w,
                                                           const float* __restrict__ gamma,
                                                           const float* __restrict__ beta, int K,
                                                           int F, bf16_t* __restrict__ w_out,
                                                           float* __restrict__ bias) {
  __shared__ float part[4];
  const int f = blockIdx.x, b = blockIdx.y;
  const bf16_t* src = w_in + (long long)f * K;
  bf16_t* dst = w_out + ((long long)b * F + f) * K;
  float s = 0.f;
  for (int c = threadIdx.x * 8; c < K; c += 256 * 8) {
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(src + c);
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float wv = (float)v[e];
      o[e] = (bf16_t)(wv * (w[c + e] * (1.f + gamma[(long long)b * K + c + e])));
      s = __builtin_fmaf(beta[(long long)b * K + c + e], wv, s);
    }
    *reinterpret_cast<bf16x8*>(dst + c) = o;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) bias[(long long)b * F + f] = (part[0] + part[1]) + (part[2] + part[3]);
}

size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

int projection_gemm_check(long long n_rows, long long rows_per_sample, int K, int F) {
  if (n_rows <= 0 || rows_per_sample <= 0 || K < kBK || F < 8) return AERIS_ERR_INVALID_SHAPE;
  if (K % kBK != 0 || F % 8 != 0 || n_rows % rows_per_sample != 0) return AERIS_ERR_NOT_DIVISIBLE;
  if (n_rows / rows_per_sample > 65535) return AERIS_ERR_INVALID_SHAPE;   // a grid dimension
  // 32-bit byte offsets inside a workgroup's operand tiles, 31-bit tile counts
  if ((long long)F * K * 2 >= (1LL << 32)) return AERIS_ERR_INVALID_SHAPE;
  const long long m_tiles = (n_rows / rows_per_sample) * ((rows_per_sample + kBM - 1) / kBM);
  const long long n_tiles = (F + kBN - 1) / kBN;
  if (((m_tiles + 63) / 64) * 64 * n_tiles >= (1LL << 31)) return AERIS_ERR_INVALID_SHAPE;
  return AERIS_OK;
}

namespace {

int check_projection(int64_t n_rows, int64_t rows_per_sample, int32_t channels, int32_t features) {
  if (n_rows <= 0 || rows_per_sample <= 0 || channels <= 0 || features <= 0)
    return AERIS_ERR_INVALID_SHAPE;
  if (channels > AERIS_MAX_PROJECTION_CHANNELS) return AERIS_ERR_INVALID_SHAPE;
  return projection_gemm_check(n_rows, rows_per_sample, channels, features);
}

bool bad16(const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) != 0; }

}  // namespace

int launch_projection_gemm(GemmParams p, hipStream_t stream) {
  p.m_tiles_per_sample = (int)((p.rows_per_sample + kBM - 1) / kBM);
  if (!allow_full_lds<norm_linear_gemm_kernel>()) return -1;
  // two operand stages; the epilogue reuses them as eight 128 x 144-byte staging regions
  constexpr size_t kSmem = kGemmWaves * 128 * 144 > 2 * kStageBytes ? kGemmWaves * 128 * 144
                                                                    : 2 * kStageBytes;
  return launch_kernel(norm_linear_gemm_kernel, dim3(gemm_grid(p)), dim3(kGemmWaves * 64), kSmem,
                       stream, p);
}

namespace {

struct Folded {
  bf16_t* w;
  float* bias;
  float* r;
};
Folded carve(void* workspace, int64_t n_rows, int64_t n_samples, int32_t channels, int32_t features) {
  char* ws = static_cast<char*>(workspace);
  Folded f;
  f.w = reinterpret_cast<bf16_t*>(ws);
  ws += round256((size_t)n_samples * features * channels * 2);
  f.bias = reinterpret_cast<float*>(ws);
  ws += round256((size_t)n_samples * features * 4);
  f.r = reinterpret_cast<float*>(ws);
  return f;
}

// Row pass + weight folding + GEMM.  features = rows of `weight`; swiglu: features = 2 * hidden.
int norm_projection(const void* x, const float* w, const float* gamma, const float* beta, float eps,
                    const void* weight, int64_t n_rows, int64_t rows_per_sample, int32_t channels,
                    int32_t features, bool swiglu, void* y, void* g, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (!x || !w || !gamma || !beta || !weight || !workspace || (!swiglu && !y) || (swiglu && !g))
    return AERIS_ERR_NULL_POINTER;
  if (const int rc = check_projection(n_rows, rows_per_sample, channels, features)) return rc;
  if (!(eps >= 0.f)) return AERIS_ERR_INVALID_SHAPE;
  if (bad16(x) || bad16(weight) || bad16(y) || bad16(g) || bad16(workspace) || bad16(w) ||
      bad16(gamma) || bad16(beta))
    return AERIS_ERR_MISALIGNED;
  if (workspace_bytes < aeris_norm_linear_workspace_bytes(n_rows, rows_per_sample, channels, features))
    return AERIS_ERR_WORKSPACE_TOO_SMALL;
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int64_t n_samples = n_rows / rows_per_sample;
  const Folded f = carve(workspace, n_rows, n_samples, channels, features);
  const long long row_blocks = (n_rows + 3) / 4;
  if (launch_kernel(rms_rows_kernel, dim3((unsigned)(row_blocks < 8192 ? row_blocks : 8192)),
                    dim3(256), 0, st, static_cast<const bf16_t*>(x), (long long)n_rows, channels,
                    eps, f.r) != 0 ||
      launch_kernel(fold_weights_kernel, dim3((unsigned)features, (unsigned)n_samples), dim3(256), 0,
                    st, static_cast<const bf16_t*>(weight), w, gamma, beta, channels, features,
                    f.w, f.bias) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  GemmParams p{};
  p.x = static_cast<const bf16_t*>(x);
  p.w = f.w;
  p.w_sample_stride = (long long)features * channels;
  p.r = f.r;
  p.bias = f.bias;
  p.y = static_cast<bf16_t*>(y);
  p.g = static_cast<bf16_t*>(g);
  p.rows_per_sample = rows_per_sample;
  p.m_tiles = (int)(n_samples * ((rows_per_sample + kBM - 1) / kBM));
  p.K = channels;
  p.F = features;
  p.swiglu = swiglu ? 1 : 0;
  p.n_tiles = swiglu ? (features / 2 + kBN / 2 - 1) / (kBN / 2) : (features + kBN - 1) / kBN;
  return launch_projection_gemm(p, st) == 0 ? AERIS_OK : AERIS_ERR_HIP_LAUNCH;
}

}  // namespace
}  // namespace aeris

using namespace aeris;

extern "C" size_t aeris_norm_linear_workspace_bytes(int64_t n_rows, int64_t rows_per_sample,
                                                    int32_t channels, int32_t out_features) {
  if (check_projection(n_rows, rows_per_sample, channels, out_features) != AERIS_OK) return 0;
  const size_t n_samples = (size_t)(n_rows / rows_per_sample);
  return round256(n_samples * out_features * channels * 2) + round256(n_samples * out_features * 4) +
         round256((size_t)n_rows * 4);
}

extern "C" int aeris_norm_linear_fwd(const void* x, const float* w, const float* gamma,
                                     const float* beta, float eps, const void* weight,
                                     int64_t n_rows, int64_t rows_per_sample, int32_t channels,
                                     int32_t out_features, void* y, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
  return norm_projection(x, w, gamma, beta, eps, weight, n_rows, rows_per_sample, channels,
                         out_features, false, y, nullptr, workspace, workspace_bytes, hip_stream);
}

extern "C" int aeris_norm_linear_swiglu_fwd(const void* x, const float* w, const float* gamma,
                                            const float* beta, float eps, const void* weight,
                                            int64_t n_rows, int64_t rows_per_sample,
                                            int32_t channels, int32_t hidden, void* g, void* uv,
                                            void* workspace, size_t workspace_bytes,
                                            void* hip_stream) {
  if (hidden <= 0 || hidden > (1 << 29)) return AERIS_ERR_INVALID_SHAPE;
  if (hidden % 8 != 0) return AERIS_ERR_NOT_DIVISIBLE;
  return norm_projection(x, w, gamma, beta, eps, weight, n_rows, rows_per_sample, channels,
                         2 * hidden, true, uv, g, workspace, workspace_bytes, hip_stream);
}

extern "C" int aeris_linear_fwd(const void* x, const void* weight, int64_t n_rows, int32_t channels,
                                int32_t out_features, void* y, void* hip_stream) {
  if (!x || !weight || !y) return AERIS_ERR_NULL_POINTER;
  if (const int rc = check_projection(n_rows, n_rows, channels, out_features)) return rc;
  if (bad16(x) || bad16(weight) || bad16(y)) return AERIS_ERR_MISALIGNED;
  GemmParams p{};
  p.x = static_cast<const bf16_t*>(x);
  p.w = static_cast<const bf16_t*>(weight);
  p.y = static_cast<bf16_t*>(y);
  p.rows_per_sample = n_rows;
  p.m_tiles = (int)((n_rows + kBM - 1) / kBM);
  p.K = channels;
  p.F = out_features;
  p.n_tiles = (out_features + kBN - 1) / kBN;
  return launch_projection_gemm(p, static_cast<hipStream_t>(hip_stream)) == 0 ? AERIS_OK : AERIS_ERR_HIP_LAUNCH;
}
