// Gradients of a projection y = x W^T of an AERIS transformer layer (paper, Model Architecture
// section: the projections of queries, keys and values, the output projection and the SwiGLU
// feed-forward part; training runs the backward pass of each): dx = dy W and dW = dy^T x;
// argument contracts in include/aeris_layer_ops.h.
//
// dx is the forward GEMM kernel on the transposed weight (a small transposing kernel writes
// W^T [C, F] first), so both of its operands are contiguous along the contraction again.
//
// dW contracts over the token rows, along which neither operand is contiguous.  One workgroup
// of eight wavefronts owns a 256 x 256 tile of dW for a range of rows; per step 64 rows of dy
// (256 features) and of x (256 channels) go global -> LDS directly as four [64][128] sub-tiles
// in the swizzled chunk layout of the attention kernels, and both MFMA operands are fetched
// with transposing reads (ds_read_b64_tr_b16), the token index landing in the registers.  The
// row range of the whole problem is split over several workgroups per tile; each writes its
// partial tile, and a second kernel adds the partials in a fixed order (no atomics: the result
// does not depend on the schedule) together with the products of the rows past the last whole
// step of 64.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "aeris_layer_ops.h"
#include "aeris_winattn.h"
#include "projection_gemm.hpp"
#include "winattn_common.hpp"
#include "winattn_launch.hpp"

namespace aeris {
namespace {

constexpr int kTF = 256;                 // features per workgroup tile
constexpr int kTC = 256;                 // channels per workgroup tile
constexpr int kTM = 64;                  // token rows per step
constexpr int kWgradWaves = 8;
constexpr int kSubTileBytes = kTM * 128 * 2;          // [64 rows][128 columns] bf16
constexpr int kWgradStageBytes = 4 * kSubTileBytes;   // dy halves, then x halves
using Sub128 = Tile<128, kWgradWaves>;

struct WgradParams {
  const bf16_t* dy;            // [M, F]
  const bf16_t* x;             // [M, C]
  float* out;                  // [splits][F, C]
  int F, C;
  int f_tiles, c_tiles;
  int cu, f_groups, c_groups;  // a unit is (32 / cu) x cu tiles
  int splits;
  int steps_per_split, steps_total;      // steps of kTM rows
};

// Workgroup id -> (split, feature tile, channel tile).  Consecutive ids go to the eight XCDs in
// turn.  The 32 workgroups an XCD runs at a time form one unit: fu x cu output tiles of the
// same row range, so that each 64-row piece of dy or x that arrives in that XCD's L2 serves cu
// or fu workgroups which walk the rows together.
__device__ __forceinline__ bool wgrad_tile(const WgradParams& p, int& split, int& ft, int& ct) {
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int unit = (slot >> 5) * 8 + xcd, t = slot & 31;
  const int fu = 32 / p.cu;
  const int cg = unit % p.c_groups;
  const int rest = unit / p.c_groups;
  const int fg = rest % p.f_groups;
  split = rest / p.f_groups;
  ct = cg * p.cu + t % p.cu;
  ft = fg * fu + t / p.cu;
  return split < p.splits && ft < p.f_tiles && ct < p.c_tiles;
}
inline unsigned wgrad_grid(const WgradParams& p) {
  const unsigned units = (unsigned)p.splits * (unsigned)p.f_groups * (unsigned)p.c_groups;
  return ((units + 7) / 8) * 8 * 32;
}

__global__ __launch_bounds__(kWgradWaves * 64, 1) void linear_wgrad_kernel(WgradParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  int split, ft, ct;
  if (!wgrad_tile(p, split, ft, ct)) return;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wf = wave >> 2, wc = wave & 3;          // 2 x 4 waves: 128 features x 64 channels
  const int li = lane & 31, g = lane >> 5;
  const int f0 = ft * kTF, c0 = ct * kTC;
  const int s0 = split * p.steps_per_split;
  const int s1 = s0 + p.steps_per_split < p.steps_total ? s0 + p.steps_per_split : p.steps_total;

  // ---- copies: instruction j (0..63) moves rows 4(j % 16) .. +3 of sub-tile j / 16; wave w
  // issues j = w + 8i, i.e. sub-tile i / 2, rows 4(w + 8(i % 2)) ..  Lane: row + lane / 16, LDS
  // chunk position lane % 16, which holds source chunk position ^ swz(row).  Columns past the
  // end of a ragged last tile are clamped into the row (their products are never stored).
  uint32_t voff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int t = i >> 1;
    const int r = 4 * (wave + 8 * (i & 1)) + (lane >> 4);
    const int chunk = (lane & 15) ^ Sub128::swz(r);
    const int ld = t < 2 ? p.F : p.C;
    int col = (t < 2 ? f0 : c0) + 128 * (t & 1) + 8 * chunk;
    col = col < ld ? col : ld - 8;
    voff[i] = (uint32_t)(((long long)r * ld + col) * 2);
  }
  const unsigned long long dybase = reinterpret_cast<unsigned long long>(p.dy);
  const unsigned long long xbase = reinterpret_cast<unsigned long long>(p.x);
  const uint32_t lds0 = lds_address(smem);
  auto copy_piece = [&](int i, uint32_t stage, int step, uint32_t enable) __attribute__((always_inline)) {
    const unsigned long long row_bytes = (unsigned long long)(i < 4 ? p.F : p.C) * 2;
    async_copy16_off(voff[i], (i < 4 ? dybase : xbase) + (unsigned long long)step * kTM * row_bytes,
                     stage + (uint32_t)((i >> 1) * kSubTileBytes + ((wave + 8 * (i & 1)) << 10)),
                     enable);
  };

  // ---- transposing operand reads: per lane two addresses per 32-column block (rows 4g..4g+3
  // and 8+4g..8+4g+3 of a 16-row group; both operands use the same row order)
  uint32_t ta[4][2], tb[2][2];
  {
    const int j = lane & 15, blk = lane >> 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int r = 8 * h + 4 * (blk >> 1) + (j >> 2);
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int c = 4 * a + 2 * (blk & 1) + ((j & 3) >> 1);
        ta[a][h] = lds0 + wf * kSubTileBytes + Sub128::chunk_offset(r, c) + (j & 1) * 8;
      }
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int c = 4 * (2 * (wc & 1) + b) + 2 * (blk & 1) + ((j & 3) >> 1);
        tb[b][h] = lds0 + (2 + (wc >> 1)) * kSubTileBytes + Sub128::chunk_offset(r, c) + (j & 1) * 8;
      }
    }
  }

  f32x16 acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

#pragma unroll
  for (int i = 0; i < 8; ++i) copy_piece(i, lds0, s0, 1);

  bf16x8 ao[2][4], bo[2][2];
  auto fetch = [&](int set, int kk, uint32_t stage_off) __attribute__((always_inline)) {
    const uint32_t off = stage_off + kk * (16 * 256);
#pragma unroll
    for (int a = 0; a < 4; ++a) ao[set][a] = Sub128::read_tr(ta[a][0] + off, ta[a][1] + off);
#pragma unroll
    for (int b = 0; b < 2; ++b) bo[set][b] = Sub128::read_tr(tb[b][0] + off, tb[b][1] + off);
  };

  for (int ks = s0; ks < s1; ++ks) {
    const uint32_t stage_off = ((ks - s0) & 1) * kWgradStageBytes;
    wait_async_loads();
    __syncthreads();               // this stage has landed; every reader of the other one is done
    const uint32_t more = ks + 1 < s1;
    const uint32_t next_stage = lds0 + (kWgradStageBytes - stage_off);
    fetch(0, 0, stage_off);
    sched_fence();
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk < 3) fetch((kk + 1) & 1, kk + 1, stage_off);
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          acc[a][b] = mfma32(ao[kk & 1][a], bo[kk & 1][b], acc[a][b]);
          // the next stage's copies ride in the first half of the step, one per two products
          if (kk < 2 && (b & 1)) copy_piece(4 * kk + a, next_stage, ks + 1, more);
        }
      sched_fence();
    }
  }

  // ---- partial tile: a lane owns one channel column, a register one feature row
  float* out = p.out + (long long)split * p.F * p.C;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int c = c0 + wc * 64 + b * 32 + li;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int f = f0 + wf * 128 + a * 32 + acc_row(e, g);
        if (f < p.F && c < p.C) out[(long long)f * p.C + c] = acc[a][b][e];
      }
    }
}

// dW = sum of the partial tiles, in the order of the splits, plus the products of the last
// n_rows % 64 rows (`tail` rows starting at row `row0`), which the tile kernel does not take:
// at most 63 multiply-adds per element, in row order.  n4: number of 4-float groups of dW.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ part,
                                                           long long n4, int splits,
                                                           const bf16_t* __restrict__ dy,
                                                           const bf16_t* __restrict__ x,
                                                           long long row0, int tail, int F, int C,
                                                           float* __restrict__ dw) {
  const long long stride = (long long)gridDim.x * 256;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < splits; ++k) {
      const f32x4 v = reinterpret_cast<const f32x4*>(part)[(long long)k * n4 + i];
      s[0] += v[0]; s[1] += v[1]; s[2] += v[2]; s[3] += v[3];
    }
    if (tail) {
      const long long e = i * 4;
      const int f = (int)(e / C), c = (int)(e - (long long)f * C);
      for (int m = 0; m < tail; ++m) {
        const float d = (float)dy[(row0 + m) * F + f];
        const bf16x4 xv = *reinterpret_cast<const bf16x4*>(x + (row0 + m) * C + c);
        s[0] = __builtin_fmaf(d, (float)xv[0], s[0]);
        s[1] = __builtin_fmaf(d, (float)xv[1], s[1]);
        s[2] = __builtin_fmaf(d, (float)xv[2], s[2]);
        s[3] = __builtin_fmaf(d, (float)xv[3], s[3]);
      }
    }
    reinterpret_cast<f32x4*>(dw)[i] = s;
  }
}

// wt [C, F] = w [F, C]^T, bf16: 64 x 64 tiles through the LDS (row pitch 65 words apart in banks).
__global__ __launch_bounds__(256) void transpose_weight_kernel(const bf16_t* __restrict__ w, int F,
                                                               int C, bf16_t* __restrict__ wt) {
  __shared__ unsigned short tile[64][66];
  const int f0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const unsigned short* src = reinterpret_cast<const unsigned short*>(w);
  unsigned short* dst = reinterpret_cast<unsigned short*>(wt);
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;
    tile[r][c] = (f0 + r < F && c0 + c < C) ? src[(long long)(f0 + r) * C + c0 + c] : (unsigned short)0;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;               // r: channel, c: feature
    if (c0 + r < C && f0 + c < F) dst[(long long)(c0 + r) * F + f0 + c] = tile[c][r];
  }
}

size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }
bool bad16(const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) != 0; }

// How the rows are split for dW: enough workgroups to fill the chip several times over, but at
// least 16 steps each and at most 64 partial tiles per output tile; among the next few counts
// the one whose units (32 tiles, one XCD's worth) fill the eight XCDs most evenly.
struct Split {
  int steps_total, steps_per_split, splits;
  int cu, f_groups, c_groups;
};
Split choose_split(int64_t n_rows, int32_t channels, int32_t features) {
  Split s;
  s.steps_total = (int)(n_rows / kTM);
  const int f_tiles = (features + kTF - 1) / kTF, c_tiles = (channels + kTC - 1) / kTC;
  s.cu = c_tiles >= 8 ? 8 : (c_tiles >= 4 ? 4 : (c_tiles >= 2 ? 2 : 1));
  s.c_groups = (c_tiles + s.cu - 1) / s.cu;
  s.f_groups = (f_tiles + 32 / s.cu - 1) / (32 / s.cu);
  const long long tiles = (long long)f_tiles * c_tiles;
  long long want = (2048 + tiles - 1) / tiles;
  want = want < 1 ? 1 : (want > 64 ? 64 : want);
  auto layout = [&](long long target, int& per_out, int& splits_out) {
    long long per = (s.steps_total + target - 1) / target;
    per = per < 16 ? 16 : per;
    per_out = (int)per;
    splits_out = (int)((s.steps_total + per - 1) / per);    // 0 if there is no whole step
  };
  layout(want, s.steps_per_split, s.splits);
  double best = -1.0;
  for (long long target = want; target < want + 8 && target <= 64; ++target) {
    int per, splits;
    layout(target, per, splits);
    if (splits == 0) break;
    const long long units = (long long)splits * s.f_groups * s.c_groups;
    const double fill = (double)units / (double)(((units + 7) / 8) * 8);
    if (fill > best + 1e-9) {
      best = fill;
      s.steps_per_split = per;
      s.splits = splits;
    }
  }
  return s;
}
// whether the tile kernel can write dW itself: one row range and no rows left over
bool direct_dw(const Split& s, int64_t n_rows) { return s.splits == 1 && n_rows % kTM == 0; }

int check_linear_bwd(int64_t n_rows, int32_t channels, int32_t features) {
  if (n_rows <= 0 || channels <= 0 || features <= 0) return AERIS_ERR_INVALID_SHAPE;
  if (channels % 64 != 0 || features % 64 != 0) return AERIS_ERR_NOT_DIVISIBLE;
  if (n_rows / kTM >= (1LL << 31)) return AERIS_ERR_INVALID_SHAPE;
  // dx: the forward kernel with the roles of channels and features exchanged
  if (const int rc = projection_gemm_check(n_rows, n_rows, features, channels)) return rc;
  // dW: 32-bit byte offsets inside a 64-row step
  if ((long long)kTM * (features > channels ? features : channels) * 2 >= (1LL << 32))
    return AERIS_ERR_INVALID_SHAPE;
  return AERIS_OK;
}

}  // namespace
}  // namespace aeris

using namespace aeris;

extern "C" size_t aeris_linear_bwd_workspace_bytes(int64_t n_rows, int32_t channels,
                                                   int32_t out_features) {
  if (check_linear_bwd(n_rows, channels, out_features) != AERIS_OK) return 0;
  const Split s = choose_split(n_rows, channels, out_features);
  return round256((size_t)out_features * channels * 2) +
         (direct_dw(s, n_rows) ? 0 : round256((size_t)s.splits * out_features * channels * 4));
}

extern "C" int aeris_linear_bwd(const void* x, const void* weight, const void* dy, int64_t n_rows,
                                int32_t channels, int32_t out_features, void* dx, float* dweight,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!dy || !workspace || (!dx && !dweight) || (dx && !weight) || (dweight && !x))
    return AERIS_ERR_NULL_POINTER;
  if (const int rc = check_linear_bwd(n_rows, channels, out_features)) return rc;
  if (bad16(x) || bad16(weight) || bad16(dy) || bad16(dx) || bad16(dweight) || bad16(workspace))
    return AERIS_ERR_MISALIGNED;
  if (workspace_bytes < aeris_linear_bwd_workspace_bytes(n_rows, channels, out_features))
    return AERIS_ERR_WORKSPACE_TOO_SMALL;
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  bf16_t* wt = reinterpret_cast<bf16_t*>(ws);
  float* part = reinterpret_cast<float*>(ws + round256((size_t)out_features * channels * 2));

  if (dx) {
    if (launch_kernel(transpose_weight_kernel,
                      dim3((unsigned)(channels / 64), (unsigned)(out_features / 64)), dim3(256), 0,
                      st, static_cast<const bf16_t*>(weight), out_features, channels, wt) != 0)
      return AERIS_ERR_HIP_LAUNCH;
    GemmParams p{};
    p.x = static_cast<const bf16_t*>(dy);
    p.w = wt;
    p.y = static_cast<bf16_t*>(dx);
    p.rows_per_sample = n_rows;
    p.m_tiles = (int)((n_rows + 255) / 256);
    p.K = out_features;
    p.F = channels;
    p.n_tiles = (channels + 255) / 256;
    if (launch_projection_gemm(p, st) != 0) return AERIS_ERR_HIP_LAUNCH;
  }
  if (dweight) {
    const Split s = choose_split(n_rows, channels, out_features);
    WgradParams p{};
    p.dy = static_cast<const bf16_t*>(dy);
    p.x = static_cast<const bf16_t*>(x);
    const bool direct = direct_dw(s, n_rows);
    p.out = direct ? dweight : part;
    p.F = out_features;
    p.C = channels;
    p.f_tiles = (out_features + kTF - 1) / kTF;
    p.c_tiles = (channels + kTC - 1) / kTC;
    p.cu = s.cu;
    p.c_groups = s.c_groups;
    p.f_groups = s.f_groups;
    p.splits = s.splits;
    p.steps_per_split = s.steps_per_split;
    p.steps_total = s.steps_total;
    if (s.splits > 0) {
      if (!allow_full_lds<linear_wgrad_kernel>()) return AERIS_ERR_HIP_LAUNCH;
      if (launch_kernel(linear_wgrad_kernel, dim3(wgrad_grid(p)), dim3(kWgradWaves * 64),
                        (size_t)2 * kWgradStageBytes, st, p) != 0)
        return AERIS_ERR_HIP_LAUNCH;
    }
    if (!direct) {
      const long long n4 = (long long)out_features * channels / 4;
      const long long blocks = (n4 + 255) / 256;
      if (launch_kernel(wgrad_reduce_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)),
                        dim3(256), 0, st, static_cast<const float*>(part), n4, s.splits,
                        static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(x),
                        (long long)s.steps_total * kTM, (int)(n_rows % kTM), (int)out_features,
                        (int)channels, dweight) != 0)
        return AERIS_ERR_HIP_LAUNCH;
    }
  }
  return AERIS_OK;
}
