// Backward shifted-window attention for gfx950 ("forward and backward pass with
// BF16 activations", AERIS paper, Software Environment section; the gradient
// formulas are the ones listed in include/aeris_winattn.h).  P is recomputed
// from the saved log-sum-exp; nothing of size T x T touches memory.
//
// Three kernels, no atomics (bitwise reproducible):
//   delta   delta_i = sum_c dO_ic O_ic, and LSE_i * log2(e)   (HBM-bound pre-pass)
//   dq      queries resident, keys streamed:   S^T, dP^T -> dS^T -> dQ^T += K^T dS^T
//   dkdv    keys resident, queries streamed:   S, dP -> P, dS -> dV^T += dO^T P,
//                                                               dK^T += Q^T dS
// Both big kernels mirror the forward kernel: the resident side sits in MFMA B
// operands / accumulator columns (one token per lane pair); the streamed side
// goes through asynchronously filled LDS tiles, read row-major for the first
// products and through transposing reads for the second.
//
// Workspace layout (floats): [0, N) delta, [N, 2N) LSE*log2(e), N = B*heads*H*W,
// both indexed like LSE.
#include "winattn_common.hpp"
#include "winattn_launch.hpp"

namespace aeris {

constexpr float kLog2e = 1.4426950408889634f;

// ----------------------------------------------------------------------------
// delta[b, head, y, x] = sum_c dO * O.  One thread per 8 channels.
// ----------------------------------------------------------------------------
__device__ __forceinline__ void load8(const bf16_t* src, float* out) {
  const u32x4 r = *reinterpret_cast<const u32x4*>(src);
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    out[2 * w] = __uint_as_float(r[w] << 16);
    out[2 * w + 1] = __uint_as_float(r[w] & 0xffff0000u);
  }
}
__device__ __forceinline__ void load8(const float* src, float* out) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(src);
  const f32x4 b = *reinterpret_cast<const f32x4*>(src + 4);
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    out[w] = a[w];
    out[4 + w] = b[w];
  }
}

template <int D, typename OT>
__global__ __launch_bounds__(kThreads) void winattn_delta_kernel(
    KParams p, long long n_items, const OT* __restrict__ o, const bf16_t* __restrict__ d_o,
    const float* __restrict__ lse, float* __restrict__ delta, float* __restrict__ lse2) {
  constexpr int kChunks = D / 8;
  const long long plane = (long long)p.H * p.W;
  for (long long gid = (long long)blockIdx.x * kThreads + threadIdx.x; gid < n_items * kChunks;
       gid += (long long)gridDim.x * kThreads) {
    const int chunk = (int)(gid % kChunks);
    const long long item = gid / kChunks;       // (token, head), head fastest
    const int head = (int)(item % p.nh);
    const long long tok = item / p.nh;           // b * plane + y*W + x
    const long long off = tok * p.o_tok + (long long)head * p.o_head + chunk * 8;
    float a[8], b[8];
    load8(o + off, a);
    load8(d_o + off, b);
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc = __builtin_fmaf(a[i], b[i], acc);
#pragma unroll
    for (int s = 1; s < kChunks; s <<= 1) acc += __shfl_xor(acc, s);
    if (chunk == 0) {
      const long long bidx = tok / plane;
      const long long idx = (bidx * p.nh + head) * plane + (tok - bidx * plane);
      delta[idx] = acc;
      lse2[idx] = lse[idx] * kLog2e;
    }
  }
}

// ----------------------------------------------------------------------------
// dQ: same skeleton as the forward kernel.  LDS: table + 2 buffers x (K, V).
// ----------------------------------------------------------------------------
template <int D>
constexpr size_t dq_smem_bytes(int T) {
  return ((T * 4 + 15) & ~15) + 4 * Tile<D>::kBytes;
}

template <int D, typename OutT>
__global__ __launch_bounds__(kThreads, 2) void winattn_dq_kernel(
    KParams p, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o,
    const float* __restrict__ delta, const float* __restrict__ lse2v, OutT* __restrict__ dq) {
  using Tl = Tile<D>;
  extern __shared__ __align__(16) unsigned char smem[];
  int* tok_grid = reinterpret_cast<int*>(smem);
  const uint32_t tiles = lds_address(smem) + ((p.T * 4 + 15) & ~15);

  int pair, qt;
  if (!block_to_work(p, pair, qt)) return;

  Window win;
  win.init(p, pair);
  build_token_table(p, win, tok_grid);
  __syncthreads();

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qi = lane & 31, g = lane >> 5;
  const int T = p.T;
  const long long plane = (long long)p.H * p.W;
  const long long qkv_base = ((long long)win.b * plane) * p.qkv_tok + (long long)win.head * p.qkv_head;
  const long long o_base = ((long long)win.b * plane) * p.o_tok + (long long)win.head * p.o_head;
  const long long stat_base = ((long long)win.b * p.nh + win.head) * plane;
  const bf16_t* kb = k + qkv_base;
  const bf16_t* vb = v + qkv_base;

  Ranges rg;
  rg.init(win, qt, wave, qi);
  const int q_grid = tok_grid[rg.tok];
  const int lo_q = rg.lo, hi_q = rg.hi;

  const int kt_begin = rg.wg_lo / kStream;
  const int kt_end = (rg.wg_hi + kStream - 1) / kStream;
  Tl::fill_async(tiles, kb, p.qkv_tok, tok_grid, kt_begin * kStream, T, wave, lane);
  Tl::fill_async(tiles + Tl::kBytes, vb, p.qkv_tok, tok_grid, kt_begin * kStream, T, wave, lane);

  bf16x8 qreg[D / 16], doreg[D / 16];
  {
    const bf16_t* qrow = q + qkv_base + (long long)q_grid * p.qkv_tok + 8 * g;
    const bf16_t* dorow = d_o + o_base + (long long)q_grid * p.o_tok + 8 * g;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      qreg[kk] = *reinterpret_cast<const bf16x8*>(qrow + kk * 16);
      doreg[kk] = *reinterpret_cast<const bf16x8*>(dorow + kk * 16);
    }
  }
  float lse2 = lse2v[stat_base + q_grid];
  float delta_q = delta[stat_base + q_grid];
  typename Tl::Lanes la;
  la.init(lane);
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    settle(qreg[kk]);
    settle(doreg[kk]);
  }
  settle(lse2);
  settle(delta_q);

  f32x16 acc[D / 32];
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;

  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const uint32_t buf = tiles + ((kt - kt_begin) & 1) * (2 * Tl::kBytes);
    wait_async_loads();
    __syncthreads();
    if (kt + 1 < kt_end) {
      const uint32_t nxt = tiles + ((kt + 1 - kt_begin) & 1) * (2 * Tl::kBytes);
      Tl::fill_async(nxt, kb, p.qkv_tok, tok_grid, (kt + 1) * kStream, T, wave, lane);
      Tl::fill_async(nxt + Tl::kBytes, vb, p.qkv_tok, tok_grid, (kt + 1) * kStream, T, wave, lane);
    }
    if (!rg.wave_active) continue;
#pragma unroll
    for (int kb2 = 0; kb2 < kStream / 32; ++kb2) {
      const int sub_lo = kt * kStream + kb2 * 32;
      if (rg.skip(sub_lo)) continue;
      const uint32_t ksub = buf + kb2 * Tl::kSubBytes;
      const uint32_t vsub = buf + Tl::kBytes + kb2 * Tl::kSubBytes;
      f32x16 s, dp;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        s = mfma32(Tl::read_rm(ksub + la.rm[kk]), qreg[kk], s);
        dp = mfma32(Tl::read_rm(vsub + la.rm[kk]), doreg[kk], dp);
      }
      if (!rg.mask_free(sub_lo)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kidx = sub_lo + acc_row(i, g);
          if (kidx < lo_q || kidx >= hi_q) s[i] = -INFINITY;
        }
      }
      float ds[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], p.scale_log2, -lse2));
        ds[i] = pr * (dp[i] - delta_q);
      }
      union { u32x4 u; bf16x8 h; } dsb[2];
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) dsb[c].u[e] = pack_bf16(ds[8 * c + 2 * e], ds[8 * c + 2 * e + 1]);
#pragma unroll
      for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const uint32_t grp = ksub + c * (16 * D * 2);
          acc[cb] = mfma32(Tl::read_tr(grp + la.tr[cb][0], grp + la.tr[cb][1]), dsb[c].h, acc[cb]);
        }
    }
  }

  if (!rg.valid) return;
  OutT* row = dq + qkv_base + (long long)q_grid * p.qkv_tok;
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int vq = 0; vq < 4; ++vq)
      store4(row + cb * 32 + 8 * vq + 4 * g, acc[cb][4 * vq] * p.scale,
             acc[cb][4 * vq + 1] * p.scale, acc[cb][4 * vq + 2] * p.scale,
             acc[cb][4 * vq + 3] * p.scale);
}

// ----------------------------------------------------------------------------
// dK, dV: keys resident (one per lane pair), queries streamed.
// LDS: table + 2 buffers x (Q tile, dO tile, 64 x LSE*log2e, 64 x delta).
// ----------------------------------------------------------------------------
template <int D>
constexpr size_t dkdv_smem_bytes(int T) {
  return ((T * 4 + 15) & ~15) + 2 * (2 * Tile<D>::kBytes + 2 * kStream * 4);
}

template <int D, typename OutT>
__global__ __launch_bounds__(kThreads, 1) void winattn_dkdv_kernel(
    KParams p, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o,
    const float* __restrict__ delta, const float* __restrict__ lse2v, OutT* __restrict__ dk,
    OutT* __restrict__ dv) {
  using Tl = Tile<D>;
  constexpr uint32_t kBufBytes = 2 * Tl::kBytes + 2 * kStream * 4;
  extern __shared__ __align__(16) unsigned char smem[];
  int* tok_grid = reinterpret_cast<int*>(smem);
  const uint32_t tiles = lds_address(smem) + ((p.T * 4 + 15) & ~15);

  int pair, kt;
  if (!block_to_work(p, pair, kt)) return;

  Window win;
  win.init(p, pair);
  build_token_table(p, win, tok_grid);
  __syncthreads();

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ki = lane & 31, g = lane >> 5;
  const int T = p.T;
  const long long plane = (long long)p.H * p.W;
  const long long qkv_base = ((long long)win.b * plane) * p.qkv_tok + (long long)win.head * p.qkv_head;
  const long long o_base = ((long long)win.b * plane) * p.o_tok + (long long)win.head * p.o_head;
  const long long stat_base = ((long long)win.b * p.nh + win.head) * plane;
  const bf16_t* qb = q + qkv_base;
  const bf16_t* dob = d_o + o_base;

  Ranges rg;
  rg.init(win, kt, wave, ki);
  const int k_grid = tok_grid[rg.tok];
  const int lo_k = rg.lo, hi_k = rg.hi;

  // one streamed tile: Q, dO (all waves), LSE*log2e (wave 0), delta (wave 1)
  auto fill = [&](uint32_t buf, int t0) {
    Tl::fill_async(buf, qb, p.qkv_tok, tok_grid, t0, T, wave, lane);
    Tl::fill_async(buf + Tl::kBytes, dob, p.o_tok, tok_grid, t0, T, wave, lane);
    if (wave < 2) {
      int t = t0 + lane;
      t = t < T ? t : T - 1;
      const float* src = (wave == 0 ? lse2v : delta) + stat_base + tok_grid[t];
      async_copy4(src, buf + 2 * Tl::kBytes + wave * (kStream * 4));
    }
  };

  const int qt_begin = rg.wg_lo / kStream;
  const int qt_end = (rg.wg_hi + kStream - 1) / kStream;
  fill(tiles, qt_begin * kStream);

  bf16x8 kreg[D / 16], vreg[D / 16];
  {
    const bf16_t* krow = k + qkv_base + (long long)k_grid * p.qkv_tok + 8 * g;
    const bf16_t* vrow = v + qkv_base + (long long)k_grid * p.qkv_tok + 8 * g;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      kreg[kk] = *reinterpret_cast<const bf16x8*>(krow + kk * 16);
      vreg[kk] = *reinterpret_cast<const bf16x8*>(vrow + kk * 16);
    }
  }
  typename Tl::Lanes la;
  la.init(lane);
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    settle(kreg[kk]);
    settle(vreg[kk]);
  }

  f32x16 dkacc[D / 32], dvacc[D / 32];
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dkacc[cb][i] = 0.f; dvacc[cb][i] = 0.f; }

  for (int qt = qt_begin; qt < qt_end; ++qt) {
    const uint32_t buf = tiles + ((qt - qt_begin) & 1) * kBufBytes;
    wait_async_loads();
    __syncthreads();
    if (qt + 1 < qt_end) fill(tiles + ((qt + 1 - qt_begin) & 1) * kBufBytes, (qt + 1) * kStream);
    if (!rg.wave_active) continue;
    const uint32_t stat = buf + 2 * Tl::kBytes;
#pragma unroll
    for (int qb2 = 0; qb2 < kStream / 32; ++qb2) {
      const int sub_lo = qt * kStream + qb2 * 32;
      if (rg.skip(sub_lo)) continue;
      const uint32_t qsub = buf + qb2 * Tl::kSubBytes;
      const uint32_t dosub = buf + Tl::kBytes + qb2 * Tl::kSubBytes;
      // S[query, key] = Q K^T,  dP[query, key] = dO V^T: rows = streamed queries
      f32x16 s, dp;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        s = mfma32(Tl::read_rm(qsub + la.rm[kk]), kreg[kk], s);
        dp = mfma32(Tl::read_rm(dosub + la.rm[kk]), vreg[kk], dp);
      }
      if (!rg.mask_free(sub_lo)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int qidx = sub_lo + acc_row(i, g);
          if (qidx < lo_k || qidx >= hi_k) s[i] = -INFINITY;
        }
      }
      float pr[16], ds[16];
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const uint32_t at = stat + (qb2 * 32 + 8 * vq + 4 * g) * 4;
        const f32x4 l4 = *reinterpret_cast<const AERIS_LDS f32x4*>(at);
        const f32x4 d4 = *reinterpret_cast<const AERIS_LDS f32x4*>(at + kStream * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * vq + e;
          pr[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], p.scale_log2, -l4[e]));
          ds[i] = pr[i] * (dp[i] - d4[e]);
        }
      }
      union { u32x4 u; bf16x8 h; } pb[2], dsb[2];
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          pb[c].u[e] = pack_bf16(pr[8 * c + 2 * e], pr[8 * c + 2 * e + 1]);
          dsb[c].u[e] = pack_bf16(ds[8 * c + 2 * e], ds[8 * c + 2 * e + 1]);
        }
#pragma unroll
      for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const uint32_t off = c * (16 * D * 2);
          dvacc[cb] = mfma32(Tl::read_tr(dosub + off + la.tr[cb][0], dosub + off + la.tr[cb][1]),
                             pb[c].h, dvacc[cb]);
          dkacc[cb] = mfma32(Tl::read_tr(qsub + off + la.tr[cb][0], qsub + off + la.tr[cb][1]),
                             dsb[c].h, dkacc[cb]);
        }
    }
  }

  if (!rg.valid) return;
  OutT* dkrow = dk + qkv_base + (long long)k_grid * p.qkv_tok;
  OutT* dvrow = dv + qkv_base + (long long)k_grid * p.qkv_tok;
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const int ch = cb * 32 + 8 * vq + 4 * g;
      store4(dkrow + ch, dkacc[cb][4 * vq] * p.scale, dkacc[cb][4 * vq + 1] * p.scale,
             dkacc[cb][4 * vq + 2] * p.scale, dkacc[cb][4 * vq + 3] * p.scale);
      store4(dvrow + ch, dvacc[cb][4 * vq], dvacc[cb][4 * vq + 1], dvacc[cb][4 * vq + 2],
             dvacc[cb][4 * vq + 3]);
    }
}

template <typename K>
static bool allow_smem(K kern, size_t smem) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                             hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)smem) == hipSuccess;
}

template <int D, typename OutT>
static int launch_bwd_t(const KParams& kp, const void* q, const void* k, const void* v,
                        const void* o, const float* lse, const void* d_o, void* dq, void* dk,
                        void* dv, float* workspace, hipStream_t stream, unsigned stages) {
  const bf16_t* qp = static_cast<const bf16_t*>(q);
  const bf16_t* kp_ = static_cast<const bf16_t*>(k);
  const bf16_t* vp = static_cast<const bf16_t*>(v);
  const bf16_t* dop = static_cast<const bf16_t*>(d_o);

  const long long n_items = (long long)kp.B * kp.H * kp.W * kp.nh;
  float* delta = workspace;
  float* lse2 = workspace + n_items;
  if (stages & 1u) {
    const long long n_thr = n_items * (D / 8);
    long long dblocks = (n_thr + kThreads - 1) / kThreads;
    if (dblocks > 256 * 64) dblocks = 256 * 64;
    hipLaunchKernelGGL((winattn_delta_kernel<D, OutT>), dim3((unsigned)dblocks), dim3(kThreads),
                       0, stream, kp, n_items, static_cast<const OutT*>(o), dop, lse, delta, lse2);
    if (hipGetLastError() != hipSuccess) return -1;
  }

  const int n_blocks = grid_blocks(kp);
  if (stages & 2u) {
    const size_t smem = dq_smem_bytes<D>(kp.T);
    auto kern = winattn_dq_kernel<D, OutT>;
    if (!allow_smem(kern, smem)) return -1;
    hipLaunchKernelGGL(kern, dim3(n_blocks), dim3(kThreads), smem, stream, kp, qp, kp_, vp, dop,
                       static_cast<const float*>(delta), static_cast<const float*>(lse2),
                       static_cast<OutT*>(dq));
    if (hipGetLastError() != hipSuccess) return -1;
  }
  if (stages & 4u) {
    const size_t smem = dkdv_smem_bytes<D>(kp.T);
    auto kern = winattn_dkdv_kernel<D, OutT>;
    if (!allow_smem(kern, smem)) return -1;
    hipLaunchKernelGGL(kern, dim3(n_blocks), dim3(kThreads), smem, stream, kp, qp, kp_, vp, dop,
                       static_cast<const float*>(delta), static_cast<const float*>(lse2),
                       static_cast<OutT*>(dk), static_cast<OutT*>(dv));
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

int launch_bwd(const KParams& kp, int head_dim, bool out_f32, const void* q, const void* k,
               const void* v, const void* o, const float* lse, const void* d_o, void* dq,
               void* dk, void* dv, float* workspace, hipStream_t stream, unsigned stages) {
#define AERIS_BWD_CASE(DD)                                                                    \
  case DD:                                                                                    \
    return out_f32 ? launch_bwd_t<DD, float>(kp, q, k, v, o, lse, d_o, dq, dk, dv, workspace, \
                                             stream, stages)                                  \
                   : launch_bwd_t<DD, bf16_t>(kp, q, k, v, o, lse, d_o, dq, dk, dv,           \
                                              workspace, stream, stages);
  switch (head_dim) {
    AERIS_BWD_CASE(32)
    AERIS_BWD_CASE(64)
    AERIS_BWD_CASE(128)
  }
#undef AERIS_BWD_CASE
  return -1;
}

}  // namespace aeris
