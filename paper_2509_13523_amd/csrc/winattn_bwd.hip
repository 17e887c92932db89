// Backward shifted-window attention for gfx950 ("forward and backward pass with
// BF16 activations", AERIS paper, Software Environment section; the gradient
// formulas are the ones listed in include/aeris_winattn.h).  P is recomputed
// from the saved log-sum-exp; nothing of size T x T touches memory.
//
// Three kernels, no atomics (bitwise reproducible):
//   delta   delta_i = sum_c dO_ic O_ic                       (HBM-bound pre-pass)
//   dq      queries resident, keys streamed:   S^T, dP^T -> dS^T -> dQ^T += K^T dS^T
//   dkdv    keys resident, queries streamed:   S, dP -> P, dS -> dV^T += dO^T P,
//                                                               dK^T += Q^T dS
// Both big kernels mirror the forward kernel: the resident side sits in MFMA B
// operands / accumulator columns (one token per lane pair), the streamed side
// goes through LDS row-major (first products) and transposed (second products).
#include "winattn_common.hpp"
#include "winattn_launch.hpp"

namespace aeris {

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
    float* __restrict__ delta) {
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
      delta[(bidx * p.nh + head) * plane + (tok - bidx * plane)] = acc;
    }
  }
}

// ----------------------------------------------------------------------------
// dQ: same skeleton as the forward kernel.
// ----------------------------------------------------------------------------
template <int D, typename OutT>
__global__ __launch_bounds__(kThreads, 2) void winattn_dq_kernel(
    KParams p, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o, const float* __restrict__ lse,
    const float* __restrict__ delta, OutT* __restrict__ dq) {
  using St = Stage<D>;
  extern __shared__ __align__(16) unsigned char smem[];
  int* tok_grid = reinterpret_cast<int*>(smem);
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem + ((p.T * 4 + 15) & ~15));
  bf16_t* Vs = Ks + St::kRowTile;
  bf16_t* Kt = Vs + St::kRowTile;

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
  const float lse2 = lse[stat_base + q_grid] * 1.4426950408889634f;
  const float delta_q = delta[stat_base + q_grid];

  f32x16 acc[D / 32];
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;

  const int kt_begin = rg.wg_lo / kStream;
  const int kt_end = (rg.wg_hi + kStream - 1) / kStream;
  St kst, vst;
  kst.load(kb, p.qkv_tok, tok_grid, kt_begin * kStream, T);
  vst.load(vb, p.qkv_tok, tok_grid, kt_begin * kStream, T);

  for (int kt = kt_begin; kt < kt_end; ++kt) {
    if (kt != kt_begin) __syncthreads();
    kst.store_rowmajor(Ks);
    kst.store_transposed(Kt);
    vst.store_rowmajor(Vs);
    __syncthreads();
    if (kt + 1 < kt_end) {
      kst.load(kb, p.qkv_tok, tok_grid, (kt + 1) * kStream, T);
      vst.load(vb, p.qkv_tok, tok_grid, (kt + 1) * kStream, T);
    }
    if (!rg.wave_active) continue;
#pragma unroll
    for (int kb2 = 0; kb2 < kStream / 32; ++kb2) {
      const int sub_lo = kt * kStream + kb2 * 32;
      if (rg.skip(sub_lo)) continue;
      f32x16 s, dp;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
      const bf16_t* krow = Ks + (kb2 * 32 + qi) * St::kRowStride + 8 * g;
      const bf16_t* vrow = Vs + (kb2 * 32 + qi) * St::kRowStride + 8 * g;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        s = mfma32(*reinterpret_cast<const bf16x8*>(krow + kk * 16), qreg[kk], s);
        dp = mfma32(*reinterpret_cast<const bf16x8*>(vrow + kk * 16), doreg[kk], dp);
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
      const bf16_t* ktrow = Kt + qi * St::kTrStride + kb2 * 32 + 8 * g;
#pragma unroll
      for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
        for (int c = 0; c < 2; ++c)
          acc[cb] = mfma32(
              *reinterpret_cast<const bf16x8*>(ktrow + cb * 32 * St::kTrStride + 16 * c),
              dsb[c].h, acc[cb]);
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
// ----------------------------------------------------------------------------
template <int D, typename OutT>
__global__ __launch_bounds__(kThreads, 1) void winattn_dkdv_kernel(
    KParams p, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o, const float* __restrict__ lse,
    const float* __restrict__ delta, OutT* __restrict__ dk, OutT* __restrict__ dv) {
  using St = Stage<D>;
  extern __shared__ __align__(16) unsigned char smem[];
  int* tok_grid = reinterpret_cast<int*>(smem);
  float* stat = reinterpret_cast<float*>(smem + ((p.T * 4 + 15) & ~15));  // lse2[64], delta[64]
  bf16_t* Qs = reinterpret_cast<bf16_t*>(stat + 2 * kStream);
  bf16_t* dOs = Qs + St::kRowTile;
  bf16_t* Qt = dOs + St::kRowTile;
  bf16_t* dOt = Qt + St::kTrTile;

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

  f32x16 dkacc[D / 32], dvacc[D / 32];
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dkacc[cb][i] = 0.f; dvacc[cb][i] = 0.f; }

  const int qt_begin = rg.wg_lo / kStream;
  const int qt_end = (rg.wg_hi + kStream - 1) / kStream;
  St qst, dost;
  float stat_reg = 0.f;
  auto load_stat = [&](int t0) {
    if (tid < 2 * kStream) {
      int t = t0 + (tid & (kStream - 1));
      t = t < T ? t : T - 1;
      const long long idx = stat_base + tok_grid[t];
      stat_reg = tid < kStream ? lse[idx] * 1.4426950408889634f : delta[idx];
    }
  };
  qst.load(qb, p.qkv_tok, tok_grid, qt_begin * kStream, T);
  dost.load(dob, p.o_tok, tok_grid, qt_begin * kStream, T);
  load_stat(qt_begin * kStream);

  for (int qt = qt_begin; qt < qt_end; ++qt) {
    if (qt != qt_begin) __syncthreads();
    qst.store_rowmajor(Qs);
    qst.store_transposed(Qt);
    dost.store_rowmajor(dOs);
    dost.store_transposed(dOt);
    if (tid < 2 * kStream) stat[tid] = stat_reg;
    __syncthreads();
    if (qt + 1 < qt_end) {
      qst.load(qb, p.qkv_tok, tok_grid, (qt + 1) * kStream, T);
      dost.load(dob, p.o_tok, tok_grid, (qt + 1) * kStream, T);
      load_stat((qt + 1) * kStream);
    }
    if (!rg.wave_active) continue;
#pragma unroll
    for (int qb2 = 0; qb2 < kStream / 32; ++qb2) {
      const int sub_lo = qt * kStream + qb2 * 32;
      if (rg.skip(sub_lo)) continue;
      // S[query, key] = Q K^T,  dP[query, key] = dO V^T: rows = streamed queries
      f32x16 s, dp;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
      const bf16_t* qrow = Qs + (qb2 * 32 + ki) * St::kRowStride + 8 * g;
      const bf16_t* dorow = dOs + (qb2 * 32 + ki) * St::kRowStride + 8 * g;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        s = mfma32(*reinterpret_cast<const bf16x8*>(qrow + kk * 16), kreg[kk], s);
        dp = mfma32(*reinterpret_cast<const bf16x8*>(dorow + kk * 16), vreg[kk], dp);
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
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(stat + qb2 * 32 + 8 * vq + 4 * g);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(stat + kStream + qb2 * 32 + 8 * vq + 4 * g);
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
      const bf16_t* qtrow = Qt + ki * St::kTrStride + qb2 * 32 + 8 * g;
      const bf16_t* dotrow = dOt + ki * St::kTrStride + qb2 * 32 + 8 * g;
#pragma unroll
      for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          dvacc[cb] = mfma32(
              *reinterpret_cast<const bf16x8*>(dotrow + cb * 32 * St::kTrStride + 16 * c),
              pb[c].h, dvacc[cb]);
          dkacc[cb] = mfma32(
              *reinterpret_cast<const bf16x8*>(qtrow + cb * 32 * St::kTrStride + 16 * c),
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

template <int D, typename OutT>
static int launch_bwd_t(const KParams& kp, const void* q, const void* k, const void* v,
                        const void* o, const float* lse, const void* d_o, void* dq, void* dk,
                        void* dv, float* delta, hipStream_t stream, unsigned stages) {
  using St = Stage<D>;
  const bf16_t* qp = static_cast<const bf16_t*>(q);
  const bf16_t* kp_ = static_cast<const bf16_t*>(k);
  const bf16_t* vp = static_cast<const bf16_t*>(v);
  const bf16_t* dop = static_cast<const bf16_t*>(d_o);

  const long long n_items = (long long)kp.B * kp.H * kp.W * kp.nh;
  const long long n_thr = n_items * (D / 8);
  long long dblocks = (n_thr + kThreads - 1) / kThreads;
  if (dblocks > 256 * 64) dblocks = 256 * 64;
  if (stages & 1u) {
    hipLaunchKernelGGL((winattn_delta_kernel<D, OutT>), dim3((unsigned)dblocks), dim3(kThreads),
                       0, stream, kp, n_items, static_cast<const OutT*>(o), dop, delta);
    if (hipGetLastError() != hipSuccess) return -1;
  }

  const int n_blocks = grid_blocks(kp);
  const size_t tab = (kp.T * 4 + 15) & ~15;
  if (stages & 2u) {
    const size_t smem = tab + (2 * St::kRowTile + St::kTrTile) * sizeof(bf16_t);
    auto kern = winattn_dq_kernel<D, OutT>;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return -1;
    hipLaunchKernelGGL(kern, dim3(n_blocks), dim3(kThreads), smem, stream, kp, qp, kp_,
                       vp, dop, lse, static_cast<const float*>(delta), static_cast<OutT*>(dq));
    if (hipGetLastError() != hipSuccess) return -1;
  }
  if (stages & 4u) {
    const size_t smem = tab + 2 * kStream * sizeof(float) +
                        (2 * St::kRowTile + 2 * St::kTrTile) * sizeof(bf16_t);
    auto kern = winattn_dkdv_kernel<D, OutT>;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return -1;
    hipLaunchKernelGGL(kern, dim3(n_blocks), dim3(kThreads), smem, stream, kp, qp, kp_,
                       vp, dop, lse, static_cast<const float*>(delta), static_cast<OutT*>(dk),
                       static_cast<OutT*>(dv));
    if (hipGetLastError() != hipSuccess) return -1;
  }
  return 0;
}

int launch_bwd(const KParams& kp, int head_dim, bool out_f32, const void* q, const void* k,
               const void* v, const void* o, const float* lse, const void* d_o, void* dq,
               void* dk, void* dv, float* delta, hipStream_t stream, unsigned stages) {
#define AERIS_BWD_CASE(DD)                                                                     \
  case DD:                                                                                     \
    return out_f32                                                                             \
               ? launch_bwd_t<DD, float>(kp, q, k, v, o, lse, d_o, dq, dk, dv, delta, stream,  \
                                         stages)                                        \
               : launch_bwd_t<DD, bf16_t>(kp, q, k, v, o, lse, d_o, dq, dk, dv, delta, stream,  \
                                          stages);
  switch (head_dim) {
    AERIS_BWD_CASE(32)
    AERIS_BWD_CASE(64)
    AERIS_BWD_CASE(128)
  }
#undef AERIS_BWD_CASE
  return -1;
}

}  // namespace aeris
