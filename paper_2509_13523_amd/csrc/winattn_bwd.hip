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
// Workspace (floats): two vectors of n_pairs * T + 64 entries, delta first, then
// LSE * log2(e); both in WINDOW order -- entry pair * T + t belongs to token t of
// that (batch, window, head) in the kernels' token enumeration -- so the
// statistics of a streamed tile are 64 consecutive floats.
#include "winattn_common.hpp"
#include "winattn_launch.hpp"

namespace aeris {

__host__ __device__ inline long long stat_entries(const KParams& p) {
  return (long long)p.n_pairs * p.T + kStream;
}

// ----------------------------------------------------------------------------
// delta and LSE*log2e in window order.  One thread per 8 channels of one token
// of one (batch, window, head); the D/8 threads of a token reduce by shuffles.
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
    KParams p, const OT* __restrict__ o, const bf16_t* __restrict__ d_o,
    const float* __restrict__ lse, float* __restrict__ delta, float* __restrict__ lse2) {
  constexpr int kChunks = D / 8;
  constexpr int kTokens = kThreads / kChunks;   // tokens per workgroup
  const int blocks_per_pair = (p.T + kTokens - 1) / kTokens;
  const int pair = blockIdx.x / blocks_per_pair;
  const int t = (blockIdx.x - pair * blocks_per_pair) * kTokens + threadIdx.x / kChunks;
  const int chunk = threadIdx.x % kChunks;
  if (blockIdx.x == 0 && threadIdx.x < kStream) {
    // padding behind the last pair: streamed tiles read up to 63 entries past a window's end
    delta[(long long)p.n_pairs * p.T + threadIdx.x] = 0.f;
    lse2[(long long)p.n_pairs * p.T + threadIdx.x] = 0.f;
  }
  if (t >= p.T) return;   // whole token groups leave together (kChunks divides 64)
  Window win;
  if (!win.init(p, pair)) {
    // a skipped window still gets finite statistics: the streamed tiles of the pair before
    // it read up to 63 entries past their own end
    if (chunk == 0) {
      delta[(long long)pair * p.T + t] = 0.f;
      lse2[(long long)pair * p.T + t] = 0.f;
    }
    return;
  }
  const long long plane = (long long)p.H * p.W;
  const int g = win.grid_index(p, t);
  const long long off = ((long long)win.b * plane + g) * p.o_tok + (long long)win.head * p.o_head +
                        chunk * 8;
  float a[8], b[8];
  load8(o + off, a);
  load8(d_o + off, b);
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) acc = __builtin_fmaf(a[i], b[i], acc);
#pragma unroll
  for (int s = 1; s < kChunks; s <<= 1) acc += __shfl_xor(acc, s);
  if (chunk == 0) {
    const long long idx = (long long)pair * p.T + t;
    delta[idx] = acc;
    lse2[idx] = lse[((long long)win.b * p.nh + win.head) * plane + g] * kLog2e;
  }
}

// ----------------------------------------------------------------------------
// dQ: same skeleton as the forward kernel.  LDS: table + 2 buffers x (K, V).
// ----------------------------------------------------------------------------
template <int D>
constexpr size_t dq_smem_bytes(int T) {
  return table_bytes(T) + 4 * Tile<D>::kBytes;
}

template <int D, typename OutT>
__global__ __launch_bounds__(kThreads, 2) void winattn_dq_kernel(
    KParams p, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o, const OutT* __restrict__ o,
    const float* __restrict__ lse, float* __restrict__ delta, float* __restrict__ lse2v,
    OutT* __restrict__ dq, int make_stats) {
  // make_stats != 0: this kernel computes delta and LSE*log2e of its resident queries itself
  // (bit for bit what winattn_delta_kernel computes) and leaves them in the workspace for the
  // dK/dV kernel, so the separate pass over O and dO is not needed; otherwise it reads them.
  using Tl = Tile<D>;
  constexpr uint32_t kBuf = 2 * Tl::kBytes;   // one buffer: K tile, V tile
  extern __shared__ __align__(16) unsigned char smem[];
  int* tok_grid = reinterpret_cast<int*>(smem);
  const uint32_t table = lds_address(smem);
  const uint32_t tiles = table + table_bytes(p.T);

  int pair, qt;
  if (!block_to_work(p, pair, qt)) return;

  if (make_stats && blockIdx.x == 0 && threadIdx.x < kStream) {
    // padding behind the last pair: streamed tiles read up to 63 entries past a window's end
    delta[(long long)p.n_pairs * p.T + threadIdx.x] = 0.f;
    lse2v[(long long)p.n_pairs * p.T + threadIdx.x] = 0.f;
  }
  Window win;
  if (!win.init(p, pair)) {
    // a skipped window still gets finite statistics (see winattn_delta_kernel)
    const int t = qt * kResident + (int)threadIdx.x;
    if (make_stats && threadIdx.x < kResident && t < p.T) {
      delta[(long long)pair * p.T + t] = 0.f;
      lse2v[(long long)pair * p.T + t] = 0.f;
    }
    return;
  }
  build_token_table(p, win, tok_grid);
  __syncthreads();

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qi = lane & 31, g = lane >> 5;
  const long long plane = (long long)p.H * p.W;
  const long long qkv_base = ((long long)win.b * plane) * p.qkv_tok + (long long)win.head * p.qkv_head;
  const long long q_base = ((long long)win.b * plane) * p.q_tok + (long long)win.head * p.q_head;
  const long long k_base = ((long long)win.b * plane) * p.k_tok + (long long)win.head * p.k_head;
  const long long o_base = ((long long)win.b * plane) * p.o_tok + (long long)win.head * p.o_head;

  Ranges rg;
  rg.init(win, qt, wave, qi);
  const int q_grid = tok_grid[rg.tok];
  const int lo_q = rg.lo, hi_q = rg.hi;

  const int kt_begin = rg.wg_lo / kStream;
  const int kt_end = (rg.wg_hi + kStream - 1) / kStream;
  typename Tl::Rows rows;
  typename Tl::Filler kfill, vfill;
  rows.init(table, wave, lane);
  kfill.init(k + k_base, p.k_tok, wave, lane);
  vfill.init(v + qkv_base, p.qkv_tok, wave, lane);
  rows.prepare(kt_begin * kStream);
  kfill.issue(tiles, rows);
  vfill.issue(tiles + Tl::kBytes, rows);
  if (kt_begin + 1 < kt_end) rows.prepare((kt_begin + 1) * kStream);

  bf16x8 qreg[D / 16], doreg[D / 16];
  {
    const bf16_t* qrow = q + q_base + (long long)q_grid * p.q_tok + 8 * g;
    const bf16_t* dorow = d_o + o_base + (long long)q_grid * p.o_tok + 8 * g;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      qreg[kk] = *reinterpret_cast<const bf16x8*>(qrow + kk * 16);
      doreg[kk] = *reinterpret_cast<const bf16x8*>(dorow + kk * 16);
    }
  }
  float lse2, delta_q;
  if (make_stats) {
    // delta = sum_c dO*O with the summation tree of winattn_delta_kernel: an fma chain over
    // the 8 channels of a chunk, then pairwise over the chunk index (bit 0 first).  This lane
    // holds chunks 2*kk + g; the partner lane (l ^ 32) holds the other chunk of every pair.
    const OutT* orow = o + o_base + (long long)q_grid * p.o_tok + 8 * g;
    float part[D / 16];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      float a[8];
      load8(orow + kk * 16, a);
      float acc1 = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc1 = __builtin_fmaf(a[i], (float)doreg[kk][i], acc1);
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc1), __float_as_uint(acc1),
                                                       false, false);
      part[kk] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);   // chunk 2kk + chunk 2kk+1
    }
#pragma unroll
    for (int s2 = 1; s2 < D / 16; s2 <<= 1)
#pragma unroll
      for (int kk = 0; kk < D / 16; kk += 2 * s2) part[kk] += part[kk + s2];
    delta_q = part[0];
    lse2 = lse[((long long)win.b * p.nh + win.head) * plane + q_grid] * kLog2e;
    if (rg.valid && g == 0) {
      delta[(long long)pair * p.T + rg.tok] = delta_q;
      lse2v[(long long)pair * p.T + rg.tok] = lse2;
    }
  } else {
    lse2 = lse2v[(long long)pair * p.T + rg.tok];
    delta_q = delta[(long long)pair * p.T + rg.tok];
  }
  typename Tl::Lanes la;
  la.init(tiles, lane);
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

  // Schedule of one 32-key block, as in the forward kernel (LDS offsets are compile-time
  // constants):
  //   logits phase   2*D/16 products S^T = K Q^T, dP^T = V dO^T.  Their operands pass through
  //                  a window of kWin contraction blocks: the first kWin were fetched during
  //                  the previous block's output phase, block kk + kWin is fetched right after
  //                  the products of block kk; copies of the next tile are issued in between;
  //   vector phase   K^T operands of this block are fetched (transposing reads), then
  //                  P = exp2(S - LSE), dS = P o (dP - delta), rounded to bf16;
  //   output phase   D/16 products dQ^T += K^T dS^T, with the first kWin operand blocks of the
  //                  NEXT block fetched and further copies issued in between.
  constexpr int kNK = D / 16;
  constexpr int kWin = kNK < 4 ? kNK : 4;
  constexpr int kF = Tl::kFillPerWave;
  bf16x8 ka[kNK], va[kNK], kta[D / 32][2];
  f32x16 sacc, dpacc;
  union { u32x4 u; bf16x8 h; } dsb[2];

  auto fetch_rows = [&](auto off, int kk) __attribute__((always_inline)) {
    constexpr uint32_t kOff = decltype(off)::value;
    ka[kk] = Tl::read_rm(la.rm[kk] + kOff);
    va[kk] = Tl::read_rm(la.rm[kk] + kOff + Tl::kBytes);
  };
  auto fetch_first = [&](auto off) __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < kWin; ++kk) fetch_rows(off, kk);
  };
  // en: non-zero if the copies are wanted (wave-uniform)
  auto logits_phase = [&](auto off, auto with_fill, const typename Tl::Filler& fill,
                          uint32_t fill_tile, uint32_t en) __attribute__((always_inline)) {
    constexpr bool kFill = decltype(with_fill)::value != 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
    sched_fence();
#pragma unroll
    for (int kk = 0; kk < kNK; ++kk) {
      sacc = mfma32(ka[kk], qreg[kk], sacc);
      dpacc = mfma32(va[kk], doreg[kk], dpacc);
      if (kk + kWin < kNK) fetch_rows(off, kk + kWin);
      if (kFill && (kk * kF) % kNK < kF && (kk * kF) / kNK < kF)
        fill.issue_one_if((kk * kF) / kNK, fill_tile, rows, en);
      sched_fence();
    }
  };
  auto vector_phase = [&](auto off, int sub_lo) __attribute__((always_inline)) {
    constexpr uint32_t kOff = decltype(off)::value;
#pragma unroll
    for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
      for (int c = 0; c < 2; ++c)
        kta[cb][c] = Tl::read_tr(la.tr[cb][0] + kOff + c * Tl::kGroupBytes,
                                 la.tr[cb][1] + kOff + c * Tl::kGroupBytes);
    if (!rg.mask_free(sub_lo)) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kidx = sub_lo + acc_row(i, g);
        if (kidx < lo_q || kidx >= hi_q) sacc[i] = -INFINITY;
      }
    }
    float ds[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i], p.scale_log2, -lse2));
      ds[i] = pr * (dpacc[i] - delta_q);
    }
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) dsb[c].u[e] = pack_bf16(ds[8 * c + 2 * e], ds[8 * c + 2 * e + 1]);
  };
  auto output_phase = [&](auto next_off, auto with_fill, const typename Tl::Filler& fill,
                          uint32_t fill_tile, uint32_t en) __attribute__((always_inline)) {
    constexpr bool kFill = decltype(with_fill)::value != 0;
    sched_fence();
#pragma unroll
    for (int j = 0; j < kNK; ++j) {
      const int c = j / (D / 32), cb = j % (D / 32);
      acc[cb] = mfma32(kta[cb][c], dsb[c].h, acc[cb]);
      if (j % 2 == 0 && j / 2 < kWin) fetch_rows(next_off, j / 2);
      if (kFill && (j & 1) && (j >> 1) < kF) fill.issue_one_if(j >> 1, fill_tile, rows, en);
      sched_fence();
    }
    if (kWin > (kNK + 1) / 2) {   // narrow heads: the output phase is shorter than the window
#pragma unroll
      for (int kk = (kNK + 1) / 2; kk < kWin; ++kk) fetch_rows(next_off, kk);
    }
  };

  // Tile kt lives in buffer (kt - kt_begin) & 1.  While it is processed, the V copies of tile
  // kt+1 are issued (its K copies were issued during tile kt-1); a barrier after the vector
  // phase of the second block publishes tile kt+1 and retires the readers of tile kt, after
  // which the K copies of tile kt+2 go into this tile's buffer.
  const int kt_last = kt_end - 1;
  auto prepare_after_next = [&](int kt) __attribute__((always_inline)) {
    rows.prepare((kt + 2 < kt_last ? kt + 2 : kt_last) * kStream);
  };
  auto tile_step = [&](auto parity, int kt) __attribute__((always_inline)) {
    constexpr uint32_t kP = decltype(parity)::value;
    constexpr uint32_t kCur = kP * kBuf, kNext = (1 - kP) * kBuf;
    const uint32_t has1 = kt + 1 < kt_end, has2 = kt + 2 < kt_end;
    logits_phase(Const<kCur>{}, Const<1>{}, vfill, tiles + kNext + Tl::kBytes, has1);
    prepare_after_next(kt);
    vector_phase(Const<kCur>{}, kt * kStream);
    output_phase(Const<kCur + Tl::kSubBytes>{}, Const<0>{}, kfill, 0, 0);
    logits_phase(Const<kCur + Tl::kSubBytes>{}, Const<0>{}, vfill, 0, 0);
    vector_phase(Const<kCur + Tl::kSubBytes>{}, kt * kStream + 32);
    wait_async_loads();
    __syncthreads();
    output_phase(Const<kNext>{}, Const<1>{}, kfill, tiles + kCur, has2);
  };
  auto idle_step = [&](int kt) __attribute__((always_inline)) {
    const uint32_t cur = tiles + ((kt - kt_begin) & 1) * kBuf, next = tiles + kBuf - (cur - tiles);
    vfill.issue_if(next + Tl::kBytes, rows, kt + 1 < kt_end);
    prepare_after_next(kt);
    wait_async_loads();
    __syncthreads();
    kfill.issue_if(cur, rows, kt + 2 < kt_end);
  };

  // This wave's tiles: [wt_lo, wt_hi) inside the workgroup's [kt_begin, kt_end).
  const int wt_lo = rg.wave_active ? rg.w_lo / kStream : kt_end;
  const int wt_hi = rg.wave_active ? (rg.w_hi + kStream - 1) / kStream : kt_end;

  wait_async_loads();
  __syncthreads();
  kfill.issue_if(tiles + kBuf, rows, kt_begin + 1 < kt_end);
  int kt = kt_begin;
  for (; kt < wt_lo; ++kt) idle_step(kt);
  if (kt < wt_hi) {
    if ((kt - kt_begin) & 1) {
      fetch_first(Const<kBuf>{});
      tile_step(Const<1>{}, kt);
      ++kt;
    } else {
      fetch_first(Const<0>{});
    }
    for (; kt + 1 < wt_hi; kt += 2) {
      tile_step(Const<0>{}, kt);
      tile_step(Const<1>{}, kt + 1);
    }
    if (kt < wt_hi) {
      tile_step(Const<0>{}, kt);
      ++kt;
    }
  }
  for (; kt < kt_end; ++kt) idle_step(kt);
  wait_async_loads();

  if (!rg.valid) return;
  OutT* row = dq + qkv_base + (long long)q_grid * p.qkv_tok;
  float p_lat = 0.f, p_lon = 0.f;
  if (p.rope) rope_position(p, q_grid, p_lat, p_lon);
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const int ch = cb * 32 + 8 * vq + 4 * g;
      float a0 = acc[cb][4 * vq] * p.scale, a1 = acc[cb][4 * vq + 1] * p.scale,
            a2 = acc[cb][4 * vq + 2] * p.scale, a3 = acc[cb][4 * vq + 3] * p.scale;
      // gradient with respect to the unrotated query: turn the pairs back
      if (p.rope) rope_unrotate4(a0, a1, a2, a3, ch, p_lat, p_lon, p.rope_c);
      store4(row + ch, a0, a1, a2, a3);
    }
}

// ----------------------------------------------------------------------------
// dK, dV: keys resident (one per lane pair), queries streamed.
// LDS: table + 2 buffers x (Q tile, dO tile, 64 x LSE*log2e, 64 x delta).
// ----------------------------------------------------------------------------
template <int D>
constexpr size_t dkdv_smem_bytes(int T) {
  return table_bytes(T) + 2 * (2 * Tile<D>::kBytes + 2 * kStream * 4);
}

template <int D, typename OutT>
__global__ __launch_bounds__(kThreads, D == 128 ? 1 : 2) void winattn_dkdv_kernel(
    KParams p, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o,
    const float* __restrict__ delta, const float* __restrict__ lse2v, OutT* __restrict__ dk,
    OutT* __restrict__ dv) {
  using Tl = Tile<D>;
  constexpr uint32_t kStat = 2 * Tl::kBytes;            // offset of the statistics in a buffer
  constexpr uint32_t kBuf = kStat + 2 * kStream * 4;    // Q tile, dO tile, LSE2[64], delta[64]
  extern __shared__ __align__(16) unsigned char smem[];
  int* tok_grid = reinterpret_cast<int*>(smem);
  const uint32_t table = lds_address(smem);
  const uint32_t tiles = table + table_bytes(p.T);

  int pair, kt;
  if (!block_to_work(p, pair, kt)) return;

  Window win;
  if (!win.init(p, pair)) return;
  build_token_table(p, win, tok_grid);
  __syncthreads();

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ki = lane & 31, g = lane >> 5;
  const long long plane = (long long)p.H * p.W;
  const long long qkv_base = ((long long)win.b * plane) * p.qkv_tok + (long long)win.head * p.qkv_head;
  const long long o_base = ((long long)win.b * plane) * p.o_tok + (long long)win.head * p.o_head;

  Ranges rg;
  rg.init(win, kt, wave, ki);
  const int k_grid = tok_grid[rg.tok];
  const int lo_k = rg.lo, hi_k = rg.hi;

  // one streamed tile: Q, dO (all waves), LSE*log2e (wave 0), delta (wave 1)
  typename Tl::Rows rows;
  typename Tl::Filler qfill, dofill;
  rows.init(table, wave, lane);
  qfill.init(q + ((long long)win.b * plane) * p.q_tok + (long long)win.head * p.q_head, p.q_tok, wave, lane);
  dofill.init(d_o + o_base, p.o_tok, wave, lane);
  const float* stat_src = (wave == 0 ? lse2v : delta) + (long long)pair * p.T + lane;
  // launches the fill of tile t0, whose table entries `rows` holds
  auto fill = [&](uint32_t buf, int t0) __attribute__((always_inline)) {
    qfill.issue(buf, rows);
    dofill.issue(buf + Tl::kBytes, rows);
    if (wave < 2) async_copy4(stat_src + t0, buf + kStat + wave * (kStream * 4));
  };

  const int qt_begin = rg.wg_lo / kStream;
  const int qt_end = (rg.wg_hi + kStream - 1) / kStream;
  rows.prepare(qt_begin * kStream);
  fill(tiles, qt_begin * kStream);
  if (qt_begin + 1 < qt_end) rows.prepare((qt_begin + 1) * kStream);

  bf16x8 kreg[D / 16], vreg[D / 16];
  {
    const bf16_t* krow = k + ((long long)win.b * plane) * p.k_tok + (long long)win.head * p.k_head +
                         (long long)k_grid * p.k_tok + 8 * g;
    const bf16_t* vrow = v + qkv_base + (long long)k_grid * p.qkv_tok + 8 * g;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      kreg[kk] = *reinterpret_cast<const bf16x8*>(krow + kk * 16);
      vreg[kk] = *reinterpret_cast<const bf16x8*>(vrow + kk * 16);
    }
  }
  typename Tl::Lanes la;
  la.init(tiles, lane);
  uint32_t stat_lane = tiles + kStat + 4 * g * 4;   // rows 8*vq + 4*g + (0..3) of a sub-block
  settle(stat_lane);
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

  // One 32-query block: kOff = compile-time LDS offset of its rows from buffer 0 /
  // sub-block 0, kStatOff = the same for its statistics.
  auto sub_block = [&](auto off, auto stat_off, int sub_lo) __attribute__((always_inline)) {
    constexpr uint32_t kOff = decltype(off)::value;
    constexpr uint32_t kStatOff = decltype(stat_off)::value;
    if (rg.skip(sub_lo)) return;
    // operand reads first, products after: LDS latency hides behind the MFMA pipeline
    bf16x8 qa[D / 16], doa[D / 16], qta[D / 32][2], dota[D / 32][2];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      qa[kk] = Tl::read_rm(la.rm[kk] + kOff);
      doa[kk] = Tl::read_rm(la.rm[kk] + kOff + Tl::kBytes);
    }
    f32x4 l4[4], d4[4];
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      l4[vq] = *reinterpret_cast<const AERIS_LDS f32x4*>(stat_lane + kStatOff + vq * 32);
      d4[vq] = *reinterpret_cast<const AERIS_LDS f32x4*>(stat_lane + kStatOff + vq * 32 +
                                                         kStream * 4);
    }
    // S[query, key] = Q K^T,  dP[query, key] = dO V^T: rows = streamed queries
    f32x16 s, dp;
#pragma unroll
    for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      s = mfma32(qa[kk], kreg[kk], s);
      dp = mfma32(doa[kk], vreg[kk], dp);
    }
#pragma unroll
    for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        dota[cb][c] = Tl::read_tr(la.tr[cb][0] + kOff + Tl::kBytes + c * Tl::kGroupBytes,
                                  la.tr[cb][1] + kOff + Tl::kBytes + c * Tl::kGroupBytes);
        qta[cb][c] = Tl::read_tr(la.tr[cb][0] + kOff + c * Tl::kGroupBytes,
                                 la.tr[cb][1] + kOff + c * Tl::kGroupBytes);
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
    for (int i = 0; i < 16; ++i) {
      pr[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], p.scale_log2, -l4[i >> 2][i & 3]));
      ds[i] = pr[i] * (dp[i] - d4[i >> 2][i & 3]);
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
        dvacc[cb] = mfma32(dota[cb][c], pb[c].h, dvacc[cb]);
        dkacc[cb] = mfma32(qta[cb][c], dsb[c].h, dkacc[cb]);
      }
  };

  auto tile_step = [&](auto parity, int qt) __attribute__((always_inline)) {
    constexpr uint32_t kP = decltype(parity)::value;
    wait_async_loads();
    __syncthreads();
    if (qt + 1 < qt_end) {
      fill(tiles + (1 - kP) * kBuf, (qt + 1) * kStream);
      if (qt + 2 < qt_end) rows.prepare((qt + 2) * kStream);
    }
    if (!rg.wave_active) return;
    sub_block(Const<kP * kBuf>{}, Const<kP * kBuf>{}, qt * kStream);
    sub_block(Const<kP * kBuf + Tl::kSubBytes>{}, Const<kP * kBuf + 32 * 4>{}, qt * kStream + 32);
  };
  for (int qt = qt_begin; qt < qt_end; qt += 2) {
    tile_step(Const<0>{}, qt);
    if (qt + 1 < qt_end) tile_step(Const<1>{}, qt + 1);
  }

  if (!rg.valid) return;
  OutT* dkrow = dk + qkv_base + (long long)k_grid * p.qkv_tok;
  OutT* dvrow = dv + qkv_base + (long long)k_grid * p.qkv_tok;
  float p_lat = 0.f, p_lon = 0.f;
  if (p.rope) rope_position(p, k_grid, p_lat, p_lon);
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const int ch = cb * 32 + 8 * vq + 4 * g;
      float a0 = dkacc[cb][4 * vq] * p.scale, a1 = dkacc[cb][4 * vq + 1] * p.scale,
            a2 = dkacc[cb][4 * vq + 2] * p.scale, a3 = dkacc[cb][4 * vq + 3] * p.scale;
      // gradient with respect to the unrotated key: turn the pairs back
      if (p.rope) rope_unrotate4(a0, a1, a2, a3, ch, p_lat, p_lon, p.rope_c);
      store4(dkrow + ch, a0, a1, a2, a3);
      store4(dvrow + ch, dvacc[cb][4 * vq], dvacc[cb][4 * vq + 1], dvacc[cb][4 * vq + 2],
             dvacc[cb][4 * vq + 3]);
    }
}

template <int D, typename OutT>
static int launch_bwd_t(const KParams& kp, const void* q, const void* k, const void* v,
                        const void* o, const float* lse, const void* d_o, void* dq, void* dk,
                        void* dv, float* workspace, hipStream_t stream, unsigned stages) {
  const bf16_t* qp = static_cast<const bf16_t*>(q);
  const bf16_t* kp_ = static_cast<const bf16_t*>(k);
  const bf16_t* vp = static_cast<const bf16_t*>(v);
  const bf16_t* dop = static_cast<const bf16_t*>(d_o);

  float* delta = workspace;
  float* lse2 = workspace + stat_entries(kp);
  // with both stages requested the dQ kernel produces the statistics itself
  const bool fused_stats = (stages & 3u) == 3u;
  if ((stages & 1u) && !fused_stats) {
    constexpr int kTokens = kThreads / (D / 8);
    const long long dblocks = (long long)kp.n_pairs * ((kp.T + kTokens - 1) / kTokens);
    if (launch_kernel(winattn_delta_kernel<D, OutT>, dim3((unsigned)dblocks), dim3(kThreads), 0,
                      stream, kp, static_cast<const OutT*>(o), dop, lse, delta, lse2) != 0)
      return -1;
  }

  const int n_blocks = grid_blocks(kp);
  if (stages & 2u) {
    const size_t smem = dq_smem_bytes<D>(kp.T);
    auto kern = winattn_dq_kernel<D, OutT>;
    if (!allow_full_lds<winattn_dq_kernel<D, OutT>>()) return -1;
    if (launch_kernel(kern, dim3(n_blocks), dim3(kThreads), smem, stream, kp, qp, kp_, vp, dop,
                      static_cast<const OutT*>(o), lse, delta, lse2, static_cast<OutT*>(dq),
                      fused_stats ? 1 : 0) != 0)
      return -1;
  }
  if constexpr (D == 128) {   // software-pipelined kernel; the generic one is not built for it
    if ((stages & 4u) && launch_dkdv_pipe128(kp, std::is_same<OutT, float>::value, q, k, v, d_o,
                                             delta, lse2, dk, dv, stream) != 0)
      return -1;
  } else if (stages & 4u) {
    const size_t smem = dkdv_smem_bytes<D>(kp.T);
    auto kern = winattn_dkdv_kernel<D, OutT>;
    if (!allow_full_lds<winattn_dkdv_kernel<D, OutT>>()) return -1;
    if (launch_kernel(kern, dim3(n_blocks), dim3(kThreads), smem, stream, kp, qp, kp_, vp, dop,
                      static_cast<const float*>(delta), static_cast<const float*>(lse2),
                      static_cast<OutT*>(dk), static_cast<OutT*>(dv)) != 0)
      return -1;
  }
  return 0;
}

size_t bwd_workspace_bytes(const KParams& kp) { return 2 * (size_t)stat_entries(kp) * sizeof(float); }

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
