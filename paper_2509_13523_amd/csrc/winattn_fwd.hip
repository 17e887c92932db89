// Forward shifted-window attention for gfx950 (AERIS paper, Model Architecture
// section: window partition + shift, then dot-product attention per window and
// head; computed flash-style: the T x T logits never leave the chip).
//
// One workgroup = 128 queries of one (batch, window, head); each of its four
// wavefronts owns 32 queries, one per lane pair (l, l+32).  Keys/values stream
// through double-buffered LDS tiles of 64 tokens, filled asynchronously.  The
// logits are produced transposed,
//     S^T[key, query] = K Q^T        (A = K tile, row-major reads; B = Q in registers)
// so every lane holds logits of ONE query: the softmax statistics are per-lane
// scalars and the row reductions need a single cross-lane exchange.  P^T then
// feeds the second product in place,
//     O^T[channel, query] += V^T P^T (A = V tile through transposing reads, B = P^T).
#include "winattn_common.hpp"
#include "winattn_launch.hpp"

namespace aeris {

template <int D>
constexpr size_t fwd_smem_bytes(int T) {
  return table_bytes(T) + 4 * Tile<D>::kBytes;   // table + 2 buffers x (K, V)
}

// W wavefronts per workgroup, 32 resident queries each.  Four waves (two workgroups per CU, so
// one's prologue and epilogue run under the other's loop) suit short windows; eight waves (one
// workgroup per CU) stream every K/V tile for twice as many queries, which halves the
// L2 -> LDS traffic and the copy instructions per product and wins once the loop is long.
template <int D, typename OutT, int W>
__global__ __launch_bounds__(W * 64, W == 4 ? 2 : 1) void winattn_fwd_kernel(
    KParams p, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, OutT* __restrict__ o, float* __restrict__ lse) {
  using Tl = Tile<D, W>;
  constexpr uint32_t kBuf = 2 * Tl::kBytes;   // one buffer: K tile, V tile
  extern __shared__ __align__(16) unsigned char smem[];
  int* tok_grid = reinterpret_cast<int*>(smem);
  const uint32_t table = lds_address(smem);
  const uint32_t tiles = table + table_bytes(p.T);

  int pair, qt;
  if (!block_to_work(p, pair, qt)) return;

  Window win;
  if (!win.init(p, pair)) return;
  build_token_table(p, win, tok_grid);
  __syncthreads();

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qi = lane & 31, g = lane >> 5;

  const long long plane = (long long)p.H * p.W;
  const long long q_base = ((long long)win.b * plane) * p.q_tok + (long long)win.head * p.q_head;
  const long long k_base = ((long long)win.b * plane) * p.k_tok + (long long)win.head * p.k_head;
  const long long v_base = ((long long)win.b * plane) * p.qkv_tok + (long long)win.head * p.qkv_head;

  // ---- this lane's query ----------------------------------------------------
  Ranges rg;
  rg.init(win, qt, wave, qi, W * 32);
  const int q_grid = tok_grid[rg.tok];
  const int lo_q = rg.lo, hi_q = rg.hi;

  const int kt_begin = rg.wg_lo / kStream;
  const int kt_end = (rg.wg_hi + kStream - 1) / kStream;
  typename Tl::Rows rows;
  typename Tl::Filler kfill, vfill;
  rows.init(table, wave, lane);
  kfill.init(k + k_base, p.k_tok, wave, lane);
  vfill.init(v + v_base, p.qkv_tok, wave, lane);
  rows.prepare(kt_begin * kStream);
  kfill.issue(tiles, rows);
  vfill.issue(tiles + Tl::kBytes, rows);
  if (kt_begin + 1 < kt_end) rows.prepare((kt_begin + 1) * kStream);

  bf16x8 qreg[D / 16];
  {
    const bf16_t* qrow = q + q_base + (long long)q_grid * p.q_tok + 8 * g;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
      qreg[kk] = *reinterpret_cast<const bf16x8*>(qrow + kk * 16);
    if (p.rope) {   // rotary embedding fused into the load of the resident queries
      float p_lat, p_lon;
      rope_position(p, q_grid, p_lat, p_lon);
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk)
        qreg[kk] = rope_rotate8(qreg[kk], kk * 16 + 8 * g, p_lat, p_lon, p.rope_c, false);
      if (p.q_rot_out && rg.valid) {   // by-product for the backward pass: no second rotation
        bf16_t* keep = p.q_rot_out + (((long long)win.b * plane + q_grid) * p.nh + win.head) * D + 8 * g;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) *reinterpret_cast<bf16x8*>(keep + kk * 16) = qreg[kk];
      }
    }
  }
  typename Tl::Lanes la;
  la.init(tiles, lane);
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) settle(qreg[kk]);

  f32x16 oacc[D / 32];
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[cb][i] = 0.f;
  float m_run = -INFINITY;   // running (lagging) row maximum, log2 domain
  float l_run = 0.f;         // this lane's share of the row sum

  // Schedule of one 32-key block (LDS offsets are compile-time constants, so every
  // operand address is a per-lane register plus an immediate):
  //   logits phase   D/16 products S^T = K Q^T, whose K operands were fetched during
  //                  the previous block; between them the V operands of this block are
  //                  fetched (they land during the softmax) and copies of the next
  //                  tile are issued;
  //   softmax phase  vector work only;
  //   output phase   D/16 products O^T += V^T P^T; between them the K operands of the
  //                  NEXT block are fetched and further copies are issued.
  // The scheduling fences keep the compiler from collapsing the phases again (it
  // otherwise serialises operand reads and products to save registers).
  bf16x8 ka[D / 16], va[D / 32][2];
  f32x16 sacc;
  union { u32x4 u; bf16x8 h; } pb[2];
  constexpr int kF = Tl::kFillPerWave;

  auto fetch_k = [&](auto off) __attribute__((always_inline)) {
    constexpr uint32_t kOff = decltype(off)::value;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) ka[kk] = Tl::read_rm(la.rm[kk] + kOff);
  };
  // en: non-zero if the copies are wanted (wave-uniform)
  auto logits_phase = [&](auto off, auto with_fill, const typename Tl::Filler& fill,
                          uint32_t fill_tile, uint32_t en) __attribute__((always_inline)) {
    constexpr uint32_t kV = decltype(off)::value + Tl::kBytes;
    constexpr bool kFill = decltype(with_fill)::value != 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
    sched_fence();
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      sacc = mfma32(ka[kk], qreg[kk], sacc);
      const int cb = kk >> 1, c = kk & 1;
      va[cb][c] = Tl::read_tr(la.tr[cb][0] + kV + c * Tl::kGroupBytes,
                              la.tr[cb][1] + kV + c * Tl::kGroupBytes);
      if (kFill && (kk & 1) && (kk >> 1) < kF) fill.issue_one_if(kk >> 1, fill_tile, rows, en);
      sched_fence();
    }
  };
  auto softmax_phase = [&](int sub_lo) __attribute__((always_inline)) {
    if (!rg.mask_free(sub_lo)) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kidx = sub_lo + acc_row(i, g);
        if (kidx < lo_q || kidx >= hi_q) sacc[i] = -INFINITY;
      }
    }
    // online softmax, log2 domain, lagging maximum.  The reference point m_run only has to keep
    // the exponentials in range, so the common case computes them straight away and looks at
    // their sum: 16 values that add up to at most 2^12 are each at most 2^12.  Only when a lane's
    // sum is larger (or not a number), or a row has no reference point yet (its first block with
    // a visible key sets it to that block's maximum, so that a row of very negative logits does
    // not underflow), is the row maximum taken and the reference point raised, for both lanes of
    // a query alike, and the block's exponentials computed again.
    float pv[16];
    float psum = 0.f;   // in fp32 over the unrounded probabilities: the saved LSE stays exact
    {
      const float m_sub = m_run == -INFINITY ? 0.f : m_run;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        pv[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i], p.scale_log2, -m_sub));
        psum += pv[i];
      }
    }
    if (__builtin_expect(__any(!(psum <= kSumLimit) || m_run == -INFINITY), 0)) {
      float mx = sacc[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sacc[i]);
      mx = wave_half_max(mx) * p.scale_log2;
      const bool grow = mx > m_run + kLazyRescale;
      const float alpha = grow ? __builtin_amdgcn_exp2f(m_run - mx) : 1.f;
      m_run = grow ? mx : m_run;
      l_run *= alpha;
#pragma unroll
      for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[cb][i] *= alpha;
      const float m_sub = m_run == -INFINITY ? 0.f : m_run;
      psum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        pv[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i], p.scale_log2, -m_sub));
        psum += pv[i];
      }
    }
    l_run += psum;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) pb[c].u[e] = pack_bf16(pv[8 * c + 2 * e], pv[8 * c + 2 * e + 1]);
  };
  auto output_phase = [&](auto k_off, auto with_fill, const typename Tl::Filler& fill,
                          uint32_t fill_tile, uint32_t en) __attribute__((always_inline)) {
    constexpr uint32_t kOff = decltype(k_off)::value;
    constexpr bool kFill = decltype(with_fill)::value != 0;
    sched_fence();
#pragma unroll
    for (int j = 0; j < D / 16; ++j) {
      const int c = j / (D / 32), cb = j % (D / 32);
      oacc[cb] = mfma32(va[cb][c], pb[c].h, oacc[cb]);
      ka[j] = Tl::read_rm(la.rm[j] + kOff);
      if (kFill && (j & 1) && (j >> 1) < kF) fill.issue_one_if(j >> 1, fill_tile, rows, en);
      sched_fence();
    }
  };

  // Tile kt lives in buffer (kt - kt_begin) & 1.  While it is processed, the V copies
  // of tile kt+1 are issued (its K copies were issued during tile kt-1); a barrier in
  // the middle of the second block publishes tile kt+1 and retires the readers of tile
  // kt, after which the K copies of tile kt+2 go into this tile's buffer.  Copies of
  // tiles past the end are branched over.
  const int kt_last = kt_end - 1;
  auto prepare_after_next = [&](int kt) __attribute__((always_inline)) {
    rows.prepare((kt + 2 < kt_last ? kt + 2 : kt_last) * kStream);
  };
  // A tile in which this wave computes both blocks (masked where needed).
  auto tile_step = [&](auto parity, int kt) __attribute__((always_inline)) {
    constexpr uint32_t kP = decltype(parity)::value;
    constexpr uint32_t kCur = kP * kBuf, kNext = (1 - kP) * kBuf;
    const uint32_t has1 = kt + 1 < kt_end, has2 = kt + 2 < kt_end;
    logits_phase(Const<kCur>{}, Const<1>{}, vfill, tiles + kNext + Tl::kBytes, has1);
    prepare_after_next(kt);
    softmax_phase(kt * kStream);
    output_phase(Const<kCur + Tl::kSubBytes>{}, Const<0>{}, kfill, 0, 0);
    logits_phase(Const<kCur + Tl::kSubBytes>{}, Const<0>{}, vfill, 0, 0);
    softmax_phase(kt * kStream + 32);
    wait_async_loads();
    __syncthreads();
    output_phase(Const<kNext>{}, Const<1>{}, kfill, tiles + kCur, has2);
  };
  // A tile none of whose keys this wave needs: keep the copies and the barrier going.
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
      fetch_k(Const<kBuf>{});
      tile_step(Const<1>{}, kt);
      ++kt;
    } else {
      fetch_k(Const<0>{});
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

  // ---- epilogue: normalise, un-shift/un-partition store -----------------------
  if (!rg.valid) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.f / l_tot;
  OutT* orow = o + ((long long)win.b * plane + q_grid) * p.o_tok + (long long)win.head * p.o_head;
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int vq = 0; vq < 4; ++vq)
      store4(orow + cb * 32 + 8 * vq + 4 * g, oacc[cb][4 * vq] * inv, oacc[cb][4 * vq + 1] * inv,
             oacc[cb][4 * vq + 2] * inv, oacc[cb][4 * vq + 3] * inv);
  if (g == 0)
    lse[((long long)win.b * p.nh + win.head) * plane + q_grid] =
        (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
}

// Windows of at least this many tokens run with eight waves per workgroup (head_dim >= 64).
constexpr int kWideFromTokens = 2048;

template <int D, typename OutT, int W>
static int launch_fwd_w(KParams kp, const void* q, const void* k, const void* v, void* o,
                        float* lse, hipStream_t stream) {
  kp.n_tiles = (kp.T + W * 32 - 1) / (W * 32);
  const int n_blocks = grid_blocks(kp);
  const size_t smem = fwd_smem_bytes<D>(kp.T);
  auto kern = winattn_fwd_kernel<D, OutT, W>;
  if (!allow_full_lds<winattn_fwd_kernel<D, OutT, W>>()) return -1;
  return launch_kernel(kern, dim3(n_blocks), dim3(W * 64), smem, stream, kp,
                       static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k),
                       static_cast<const bf16_t*>(v), static_cast<OutT*>(o), lse);
}

template <int D, typename OutT>
static int launch_fwd_t(const KParams& kp, const void* q, const void* k, const void* v, void* o,
                        float* lse, hipStream_t stream) {
  if constexpr (D >= 64) {
    if (kp.T >= kWideFromTokens) return launch_fwd_w<D, OutT, 8>(kp, q, k, v, o, lse, stream);
  }
  return launch_fwd_w<D, OutT, 4>(kp, q, k, v, o, lse, stream);
}

int launch_fwd(const KParams& kp, int head_dim, bool out_f32, const void* q, const void* k,
               const void* v, void* o, float* lse, hipStream_t stream) {
#define AERIS_FWD_CASE(DD)                                                             \
  case DD:                                                                             \
    return out_f32 ? launch_fwd_t<DD, float>(kp, q, k, v, o, lse, stream)              \
                   : launch_fwd_t<DD, bf16_t>(kp, q, k, v, o, lse, stream);
  switch (head_dim) {
    AERIS_FWD_CASE(32)
    AERIS_FWD_CASE(64)
    AERIS_FWD_CASE(128)
  }
#undef AERIS_FWD_CASE
  return -1;
}

}  // namespace aeris
