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

template <int D, typename OutT>
__global__ __launch_bounds__(kThreads, 2) void winattn_fwd_kernel(
    KParams p, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, OutT* __restrict__ o, float* __restrict__ lse) {
  using Tl = Tile<D>;
  constexpr uint32_t kBuf = 2 * Tl::kBytes;   // one buffer: K tile, V tile
  extern __shared__ __align__(16) unsigned char smem[];
  int* tok_grid = reinterpret_cast<int*>(smem);
  const uint32_t table = lds_address(smem);
  const uint32_t tiles = table + table_bytes(p.T);

  int pair, qt;
  if (!block_to_work(p, pair, qt)) return;

  Window win;
  win.init(p, pair);
  build_token_table(p, win, tok_grid);
  __syncthreads();

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qi = lane & 31, g = lane >> 5;

  const long long plane = (long long)p.H * p.W;
  const long long qkv_base = ((long long)win.b * plane) * p.qkv_tok + (long long)win.head * p.qkv_head;

  // ---- this lane's query ----------------------------------------------------
  Ranges rg;
  rg.init(win, qt, wave, qi);
  const int q_grid = tok_grid[rg.tok];
  const int lo_q = rg.lo, hi_q = rg.hi;

  const int kt_begin = rg.wg_lo / kStream;
  const int kt_end = (rg.wg_hi + kStream - 1) / kStream;
  typename Tl::Rows rows;
  typename Tl::Filler kfill, vfill;
  rows.init(table, wave, lane);
  kfill.init(k + qkv_base, p.qkv_tok, wave, lane);
  vfill.init(v + qkv_base, p.qkv_tok, wave, lane);
  rows.prepare(kt_begin * kStream);
  kfill.issue(tiles, rows);
  vfill.issue(tiles + Tl::kBytes, rows);
  if (kt_begin + 1 < kt_end) rows.prepare((kt_begin + 1) * kStream);

  bf16x8 qreg[D / 16];
  {
    const bf16_t* qrow = q + qkv_base + (long long)q_grid * p.qkv_tok + 8 * g;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
      qreg[kk] = *reinterpret_cast<const bf16x8*>(qrow + kk * 16);
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

  // One 32-key block at compile-time LDS offset kOff from buffer 0 / sub-block 0:
  // every operand address is a per-lane register plus an immediate.
  auto sub_block = [&](auto off, int sub_lo) __attribute__((always_inline)) {
    constexpr uint32_t kOff = decltype(off)::value;
    if (rg.skip(sub_lo)) return;   // wave-uniform
    // ---- operand reads first, products after: LDS latency hides behind the MFMA
    //      pipeline; the V operands land during the softmax ------------------------
    bf16x8 ka[D / 16], va[D / 32][2];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) ka[kk] = Tl::read_rm(la.rm[kk] + kOff);
#pragma unroll
    for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        constexpr uint32_t kV = kOff + Tl::kBytes;
        va[cb][c] = Tl::read_tr(la.tr[cb][0] + kV + c * Tl::kGroupBytes,
                                la.tr[cb][1] + kV + c * Tl::kGroupBytes);
      }
    // ---- S^T = K Q^T ---------------------------------------------------------
    f32x16 s;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) s = mfma32(ka[kk], qreg[kk], s);
    // ---- mask ----------------------------------------------------------------
    if (!rg.mask_free(sub_lo)) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kidx = sub_lo + acc_row(i, g);
        if (kidx < lo_q || kidx >= hi_q) s[i] = -INFINITY;
      }
    }
    // ---- online softmax (log2 domain, lagging maximum) --------------------------
    float mx = s[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i]);
    mx = wave_half_max(mx) * p.scale_log2;
    const bool grow = mx > m_run + kLazyRescale;
    if (__builtin_expect(__any(grow), 0)) {
      const float alpha = grow ? __builtin_amdgcn_exp2f(m_run - mx) : 1.f;
      m_run = grow ? mx : m_run;
      l_run *= alpha;
#pragma unroll
      for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[cb][i] *= alpha;
    }
    const float m_sub = m_run == -INFINITY ? 0.f : m_run;
    float pv[16];
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      pv[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], p.scale_log2, -m_sub));
      psum += pv[i];
    }
    l_run += psum;
    // ---- O^T += V^T P^T ----------------------------------------------------------
    union { u32x4 u; bf16x8 h; } pb[2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) pb[c].u[e] = pack_bf16(pv[8 * c + 2 * e], pv[8 * c + 2 * e + 1]);
#pragma unroll
    for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
      for (int c = 0; c < 2; ++c) oacc[cb] = mfma32(va[cb][c], pb[c].h, oacc[cb]);
  };

  // One streamed tile held in buffer kP (compile time); the next one flies into
  // the other buffer during the math.  One barrier per tile: it publishes tile
  // kt and retires the readers of tile kt-1, whose buffer the new fill reuses.
  auto tile_step = [&](auto parity, int kt) __attribute__((always_inline)) {
    constexpr uint32_t kP = decltype(parity)::value;
    wait_async_loads();
    __syncthreads();
    if (kt + 1 < kt_end) {     // table entries were read one tile ago
      kfill.issue(tiles + (1 - kP) * kBuf, rows);
      vfill.issue(tiles + (1 - kP) * kBuf + Tl::kBytes, rows);
      if (kt + 2 < kt_end) rows.prepare((kt + 2) * kStream);
    }
    if (!rg.wave_active) return;
    sub_block(Const<kP * kBuf>{}, kt * kStream);
    sub_block(Const<kP * kBuf + Tl::kSubBytes>{}, kt * kStream + 32);
  };
  for (int kt = kt_begin; kt < kt_end; kt += 2) {
    tile_step(Const<0>{}, kt);
    if (kt + 1 < kt_end) tile_step(Const<1>{}, kt + 1);
  }

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

template <int D, typename OutT>
static int launch_fwd_t(const KParams& kp, const void* q, const void* k, const void* v, void* o,
                        float* lse, hipStream_t stream) {
  const int n_blocks = grid_blocks(kp);
  const size_t smem = fwd_smem_bytes<D>(kp.T);
  auto kern = winattn_fwd_kernel<D, OutT>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
    return -1;
  hipLaunchKernelGGL(kern, dim3(n_blocks), dim3(kThreads), smem, stream, kp,
                     static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k),
                     static_cast<const bf16_t*>(v), static_cast<OutT*>(o), lse);
  return hipGetLastError() == hipSuccess ? 0 : -1;
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
