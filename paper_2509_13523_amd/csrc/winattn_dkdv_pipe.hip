// dK/dV kernel, software-pipelined variant (used for head_dim 128, where the
// two 128x32 accumulators leave room for only one wave per SIMD, so nothing but
// the instruction order inside the wave can overlap matrix and vector work).
//
// Same mathematics and data flow as winattn_dkdv_kernel (see winattn_bwd.hip):
// keys resident, queries streamed through LDS tiles, S = Q K^T and dP = dO V^T
// by row-major reads, dV^T += dO^T P and dK^T += Q^T dS by transposing reads.
// What differs is the schedule.  Per 32-query block j:
//     stage A(j):  16 MFMA   logits S_j, dP_j
//     stage B(j):  ~100 VALU P_j = exp2(S_j*c - LSE2), dS_j = P_j (dP_j - delta)
//     stage C(j):  16 MFMA   dV^T += dO_j^T P_j, dK^T += Q_j^T dS_j
// and the instruction stream is A(j+1) interleaved with B(j) -- one MFMA, then
// one logit's worth of vector work -- followed by C(j).  On gfx950 a 32x32x16
// MFMA keeps the matrix pipe busy for 32 cycles but blocks instruction issue for
// only about half of that, so the vector work of B rides under the MFMAs of A.
// Three LDS buffers: tile t+2 streams in while A reads tile t+1 and C reads t.
#include "winattn_common.hpp"
#include "winattn_launch.hpp"


namespace aeris {

// c += a b with c pinned to accumulation registers.  This file is compiled with MFMA results
// in ordinary VGPRs by default, so that the vector stage reads the logits where the products
// deliver them; the 2 x 128 gradient accumulators, which only MFMAs touch inside the loop,
// are kept in accumulation registers by this statement.  Products on one accumulator are two
// MFMAs apart, and the epilogue waits out the MFMA latency before it reads them.
__device__ __forceinline__ void mfma32_acc(bf16x8 a, bf16x8 b, f32x16& c) {
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

template <int D>
constexpr size_t dkdv_pipe_smem_bytes(int T) {
  return table_bytes(T) + 3 * (2 * Tile<D>::kBytes + 2 * kStream * 4);
}

template <int D, typename OutT>
__global__ __launch_bounds__(kThreads, 1) void winattn_dkdv_pipe_kernel(
    KParams p, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o,
    const float* __restrict__ delta, const float* __restrict__ lse2v, OutT* __restrict__ dk,
    OutT* __restrict__ dv) {
  using Tl = Tile<D>;
  constexpr uint32_t kStat = 2 * Tl::kBytes;            // offset of the statistics in a buffer
  constexpr uint32_t kBuf = kStat + 2 * kStream * 4;    // Q tile, dO tile, LSE2[64], delta[64]
  constexpr int kNK = D / 16;                           // contraction blocks of the first products
  constexpr int kNA = 2 * kNK;                          // MFMAs of stage A
  constexpr int kNC = 4 * (D / 32);                     // MFMAs of stage C
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

  bf16x8 kreg[kNK], vreg[kNK];
  {
    const bf16_t* krow = k + ((long long)win.b * plane) * p.k_tok + (long long)win.head * p.k_head +
                         (long long)k_grid * p.k_tok + 8 * g;
    const bf16_t* vrow = v + qkv_base + (long long)k_grid * p.qkv_tok + 8 * g;
#pragma unroll
    for (int kk = 0; kk < kNK; ++kk) {
      kreg[kk] = *reinterpret_cast<const bf16x8*>(krow + kk * 16);
      vreg[kk] = *reinterpret_cast<const bf16x8*>(vrow + kk * 16);
    }
  }
  // Per-lane LDS addresses.  `rm` (row-major reads, stage A) points into the
  // buffer of the tile stage A works on; `tr` (transposing reads, stage C) and
  // `st` (statistics, stage B) into the buffer of the tile stages B and C work
  // on.  They advance by one buffer per tile, independently.
  typename Tl::Lanes la;
  la.init(tiles, lane);
  uint32_t st = tiles + kStat + 4 * g * 4;   // rows 8*vq + 4*g + (0..3) of a sub-block
  settle(st);
#pragma unroll
  for (int kk = 0; kk < kNK; ++kk) {
    settle(kreg[kk]);
    settle(vreg[kk]);
  }

  f32x16 dkacc[D / 32], dvacc[D / 32];
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dkacc[cb][i] = 0.f; dvacc[cb][i] = 0.f; }

  // Logits of the block stage B consumes next.  Two sets: while stage B reads one, stage A
  // of the following block accumulates into the other (no copies between stages).
  f32x16 s0, dp0, s1, dp1;
  union Packed { u32x4 u; bf16x8 h; };
  Packed pb[2], dsb[2];                           // P, dS of the block stage C consumes

  // operand i of stage A: even -> Q rows, odd -> dO rows, contraction block i/2
  auto a_operand = [&](int i, uint32_t sub) __attribute__((always_inline)) {
    return Tl::read_rm(la.rm[i >> 1] + sub + ((i & 1) ? Tl::kBytes : 0));
  };
  // operand i of stage C: channel block i/4, 16-query group (i/2)%2, even -> dO^T, odd -> Q^T
  auto c_operand = [&](int i, uint32_t sub) __attribute__((always_inline)) {
    const int cb = i >> 2, c = (i >> 1) & 1;
    const uint32_t off = sub + c * Tl::kGroupBytes + ((i & 1) ? 0 : Tl::kBytes);
    return Tl::read_tr(la.tr[cb][0] + off, la.tr[cb][1] + off);
  };

  // Stage A alone (pipeline prologue).
  auto stage_a = [&](uint32_t sub) __attribute__((always_inline)) {
    bf16x8 op[kNA];
#pragma unroll
    for (int i = 0; i < kNA; ++i) op[i] = a_operand(i, sub);
#pragma unroll
    for (int i = 0; i < 16; ++i) { s0[i] = 0.f; dp0[i] = 0.f; }
#pragma unroll
    for (int i = 0; i < kNA; ++i) {
      if (i & 1) dp0 = mfma32(op[i], vreg[i >> 1], dp0);
      else s0 = mfma32(op[i], kreg[i >> 1], s0);
    }
  };

  // Vector work for logit e of the current block (statistics l, d of its query row).
  auto b_element = [&](auto masked, const f32x16& s, const f32x16& dp, int e, float l, float d,
                       int sub_lo, float* pr, float* ds) __attribute__((always_inline)) {
    float se = s[e];
    if (decltype(masked)::value) {
      const int qidx = sub_lo + acc_row(e, g);
      if (qidx < lo_k || qidx >= hi_k) se = -INFINITY;
    }
    pr[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(se, p.scale_log2, -l));
    ds[e] = pr[e] * (dp[e] - d);
  };

  // piece i (0 .. 2*kFillPerWave) of a tile fill whose table entries were prepared
  // earlier: Q rows, dO rows, statistics
  auto fill_piece = [&](int i, uint32_t buf, int t0) __attribute__((always_inline)) {
    if (i < Tl::kFillPerWave) qfill.issue_one(i, buf, rows);
    else if (i < 2 * Tl::kFillPerWave) dofill.issue_one(i - Tl::kFillPerWave, buf + Tl::kBytes, rows);
    else if (wave < 2) async_copy4(stat_src + t0, buf + kStat + wave * (kStream * 4));
  };

  // Stage B(cur) interleaved with stage A(next) when kNext, else B alone.
  //   nsub: LDS offset of the next block's rows relative to `rm`;
  //   csub_stat: offset of the current block's statistics relative to `st`.
  //   s, dp: logits of the current block; sn, dpn: receive those of the next one.
  //   do_fill (wave-uniform): the pieces of a tile fill are dropped into the first slots, one
  //   per slot (issued as a burst they stall the wave until the memory pipeline drains).  They
  //   ride here rather than in stage C because stage C keeps the LDS busier (transposing reads
  //   run at half the rate of row reads) and the copies land in the LDS too.
  auto stage_ab = [&](auto has_next, auto masked, const f32x16& s, const f32x16& dp, f32x16& sn,
                      f32x16& dpn, uint32_t nsub, uint32_t csub_stat, int sub_lo, bool do_fill,
                      uint32_t fill_buf, int fill_t0) __attribute__((always_inline)) {
    constexpr bool kNext = decltype(has_next)::value;
    constexpr int kAhead = 3;                     // LDS reads run this many MFMAs ahead
    bf16x8 op[kNA];
    f32x4 l4[4], d4[4];
    float pr[16], ds[16];
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      l4[vq] = *reinterpret_cast<const AERIS_LDS f32x4*>(st + csub_stat + vq * 32);
      d4[vq] = *reinterpret_cast<const AERIS_LDS f32x4*>(st + csub_stat + vq * 32 + kStream * 4);
    }
    if (kNext) {
#pragma unroll
      for (int i = 0; i < kAhead; ++i) op[i] = a_operand(i, nsub);
#pragma unroll
      for (int i = 0; i < 16; ++i) { sn[i] = 0.f; dpn[i] = 0.f; }
    }
    __builtin_amdgcn_sched_barrier(0);
    // 16 slots: slot e carries logit e, and MFMAs e*kNA/16 .. of stage A
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      if (kNext) {
#pragma unroll
        for (int i = e * kNA / 16; i < (e + 1) * kNA / 16; ++i) {
          if (i + kAhead < kNA) op[i + kAhead] = a_operand(i + kAhead, nsub);
          if (i & 1) dpn = mfma32(op[i], vreg[i >> 1], dpn);
          else sn = mfma32(op[i], kreg[i >> 1], sn);
        }
      }
      if (e <= 2 * Tl::kFillPerWave && do_fill) fill_piece(e, fill_buf, fill_t0);
      b_element(masked, s, dp, e, l4[e >> 2][e & 3], d4[e >> 2][e & 3], sub_lo, pr, ds);
      if (e & 1) {
        const int c = e >> 3, w = (e >> 1) & 3;
        pb[c].u[w] = pack_bf16(pr[e - 1], pr[e]);
        dsb[c].u[w] = pack_bf16(ds[e - 1], ds[e]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Stage C: the 16 accumulating products of the current block.
  auto stage_c = [&](uint32_t sub) __attribute__((always_inline)) {
    constexpr int kAhead = 3;
    bf16x8 op[kNC];
#pragma unroll
    for (int i = 0; i < kAhead; ++i) op[i] = c_operand(i, sub);
#pragma unroll
    for (int i = 0; i < kNC; ++i) {
      if (i + kAhead < kNC) op[i + kAhead] = c_operand(i + kAhead, sub);
      const int cb = i >> 2, c = (i >> 1) & 1;
      if (i & 1) mfma32_acc(op[i], dsb[c].h, dkacc[cb]);
      else mfma32_acc(op[i], pb[c].h, dvacc[cb]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  auto run_ab = [&](bool has_next, const f32x16& s, const f32x16& dp, f32x16& sn, f32x16& dpn,
                    uint32_t nsub, uint32_t csub_stat, int sub_lo, bool do_fill, uint32_t fill_buf,
                    int fill_t0) __attribute__((always_inline)) {
    const bool mf = rg.mask_free(sub_lo);
    if (has_next) {
      if (mf) stage_ab(std::true_type{}, std::false_type{}, s, dp, sn, dpn, nsub, csub_stat, sub_lo, do_fill, fill_buf, fill_t0);
      else stage_ab(std::true_type{}, std::true_type{}, s, dp, sn, dpn, nsub, csub_stat, sub_lo, do_fill, fill_buf, fill_t0);
    } else {
      if (mf) stage_ab(std::false_type{}, std::false_type{}, s, dp, sn, dpn, nsub, csub_stat, sub_lo, do_fill, fill_buf, fill_t0);
      else stage_ab(std::false_type{}, std::true_type{}, s, dp, sn, dpn, nsub, csub_stat, sub_lo, do_fill, fill_buf, fill_t0);
    }
  };

  // ---- prologue: first tile visible, second one requested, logits of block 0 ----
  wait_async_loads();
  __syncthreads();
  if (qt_begin + 1 < qt_end) {
    rows.prepare((qt_begin + 1) * kStream);
    fill(tiles + kBuf, (qt_begin + 1) * kStream);
  }
  if (rg.wave_active) stage_a(0);
  int a_buf = 0, c_buf = 0;   // buffer index `rm` / `tr`,`st` point into
  // Two of the four waves take the tile barrier one stage earlier (before the accumulating
  // stage of block 0 instead of after it).  Both places lie after every read of the previous
  // tile's buffer and before the first read of the next tile, so the barrier means the same
  // for both; but from then on one pair of waves is in a vector stage (light on the LDS) while
  // the other is in an accumulating stage (transposing reads at the rate the LDS delivers),
  // instead of all four hitting the LDS, and then the vector pipe, together.
  const bool early_barrier = wave >= 2;

  for (int qt = qt_begin; qt < qt_end; ++qt) {
    const bool more = qt + 1 < qt_end;
    if (qt + 2 < qt_end) rows.prepare((qt + 2) * kStream);   // table entries of tile qt+2: used two stages later
    // first half: A(tile qt, block 1) with B(tile qt, block 0); then C(block 0)
    if (rg.wave_active) {
      run_ab(true, s0, dp0, s1, dp1, Tl::kSubBytes, 0, qt * kStream, false, 0, 0);
      if (!early_barrier) stage_c(0);
    }
    // tile qt+1 must be visible before stage A touches it; this barrier also
    // retires every reader of tile qt-1, whose buffer the new fill reuses
    const bool do_fill = qt + 2 < qt_end;               // tile qt+2 goes to buffer (a_buf + 2) % 3
    const uint32_t fill_buf = tiles + (a_buf == 0 ? 2 : a_buf - 1) * kBuf;
    const int fill_t0 = (qt + 2) * kStream;
    if (more) {
      wait_async_loads();
      __syncthreads();
      const uint32_t step = a_buf == 2 ? (uint32_t)(-2 * (int)kBuf) : kBuf;
      a_buf = a_buf == 2 ? 0 : a_buf + 1;
#pragma unroll
      for (int kk = 0; kk < kNK; ++kk) la.rm[kk] += step;
    }
    if (early_barrier && rg.wave_active) stage_c(0);
    // second half: A(tile qt+1, block 0) with B(tile qt, block 1); then C(block 1)
    if (rg.wave_active) {
      run_ab(more, s1, dp1, s0, dp0, 0, 32 * 4, qt * kStream + 32, do_fill, fill_buf, fill_t0);
      stage_c(Tl::kSubBytes);
    } else if (do_fill) {        // waves without real keys still move their share of the tile
#pragma unroll
      for (int i = 0; i <= 2 * Tl::kFillPerWave; ++i) fill_piece(i, fill_buf, fill_t0);
    }
    {
      const uint32_t step = c_buf == 2 ? (uint32_t)(-2 * (int)kBuf) : kBuf;
      c_buf = c_buf == 2 ? 0 : c_buf + 1;
#pragma unroll
      for (int cb = 0; cb < D / 32; ++cb) {
        la.tr[cb][0] += step;
        la.tr[cb][1] += step;
      }
      st += step;
    }
  }
  // The accumulating MFMAs are assembly statements, so the compiler does not know their
  // latency: wait it out (8 passes of 4 cycles plus write-back, with a wide margin) before the
  // epilogue reads the accumulators.
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");

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
static int launch_t(const KParams& kp, const void* q, const void* k, const void* v,
                    const void* d_o, const float* delta, const float* lse2, void* dk, void* dv,
                    hipStream_t stream) {
  const size_t smem = dkdv_pipe_smem_bytes<D>(kp.T);
  auto kern = winattn_dkdv_pipe_kernel<D, OutT>;
  if (!allow_full_lds<winattn_dkdv_pipe_kernel<D, OutT>>()) return -1;
  return launch_kernel(kern, dim3(grid_blocks(kp)), dim3(kThreads), smem, stream, kp,
                       static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k),
                       static_cast<const bf16_t*>(v), static_cast<const bf16_t*>(d_o), delta, lse2,
                       static_cast<OutT*>(dk), static_cast<OutT*>(dv));
}

int launch_dkdv_pipe128(const KParams& kp, bool out_f32, const void* q, const void* k,
                        const void* v, const void* d_o, const float* delta, const float* lse2,
                        void* dk, void* dv, hipStream_t stream) {
  return out_f32 ? launch_t<128, float>(kp, q, k, v, d_o, delta, lse2, dk, dv, stream)
                 : launch_t<128, bf16_t>(kp, q, k, v, d_o, delta, lse2, dk, dv, stream);
}

}  // namespace aeris

