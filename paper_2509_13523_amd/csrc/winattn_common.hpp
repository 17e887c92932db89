// Shared device-side pieces of the gfx950 shifted-window attention kernels:
// kernel parameter block, window geometry (cyclic shift + partition + region
// ordering), MFMA operand types, streamed LDS tiles.
//
// Window geometry follows the AERIS paper's Model Architecture section (square
// windows, shifted on alternating layers) with the cyclic wrap of Fig. 2a; the
// region/mask rules are the ones stated in include/aeris_winattn.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace aeris {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int N>
using Const = std::integral_constant<int, N>;

constexpr int kThreads = 256;      // 4 wavefronts of 64 lanes
constexpr int kWaves = 4;
constexpr int kResident = 128;     // tokens a workgroup keeps in registers (32 per wave)
constexpr int kStream = 64;        // tokens per streamed LDS tile
constexpr float kLazyRescale = 8.0f;  // log2 units a row maximum may lag behind
constexpr float kSumLimit = 4096.0f;  // a lane's 16 exponentials of a block may add up to this
constexpr float kLog2e = 1.4426950408889634f;

// Host-filled launch parameters (plain data, passed by value).
struct KParams {
  int B, H, W, nh;
  int ws_h, ws_w, s_h, s_w;
  int mask;            // AERIS_MASK_*
  int nWy, nWx;        // windows along latitude / longitude
  int n_win;           // windows processed per batch member: nWy*nWx, or the length of win_list
  const int* win_list; // device array of n_win window indices wy*nWx + wx, or null = all windows
  int T;               // tokens per window
  int n_tiles;         // resident-side tiles per window = ceil(T / kResident)
  int n_pairs;         // B * n_win * nh
  float scale;         // softmax scale
  float scale_log2;    // scale * log2(e)
  long long qkv_tok, qkv_head;  // element strides of v and of dq, dk, dv
  long long q_tok, q_head;      // element strides of the q the kernel reads
  long long k_tok, k_head;      // element strides of the k the kernel reads
  long long o_tok, o_head;      // element strides of o, dO
  // Rotary embedding of queries and keys (Model Architecture section; off when rope == 0).
  int rope;            // 1: the resident q of the forward kernel is rotated as it is loaded,
                       //    dq and dk are rotated back as they are stored
  int rope_pos;        // AERIS_ROPE_POS_*
  float rope_c;        // log2(base) / (head_dim / 4): theta_t = 2^(-t * rope_c)
  bf16_t* q_rot_out;   // forward kernel, rope == 1: if not null, the rotated queries are also
                       // stored here (compact [B, H, W, heads, head_dim]) for the backward pass
};

// Bytes of the per-window token table: one int per token, padded to a whole
// streamed tile (the padding repeats the last token, so loads never need a clamp).
__host__ __device__ inline int table_bytes(int T) { return ((T + kStream - 1) / kStream) * kStream * 4; }

// ----------------------------------------------------------------------------
// Workgroup id -> (pair, tile).  Hardware deals consecutive workgroup ids to
// the eight XCDs in turn.  Pairs (batch, window, head) are dealt to XCDs
// round-robin (pair % 8), which balances seam windows -- they carry less work
// -- across XCDs, and all tiles of one pair run on that one XCD, so the K/V
// (or Q/dO) rows they all stream are shared through its L2.
// Grid size: 8 * ceil(n_pairs / 8) * n_tiles.  Returns false for padding.
// ----------------------------------------------------------------------------
__device__ __forceinline__ bool block_to_work(const KParams& p, int& pair, int& tile) {
  const int id = blockIdx.x;
  const int xcd = id & 7, slot = id >> 3;
  const int pair_local = slot / p.n_tiles;
  tile = slot - pair_local * p.n_tiles;
  pair = pair_local * 8 + xcd;
  return pair < p.n_pairs;
}
__host__ __device__ inline int grid_blocks(const KParams& p) {
  return 8 * ((p.n_pairs + 7) / 8) * p.n_tiles;
}

// One (batch, window, head) and how its tokens are enumerated.
//
// Tokens of a window are enumerated region by region (at most a 2x2 split of
// the window by the seam rows/columns), row-major inside a region.  Attention
// inside a window does not depend on the enumeration order, and with this one
// every token's visible keys form one contiguous index range [lo, hi), so
// masked blocks are skipped whole and the rest is masked by two compares.
struct Window {
  int b, head, wy, wx;
  int split_r, split_c;   // first row / column of the second region (== side if no seam)
  int wc0, wc1;           // columns in the left / right region
  float inv_wc0, inv_wc1; // their reciprocals (for the row/column split in grid_index)
  int s01, s10, s11, T;   // enumeration start of regions (0,1), (1,0), (1,1)

  // False (uniformly for the workgroup) if a listed window index is out of range: the
  // caller then leaves before touching memory.
  __device__ __forceinline__ bool init(const KParams& p, int pair) {
    head = pair % p.nh;
    const int w = pair / p.nh;
    b = w / p.n_win;
    int idx = w - b * p.n_win;
    if (p.win_list) idx = p.win_list[idx];
    if ((unsigned)idx >= (unsigned)(p.nWy * p.nWx)) return false;
    wy = idx / p.nWx;
    wx = idx - wy * p.nWx;
    const bool lat_seam = p.mask != 0 && wy == p.nWy - 1 && p.s_h > 0;
    const bool lon_seam = p.mask == 2 && wx == p.nWx - 1 && p.s_w > 0;
    split_r = lat_seam ? p.ws_h - p.s_h : p.ws_h;
    split_c = lon_seam ? p.ws_w - p.s_w : p.ws_w;
    wc0 = split_c;
    wc1 = p.ws_w - split_c;
    inv_wc0 = 1.0f / (float)wc0;
    inv_wc1 = 1.0f / (float)(wc1 > 0 ? wc1 : 1);
    const int hr0 = split_r, hr1 = p.ws_h - split_r;
    s01 = hr0 * wc0;
    s10 = s01 + hr0 * wc1;
    s11 = s10 + hr1 * wc0;
    T = p.T;
    return true;
  }
  // Visible key range of token t.
  __device__ __forceinline__ void range(int t, int& lo, int& hi) const {
    if (t < s01) { lo = 0; hi = s01; }
    else if (t < s10) { lo = s01; hi = s10; }
    else if (t < s11) { lo = s10; hi = s11; }
    else { lo = s11; hi = T; }
  }
  // Grid point (row-major index y*W + x) of token t: partition + cyclic shift.
  __device__ __forceinline__ int grid_index(const KParams& p, int t) const {
    int lo, w, r0, c0;
    float inv;
    if (t < s01) { lo = 0; w = wc0; inv = inv_wc0; r0 = 0; c0 = 0; }
    else if (t < s10) { lo = s01; w = wc1; inv = inv_wc1; r0 = 0; c0 = split_c; }
    else if (t < s11) { lo = s10; w = wc0; inv = inv_wc0; r0 = split_r; c0 = 0; }
    else { lo = s11; w = wc1; inv = inv_wc1; r0 = split_r; c0 = split_c; }
    // u / w without an integer division: u < 8192, so the float quotient is off by at most
    // one, which the remainder test repairs (a workgroup evaluates this T/256 times per thread)
    const int u = t - lo;
    int rr = (int)((float)u * inv);
    int cc = u - rr * w;
    if (cc < 0) { rr -= 1; cc += w; }
    else if (cc >= w) { rr += 1; cc -= w; }
    int y = wy * p.ws_h + r0 + rr + p.s_h;
    int x = wx * p.ws_w + c0 + cc + p.s_w;
    if (y >= p.H) y -= p.H;
    if (x >= p.W) x -= p.W;
    return y * p.W + x;
  }
};

// Visible-range bookkeeping for the 128 resident tokens of a workgroup (32 per
// wave, token `first + lane%32` per lane).  Tokens are enumerated region by
// region, so range starts and ends are non-decreasing in the token index.
struct Ranges {
  int tok;            // this lane's resident token, clamped to T-1
  bool valid;         // false for phantom tokens past the window's end
  bool wave_active;   // wave owns at least one real token
  int lo, hi;         // visible streamed tokens of this lane
  int w_lo, w_hi;     // union over the wave (skip streamed blocks outside)
  int lo_max, hi_min; // intersection over the wave (blocks inside need no mask)
  int wg_lo, wg_hi;   // union over the workgroup (loop bounds)

  // resident: tokens a workgroup keeps in registers (32 per wave)
  __device__ __forceinline__ void init(const Window& win, int tile, int wave, int qi,
                                       int resident = kResident) {
    const int T = win.T;
    const int wave_t0 = tile * resident + wave * 32;
    wave_active = wave_t0 < T;
    const int t = wave_t0 + qi;
    valid = t < T;
    tok = valid ? t : T - 1;
    win.range(tok, lo, hi);
    int unused;
    const int wg_last = tile * resident + resident - 1;
    win.range(tile * resident, wg_lo, unused);
    win.range(wg_last < T ? wg_last : T - 1, unused, wg_hi);
    w_lo = w_hi = lo_max = hi_min = 0;
    if (wave_active) {
      const int last = wave_t0 + 31;
      win.range(wave_t0, w_lo, hi_min);
      win.range(last < T ? last : T - 1, lo_max, w_hi);
    }
    // wave-uniform by construction: keep them in scalar registers, so that skip()
    // and mask_free() become scalar branches instead of predicated vector code
    w_lo = __builtin_amdgcn_readfirstlane(w_lo);
    w_hi = __builtin_amdgcn_readfirstlane(w_hi);
    lo_max = __builtin_amdgcn_readfirstlane(lo_max);
    hi_min = __builtin_amdgcn_readfirstlane(hi_min);
    wg_lo = __builtin_amdgcn_readfirstlane(wg_lo);
    wg_hi = __builtin_amdgcn_readfirstlane(wg_hi);
  }
  // Block [s, s+32) of streamed tokens: does this wave need it, and masked?
  __device__ __forceinline__ bool skip(int s) const { return s + 32 <= w_lo || s >= w_hi; }
  __device__ __forceinline__ bool mask_free(int s) const { return s >= lo_max && s + 32 <= hi_min; }
};

// Fill the per-window table token -> y*W + x (in LDS), padding included.
// Caller barriers.
__device__ __forceinline__ void build_token_table(const KParams& p, const Window& win,
                                                  int* tok_grid) {
  const int padded = table_bytes(p.T) / 4;
  for (int t = threadIdx.x; t < padded; t += blockDim.x)
    tok_grid[t] = win.grid_index(p, t < p.T ? t : p.T - 1);
}

// ----------------------------------------------------------------------------
// MFMA wrappers.  v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32].
// Lane l supplies A[l%32][8*(l/32) .. +8] and B[8*(l/32) .. +8][l%32]; it
// receives D[8*(v/4) + 4*(l/32) + v%4][l%32] in accumulator register v.
// Because the eight contraction indices a lane supplies only have to agree
// between A and B, a D tile can be fed back as the B operand of the next
// product without any cross-lane movement: registers 8c..8c+7 of lane l hold
// rows {16c + 4*(l/32) + (0..3), 16c + 8 + 4*(l/32) + (0..3)}, and the A
// operand is fetched in that same row order (Tile::read_tr).
// ----------------------------------------------------------------------------
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of a 32x32 accumulator tile held in register v by a lane of half g.
__device__ __forceinline__ int acc_row(int v, int g) { return 8 * (v >> 2) + 4 * g + (v & 3); }

// max over the lane pair (l, l ^ 32).  v_permlane32_swap hands every lane the value
// of lane l % 32 and the value of lane 32 + l % 32 without a trip through the LDS.
__device__ __forceinline__ float wave_half_max(float x) {
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return *reinterpret_cast<uint32_t*>(&r);
}

// ----------------------------------------------------------------------------
// Axial-frequency 2-D rotary embedding (Model Architecture section).  Channel pair
// j = (2j, 2j+1) of a head turns by theta_t * position, t = j / 2, theta_t =
// base^(-t / (d/4)); even pairs use the longitude position, odd pairs the latitude
// position.  Positions are grid coordinates, or coordinates inside the window in the
// shifted frame.
// ----------------------------------------------------------------------------
__device__ __forceinline__ void rope_position(const KParams& p, int grid_index, float& p_lat,
                                              float& p_lon) {
  int y = grid_index / p.W;
  int x = grid_index - y * p.W;
  if (p.rope_pos == 0) {
    y -= p.s_h;
    if (y < 0) y += p.H;
    y %= p.ws_h;
    x -= p.s_w;
    if (x < 0) x += p.W;
    x %= p.ws_w;
  }
  p_lat = (float)y;
  p_lon = (float)x;
}

// cos and sin of theta_t * pos.  The angle is formed in revolutions with the rounding
// error of the product recovered by an fma, and reduced by fract() before the hardware
// sine/cosine, so the error stays near 1e-7 of a revolution at any position.
__device__ __forceinline__ void rope_cos_sin(float pos, int t, float c, float& cs, float& sn) {
  const float w = __builtin_amdgcn_exp2f(-(float)t * c) * 0.15915494309189535f;
  const float hi = pos * w;
  const float lo = __builtin_fmaf(pos, w, -hi);
  const float rev = __builtin_amdgcn_fractf(hi) + lo;
  cs = __builtin_amdgcn_cosf(rev);
  sn = __builtin_amdgcn_sinf(rev);
}

// Turns four consecutive pairs (eight channels starting at channel ch0, a multiple of 8).
__device__ __forceinline__ bf16x8 rope_rotate8(bf16x8 v, int ch0, float p_lat, float p_lon, float c,
                                               bool inverse) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int j = (ch0 >> 1) + e;
    float cs, sn;
    rope_cos_sin((e & 1) ? p_lat : p_lon, j >> 1, c, cs, sn);
    if (inverse) sn = -sn;
    const float a = (float)v[2 * e], b = (float)v[2 * e + 1];
    r[2 * e] = (bf16_t)__builtin_fmaf(a, cs, -(b * sn));
    r[2 * e + 1] = (bf16_t)__builtin_fmaf(a, sn, b * cs);
  }
  return r;
}

// Turns the two pairs (a0, a1), (a2, a3) at channels ch0 .. ch0+3 (ch0 a multiple of 4)
// back by their angles: the transpose of the embedding, applied to a gradient.
__device__ __forceinline__ void rope_unrotate4(float& a0, float& a1, float& a2, float& a3, int ch0,
                                               float p_lat, float p_lon, float c) {
  const int t = ch0 >> 2;
  float cs, sn;
  rope_cos_sin(p_lon, t, c, cs, sn);
  const float b0 = __builtin_fmaf(a1, sn, a0 * cs), b1 = __builtin_fmaf(-a0, sn, a1 * cs);
  rope_cos_sin(p_lat, t, c, cs, sn);
  const float b2 = __builtin_fmaf(a3, sn, a2 * cs), b3 = __builtin_fmaf(-a2, sn, a3 * cs);
  a0 = b0;
  a1 = b1;
  a2 = b2;
  a3 = b3;
}

// ----------------------------------------------------------------------------
// Streamed tiles in LDS.
//
// A tile is kStream tokens x D channels, row-major, unpadded; the 16-byte
// chunks of token row r sit at chunk position c ^ swz(r).  It is filled
// straight from global memory (global_load_lds_dwordx4: no registers, no VALU
// besides addresses; each wave instruction deposits 64 consecutive chunks, and
// every lane fetches the source chunk that belongs in its slot, so the swizzle
// costs nothing).  It is read two ways:
//   * row-major, ds_read_b128: lane (row l%32, chunk 2*kk + l/32): the A
//     operand of the first products (contraction over channels);
//   * transposed, ds_read_b64_tr_b16: a 16-lane block fetches 4 token rows x
//     16 channels and each lane receives the 4 tokens of ONE channel: the A
//     operand of the second products (contraction over tokens), in the row
//     order {4g..4g+3, 8+4g..8+4g+3} that matches the accumulator layout.
// swz() makes both access patterns bank-conflict free: 16 consecutive rows at
// one logical chunk hit 16 different chunk positions, and 4 consecutive rows x
// 4 consecutive chunks hit 16 different positions.
// ----------------------------------------------------------------------------
#define AERIS_LDS __attribute__((address_space(3)))

__device__ __forceinline__ uint32_t lds_address(const void* generic) {
  return (uint32_t)(uintptr_t)(AERIS_LDS const void*)generic;
}

// 16 bytes per lane, global -> LDS, asynchronously: lane l's data lands at LDS
// byte address lds_base + 16*l (lds_base wave-uniform).  Written as assembly so
// that the compiler does not serialise later LDS reads of OTHER buffers behind
// it; completion is awaited explicitly with wait_async_loads() + a barrier.
__device__ __forceinline__ void async_copy16(const void* src, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(src), "s"(__builtin_amdgcn_readfirstlane(lds_base))
               : "memory");
}
// The same, executed only if `enable` (wave-uniform) is non-zero.  The scalar branch
// sits inside the statement, so a hand-placed schedule keeps the copy at a fixed
// place without the compiler splitting the surrounding code into blocks.
__device__ __forceinline__ void async_copy16_if(const void* src, uint32_t lds_base,
                                                uint32_t enable) {
  asm volatile(
      "s_cmp_eq_u32 %2, 0\n\t"
      "s_cbranch_scc1 1f\n\t"
      "s_mov_b32 m0, %1\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, off\n"
      "1:"
      :
      : "v"(src), "s"(__builtin_amdgcn_readfirstlane(lds_base)),
        "s"(__builtin_amdgcn_readfirstlane(enable))
      : "memory", "scc");
}
// 4 bytes per lane: lane l's dword lands at lds_base + 4*l.
__device__ __forceinline__ void async_copy4(const void* src, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :
               : "v"(src), "s"(__builtin_amdgcn_readfirstlane(lds_base))
               : "memory");
}
// The same copy with the source given as a wave-uniform 64-bit base plus a 32-bit unsigned
// byte offset per lane; executed only if `enable` (wave-uniform) is non-zero.
__device__ __forceinline__ void async_copy16_off(uint32_t offset, unsigned long long base,
                                                 uint32_t lds_base, uint32_t enable = 1) {
  asm volatile(
      "s_cmp_eq_u32 %3, 0\n\t"
      "s_cbranch_scc1 1f\n\t"
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1\n"
      "1:"
      :
      : "v"(offset), "s"(base), "s"(__builtin_amdgcn_readfirstlane(lds_base)),
        "s"(__builtin_amdgcn_readfirstlane(enable))
      : "memory", "scc");
}
__device__ __forceinline__ void wait_async_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Makes the compiler finish the loads that produce `v` here (it then places its
// own wait before this point instead of inside the main loop, where a vmcnt
// wait would also wait for the prefetch of the next tile).
template <typename V>
__device__ __forceinline__ void settle(V& v) {
  asm volatile("" : "+v"(v));
}

// Nothing is scheduled across this point: pins a hand-made interleaving of
// products, operand reads and copies.
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

// W: wavefronts of the workgroup (they share the filling of a tile).
template <int D, int W = kWaves>
struct Tile {
  static constexpr int NC = D / 8;                  // 16-byte chunks per token row
  static constexpr int kBytes = kStream * D * 2;
  static constexpr int kSubBytes = 32 * D * 2;      // 32-token sub-block
  static constexpr int kGroupBytes = 16 * D * 2;    // 16-token group of a second product
  static constexpr int kFillPerWave = NC / W;       // wave instructions per tile and wave
  static_assert(NC % W == 0, "every wave must issue a whole number of copies per tile");

  __device__ __forceinline__ static int swz(int r) {
    if (D == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
    if (D == 64) return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
    return (r >> 2) & 3;
  }
  // Byte offset, inside a tile, of chunk c of token row r.
  __device__ __forceinline__ static int chunk_offset(int r, int c) {
    return (r * NC + (c ^ swz(r))) * 16;
  }

  // Asynchronous tile fill.  A wave instruction moves 64 chunks = kRowsPerInst token
  // rows.  Instruction i of wave w covers rows
  //   i * kRowStep + w * kRowsPerInst + lane / NC,      kRowStep = kRowsPerInst * W,
  // and because swz() has period 16 (which divides kRowStep) the lane's source chunk is
  // the same in every instruction: per 16 bytes moved the source is
  //   src + table[t0 + row_i] * stride_bytes
  // (one LDS table read and one 64-bit multiply-add), with ONE pointer per tensor.
  // Two phases, so the table read's latency is never exposed and the copies can be
  // spread over a compute phase (a burst of them stalls the issuing wave until the
  // memory pipeline drains): Rows::prepare() reads the table entries of a tile into
  // registers; Filler::issue_one()/issue() launch the copies of one tensor.  Tensors
  // streamed together (K and V, or Q and dO) share one Rows.
  static constexpr int kRowsPerInst = 64 / NC;
  static constexpr int kRowStep = kRowsPerInst * W;
  static constexpr int kInstStep = kRowStep * D * 2;   // LDS bytes between instructions
  static_assert(kRowStep % 16 == 0, "swizzle period must divide the instruction row step");
  struct Rows {
    uint32_t tab;                    // LDS byte address of table[row of instruction 0]
    uint32_t g[kFillPerWave];        // grid index of the lane's row in each instruction
    __device__ __forceinline__ void init(uint32_t table_lds, int wave, int lane) {
      tab = table_lds + (wave * kRowsPerInst + lane / NC) * 4;
    }
    // t0: first token of the tile (multiple of kStream)
    __device__ __forceinline__ void prepare(int t0) {
      const uint32_t row0 = tab + t0 * 4;
#pragma unroll
      for (int i = 0; i < kFillPerWave; ++i)
        g[i] = *reinterpret_cast<const AERIS_LDS uint32_t*>(row0 + i * kRowStep * 4);
    }
  };
  struct Filler {
    const char* src;                 // tensor origin of this (batch, head) + lane's chunk
    uint32_t dst;                    // byte offset of this wave's first instruction in a tile
    uint32_t stride_bytes;

    __device__ __forceinline__ void init(const bf16_t* origin, long long tok_stride, int wave,
                                         int lane) {
      stride_bytes = (uint32_t)(tok_stride * 2);
      dst = wave * 1024;
      const int r = wave * kRowsPerInst + lane / NC;
      src = reinterpret_cast<const char*>(origin) + ((lane % NC) ^ swz(r)) * 16;
    }
    // tile: LDS byte address (wave-uniform)
    __device__ __forceinline__ void issue_one(int i, uint32_t tile, const Rows& rows) const {
      async_copy16(src + (unsigned long long)rows.g[i] * stride_bytes, tile + dst + i * kInstStep);
    }
    __device__ __forceinline__ void issue(uint32_t tile, const Rows& rows) const {
#pragma unroll
      for (int i = 0; i < kFillPerWave; ++i) issue_one(i, tile, rows);
    }
    // enable: wave-uniform, non-zero = issue
    __device__ __forceinline__ void issue_one_if(int i, uint32_t tile, const Rows& rows,
                                                 uint32_t enable) const {
      async_copy16_if(src + (unsigned long long)rows.g[i] * stride_bytes,
                      tile + dst + i * kInstStep, enable);
    }
    __device__ __forceinline__ void issue_if(uint32_t tile, const Rows& rows,
                                             uint32_t enable) const {
#pragma unroll
      for (int i = 0; i < kFillPerWave; ++i) issue_one_if(i, tile, rows, enable);
    }
  };

  // Per-lane LDS byte addresses (buffer 0, sub-block 0) of the operand reads.
  struct Lanes {
    uint32_t rm[D / 16];        // row-major: contraction block kk
    uint32_t tr[D / 32][2];     // transposed: channel block cb, first/second four tokens

    __device__ __forceinline__ void init(uint32_t tile0, int lane) {
      const int row = lane & 31, g = lane >> 5;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) rm[kk] = tile0 + chunk_offset(row, 2 * kk + g);
      const int j = lane & 15, blk = lane >> 4;
#pragma unroll
      for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int r = 8 * h + 4 * (blk >> 1) + (j >> 2);
          const int c = 4 * cb + 2 * (blk & 1) + ((j & 3) >> 1);
          tr[cb][h] = tile0 + chunk_offset(r, c) + (j & 1) * 8;
        }
      // keep the finished addresses in registers (reads then need no VALU at all)
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) settle(rm[kk]);
#pragma unroll
      for (int cb = 0; cb < D / 32; ++cb) {
        settle(tr[cb][0]);
        settle(tr[cb][1]);
      }
    }
  };

  __device__ __forceinline__ static bf16x8 read_rm(uint32_t addr) {
    return *reinterpret_cast<const AERIS_LDS bf16x8*>(addr);
  }
  // A operand of a second product: channel block cb, tokens of 16-token group at `addr_*`.
  __device__ __forceinline__ static bf16x8 read_tr(uint32_t addr_first, uint32_t addr_second) {
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        reinterpret_cast<AERIS_LDS bf16x4*>(addr_first));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        reinterpret_cast<AERIS_LDS bf16x4*>(addr_second));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }
};

// Output element stores: four consecutive channels of one token.
__device__ __forceinline__ void store4(bf16_t* dst, float a, float b, float c, float d) {
  u32x2 v = {pack_bf16(a, b), pack_bf16(c, d)};
  *reinterpret_cast<u32x2*>(dst) = v;
}
__device__ __forceinline__ void store4(float* dst, float a, float b, float c, float d) {
  f32x4 v = {a, b, c, d};
  *reinterpret_cast<f32x4*>(dst) = v;
}

}  // namespace aeris
