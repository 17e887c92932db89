// Axial-frequency 2-D rotary embedding of a [B, H_lat, W_lon, heads, head_dim] bf16
// tensor (AERIS paper, Model Architecture section: queries and keys are rotated before
// the dot-product attention).  Elementwise and bound by HBM traffic: every 16-byte chunk
// (four channel pairs) is read once and written once.
//
// The attention kernels stream one operand from global memory into the LDS without
// passing registers, so that operand cannot be rotated on the way; it is rotated once
// by this kernel into a workspace instead.  The operand a kernel keeps in registers is
// rotated as it is loaded, and gradients are rotated back as they are stored (see the
// attention kernels).
#include "winattn_common.hpp"
#include "winattn_launch.hpp"

namespace aeris {

__global__ __launch_bounds__(256) void rope2d_kernel(KParams p, int chunks_per_head,
                                                     const bf16_t* x, long long x_tok,
                                                     long long x_head, bf16_t* y,
                                                     long long y_tok, long long y_head, int inverse,
                                                     long long n_chunks) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  const long long plane = (long long)p.H * p.W;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n_chunks; i += stride) {
    const int c = (int)(i % chunks_per_head);
    const long long r = i / chunks_per_head;
    const int head = (int)(r % p.nh);
    const long long tok = r / p.nh;                    // b * plane + grid index
    const int grid_index = (int)(tok % plane);
    float p_lat, p_lon;
    rope_position(p, grid_index, p_lat, p_lon);
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(x + tok * x_tok + head * x_head + c * 8);
    *reinterpret_cast<bf16x8*>(y + tok * y_tok + head * y_head + c * 8) =
        rope_rotate8(v, c * 8, p_lat, p_lon, p.rope_c, inverse != 0);
  }
}

// The same rotation for the tokens of the listed windows only (a rank's share): chunk i ->
// (pair, token of its window, chunk of the head); positions outside the listed windows are
// neither read nor written.
__global__ __launch_bounds__(256) void rope2d_windows_kernel(
    KParams p, int chunks_per_head, const bf16_t* x, long long x_tok, long long x_head, bf16_t* y,
    long long y_tok, long long y_head, int inverse,
    long long n_chunks) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  const long long plane = (long long)p.H * p.W;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n_chunks; i += stride) {
    const int c = (int)(i % chunks_per_head);
    const long long r = i / chunks_per_head;
    const int t = (int)(r % p.T);
    const int pair = (int)(r / p.T);
    Window win;
    if (!win.init(p, pair)) continue;   // list entry outside the grid of windows
    const int grid_index = win.grid_index(p, t);
    const long long tok = (long long)win.b * plane + grid_index;
    float p_lat, p_lon;
    rope_position(p, grid_index, p_lat, p_lon);
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(x + tok * x_tok + win.head * x_head + c * 8);
    *reinterpret_cast<bf16x8*>(y + tok * y_tok + win.head * y_head + c * 8) =
        rope_rotate8(v, c * 8, p_lat, p_lon, p.rope_c, inverse != 0);
  }
}

int launch_rope(const KParams& kp, int head_dim, const void* x, long long x_tok, long long x_head,
                void* y, long long y_tok, long long y_head, bool inverse, hipStream_t stream) {
  const int chunks_per_head = head_dim / 8;
  const bool listed = kp.win_list != nullptr;
  const long long n_chunks = listed ? (long long)kp.n_pairs * kp.T * chunks_per_head
                                    : (long long)kp.B * kp.H * kp.W * kp.nh * chunks_per_head;
  long long blocks = (n_chunks + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;           // grid-stride: 32 workgroups per CU
  return launch_kernel(listed ? rope2d_windows_kernel : rope2d_kernel, dim3((unsigned)blocks),
                       dim3(256), 0, stream, kp, chunks_per_head, static_cast<const bf16_t*>(x),
                       x_tok, x_head, static_cast<bf16_t*>(y), y_tok, y_head, inverse ? 1 : 0,
                       n_chunks);
}

}  // namespace aeris
