// C ABI of the shifted-window attention library: argument validation,
// parameter derivation and dispatch.  See include/aeris_winattn.h for the
// contract of every entry point.
#include "aeris_winattn.h"

#include "aeris_probe.h"

#include <math.h>

#include <atomic>

#include "winattn_launch.hpp"

// Scratch of aeris_winattn_bwd_static: the backward kernels' per-token statistics (delta and
// LSE * log2 e), which the other backward entry points keep in the caller's workspace.  One copy
// per GPU the library is loaded on, held until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress; kernels receive the device address that call returns.
static __device__ __align__(256) unsigned char scratch[AERIS_BWD_STATIC_SCRATCH_BYTES];

namespace {

struct Strides {
  long long qkv_tok, qkv_head, o_tok, o_head;
};

int resolve(const aeris_winattn_params* p, Strides* s) {
  if (!p) return AERIS_ERR_NULL_POINTER;
  if (p->B <= 0 || p->H_lat <= 0 || p->W_lon <= 0 || p->heads <= 0 || p->win_h <= 0 ||
      p->win_w <= 0)
    return AERIS_ERR_INVALID_SHAPE;
  if (p->head_dim != 32 && p->head_dim != 64 && p->head_dim != 128)
    return AERIS_ERR_UNSUPPORTED_HEAD_DIM;
  if (p->H_lat % p->win_h != 0 || p->W_lon % p->win_w != 0) return AERIS_ERR_NOT_DIVISIBLE;
  if (p->shift_h < 0 || p->shift_h >= p->win_h || p->shift_w < 0 || p->shift_w >= p->win_w)
    return AERIS_ERR_BAD_SHIFT;
  if (p->mask_policy != AERIS_MASK_NONE && p->mask_policy != AERIS_MASK_LAT &&
      p->mask_policy != AERIS_MASK_SWIN)
    return AERIS_ERR_BAD_MASK;
  if (p->out_dtype != AERIS_DT_BF16 && p->out_dtype != AERIS_DT_F32) return AERIS_ERR_BAD_DTYPE;
  if ((long long)p->win_h * p->win_w > AERIS_MAX_WINDOW_TOKENS) return AERIS_ERR_WINDOW_TOO_LARGE;
  if ((long long)p->H_lat * p->W_lon >= (1LL << 31)) return AERIS_ERR_INVALID_SHAPE;
  if ((long long)p->B * p->heads * (p->H_lat / p->win_h) * (p->W_lon / p->win_w) *
          (((long long)p->win_h * p->win_w + 127) / 128) >= (1LL << 31) - 8)
    return AERIS_ERR_INVALID_SHAPE;
  const long long d = p->head_dim;
  s->qkv_head = p->qkv_head_stride ? p->qkv_head_stride : d;
  s->o_head = p->o_head_stride ? p->o_head_stride : d;
  s->qkv_tok = p->qkv_tok_stride ? p->qkv_tok_stride : (long long)p->heads * d;
  s->o_tok = p->o_tok_stride ? p->o_tok_stride : (long long)p->heads * d;
  if (s->qkv_head < d || s->o_head < d) return AERIS_ERR_INVALID_SHAPE;
  if (s->qkv_tok < (p->heads - 1) * s->qkv_head + d) return AERIS_ERR_INVALID_SHAPE;
  if (s->o_tok < (p->heads - 1) * s->o_head + d) return AERIS_ERR_INVALID_SHAPE;
  if ((s->qkv_head | s->qkv_tok | s->o_head | s->o_tok) & 7) return AERIS_ERR_MISALIGNED;
  return AERIS_OK;
}

aeris::KParams derive(const aeris_winattn_params* p, const Strides& s) {
  aeris::KParams k;
  k.B = p->B;
  k.H = p->H_lat;
  k.W = p->W_lon;
  k.nh = p->heads;
  k.ws_h = p->win_h;
  k.ws_w = p->win_w;
  k.s_h = p->shift_h;
  k.s_w = p->shift_w;
  k.mask = p->mask_policy;
  k.nWy = p->H_lat / p->win_h;
  k.nWx = p->W_lon / p->win_w;
  k.T = p->win_h * p->win_w;
  k.n_tiles = (k.T + aeris::kResident - 1) / aeris::kResident;
  k.n_win = k.nWy * k.nWx;
  k.win_list = nullptr;
  k.n_pairs = k.B * k.n_win * k.nh;
  k.scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.f / sqrtf((float)p->head_dim);
  k.scale_log2 = k.scale * 1.4426950408889634f;
  k.qkv_tok = k.q_tok = k.k_tok = s.qkv_tok;
  k.qkv_head = k.q_head = k.k_head = s.qkv_head;
  k.o_tok = s.o_tok;
  k.o_head = s.o_head;
  k.rope = 0;
  k.rope_pos = 0;
  k.rope_c = 0.f;
  k.q_rot_out = nullptr;
  return k;
}

int resolve_rope(const aeris_winattn_params* p, const aeris_rope_params* r, aeris::KParams* k) {
  if (!r) return AERIS_ERR_NULL_POINTER;
  if (!(r->base > 1.f) || !isfinite(r->base)) return AERIS_ERR_BAD_ROPE;
  if (r->positions != AERIS_ROPE_POS_WINDOW && r->positions != AERIS_ROPE_POS_GRID)
    return AERIS_ERR_BAD_ROPE;
  k->rope = 1;
  k->rope_pos = r->positions;
  k->rope_c = log2f(r->base) / (float)(p->head_dim / 4);
  return AERIS_OK;
}

// Bytes of one compact [B, H, W, heads, head_dim] bf16 tensor, rounded up to 256.
size_t dense_tensor_bytes(const aeris_winattn_params* p) {
  const size_t n = (size_t)p->B * p->H_lat * p->W_lon * p->heads * p->head_dim * 2;
  return (n + 255) & ~(size_t)255;
}

bool misaligned(const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) != 0; }

}  // namespace

extern "C" {

int aeris_winattn_validate(const aeris_winattn_params* p) {
  Strides s;
  return resolve(p, &s);
}

int aeris_winattn_fwd(const aeris_winattn_params* p, const void* q, const void* k, const void* v,
                      void* o, float* lse, void* hip_stream) {
  Strides s;
  const int rc = resolve(p, &s);
  if (rc != AERIS_OK) return rc;
  if (!q || !k || !v || !o || !lse) return AERIS_ERR_NULL_POINTER;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse))
    return AERIS_ERR_MISALIGNED;
  const aeris::KParams kp = derive(p, s);
  if (aeris::launch_fwd(kp, p->head_dim, p->out_dtype == AERIS_DT_F32, q, k, v, o, lse,
                        static_cast<hipStream_t>(hip_stream)) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  return AERIS_OK;
}

// Restricts derived parameters to a list of windows.
int restrict_windows(aeris::KParams* k, const int32_t* windows, int32_t n_windows) {
  if (!windows) return AERIS_ERR_NULL_POINTER;
  if (n_windows <= 0 || n_windows > k->nWy * k->nWx) return AERIS_ERR_INVALID_SHAPE;
  if (reinterpret_cast<uintptr_t>(windows) & 3) return AERIS_ERR_MISALIGNED;
  k->win_list = windows;
  k->n_win = n_windows;
  k->n_pairs = k->B * k->n_win * k->nh;
  return AERIS_OK;
}

int aeris_winattn_fwd_windows(const aeris_winattn_params* p, const int32_t* windows,
                              int32_t n_windows, const void* q, const void* k, const void* v,
                              void* o, float* lse, void* hip_stream) {
  Strides s;
  int rc = resolve(p, &s);
  if (rc != AERIS_OK) return rc;
  if (!q || !k || !v || !o || !lse) return AERIS_ERR_NULL_POINTER;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse))
    return AERIS_ERR_MISALIGNED;
  aeris::KParams kp = derive(p, s);
  rc = restrict_windows(&kp, windows, n_windows);
  if (rc != AERIS_OK) return rc;
  if (aeris::launch_fwd(kp, p->head_dim, p->out_dtype == AERIS_DT_F32, q, k, v, o, lse,
                        static_cast<hipStream_t>(hip_stream)) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  return AERIS_OK;
}

int aeris_winattn_bwd_windows(const aeris_winattn_params* p, const int32_t* windows,
                              int32_t n_windows, const void* q, const void* k, const void* v,
                              const void* o, const float* lse, const void* d_o, void* dq, void* dk,
                              void* dv, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  Strides s;
  int rc = resolve(p, &s);
  if (rc != AERIS_OK) return rc;
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !workspace)
    return AERIS_ERR_NULL_POINTER;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) ||
      misaligned(d_o) || misaligned(dq) || misaligned(dk) || misaligned(dv) ||
      misaligned(workspace))
    return AERIS_ERR_MISALIGNED;
  aeris::KParams kp = derive(p, s);
  rc = restrict_windows(&kp, windows, n_windows);
  if (rc != AERIS_OK) return rc;
  if (workspace_bytes < aeris::bwd_workspace_bytes(kp)) return AERIS_ERR_WORKSPACE_TOO_SMALL;
  if (aeris::launch_bwd(kp, p->head_dim, p->out_dtype == AERIS_DT_F32, q, k, v, o, lse, d_o, dq,
                        dk, dv, static_cast<float*>(workspace),
                        static_cast<hipStream_t>(hip_stream), AERIS_BWD_ALL) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  return AERIS_OK;
}

size_t aeris_winattn_bwd_workspace_bytes(const aeris_winattn_params* p) {
  Strides s;
  if (resolve(p, &s) != AERIS_OK) return 0;
  return aeris::bwd_workspace_bytes(derive(p, s));
}

int aeris_winattn_bwd(const aeris_winattn_params* p, const void* q, const void* k, const void* v,
                      const void* o, const float* lse, const void* d_o, void* dq, void* dk,
                      void* dv, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return aeris_winattn_bwd_stages(p, q, k, v, o, lse, d_o, dq, dk, dv, workspace, workspace_bytes,
                                  hip_stream, AERIS_BWD_ALL);
}

int aeris_winattn_bwd_stages(const aeris_winattn_params* p, const void* q, const void* k,
                             const void* v, const void* o, const float* lse, const void* d_o,
                             void* dq, void* dk, void* dv, void* workspace,
                             size_t workspace_bytes, void* hip_stream, unsigned stages) {
  Strides s;
  const int rc = resolve(p, &s);
  if (rc != AERIS_OK) return rc;
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !workspace)
    return AERIS_ERR_NULL_POINTER;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) ||
      misaligned(d_o) || misaligned(dq) || misaligned(dk) || misaligned(dv) ||
      misaligned(workspace))
    return AERIS_ERR_MISALIGNED;
  if (workspace_bytes < aeris_winattn_bwd_workspace_bytes(p)) return AERIS_ERR_WORKSPACE_TOO_SMALL;
  const aeris::KParams kp = derive(p, s);
  if (aeris::launch_bwd(kp, p->head_dim, p->out_dtype == AERIS_DT_F32, q, k, v, o, lse, d_o, dq,
                        dk, dv, static_cast<float*>(workspace),
                        static_cast<hipStream_t>(hip_stream), stages & AERIS_BWD_ALL) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  return AERIS_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
static int static_scratch_address(float** out) {
  static std::atomic<void*> address[aeris::kMaxTrackedDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= aeris::kMaxTrackedDevices)
    return AERIS_ERR_HIP_SYMBOL;
  void* ptr = address[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr)
      return AERIS_ERR_HIP_SYMBOL;
    address[dev].store(ptr, std::memory_order_release);
  }
  *out = static_cast<float*>(ptr);
  return AERIS_OK;
}

int aeris_winattn_bwd_static(const aeris_winattn_params* p, const void* q, const void* k,
                             const void* v, const void* o, const float* lse, const void* d_o,
                             void* dq, void* dk, void* dv, void* hip_stream) {
  Strides s;
  int rc = resolve(p, &s);
  if (rc != AERIS_OK) return rc;
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv) return AERIS_ERR_NULL_POINTER;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) ||
      misaligned(d_o) || misaligned(dq) || misaligned(dk) || misaligned(dv))
    return AERIS_ERR_MISALIGNED;
  const aeris::KParams kp = derive(p, s);
  if (aeris::bwd_workspace_bytes(kp) > (size_t)AERIS_BWD_STATIC_SCRATCH_BYTES)
    return AERIS_ERR_STATIC_SCRATCH_TOO_SMALL;
  float* stats = nullptr;
  rc = static_scratch_address(&stats);
  if (rc != AERIS_OK) return rc;
  // Nothing in the array has to start at zero: the dQ kernel writes every statistic the dK/dV
  // kernel reads (all tokens of all pairs plus the padding behind the last pair) in this call.
  if (aeris::launch_bwd(kp, p->head_dim, p->out_dtype == AERIS_DT_F32, q, k, v, o, lse, d_o, dq,
                        dk, dv, stats, static_cast<hipStream_t>(hip_stream), AERIS_BWD_ALL) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  return AERIS_OK;
}

int aeris_rope2d_apply(const aeris_winattn_params* p, const aeris_rope_params* r, const void* x,
                       void* y, int32_t inverse, void* hip_stream) {
  Strides s;
  int rc = resolve(p, &s);
  if (rc != AERIS_OK) return rc;
  aeris::KParams kp = derive(p, s);
  rc = resolve_rope(p, r, &kp);
  if (rc != AERIS_OK) return rc;
  if (!x || !y) return AERIS_ERR_NULL_POINTER;
  if (misaligned(x) || misaligned(y)) return AERIS_ERR_MISALIGNED;
  if (aeris::launch_rope(kp, p->head_dim, x, s.qkv_tok, s.qkv_head, y, s.qkv_tok, s.qkv_head,
                         inverse != 0, static_cast<hipStream_t>(hip_stream)) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  return AERIS_OK;
}

size_t aeris_winattn_rope_fwd_workspace_bytes(const aeris_winattn_params* p) {
  Strides s;
  if (resolve(p, &s) != AERIS_OK) return 0;
  return 2 * dense_tensor_bytes(p);
}

size_t aeris_winattn_rope_bwd_workspace_bytes(const aeris_winattn_params* p) {
  Strides s;
  if (resolve(p, &s) != AERIS_OK) return 0;
  return 2 * dense_tensor_bytes(p) + aeris::bwd_workspace_bytes(derive(p, s));
}

// windows == nullptr: all windows
static int rope_fwd_impl(const aeris_winattn_params* p, const aeris_rope_params* r,
                         const int32_t* windows, int32_t n_windows, bool listed, const void* q,
                         const void* k, const void* v, void* o, float* lse, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  Strides s;
  int rc = resolve(p, &s);
  if (rc != AERIS_OK) return rc;
  aeris::KParams kp = derive(p, s);
  rc = resolve_rope(p, r, &kp);
  if (rc != AERIS_OK) return rc;
  if (!q || !k || !v || !o || !lse || !workspace) return AERIS_ERR_NULL_POINTER;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) ||
      misaligned(workspace))
    return AERIS_ERR_MISALIGNED;
  if (listed) {
    rc = restrict_windows(&kp, windows, n_windows);
    if (rc != AERIS_OK) return rc;
  }
  if (workspace_bytes < aeris_winattn_rope_fwd_workspace_bytes(p))
    return AERIS_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // rotated keys, compact layout
  const long long d = p->head_dim, dense_tok = (long long)p->heads * d;
  if (aeris::launch_rope(kp, p->head_dim, k, s.qkv_tok, s.qkv_head, workspace, dense_tok, d, false,
                         stream) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  kp.k_tok = dense_tok;
  kp.k_head = d;
  // the kernel rotates its resident queries as it loads them and leaves a copy behind the
  // rotated keys: together they are what the backward pass multiplies with
  kp.q_rot_out = reinterpret_cast<aeris::bf16_t*>(static_cast<char*>(workspace) +
                                                  dense_tensor_bytes(p));
  if (aeris::launch_fwd(kp, p->head_dim, p->out_dtype == AERIS_DT_F32, q, workspace, v, o, lse,
                        stream) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  return AERIS_OK;
}

static int rope_bwd_impl(const aeris_winattn_params* p, const aeris_rope_params* r,
                         const int32_t* windows, int32_t n_windows, bool listed, const void* q,
                         const void* k, const void* v, const void* o, const float* lse,
                         const void* d_o, void* dq, void* dk, void* dv, const void* saved,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  Strides s;
  int rc = resolve(p, &s);
  if (rc != AERIS_OK) return rc;
  aeris::KParams kp = derive(p, s);
  rc = resolve_rope(p, r, &kp);
  if (rc != AERIS_OK) return rc;
  if ((!saved && (!q || !k)) || !v || !o || !lse || !d_o || !dq || !dk || !dv || !workspace)
    return AERIS_ERR_NULL_POINTER;
  if ((!saved && (misaligned(q) || misaligned(k))) || misaligned(v) || misaligned(o) ||
      misaligned(lse) || misaligned(d_o) || misaligned(dq) || misaligned(dk) || misaligned(dv) ||
      misaligned(saved) || misaligned(workspace))
    return AERIS_ERR_MISALIGNED;
  if (listed) {
    rc = restrict_windows(&kp, windows, n_windows);
    if (rc != AERIS_OK) return rc;
  }
  const size_t tensor = dense_tensor_bytes(p);
  const size_t need = saved ? aeris::bwd_workspace_bytes(derive(p, s))
                            : aeris_winattn_rope_bwd_workspace_bytes(p);
  if (workspace_bytes < need) return AERIS_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const long long d = p->head_dim, dense_tok = (long long)p->heads * d;
  const void *q_rot, *k_rot;
  float* stats;
  if (saved) {
    // what the forward call left in its workspace: rotated k | rotated q
    k_rot = saved;
    q_rot = static_cast<const char*>(saved) + tensor;
    stats = static_cast<float*>(workspace);
  } else {
    // workspace: rotated q | rotated k | statistics of the backward kernels
    char* ws = static_cast<char*>(workspace);
    q_rot = ws;
    k_rot = ws + tensor;
    stats = reinterpret_cast<float*>(ws + 2 * tensor);
    if (aeris::launch_rope(kp, p->head_dim, q, s.qkv_tok, s.qkv_head, ws, dense_tok, d, false,
                           stream) != 0 ||
        aeris::launch_rope(kp, p->head_dim, k, s.qkv_tok, s.qkv_head, ws + tensor, dense_tok, d,
                           false, stream) != 0)
      return AERIS_ERR_HIP_LAUNCH;
  }
  kp.q_tok = kp.k_tok = dense_tok;
  kp.q_head = kp.k_head = d;
  if (aeris::launch_bwd(kp, p->head_dim, p->out_dtype == AERIS_DT_F32, q_rot, k_rot, v, o, lse,
                        d_o, dq, dk, dv, stats, stream, AERIS_BWD_ALL) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  return AERIS_OK;
}

int aeris_winattn_rope_fwd(const aeris_winattn_params* p, const aeris_rope_params* r,
                           const void* q, const void* k, const void* v, void* o, float* lse,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  return rope_fwd_impl(p, r, nullptr, 0, false, q, k, v, o, lse, workspace, workspace_bytes,
                       hip_stream);
}

int aeris_winattn_rope_bwd(const aeris_winattn_params* p, const aeris_rope_params* r,
                           const void* q, const void* k, const void* v, const void* o,
                           const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                           const void* saved, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
  return rope_bwd_impl(p, r, nullptr, 0, false, q, k, v, o, lse, d_o, dq, dk, dv, saved, workspace,
                       workspace_bytes, hip_stream);
}

int aeris_winattn_rope_fwd_windows(const aeris_winattn_params* p, const aeris_rope_params* r,
                                   const int32_t* windows, int32_t n_windows, const void* q,
                                   const void* k, const void* v, void* o, float* lse,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  return rope_fwd_impl(p, r, windows, n_windows, true, q, k, v, o, lse, workspace,
                       workspace_bytes, hip_stream);
}

int aeris_winattn_rope_bwd_windows(const aeris_winattn_params* p, const aeris_rope_params* r,
                                   const int32_t* windows, int32_t n_windows, const void* q,
                                   const void* k, const void* v, const void* o, const float* lse,
                                   const void* d_o, void* dq, void* dk, void* dv, const void* saved,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  return rope_bwd_impl(p, r, windows, n_windows, true, q, k, v, o, lse, d_o, dq, dk, dv, saved,
                       workspace, workspace_bytes, hip_stream);
}

int aeris_mfma_loop_probe(int32_t blocks, int32_t iters, int32_t random_operands, float* sink,
                          void* hip_stream) {
  if (!sink) return AERIS_ERR_NULL_POINTER;
  if (blocks < 1 || blocks > 65536 || iters < 1) return AERIS_ERR_INVALID_SHAPE;
  if (misaligned(sink)) return AERIS_ERR_MISALIGNED;
  if (aeris::launch_mfma_loop(blocks, iters, random_operands != 0, sink,
                              static_cast<hipStream_t>(hip_stream)) != 0)
    return AERIS_ERR_HIP_LAUNCH;
  return AERIS_OK;
}

const char* aeris_winattn_strerror(int code) {
  switch (code) {
    case AERIS_OK: return "ok";
    case AERIS_ERR_NULL_POINTER: return "null pointer argument";
    case AERIS_ERR_INVALID_SHAPE: return "invalid shape or stride";
    case AERIS_ERR_NOT_DIVISIBLE: return "window does not divide the grid";
    case AERIS_ERR_BAD_SHIFT: return "shift must satisfy 0 <= shift < window";
    case AERIS_ERR_BAD_MASK: return "unknown mask policy";
    case AERIS_ERR_UNSUPPORTED_HEAD_DIM: return "head_dim must be 32, 64 or 128";
    case AERIS_ERR_MISALIGNED: return "pointer or stride not 16-byte aligned";
    case AERIS_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case AERIS_ERR_WINDOW_TOO_LARGE: return "window has more tokens than AERIS_MAX_WINDOW_TOKENS";
    case AERIS_ERR_BAD_DTYPE: return "unknown output dtype";
    case AERIS_ERR_HIP_LAUNCH: return "HIP kernel launch failed";
    case AERIS_ERR_BAD_ROPE: return "rotary base must be > 1 and the position mode known";
    case AERIS_ERR_STATIC_SCRATCH_TOO_SMALL:
      return "problem needs more backward scratch than AERIS_BWD_STATIC_SCRATCH_BYTES";
    case AERIS_ERR_HIP_SYMBOL: return "address of the static scratch array not available on this device";
  }
  return "unknown error code";
}

int aeris_winattn_version(void) { return 2 * 10000 + 0 * 100 + 0; }

}  // extern "C"
