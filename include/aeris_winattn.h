/*
 * aeris_winattn.h -- C ABI of the MI355X (gfx950) shifted-window attention library.
 *
 * The operation is the attention step of the AERIS Swin diffusion transformer
 * (paper, "AERIS Model Architecture": the embedded image is partitioned into
 * square windows that are shifted on alternating layers, queries/keys/values
 * are projected per head, and dot-product attention runs inside each window;
 * "SWiPe", Overview: windows are disjoint, no halo).  Pixel-level tokens live
 * on a [B, H_lat, W_lon, heads, head_dim] grid.
 *
 * For window (wy, wx) and local token (r, c) the grid point is
 *     y = (wy*win_h + r + shift_h) mod H_lat,  x = (wx*win_w + c + shift_w) mod W_lon
 * (cyclic in both axes; Fig. 2a, right panel).  Within a window and head
 *     S = softmax_scale * Q K^T,  masked where region(i) != region(j),
 *     LSE_i = ln sum_j exp(S_ij),  P = exp(S - LSE),  O = P V,
 * and for the backward pass, given dO,
 *     dV = P^T dO,  dP = dO V^T,  delta_i = sum_c dO_ic O_ic,
 *     dS = P o (dP - delta),  dQ = scale * dS K,  dK = scale * dS^T Q.
 * Results are written at the original (unshifted) grid coordinates.
 *
 * The paper does not mention a boundary mask for shifted windows.  Three
 * policies are offered; regions are defined in the shifted frame, per axis of
 * length L, window side ws, shift s: coordinate u is in region 0 if u < L-ws,
 * 1 if L-ws <= u < L-s, 2 otherwise.
 *     AERIS_MASK_NONE  no mask (periodic wrap on both axes)
 *     AERIS_MASK_LAT   latitude regions separate (the pole-to-pole seam), the
 *                      longitude seam stays periodic
 *     AERIS_MASK_SWIN  latitude and longitude regions both separate, as in the
 *                      masked shifted-window attention of the Swin paper
 *
 * Arithmetic: bf16 operands, fp32 accumulation (paper, "Mixed precision"),
 * P rounded to bf16 before the P V product, outputs rounded to nearest even.
 *
 * All pointers are DEVICE pointers on the current HIP device unless stated.
 * The caller owns every buffer.  The library allocates nothing, frees nothing
 * and never synchronises: every call only enqueues kernels on `hip_stream`
 * (a hipStream_t passed as void*; NULL is the default stream).  Inputs are
 * read-only, outputs are fully overwritten.  Calls are thread-safe.  The only
 * process-wide state is a per-device flag per kernel ("this kernel may use the
 * whole LDS", set on the first launch on that device; not valid across
 * hipDeviceReset) and, for aeris_winattn_bwd_static alone, its static scratch
 * array.  Arguments are validated before anything is launched, so every error
 * except AERIS_ERR_HIP_LAUNCH and AERIS_ERR_HIP_SYMBOL is reachable without a GPU.
 */
#ifndef AERIS_WINATTN_H
#define AERIS_WINATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { AERIS_MASK_NONE = 0, AERIS_MASK_LAT = 1, AERIS_MASK_SWIN = 2 };
enum { AERIS_DT_BF16 = 0, AERIS_DT_F32 = 1 };

enum {
  AERIS_OK = 0,
  AERIS_ERR_NULL_POINTER = -1,
  AERIS_ERR_INVALID_SHAPE = -2,        /* a dimension <= 0, or a stride too small   */
  AERIS_ERR_NOT_DIVISIBLE = -3,        /* window does not divide the grid           */
  AERIS_ERR_BAD_SHIFT = -4,            /* need 0 <= shift < window                  */
  AERIS_ERR_BAD_MASK = -5,
  AERIS_ERR_UNSUPPORTED_HEAD_DIM = -6, /* head_dim must be 32, 64 or 128            */
  AERIS_ERR_MISALIGNED = -7,           /* 16-byte alignment of pointers and strides */
  AERIS_ERR_WORKSPACE_TOO_SMALL = -8,
  AERIS_ERR_WINDOW_TOO_LARGE = -9,     /* win_h*win_w > AERIS_MAX_WINDOW_TOKENS     */
  AERIS_ERR_BAD_DTYPE = -10,
  AERIS_ERR_HIP_LAUNCH = -11,          /* the launch call reported an error         */
  AERIS_ERR_BAD_ROPE = -12,            /* rotary base <= 1 or unknown position mode */
  AERIS_ERR_STATIC_SCRATCH_TOO_SMALL = -13, /* aeris_winattn_bwd_static: problem too large */
  AERIS_ERR_HIP_SYMBOL = -14           /* aeris_winattn_bwd_static: no device address of its
                                          scratch array (hipGetSymbolAddress failed, or device
                                          ordinal >= 64)                            */
};

/* Largest window (tokens) the kernels' on-chip offset table holds. */
#define AERIS_MAX_WINDOW_TOKENS 8192

typedef struct {
  int32_t B, H_lat, W_lon, heads, head_dim; /* grid; head_dim in {32, 64, 128}               */
  int32_t win_h, win_w;                     /* window; must divide H_lat, W_lon              */
  int32_t shift_h, shift_w;                 /* cyclic shift, 0 <= shift < win                */
  int32_t mask_policy;                      /* AERIS_MASK_*                                  */
  float softmax_scale;                      /* <= 0 selects 1/sqrt(head_dim)                 */
  int32_t out_dtype;                        /* AERIS_DT_*: type of O, dQ, dK, dV             */
  /* Element strides between tokens and between heads.  0 selects the compact
   * layout (tok = heads*head_dim, head = head_dim).  qkv_* apply to q, k, v and
   * to dq, dk, dv (a packed QKV buffer is passed without a copy); o_* apply to
   * o and d_o.  Batch and row strides follow: row = W_lon*tok, batch = H_lat*row.
   * Strides must be multiples of 8 elements. */
  int64_t qkv_tok_stride, qkv_head_stride;
  int64_t o_tok_stride, o_head_stride;
} aeris_winattn_params;

/*
 * Forward (Model Architecture section: window partition + shift, dot-product
 * attention per window and head).
 *   q, k, v : bf16 [B, H_lat, W_lon, heads, head_dim] with the qkv strides, read-only
 *   o       : out_dtype, same logical shape with the o strides, overwritten
 *   lse     : float32 [B, heads, H_lat, W_lon] compact, natural-log LSE of the
 *             scaled, masked logits, at original grid coordinates, overwritten
 * Returns AERIS_OK or a negative AERIS_ERR_* code; on error nothing was launched
 * (except AERIS_ERR_HIP_LAUNCH, which reports a failed launch).
 */
int aeris_winattn_fwd(const aeris_winattn_params* p, const void* q, const void* k,
                      const void* v, void* o, float* lse, void* hip_stream);

/* Bytes of device workspace the backward pass needs (two float32 vectors with one
 * entry per token and head, plus padding: delta and the LSE in log2 units, in
 * the kernels' window order).  Returns 0 if the parameters are invalid. */
size_t aeris_winattn_bwd_workspace_bytes(const aeris_winattn_params* p);

/*
 * Backward ("forward and backward pass with BF16 activations", Software
 * Environment section; formulas above).  Recomputes P from the saved LSE.
 *   q, k, v     : as in the forward call, read-only
 *   o, lse      : the forward outputs (o in out_dtype, as the forward call with the
 *                 same parameter block wrote it), read-only
 *   d_o         : bf16, layout of o, read-only
 *   dq, dk, dv  : out_dtype, layout of q/k/v, overwritten
 *   workspace   : >= aeris_winattn_bwd_workspace_bytes(p) bytes, 16-byte aligned,
 *                 contents undefined before and after
 * Deterministic: no atomics are used, results are bitwise reproducible.
 */
int aeris_winattn_bwd(const aeris_winattn_params* p, const void* q, const void* k,
                      const void* v, const void* o, const float* lse, const void* d_o,
                      void* dq, void* dk, void* dv, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/*
 * aeris_winattn_bwd for callers that cannot allocate or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the kernels' scratch -- the
 * two per-token statistics vectors that aeris_winattn_bwd keeps in `workspace` -- lives in a
 * static device array of AERIS_BWD_STATIC_SCRATCH_BYTES inside the library (one copy per GPU,
 * held until the process ends).  The call allocates nothing, frees nothing and only enqueues
 * the same kernels on `hip_stream`; results are bit-identical to aeris_winattn_bwd.
 * Arguments as aeris_winattn_bwd without the workspace.  Problems whose
 * aeris_winattn_bwd_workspace_bytes(p) exceeds AERIS_BWD_STATIC_SCRATCH_BYTES (8 bytes per
 * token and head: about 8.3 million (token, head) entries, e.g. 97 windows of 60x60 x 24
 * heads) are rejected with AERIS_ERR_STATIC_SCRATCH_TOO_SMALL before anything is launched.
 * The first call on a device looks up the array's device address (hipGetSymbolAddress, no
 * allocation); make that call outside a graph capture.  All calls on one GPU share the one
 * array: calls that overlap in time on the same GPU (different streams or threads) race and
 * must be serialised by the caller; the array's contents are undefined between calls.
 */
#define AERIS_BWD_STATIC_SCRATCH_BYTES (64u << 20)
int aeris_winattn_bwd_static(const aeris_winattn_params* p, const void* q, const void* k,
                             const void* v, const void* o, const float* lse, const void* d_o,
                             void* dq, void* dk, void* dv, void* hip_stream);

/* The backward pass has three stages; this variant runs a subset, in the order
 * delta, dq, dkdv (for profiling one kernel, or to put dq and dkdv on different
 * streams).  AERIS_BWD_DQ and AERIS_BWD_DKDV read what AERIS_BWD_DELTA left in
 * `workspace`, so that stage must have completed on it first.  When DELTA and DQ
 * are selected together the dQ kernel produces the statistics itself (the same
 * bits) and no separate pass over o and d_o is launched.  Outputs of stages that
 * are not selected are left untouched.  stages == AERIS_BWD_ALL is
 * aeris_winattn_bwd. */
enum { AERIS_BWD_DELTA = 1, AERIS_BWD_DQ = 2, AERIS_BWD_DKDV = 4, AERIS_BWD_ALL = 7 };
int aeris_winattn_bwd_stages(const aeris_winattn_params* p, const void* q, const void* k,
                             const void* v, const void* o, const float* lse, const void* d_o,
                             void* dq, void* dk, void* dv, void* workspace,
                             size_t workspace_bytes, void* hip_stream, unsigned stages);

/*
 * The same passes over a subset of the windows (SWiPe section: with window parallelism a
 * rank holds a round-robin subset of the attention windows; the windows of one operation
 * are independent, so a share is processed exactly as the whole).
 *   windows   : DEVICE array of n_windows int32 window indices wy * (W_lon/win_w) + wx in
 *               the shifted frame, 4-byte aligned, read-only; the same subset is
 *               processed for every batch member and head.  1 <= n_windows <= number of
 *               windows.  An index outside the grid of windows is skipped.  A window
 *               listed twice is computed twice (same values written twice).
 * Tensors keep the full-grid layout; only the tokens of the listed windows are read, and
 * only their entries of o, lse, dq, dk, dv are written -- everything else is left
 * untouched.  A workspace of aeris_winattn_bwd_workspace_bytes(p) bytes is always
 * sufficient (the need shrinks in proportion to n_windows).
 */
int aeris_winattn_fwd_windows(const aeris_winattn_params* p, const int32_t* windows,
                              int32_t n_windows, const void* q, const void* k, const void* v,
                              void* o, float* lse, void* hip_stream);
int aeris_winattn_bwd_windows(const aeris_winattn_params* p, const int32_t* windows,
                              int32_t n_windows, const void* q, const void* k, const void* v,
                              const void* o, const float* lse, const void* d_o, void* dq,
                              void* dk, void* dv, void* workspace, size_t workspace_bytes,
                              void* hip_stream);

/*
 * Rotary embedding of queries and keys (Model Architecture section: queries and keys
 * pass through an axial-frequency 2-D rotary position embedding before the dot-product
 * attention).  The paper gives no formula; this library takes the axial-frequency form
 * of the work it cites:
 *   - the head_dim channels of a head are head_dim/2 pairs (2j, 2j+1);
 *   - theta_t = base^(-t / (head_dim/4)), t = 0 .. head_dim/4 - 1;
 *   - pair 2t turns by theta_t * (longitude position), pair 2t+1 by
 *     theta_t * (latitude position); a pair (a, b) turns as the complex number a + ib;
 *   - positions: AERIS_ROPE_POS_WINDOW: coordinates inside the attention window in the
 *     shifted frame, ((y - shift_h) mod H_lat) mod win_h and likewise for x;
 *     AERIS_ROPE_POS_GRID: grid coordinates (y, x).
 * Rotated values are rounded to bf16, the type the products multiply in.
 */
enum { AERIS_ROPE_POS_WINDOW = 0, AERIS_ROPE_POS_GRID = 1 };
typedef struct {
  float base;        /* > 1 */
  int32_t positions; /* AERIS_ROPE_POS_* */
} aeris_rope_params;

/*
 * y = R x (inverse == 0) or y = R^T x (inverse != 0) for one tensor.
 *   x : bf16 [B, H_lat, W_lon, heads, head_dim] with the qkv strides of p, read-only
 *   y : bf16, same layout, overwritten; may equal x (in place)
 * Elementwise; bound by memory traffic.
 */
int aeris_rope2d_apply(const aeris_winattn_params* p, const aeris_rope_params* r, const void* x,
                       void* y, int32_t inverse, void* hip_stream);

/* Bytes of workspace of the two calls below.  Forward: room for the rotated keys and the
 * rotated queries (two compact tensors).  Backward without the forward's saved rotations: room
 * for rotated copies of q and k plus the backward statistics; with them,
 * aeris_winattn_bwd_workspace_bytes(p) is enough.  0 if the parameters are invalid. */
size_t aeris_winattn_rope_fwd_workspace_bytes(const aeris_winattn_params* p);
size_t aeris_winattn_rope_bwd_workspace_bytes(const aeris_winattn_params* p);

/*
 * aeris_winattn_fwd on rotated queries and keys: o, lse = attention(R q, R k, v).
 * The keys stream from global memory into the LDS without passing registers, so they
 * are rotated once into the workspace by a memory-bound pass; the queries, which the
 * kernel keeps in registers, are rotated as they are loaded and a copy of the rotated rows
 * is stored behind the rotated keys.  Arguments as aeris_winattn_fwd; workspace:
 * >= aeris_winattn_rope_fwd_workspace_bytes(p) bytes, 16-byte aligned.  After the call it
 * holds [rotated k | rotated q] (compact layout, bf16): pass it unchanged as `saved` to
 * aeris_winattn_rope_bwd and the backward pass rotates nothing again.
 */
int aeris_winattn_rope_fwd(const aeris_winattn_params* p, const aeris_rope_params* r,
                           const void* q, const void* k, const void* v, void* o, float* lse,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward of aeris_winattn_rope_fwd: gradients with respect to the UNROTATED q and k
 * (dq = R^T dq', dk = R^T dk', rotated back in the epilogues of the kernels that
 * accumulate them) and v.  o, lse are the outputs of aeris_winattn_rope_fwd.
 *   saved     : the workspace of the matching aeris_winattn_rope_fwd call, untouched since
 *               (read-only), or NULL.  With it q and k are not read (they may be NULL) and
 *               workspace needs aeris_winattn_bwd_workspace_bytes(p) bytes; without it q and
 *               k are rotated again into the workspace, which then needs
 *               aeris_winattn_rope_bwd_workspace_bytes(p) bytes.  Same results either way.
 * Other arguments as aeris_winattn_bwd.
 */
int aeris_winattn_rope_bwd(const aeris_winattn_params* p, const aeris_rope_params* r,
                           const void* q, const void* k, const void* v, const void* o,
                           const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                           const void* saved, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * The two calls above for a listed subset of the windows (SWiPe: a rank's share of the windows
 * runs the same rotary attention): `windows`, `n_windows` as in aeris_winattn_fwd_windows.  Only
 * tokens of the listed windows are rotated, read or written; the workspaces have the size of the
 * full-grid calls (the rotated copies keep the full-grid layout), and `saved` must come from a
 * forward call over the same list.
 */
int aeris_winattn_rope_fwd_windows(const aeris_winattn_params* p, const aeris_rope_params* r,
                                   const int32_t* windows, int32_t n_windows, const void* q,
                                   const void* k, const void* v, void* o, float* lse,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);
int aeris_winattn_rope_bwd_windows(const aeris_winattn_params* p, const aeris_rope_params* r,
                                   const int32_t* windows, int32_t n_windows, const void* q,
                                   const void* k, const void* v, const void* o, const float* lse,
                                   const void* d_o, void* dq, void* dk, void* dv,
                                   const void* saved, void* workspace, size_t workspace_bytes,
                                   void* hip_stream);

/* Checks a parameter block without launching (host only): AERIS_OK or an error. */
int aeris_winattn_validate(const aeris_winattn_params* p);

/* Static, never-freed description of an error code. */
const char* aeris_winattn_strerror(int code);

/* Library version: major*10000 + minor*100 + patch. */
int aeris_winattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AERIS_WINATTN_H */
