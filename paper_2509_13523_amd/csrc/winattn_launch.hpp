// Host-side launchers implemented next to their kernels.  Each returns 0 when
// the launches were enqueued and -1 when HIP reported a launch error.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <tuple>

#include "winattn_common.hpp"

namespace aeris {

// Lets kernel `Kern` use the whole LDS of a CU (160 KB on gfx950) as dynamic shared memory.
// The attribute is set once per kernel and device and remembered (one flag per device ordinal,
// the only process-wide state of the library), which keeps it off the launch path of small
// problems; what a launch actually requests still decides occupancy.  Devices beyond the
// table are configured on every launch.
constexpr int kMaxTrackedDevices = 64;
template <auto Kern>
inline bool allow_full_lds() {
  static std::atomic<unsigned char> configured[kMaxTrackedDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  const bool tracked = dev >= 0 && dev < kMaxTrackedDevices;
  if (tracked && configured[dev].load(std::memory_order_acquire)) return true;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(Kern),
                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
    return false;
  if (tracked) configured[dev].store(1, std::memory_order_release);
  return true;
}

// Enqueues `kern` and returns THIS launch's status (0 ok, -1 failed): the status comes back
// from the launch call itself, so an earlier, unrelated error of the calling thread is neither
// cleared nor reported as this library's.
template <typename... Params, typename... Args>
inline int launch_kernel(void (*kern)(Params...), dim3 grid, dim3 block, size_t smem,
                         hipStream_t stream, Args... args) {
  std::tuple<Params...> values{static_cast<Params>(args)...};
  void* ptrs[sizeof...(Params)];
  int i = 0;
  std::apply([&](auto&... v) { ((ptrs[i++] = (void*)&v), ...); }, values);
  return hipLaunchKernel(reinterpret_cast<const void*>(kern), grid, block, ptrs, smem, stream) ==
                 hipSuccess
             ? 0
             : -1;
}

int launch_fwd(const KParams& kp, int head_dim, bool out_f32, const void* q, const void* k,
               const void* v, void* o, float* lse, hipStream_t stream);

int launch_bwd(const KParams& kp, int head_dim, bool out_f32, const void* q, const void* k,
               const void* v, const void* o, const float* lse, const void* d_o, void* dq,
               void* dk, void* dv, float* workspace, hipStream_t stream, unsigned stages);

// Software-pipelined dK/dV kernel for head_dim 128 (same contract as the dK/dV stage of
// launch_bwd; delta and lse2 are the two workspace vectors).
int launch_dkdv_pipe128(const KParams& kp, bool out_f32, const void* q, const void* k,
                        const void* v, const void* d_o, const float* delta, const float* lse2,
                        void* dk, void* dv, hipStream_t stream);

// y = rotary embedding of x (inverse: the rotation by the negated angles); both
// [B, H, W, heads, head_dim] bf16 with the given element strides.  Uses kp.rope_pos, kp.rope_c.
int launch_rope(const KParams& kp, int head_dim, const void* x, long long x_tok, long long x_head,
                void* y, long long y_tok, long long y_head, bool inverse, hipStream_t stream);

// Measurement aid: `blocks` workgroups each issue 8 * iters MFMAs (32x32x16 bf16) per wave on
// register operands and write one float per thread to sink[blocks * 256].
int launch_mfma_loop(int blocks, int iters, bool random_operands, float* sink, hipStream_t stream);

// Bytes of device workspace launch_bwd needs for these parameters.
size_t bwd_workspace_bytes(const KParams& kp);

}  // namespace aeris
