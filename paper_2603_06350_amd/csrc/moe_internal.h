// Internal helpers shared by the gfx950 kernels of the MoE-layer library.
// Not part of the public boundary (that is include/moe.h).
#ifndef MOE_INTERNAL_H
#define MOE_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe.h"

#define MOE_MAX_E 256
#define MOE_MAX_K 64
#define MOE_WAVE 64
// moe_route_ws: largest batch whose gate product runs as a kernel of its own (T x E fp32 scores in
// the workspace between the two kernels)
#ifndef MOE_ROUTE_WS_MAX_T
#define MOE_ROUTE_WS_MAX_T 8191
#endif

namespace moe {

// ---- host-side argument checks ------------------------------------------------------------
inline int elem_bytes(int dtype) { return dtype == MOE_F32 ? 4 : 2; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks everything that does not depend on a particular call's pointers.
inline int check_shape(const moe_shape_t* s) {
  if (!s) return MOE_ERR_INVALID_ARG;
  if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
  if (s->T < 0 || s->d < 1 || s->E < 1 || s->k < 1 || s->F < 1) return MOE_ERR_INVALID_ARG;
  if (s->k > s->E) return MOE_ERR_INVALID_ARG;
  if (s->renorm != 0 && s->renorm != 1) return MOE_ERR_INVALID_ARG;
  const int b = elem_bytes(s->dtype);
  if ((static_cast<int64_t>(s->d) * b) % 16 != 0) return MOE_ERR_INVALID_ARG;
  if ((static_cast<int64_t>(s->F) * b) % 16 != 0) return MOE_ERR_INVALID_ARG;
  if (s->E > MOE_MAX_E || s->k > MOE_MAX_K) return MOE_ERR_UNSUPPORTED;
  if (static_cast<int64_t>(s->T) * s->k >= (int64_t(1) << 31)) return MOE_ERR_UNSUPPORTED;
  return MOE_OK;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP; }

// Raises a kernel's dynamic-LDS limit once per device.  `done` is the caller's per-kernel flag
// array (one static array per kernel); setting the attribute twice is harmless, so a race between
// two first calls needs no lock.
constexpr int MOE_MAX_DEVICES = 64;
struct LdsOnce {
  bool done[MOE_MAX_DEVICES] = {};
};
inline int ensure_dynamic_lds(LdsOnce& once, const void* kernel, int bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MOE_MAX_DEVICES) return MOE_ERR_HIP;
  if (once.done[dev]) return MOE_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return MOE_ERR_HIP;
  once.done[dev] = true;
  return MOE_OK;
}

// ---- device helpers -------------------------------------------------------------------------
typedef uint16_t bf16_t;  // bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// float -> bfloat16, round to nearest even: gfx950 has the conversion in hardware
// (v_cvt_pk_bf16_f32, two values per instruction)
typedef __bf16 moe_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float moe_f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const moe_f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, moe_bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return static_cast<bf16_t>(pack_bf16x2(f, 0.f) & 0xFFFFu);
}
__device__ __forceinline__ float bf16lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (MOE_WAVE - 1); }

}  // namespace moe
#endif
