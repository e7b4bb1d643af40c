// Shared host/device helpers of the codistillation-step library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <mutex>
#include "codistill.h"

namespace cd {

// ---- errors -------------------------------------------------------------------------------
int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int check_launch(const char* what);  // hipGetLastError -> CD_ERR_HIP

#define CD_REQUIRE(cond, ...)                                   \
  do {                                                          \
    if (!(cond)) return cd::set_error(CD_ERR_INVALID_ARG, __VA_ARGS__); \
  } while (0)

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- per-kernel-class timer ---------------------------------------------------------------
// RAII bracket around one launch (or a short group of launches of one class).
struct ProfScope {
  ProfScope(int cls, hipStream_t s, double flops, double bytes);
  ~ProfScope();
  int idx;
  hipStream_t stream;
};

// ---- second stream for work that forks off the caller's stream ----------------------------
// One per process, default priority, created on first use together with a pool of timing-free
// events; nullptr if the runtime refuses.  timer_enabled(): the per-launch timer is on, callers then
// keep everything on one stream so that a launch's duration is its own.
hipStream_t side_stream();
hipEvent_t side_event(int i);      // creates events 0..i on first use; nullptr if the runtime refuses
std::mutex& side_mutex();          // held by a call from its first fork onto the side stream to its join
bool timer_enabled();

// ---- bf16 ---------------------------------------------------------------------------------
typedef uint16_t bf16_t;  // upper half of an IEEE float32

__host__ __device__ static inline float bf16_to_f32(bf16_t v) {
  union { uint32_t u; float f; } c;
  c.u = static_cast<uint32_t>(v) << 16;
  return c.f;
}
// round to nearest even; NaN stays NaN.  Device code uses the gfx950 conversion instruction
// (v_cvt_pk_bf16_f32: the same rounding), host code the integer formula.
__host__ __device__ static inline bf16_t f32_to_bf16(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_bit_cast(bf16_t, static_cast<__bf16>(f));
#endif
  union { uint32_t u; float f; } c;
  c.f = f;
  if ((c.u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((c.u >> 16) | 0x40);
  uint32_t r = ((c.u >> 16) & 1u) + 0x7fffu;
  return static_cast<bf16_t>((c.u + r) >> 16);
}

template <typename T> struct Cvt;
template <> struct Cvt<float> {
  __device__ static inline float ld(float v) { return v; }
  __device__ static inline float st(float v) { return v; }
};
template <> struct Cvt<bf16_t> {
  __device__ static inline float ld(bf16_t v) { return bf16_to_f32(v); }
  __device__ static inline bf16_t st(float v) { return f32_to_bf16(v); }
};

// ---- wave / block reductions (64-wide wavefronts) -----------------------------------------
__device__ static inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ static inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace cd
