// Internal helpers shared by the kernels of libsynk (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/synk.h"

#define SYNK_HIP_TRY(expr)                         \
  do {                                             \
    if ((expr) != hipSuccess) return SYNK_ERR_HIP; \
  } while (0)

// Kernel launches report configuration errors through hipGetLastError.
#define SYNK_LAUNCH_CHECK()                                   \
  do {                                                        \
    if (hipGetLastError() != hipSuccess) return SYNK_ERR_HIP; \
  } while (0)

namespace synk {

// Events handed in by synk_profile_next_launch[_of] (consumed by the first launch
// made on this host thread through SYNK_LAUNCH_TIMED_AS with the kernel id they
// were handed in for).
bool take_profile_events(int kernel_id, hipEvent_t* start, hipEvent_t* stop);

// While one of these lives on this host thread no launch takes the pending pair: an entry point
// that calls another one on the way (the gather inside an indexed call) keeps the pair for its
// own kernels.
struct ProfileHold {
  ProfileHold();
  ~ProfileHold();
  ProfileHold(const ProfileHold&) = delete;
  ProfileHold& operator=(const ProfileHold&) = delete;
};

}  // namespace synk

// Launch of a kernel that a caller may want timed on its own: with events
// pending, they are attached to this very dispatch (start/stop timestamps of
// the kernel, not of the gaps around it).
#define SYNK_LAUNCH_TIMED_AS(ID, KERNEL, GRID, BLOCK, SHMEM, STREAM, ...)                            \
  do {                                                                                               \
    hipEvent_t e0_, e1_;                                                                             \
    if (synk::take_profile_events(ID, &e0_, &e1_))                                                   \
      hipExtLaunchKernelGGL(KERNEL, GRID, BLOCK, SHMEM, STREAM, e0_, e1_, 0, __VA_ARGS__);           \
    else                                                                                             \
      hipLaunchKernelGGL(KERNEL, GRID, BLOCK, SHMEM, STREAM, __VA_ARGS__);                           \
  } while (0)
// a call's main kernel
#define SYNK_LAUNCH_TIMED(KERNEL, GRID, BLOCK, SHMEM, STREAM, ...) \
  SYNK_LAUNCH_TIMED_AS(SYNK_KERNEL_MAIN, KERNEL, GRID, BLOCK, SHMEM, STREAM, __VA_ARGS__)

namespace synk {

// Native vector types (what the nontemporal builtins and MFMA builtins take).
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kNumCU = 256;

static inline bool aligned_to(const void* p, size_t a) {
  return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0;
}

static inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// share i of `count` points over `parts`: [start, start+size)
static inline void share(int64_t count, int parts, int i, int64_t* start, int64_t* size) {
  const int64_t base = count / parts, extra = count % parts;
  *size = base + (i < extra ? 1 : 0);
  *start = base * i + (i < extra ? i : extra);
}

// float -> bfloat16 bits, round to nearest even (NaN stays NaN): the conversion instruction of
// gfx950 (v_cvt_pk_bf16_f32), which the compiler selects for these casts.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  return __builtin_bit_cast(uint16_t, (__bf16)f);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float(((uint32_t)h) << 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Device-side form of the split rule: which share holds point j, and where
// that share starts.  Counts handled on the device fit 31 bits (grid and row
// limits), so the divisions are 32-bit.
__device__ __forceinline__ void share_of(int64_t count64, int parts, int64_t j64, int* which,
                                         int64_t* start) {
  const uint32_t count = (uint32_t)count64, j = (uint32_t)j64, n = (uint32_t)parts;
  const uint32_t base = count / n, extra = count % n;
  const uint32_t big = extra * (base + 1);
  if (j < big) {
    const uint32_t w = j / (base + 1);
    *which = (int)w;
    *start = (int64_t)(w * (base + 1));
  } else {
    const uint32_t w = extra + (base > 0 ? (j - big) / base : 0);
    *which = (int)w;
    *start = (int64_t)(big + (w - extra) * base);
  }
}

}  // namespace synk
