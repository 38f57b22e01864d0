// Host-side helpers of the C ABI: status/error reporting and argument checks.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/photon.h"

namespace photon {

char* error_buffer();                       // thread-local, 512 bytes
int32_t fail(int32_t code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t dtype_size(photon_dtype dt) { return dt == PHOTON_BF16 ? 2 : dt == PHOTON_FP8_E4M3 ? 1 : 4; }
inline bool valid_dtype(photon_dtype dt) { return dt == PHOTON_F32 || dt == PHOTON_BF16; }

// Report a launch failure of the kernel just enqueued (does not synchronise).
inline int32_t check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PHOTON_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return PHOTON_OK;
}

// ---- optional per-kernel-class timing with HIP events (photon_profile_* entry points) ----
enum KernelClass {
  KC_COARSE_ATTN = 0, KC_COARSE_MERGE, KC_LOCAL_ATTN, KC_SKINNY_GEMM, KC_GEMM_F32, KC_REDUCE_SPLITS, KC_CHUNKER_GEMM,
  KC_NORM, KC_ROPE_APPEND, KC_SILU_MUL, KC_CHOOSE_TOKEN, KC_MISC, KC_PERSISTENT, KC_COUNT
};
extern bool g_profile_on;
// A fresh event pair recorded under class `cls`; false when events cannot be created (the launch then goes untimed).
bool profile_pair(int cls, hipEvent_t* start, hipEvent_t* stop);
#define PHOTON_TRY(expr) do { const int32_t rc_ = (expr); if (rc_ != PHOTON_OK) return rc_; } while (0)
// Launch `kern` on `st`.  While profiling, the event pair is attached to the dispatch itself (start and end of the
// kernel as the command processor stamps them), so the measured time is the kernel's, without the gap to its neighbours.
#define PHOTON_LAUNCH(cls, stream, kern, grid, block, shmem, st, ...)                                              \
  do {                                                                                                             \
    hipEvent_t prof_a_ = nullptr, prof_b_ = nullptr;                                                               \
    if (::photon::g_profile_on && ::photon::profile_pair((cls), &prof_a_, &prof_b_))                               \
      hipExtLaunchKernelGGL(kern, grid, block, shmem, st, prof_a_, prof_b_, 0, __VA_ARGS__);                       \
    else                                                                                                           \
      hipLaunchKernelGGL(kern, grid, block, shmem, st, __VA_ARGS__);                                               \
  } while (0)

#define PHOTON_REQUIRE(cond, code, ...) \
  do { if (!(cond)) return ::photon::fail((code), __VA_ARGS__); } while (0)
#define PHOTON_REQUIRE_PTR(p) \
  PHOTON_REQUIRE((p) != nullptr && ::photon::aligned16(p), PHOTON_ERR_INVALID_ARG, \
                 "%s: %s must be a non-null, 16-byte aligned device pointer", __func__, #p)

}  // namespace photon
