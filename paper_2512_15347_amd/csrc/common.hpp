// Shared host-side helpers of the library: status plumbing and launch checks.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <cstdio>
#include <cstdint>
#include "../../include/progrpo.h"

namespace pg {

char* error_buffer();                       // thread-local message of the last failure
pg_status fail(pg_status st, const char* fmt, ...);

inline pg_status hip_fail(hipError_t e, const char* what) {
  return fail(PG_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define PG_HIP(call)                                              \
  do {                                                            \
    hipError_t e__ = (call);                                      \
    if (e__ != hipSuccess) return ::pg::hip_fail(e__, #call);     \
  } while (0)

#define PG_LAUNCH_CHECK(name)                                     \
  do {                                                            \
    hipError_t e__ = hipGetLastError();                           \
    if (e__ != hipSuccess) return ::pg::hip_fail(e__, name);      \
  } while (0)

#define PG_TRY(expr)                                              \
  do {                                                            \
    pg_status s__ = (expr);                                       \
    if (s__ != PG_OK) return s__;                                 \
  } while (0)

constexpr int WAVE = 64;

// elements of one trajectory handled by one workgroup of the streaming kernels
constexpr int STREAM_THREADS = 256;
constexpr int STREAM_ITERS = 4;
constexpr int STREAM_CHUNK = STREAM_THREADS * STREAM_ITERS * 4;   // floats

inline int64_t chunks_per_traj(int64_t d) { return (d + STREAM_CHUNK - 1) / STREAM_CHUNK; }

}  // namespace pg
