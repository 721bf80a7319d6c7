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

// Optional measurement: when switched on (pg_profile_begin) the launches of the heavy kernels are
// bracketed by HIP events on their own stream; `work` is the algorithmic flop or byte count.
enum ProfKind { PROF_GEMM = 0, PROF_ATTENTION = 1, PROF_SDE_STEP = 2, PROF_PREVIEW = 3, PROF_KINDS = 4 };
int prof_open(int kind, double work, hipStream_t s);     // returns a record index or -1 when off
void prof_close(int rec, hipStream_t s);

}  // namespace pg
