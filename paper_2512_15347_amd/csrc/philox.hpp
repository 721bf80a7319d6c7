// Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) and the Box-Muller map used for the
// initial latents and the per-step noise of the Euler-Maruyama update (paper Sec. 5.1, Eq. 13).
// Counter = (element / 4, step, original trajectory id, stream), key = (seed lo, seed hi): the
// noise a trajectory sees does not depend on where pruning has packed it.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace pg {

constexpr uint32_t PHILOX_M0 = 0xD2511F53u;
constexpr uint32_t PHILOX_M1 = 0xCD9E8D57u;
constexpr uint32_t PHILOX_W0 = 0x9E3779B9u;
constexpr uint32_t PHILOX_W1 = 0xBB67AE85u;

constexpr uint32_t STREAM_INIT = 0u;
constexpr uint32_t STREAM_STEP = 1u;

struct u32x4 { uint32_t x, y, z, w; };
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 philox4x32_10(u32x4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)PHILOX_M0 * c.x;
    const uint64_t p1 = (uint64_t)PHILOX_M1 * c.z;
    u32x4 n;
    n.x = (uint32_t)(p1 >> 32) ^ c.y ^ k0;
    n.y = (uint32_t)p1;
    n.z = (uint32_t)(p0 >> 32) ^ c.w ^ k1;
    n.w = (uint32_t)p0;
    c = n;
    k0 += PHILOX_W0;
    k1 += PHILOX_W1;
  }
  return c;
}

// Two normals from two 32-bit words: u = (n + 1/2) / 2^32, z = sqrt(-2 ln ua) (cos, sin)(2 pi ub).
// The hardware sine/cosine take their argument in revolutions, so 2 pi never appears.
__device__ __forceinline__ void box_muller(uint32_t na, uint32_t nb, float& z0, float& z1) {
  const float ua = ((float)na + 0.5f) * 2.3283064365386963e-10f;
  const float ub = ((float)nb + 0.5f) * 2.3283064365386963e-10f;
  // -2 ln(ua) = -2 ln2 * log2(ua)
  const float r = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(ua));
  z0 = r * __builtin_amdgcn_cosf(ub);
  z1 = r * __builtin_amdgcn_sinf(ub);
}

__device__ __forceinline__ f32x4 philox_normal4(uint32_t blk, uint32_t step, uint32_t orig_id,
                                                 uint32_t stream, uint32_t k0, uint32_t k1) {
  const u32x4 w = philox4x32_10(u32x4{blk, step, orig_id, stream}, k0, k1);
  float a, b, c, d;
  box_muller(w.x, w.y, a, b);
  box_muller(w.z, w.w, c, d);
  return f32x4{a, b, c, d};
}

}  // namespace pg
