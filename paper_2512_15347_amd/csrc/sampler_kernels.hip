// Streaming (HBM-bound) kernels of the sampling loop: initial latents, the fused Euler-Maruyama
// update + Gaussian log-prob (paper Eq. 13 and the policy of Eq. 19), the one-step ODE preview with
// the linear reward proxy (Eq. 15-16), and the ragged survivor gather (Sec. 5.1, early termination).
//
// Work decomposition: one workgroup of 256 lanes owns one STREAM_CHUNK (4096 floats) of one
// trajectory and moves it with 16-byte accesses; per-trajectory sums are written as one partial per
// workgroup and finished by a second tiny kernel in a fixed order (fp64), so results do not depend
// on scheduling.
#include "ctx.hpp"
#include "philox.hpp"

namespace pg {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, WAVE);
  return v;
}

// Sum over the 256 lanes of the workgroup; valid in lane 0 of wave 0.
__device__ __forceinline__ float block_sum_256(float v) {
  __shared__ float part[STREAM_THREADS / WAVE];
  v = wave_sum(v);
  const int lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
  if (lane == 0) part[wv] = v;
  __syncthreads();
  float t = 0.f;
  if (threadIdx.x == 0) t = (part[0] + part[1]) + (part[2] + part[3]);
  return t;
}

__global__ __launch_bounds__(STREAM_THREADS) void init_latents_kernel(
    float* __restrict__ x, const int32_t* __restrict__ orig_id, int d4, int chunks, uint32_t k0,
    uint32_t k1) {
  const int r = blockIdx.x / chunks, c = blockIdx.x - r * chunks;
  const uint32_t id = (uint32_t)orig_id[r];
  f32x4* xr = reinterpret_cast<f32x4*>(x) + (size_t)r * d4;
#pragma unroll
  for (int it = 0; it < STREAM_ITERS; ++it) {
    const int e4 = c * (STREAM_CHUNK / 4) + it * STREAM_THREADS + threadIdx.x;
    if (e4 < d4) xr[e4] = philox_normal4((uint32_t)e4, 0u, id, STREAM_INIT, k0, k1);
  }
}

// x_out[r] = A x[q] + B u[q] + C xi, q = src ? src[r] : r; partial of sum xi^2 per workgroup.
__global__ __launch_bounds__(STREAM_THREADS) void sde_step_kernel(
    const float* __restrict__ x, const float* __restrict__ u, float* __restrict__ x_out,
    const int32_t* __restrict__ src, const int32_t* __restrict__ orig_id, int d4, int chunks, float A,
    float B, float C, uint32_t k0, uint32_t k1, uint32_t step, float* __restrict__ partials,
    float* __restrict__ hist_next) {
  const int r = blockIdx.x / chunks, c = blockIdx.x - r * chunks;
  const int q = src ? src[r] : r;
  const uint32_t id = (uint32_t)orig_id[r];
  f32x4* hn = hist_next ? reinterpret_cast<f32x4*>(hist_next) + (size_t)id * d4 : nullptr;
  const f32x4* xq = reinterpret_cast<const f32x4*>(x) + (size_t)q * d4;
  const f32x4* uq = reinterpret_cast<const f32x4*>(u) + (size_t)q * d4;
  f32x4* xo = reinterpret_cast<f32x4*>(x_out) + (size_t)r * d4;
  f32x4 xv[STREAM_ITERS], uv[STREAM_ITERS];
  int e4[STREAM_ITERS];
#pragma unroll
  for (int it = 0; it < STREAM_ITERS; ++it) {
    e4[it] = c * (STREAM_CHUNK / 4) + it * STREAM_THREADS + threadIdx.x;
    if (e4[it] < d4) {
      xv[it] = __builtin_nontemporal_load(xq + e4[it]);
      uv[it] = __builtin_nontemporal_load(uq + e4[it]);
    }
  }
  float acc = 0.f;
#pragma unroll
  for (int it = 0; it < STREAM_ITERS; ++it) {
    if (e4[it] < d4) {
      const f32x4 z = philox_normal4((uint32_t)e4[it], step, id, STREAM_STEP, k0, k1);
      f32x4 o;
      o.x = A * xv[it].x + B * uv[it].x + C * z.x;
      o.y = A * xv[it].y + B * uv[it].y + C * z.y;
      o.z = A * xv[it].z + B * uv[it].z + C * z.z;
      o.w = A * xv[it].w + B * uv[it].w + C * z.w;
      __builtin_nontemporal_store(o, xo + e4[it]);
      if (hn) __builtin_nontemporal_store(o, hn + e4[it]);      // trajectory record by original id
      acc += (z.x * z.x + z.y * z.y) + (z.z * z.z + z.w * z.w);
    }
  }
  const float t = block_sum_256(acc);
  if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

// The same update with the latents and the network output stored as bf16 (6 instead of 12 bytes per element):
// arithmetic in fp32, the result rounded to nearest-even.  A lane handles 8 elements per access (two Philox
// blocks); the noise of an element does not depend on the storage format.
typedef uint32_t u32x4s __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float bf_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t bf_pack(float a, float b) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)a) | ((uint32_t)__builtin_bit_cast(uint16_t, (__bf16)b) << 16);
}

__global__ __launch_bounds__(STREAM_THREADS) void sde_step_bf16_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ u, uint16_t* __restrict__ x_out,
    const int32_t* __restrict__ src, const int32_t* __restrict__ orig_id, int d8, int chunks, float A, float B,
    float C, uint32_t k0, uint32_t k1, uint32_t step, float* __restrict__ partials) {
  const int r = blockIdx.x / chunks, c = blockIdx.x - r * chunks;
  const int q = src ? src[r] : r;
  const uint32_t id = (uint32_t)orig_id[r];
  const u32x4s* xq = reinterpret_cast<const u32x4s*>(x) + (size_t)q * d8;
  const u32x4s* uq = reinterpret_cast<const u32x4s*>(u) + (size_t)q * d8;
  u32x4s* xo = reinterpret_cast<u32x4s*>(x_out) + (size_t)r * d8;
  constexpr int ITERS = STREAM_CHUNK / 8 / STREAM_THREADS;         // 16-byte accesses per lane and chunk
  float acc = 0.f;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int e8 = c * (STREAM_CHUNK / 8) + it * STREAM_THREADS + threadIdx.x;
    if (e8 < d8) {
      const u32x4s xv = __builtin_nontemporal_load(xq + e8);
      const u32x4s uv = __builtin_nontemporal_load(uq + e8);
      const f32x4 z0 = philox_normal4((uint32_t)(2 * e8), step, id, STREAM_STEP, k0, k1);
      const f32x4 z1 = philox_normal4((uint32_t)(2 * e8 + 1), step, id, STREAM_STEP, k0, k1);
      u32x4s o;
      o.x = bf_pack(A * bf_lo(xv.x) + B * bf_lo(uv.x) + C * z0.x, A * bf_hi(xv.x) + B * bf_hi(uv.x) + C * z0.y);
      o.y = bf_pack(A * bf_lo(xv.y) + B * bf_lo(uv.y) + C * z0.z, A * bf_hi(xv.y) + B * bf_hi(uv.y) + C * z0.w);
      o.z = bf_pack(A * bf_lo(xv.z) + B * bf_lo(uv.z) + C * z1.x, A * bf_hi(xv.z) + B * bf_hi(uv.z) + C * z1.y);
      o.w = bf_pack(A * bf_lo(xv.w) + B * bf_lo(uv.w) + C * z1.z, A * bf_hi(xv.w) + B * bf_hi(uv.w) + C * z1.w);
      __builtin_nontemporal_store(o, xo + e8);
      acc += ((z0.x * z0.x + z0.y * z0.y) + (z0.z * z0.z + z0.w * z0.w)) +
             ((z1.x * z1.x + z1.y * z1.y) + (z1.z * z1.z + z1.w * z1.w));
    }
  }
  const float t = block_sum_256(acc);
  if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

// logp[r] = -1/2 sum_c partial[r, c] - d (ln C + 1/2 ln 2 pi); history and running sum by original id.
__global__ void logprob_finish_kernel(const float* __restrict__ partials, int chunks, int n_traj,
                                      double log_norm, const int32_t* __restrict__ orig_id,
                                      float* __restrict__ logp, float* __restrict__ logp_hist,
                                      float* __restrict__ logp_sum) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_traj) return;
  double s = 0.0;
  for (int c = 0; c < chunks; ++c) s += (double)partials[(size_t)r * chunks + c];
  const float lp = (float)(-0.5 * s - log_norm);
  if (logp) logp[r] = lp;
  const int id = orig_id[r];
  if (logp_hist) logp_hist[id] = lp;
  if (logp_sum) logp_sum[id] += lp;
}

// partial of <w, Pc x + Qc u> per workgroup
template <bool WITH_U>
__global__ __launch_bounds__(STREAM_THREADS) void preview_reward_kernel(
    const float* __restrict__ x, const float* __restrict__ u, const float* __restrict__ w, int d4,
    int chunks, float Pc, float Qc, float* __restrict__ partials) {
  const int r = blockIdx.x / chunks, c = blockIdx.x - r * chunks;
  const f32x4* xr = reinterpret_cast<const f32x4*>(x) + (size_t)r * d4;
  const f32x4* ur = reinterpret_cast<const f32x4*>(u) + (size_t)r * d4;
  const f32x4* w4 = reinterpret_cast<const f32x4*>(w);
  float acc = 0.f;
#pragma unroll
  for (int it = 0; it < STREAM_ITERS; ++it) {
    const int e4 = c * (STREAM_CHUNK / 4) + it * STREAM_THREADS + threadIdx.x;
    if (e4 < d4) {
      const f32x4 xv = __builtin_nontemporal_load(xr + e4);
      const f32x4 wv = w4[e4];
      f32x4 h;
      if (WITH_U) {
        const f32x4 uv = __builtin_nontemporal_load(ur + e4);
        h.x = Pc * xv.x + Qc * uv.x; h.y = Pc * xv.y + Qc * uv.y;
        h.z = Pc * xv.z + Qc * uv.z; h.w = Pc * xv.w + Qc * uv.w;
      } else {
        h.x = Pc * xv.x; h.y = Pc * xv.y; h.z = Pc * xv.z; h.w = Pc * xv.w;
      }
      acc += (wv.x * h.x + wv.y * h.y) + (wv.z * h.z + wv.w * h.w);
    }
  }
  const float t = block_sum_256(acc);
  if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

__global__ void reward_finish_kernel(const float* __restrict__ partials, int chunks, int n_traj,
                                     double bias, float* __restrict__ rewards) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_traj) return;
  double s = 0.0;
  for (int c = 0; c < chunks; ++c) s += (double)partials[(size_t)r * chunks + c];
  rewards[r] = (float)(bias + s);
}

__global__ __launch_bounds__(STREAM_THREADS) void compact_gather_kernel(
    const float* __restrict__ x, float* __restrict__ out, const int32_t* __restrict__ src, int d4,
    int chunks) {
  const int r = blockIdx.x / chunks, c = blockIdx.x - r * chunks;
  const int q = src[r];
  const f32x4* xq = reinterpret_cast<const f32x4*>(x) + (size_t)q * d4;
  f32x4* xo = reinterpret_cast<f32x4*>(out) + (size_t)r * d4;
  f32x4 v[STREAM_ITERS];
  int e4[STREAM_ITERS];
#pragma unroll
  for (int it = 0; it < STREAM_ITERS; ++it) {
    e4[it] = c * (STREAM_CHUNK / 4) + it * STREAM_THREADS + threadIdx.x;
    if (e4[it] < d4) v[it] = __builtin_nontemporal_load(xq + e4[it]);
  }
#pragma unroll
  for (int it = 0; it < STREAM_ITERS; ++it)
    if (e4[it] < d4) __builtin_nontemporal_store(v[it], xo + e4[it]);
}

// Stored transition (x, x_next) of a survivor under another network output u (Eq. 19): two partials per
// workgroup, the squared residual |x_next - (A x + B u)|^2 and, with xi the noise the sampler drew for this
// element (regenerated from its counter) and w = residual / C the noise the new policy would need,
// sum (xi - w)(xi + w) = sum xi^2 - sum w^2 = 2 (log pi_new - log pi_old): the log-ratio is summed from its small
// per-element terms instead of being the difference of two large log-probs.
__global__ __launch_bounds__(STREAM_THREADS) void transition_sq_kernel(
    const float* __restrict__ x, const float* __restrict__ u, const float* __restrict__ x_next_by_id,
    const int32_t* __restrict__ orig_id, int d4, int chunks, float A, float B, float C, uint32_t k0, uint32_t k1,
    uint32_t step, float* __restrict__ partials) {
  __shared__ float part[2][STREAM_THREADS / WAVE];
  const int r = blockIdx.x / chunks, c = blockIdx.x - r * chunks;
  const uint32_t id = (uint32_t)orig_id[r];
  const f32x4* xr = reinterpret_cast<const f32x4*>(x) + (size_t)r * d4;
  const f32x4* ur = reinterpret_cast<const f32x4*>(u) + (size_t)r * d4;
  const f32x4* nr = reinterpret_cast<const f32x4*>(x_next_by_id) + (size_t)id * d4;
  float acc = 0.f, dif = 0.f;
#pragma unroll
  for (int it = 0; it < STREAM_ITERS; ++it) {
    const int e4 = c * (STREAM_CHUNK / 4) + it * STREAM_THREADS + threadIdx.x;
    if (e4 < d4) {
      const f32x4 xv = __builtin_nontemporal_load(xr + e4), uv = __builtin_nontemporal_load(ur + e4);
      const f32x4 nv = __builtin_nontemporal_load(nr + e4);
      const f32x4 z = philox_normal4((uint32_t)e4, step, id, STREAM_STEP, k0, k1);
      const float a0 = nv.x - (A * xv.x + B * uv.x), a1 = nv.y - (A * xv.y + B * uv.y);
      const float a2 = nv.z - (A * xv.z + B * uv.z), a3 = nv.w - (A * xv.w + B * uv.w);
      acc += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
      // divided by the very fp32 scale the sampler multiplied its noise with: a rounded reciprocal would bias every
      // term the same way, and the bias would add up over the d elements
      const float w0 = a0 / C, w1 = a1 / C, w2 = a2 / C, w3 = a3 / C;
      dif += ((z.x - w0) * (z.x + w0) + (z.y - w1) * (z.y + w1)) + ((z.z - w2) * (z.z + w2) + (z.w - w3) * (z.w + w3));
    }
  }
  acc = wave_sum(acc);
  dif = wave_sum(dif);
  const int lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
  if (lane == 0) { part[0][wv] = acc; part[1][wv] = dif; }
  __syncthreads();
  if (threadIdx.x == 0) {
    partials[2 * (size_t)blockIdx.x] = (part[0][0] + part[0][1]) + (part[0][2] + part[0][3]);
    partials[2 * (size_t)blockIdx.x + 1] = (part[1][0] + part[1][1]) + (part[1][2] + part[1][3]);
  }
}

// logp[id] = -sum / (2 C^2) - d (ln C + 1/2 ln 2 pi);  log_ratio[id] = 1/2 sum (xi - w)(xi + w), kept in fp64
__global__ void transition_finish_kernel(const float* __restrict__ partials, int chunks, int n_traj, double inv_2c2,
                                         double log_norm, const int32_t* __restrict__ orig_id,
                                         float* __restrict__ logp_by_id, double* __restrict__ log_ratio_by_id) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_traj) return;
  double s = 0.0, dsum = 0.0;
  for (int c = 0; c < chunks; ++c) {
    s += (double)partials[2 * ((size_t)r * chunks + c)];
    dsum += (double)partials[2 * ((size_t)r * chunks + c) + 1];
  }
  logp_by_id[orig_id[r]] = (float)(-s * inv_2c2 - log_norm);
  log_ratio_by_id[orig_id[r]] = 0.5 * dsum;
}

// Eq. 19 and the first term of Eq. 20 per group: one wave per group, lanes over survivors
__global__ __launch_bounds__(256) void surrogate_kernel(const double* __restrict__ log_ratio,
                                                        const float* __restrict__ adv,
                                                        const int32_t* __restrict__ offsets,
                                                        const int32_t* __restrict__ orig_id, int n_groups, int T,
                                                        int M0, float lo, float hi, float* __restrict__ ratio,
                                                        float* __restrict__ J) {
  const int wv = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
  const int g = blockIdx.x * 4 + wv;
  if (g >= n_groups) return;
  const int b = offsets[g], e = offsets[g + 1];
  double acc = 0.0;
  for (int i = b + lane; i < e; i += WAVE) {
    const int id = orig_id[i];
    const double a = (double)adv[i];
    for (int s = 0; s < T; ++s) {
      const double r = exp(log_ratio[(size_t)s * M0 + id]);
      ratio[(size_t)s * M0 + id] = (float)r;
      const double rc = fmin(fmax(r, (double)lo), (double)hi);
      acc += fmin(r * a, rc * a);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, WAVE);
  if (lane == 0) J[g] = (e > b) ? (float)(acc / ((double)(e - b) * T)) : 0.f;
}

static pg_status check_stream_shape(int64_t n_traj, int64_t d) {
  if (n_traj < 0 || d <= 0) return fail(PG_EINVAL, "n_traj = %lld, d = %lld", (long long)n_traj, (long long)d);
  if (d % 4 != 0) return fail(PG_ESHAPE, "latent size d = %lld must be a multiple of 4", (long long)d);
  if (d / 4 > INT32_MAX || n_traj * chunks_per_traj(d) > INT32_MAX)
    return fail(PG_ESHAPE, "n_traj * ceil(d/4096) exceeds the grid limit");
  return PG_OK;
}

}  // namespace pg

using namespace pg;

extern "C" int64_t pg_step_scratch_floats(int64_t n_traj, int64_t d) {
  if (n_traj <= 0 || d <= 0) return 0;
  return n_traj * chunks_per_traj(d);
}

extern "C" pg_status pg_init_latents(float* x, const int32_t* orig_id, int64_t n_traj, int64_t d,
                                     uint64_t seed, void* stream) {
  PG_TRY(check_stream_shape(n_traj, d));
  if (n_traj == 0) return PG_OK;
  if (!x || !orig_id) return fail(PG_EINVAL, "pg_init_latents: null pointer");
  const int chunks = (int)chunks_per_traj(d);
  init_latents_kernel<<<dim3((unsigned)(n_traj * chunks)), dim3(STREAM_THREADS), 0, (hipStream_t)stream>>>(
      x, orig_id, (int)(d / 4), chunks, (uint32_t)seed, (uint32_t)(seed >> 32));
  PG_LAUNCH_CHECK("init_latents_kernel");
  return PG_OK;
}

namespace pg {
pg_status launch_sde_step(const float* x, const float* u, float* x_out, float* logp, float* logp_hist,
                          float* logp_sum, const int32_t* src, const int32_t* orig_id, int64_t n_traj, int64_t d,
                          double A, double B, double C, uint64_t seed, uint32_t step, float* partials,
                          float* hist_next, hipStream_t stream) {
  PG_TRY(check_stream_shape(n_traj, d));
  if (n_traj == 0) return PG_OK;
  if (!x || !u || !x_out || !orig_id || !partials) return fail(PG_EINVAL, "pg_sde_step_logprob: null pointer");
  if (x_out == x) return fail(PG_EINVAL, "pg_sde_step_logprob: x_out must not alias x");
  if (!(C > 0.0)) return fail(PG_EINVAL, "pg_sde_step_logprob: noise scale C = %g must be > 0", C);
  const int chunks = (int)chunks_per_traj(d);
  const int rec = prof_open(PROF_SDE_STEP, 12.0 * (double)n_traj * (double)d, stream);
  sde_step_kernel<<<dim3((unsigned)(n_traj * chunks)), dim3(STREAM_THREADS), 0, stream>>>(
      x, u, x_out, src, orig_id, (int)(d / 4), chunks, (float)A, (float)B, (float)C, (uint32_t)seed,
      (uint32_t)(seed >> 32), step, partials, hist_next);
  prof_close(rec, stream);
  PG_LAUNCH_CHECK("sde_step_kernel");
  const double log_norm = (double)d * (log(C) + 0.5 * log(2.0 * M_PI));
  logprob_finish_kernel<<<dim3((unsigned)((n_traj + 127) / 128)), dim3(128), 0, stream>>>(
      partials, chunks, (int)n_traj, log_norm, orig_id, logp, logp_hist, logp_sum);
  PG_LAUNCH_CHECK("logprob_finish_kernel");
  return PG_OK;
}

pg_status launch_transition_logprob(const float* x, const float* u, const float* x_next_by_id,
                                    const int32_t* orig_id, int64_t n_traj, int64_t d, double A, double B, double C,
                                    uint64_t seed, uint32_t step, float* logp_by_id, double* log_ratio_by_id,
                                    float* partials, hipStream_t stream) {
  PG_TRY(check_stream_shape(n_traj, d));
  if (n_traj == 0) return PG_OK;
  const int chunks = (int)chunks_per_traj(d);
  transition_sq_kernel<<<dim3((unsigned)(n_traj * chunks)), dim3(STREAM_THREADS), 0, stream>>>(
      x, u, x_next_by_id, orig_id, (int)(d / 4), chunks, (float)A, (float)B, (float)C, (uint32_t)seed,
      (uint32_t)(seed >> 32), step, partials);
  PG_LAUNCH_CHECK("transition_sq_kernel");
  transition_finish_kernel<<<dim3((unsigned)((n_traj + 127) / 128)), dim3(128), 0, stream>>>(
      partials, chunks, (int)n_traj, 1.0 / (2.0 * C * C), (double)d * (log(C) + 0.5 * log(2.0 * M_PI)), orig_id,
      logp_by_id, log_ratio_by_id);
  PG_LAUNCH_CHECK("transition_finish_kernel");
  return PG_OK;
}

pg_status launch_surrogate(const double* log_ratio, const float* adv, const int32_t* offsets,
                           const int32_t* orig_id, int n_groups, int T, int M0, double clip_eps, float* ratio,
                           float* J, hipStream_t stream) {
  surrogate_kernel<<<dim3((n_groups + 3) / 4), dim3(256), 0, stream>>>(
      log_ratio, adv, offsets, orig_id, n_groups, T, M0, (float)(1.0 - clip_eps), (float)(1.0 + clip_eps),
      ratio, J);
  PG_LAUNCH_CHECK("surrogate_kernel");
  return PG_OK;
}
}  // namespace pg

extern "C" pg_status pg_sde_step_logprob(const float* x, const float* u, float* x_out, float* logp,
                                         float* logp_hist, float* logp_sum, const int32_t* src,
                                         const int32_t* orig_id, int64_t n_traj, int64_t d, double A,
                                         double B, double C, uint64_t seed, uint32_t step,
                                         float* partials, void* stream) {
  return launch_sde_step(x, u, x_out, logp, logp_hist, logp_sum, src, orig_id, n_traj, d, A, B, C, seed, step,
                         partials, nullptr, (hipStream_t)stream);
}

extern "C" pg_status pg_sde_step_logprob_bf16(const uint16_t* x, const uint16_t* u, uint16_t* x_out, float* logp,
                                              float* logp_hist, float* logp_sum, const int32_t* src,
                                              const int32_t* orig_id, int64_t n_traj, int64_t d, double A,
                                              double B, double C, uint64_t seed, uint32_t step,
                                              float* partials, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  PG_TRY(check_stream_shape(n_traj, d));
  if (d % 8) return fail(PG_ESHAPE, "pg_sde_step_logprob_bf16: d = %lld must be a multiple of 8", (long long)d);
  if (n_traj == 0) return PG_OK;
  if (!x || !u || !x_out || !orig_id || !partials) return fail(PG_EINVAL, "pg_sde_step_logprob_bf16: null pointer");
  if (x_out == x) return fail(PG_EINVAL, "pg_sde_step_logprob_bf16: x_out must not alias x");
  if (!(C > 0.0)) return fail(PG_EINVAL, "pg_sde_step_logprob_bf16: noise scale C = %g must be > 0", C);
  const int chunks = (int)chunks_per_traj(d);
  sde_step_bf16_kernel<<<dim3((unsigned)(n_traj * chunks)), dim3(STREAM_THREADS), 0, stream>>>(
      x, u, x_out, src, orig_id, (int)(d / 8), chunks, (float)A, (float)B, (float)C, (uint32_t)seed,
      (uint32_t)(seed >> 32), step, partials);
  PG_LAUNCH_CHECK("sde_step_bf16_kernel");
  const double log_norm = (double)d * (log(C) + 0.5 * log(2.0 * M_PI));
  logprob_finish_kernel<<<dim3((unsigned)((n_traj + 127) / 128)), dim3(128), 0, stream>>>(
      partials, chunks, (int)n_traj, log_norm, orig_id, logp, logp_hist, logp_sum);
  PG_LAUNCH_CHECK("logprob_finish_kernel");
  return PG_OK;
}

extern "C" pg_status pg_preview_reward(const float* x, const float* u, const float* w, float* rewards,
                                       int64_t n_traj, int64_t d, double Pc, double Qc, double bias,
                                       float* partials, void* stream) {
  PG_TRY(check_stream_shape(n_traj, d));
  if (n_traj == 0) return PG_OK;
  if (!x || !w || !rewards || !partials) return fail(PG_EINVAL, "pg_preview_reward: null pointer");
  if (!u && Qc != 0.0) return fail(PG_EINVAL, "pg_preview_reward: u is NULL but Qc = %g", Qc);
  const int chunks = (int)chunks_per_traj(d);
  const dim3 grid((unsigned)(n_traj * chunks)), block(STREAM_THREADS);
  const int rec = prof_open(PROF_PREVIEW, ((u && Qc != 0.0) ? 8.0 : 4.0) * (double)n_traj * (double)d, (hipStream_t)stream);
  if (u && Qc != 0.0)
    preview_reward_kernel<true><<<grid, block, 0, (hipStream_t)stream>>>(x, u, w, (int)(d / 4), chunks,
                                                                          (float)Pc, (float)Qc, partials);
  else
    preview_reward_kernel<false><<<grid, block, 0, (hipStream_t)stream>>>(x, x, w, (int)(d / 4), chunks,
                                                                           (float)Pc, 0.f, partials);
  prof_close(rec, (hipStream_t)stream);
  PG_LAUNCH_CHECK("preview_reward_kernel");
  reward_finish_kernel<<<dim3((unsigned)((n_traj + 127) / 128)), dim3(128), 0, (hipStream_t)stream>>>(
      partials, chunks, (int)n_traj, bias, rewards);
  PG_LAUNCH_CHECK("reward_finish_kernel");
  return PG_OK;
}

extern "C" pg_status pg_compact_gather(const float* x, float* out, const int32_t* src, int64_t n_out,
                                       int64_t d, void* stream) {
  PG_TRY(check_stream_shape(n_out, d));
  if (n_out == 0) return PG_OK;
  if (!x || !out || !src) return fail(PG_EINVAL, "pg_compact_gather: null pointer");
  if (out == x) return fail(PG_EINVAL, "pg_compact_gather: out must not alias x");
  const int chunks = (int)chunks_per_traj(d);
  compact_gather_kernel<<<dim3((unsigned)(n_out * chunks)), dim3(STREAM_THREADS), 0, (hipStream_t)stream>>>(
      x, out, src, (int)(d / 4), chunks);
  PG_LAUNCH_CHECK("compact_gather_kernel");
  return PG_OK;
}
