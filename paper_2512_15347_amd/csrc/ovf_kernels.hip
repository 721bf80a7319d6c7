// Optimal Variance Filtering per group (paper Sec. 4.2, Eq. 10; in-loop form in Sec. 5.1), the
// group-normalised advantages (Eq. 5, Eq. 18) and the small index kernels around a prune.
//
// One 64-lane wavefront owns one group (the paper's groups have at most 64 members, cf. the
// group-size ablation): ranks by all-pairs comparison over lane broadcasts, fp64 prefix sums by a
// six-step shuffle-up scan, k+1 candidate scores in lanes 0..k, a butterfly arg-max, and a ballot
// for the survivor mask.  Why k+1 candidates are enough: with the other members fixed the variance
// is a convex quadratic in one member's value, so some optimum is "j lowest and k-j highest".
#include <mutex>
#include "common.hpp"
#include "philox.hpp"

namespace pg {

constexpr int OVF_WAVES = 4;           // groups per workgroup
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;          // groups per lane in the offsets scan
constexpr int SCAN_BLOCK = SCAN_THREADS * SCAN_ITEMS;

__device__ __forceinline__ double shfl_up_f64(double v, int delta) { return __shfl_up(v, delta, WAVE); }

// Inclusive prefix sum across the wave by the doubling recurrence: after the pass with distance dd
// lane i holds the sum of lanes max(0, i-2dd+1) .. i.  The order of additions is part of the
// library's bit-exactness contract.
__device__ __forceinline__ double wave_scan_f64(double a, int lane) {
#pragma unroll
  for (int dd = 1; dd < WAVE; dd <<= 1) {
    const double t = shfl_up_f64(a, dd);
    if (lane >= dd) a = __dadd_rn(a, t);
  }
  return a;
}

// A group whose size or count the selection cannot take (size outside 1..limit, k outside 1..size): its mask is
// empty and the error flag is raised, but the k slots that the offsets scan reserved for it in sel_idx are still
// filled with row indices that exist (its own rows, else row 0), so that a caller who gathers before reading
// the status stays in bounds.  The scan counts a negative k as 0.
__device__ __forceinline__ int counted_k(int k) { return k > 0 ? k : 0; }
__device__ __forceinline__ void fill_bad_group(int32_t* __restrict__ sel_idx, int out0, int b, int n, int k, int lane,
                                               int lanes) {
  for (int i = lane; i < k; i += lanes) sel_idx[out0 + i] = n >= 1 ? b + (i < n ? i : n - 1) : 0;
}

__global__ __launch_bounds__(OVF_WAVES * WAVE) void ovf_select_kernel(
    const float* __restrict__ rewards, const int32_t* __restrict__ offsets, const int32_t* __restrict__ kk,
    int n_groups, const int32_t* __restrict__ new_offsets, uint64_t* __restrict__ masks,
    int32_t* __restrict__ sel_idx, int32_t* __restrict__ status) {
  __shared__ float sorted[OVF_WAVES][WAVE];
  const int wv = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
  const int g = blockIdx.x * OVF_WAVES + wv;
  if (g >= n_groups) return;                        // whole wave leaves together
  const int b = offsets[g];
  const int n = offsets[g + 1] - b;
  const int k = kk[g];
  const int out0 = new_offsets[g];
  if (n < 1 || n > WAVE || k < 1 || k > n) {        // nothing to select: empty mask; flag unless the
    if (lane == 0) {                                // group is simply empty (n = k = 0)
      if (!(n == 0 && k == 0)) atomicOr(status, 2);
      masks[g] = 0ull;
    }
    fill_bad_group(sel_idx, out0, b, n, k, lane, WAVE);
    return;
  }
  const bool live = lane < n;
  float v = live ? rewards[b + lane] + 0.0f : 0.0f;  // -0.0 becomes +0.0
  const bool bad = live && !(__builtin_fabsf(v) <= 3.4028234663852886e38f);
  if (__ballot(bad) != 0ull || k == n) {
    // k == n keeps everything; a non-finite reward is flagged and the first k slots are kept so
    // that every index written stays valid for the kernels that follow
    if (__ballot(bad) != 0ull && lane == 0) atomicOr(status, 1);
    if (lane < k) sel_idx[out0 + lane] = b + lane;
    if (lane == 0) masks[g] = (k == WAVE) ? ~0ull : ((1ull << k) - 1ull);
    return;
  }
  // rank under the strict order (value, slot)
  int rank = 0;
  for (int l = 0; l < n; ++l) {
    const float vl = __shfl(v, l, WAVE);
    rank += (vl < v || (vl == v && l < lane)) ? 1 : 0;
  }
  sorted[wv][lane] = 0.0f;
  __builtin_amdgcn_wave_barrier();
  if (live) sorted[wv][rank] = v;
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  const double y = (double)sorted[wv][lane];                       // ascending, zero padded
  const double z = live ? (double)sorted[wv][n - 1 - lane] : 0.0;  // descending, zero padded
  const double s_lo = wave_scan_f64(y, lane);
  const double s_lo2 = wave_scan_f64(__dmul_rn(y, y), lane);
  const double s_hi = wave_scan_f64(z, lane);
  const double s_hi2 = wave_scan_f64(__dmul_rn(z, z), lane);
  // candidate j (lane j, 0 <= j <= k <= 63): j lowest + (k - j) highest
  const int j = lane;
  const int m = k - j;                                              // taken from the top
  double lo = shfl_up_f64(s_lo, 1), lo2 = shfl_up_f64(s_lo2, 1);
  if (j == 0) { lo = 0.0; lo2 = 0.0; }
  const int srcl = (m >= 1) ? (m - 1) : 0;
  double hi = __shfl(s_hi, srcl, WAVE), hi2 = __shfl(s_hi2, srcl, WAVE);
  if (m < 1) { hi = 0.0; hi2 = 0.0; }
  const double s1 = __dadd_rn(lo, hi);
  const double s2 = __dadd_rn(lo2, hi2);
  double score = __dsub_rn(__dmul_rn((double)k, s2), __dmul_rn(s1, s1));
  int best = j;
  if (j > k) score = -__builtin_huge_val();
  // arg-max, ties to the smaller j
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const double os = __shfl_xor(score, o, WAVE);
    const int ob = __shfl_xor(best, o, WAVE);
    if (os > score || (os == score && ob < best)) { score = os; best = ob; }
  }
  const bool keep = live && (rank < best || rank >= n - (k - best));
  const uint64_t mask = __ballot(keep);
  if (keep) sel_idx[out0 + __popcll(mask & ((1ull << lane) - 1ull))] = b + lane;
  if (lane == 0) masks[g] = mask;
}

// ---- the same selection for groups of up to 1024 members (beyond the paper's group sizes): one
// workgroup of 1024 lanes per group, one member per lane.  Same evaluation order as above with the
// prefix sums taken over S zero-padded slots, S = 64 up to 64 members, else the next power of two.
constexpr int OVF_LARGE = 1024;

__global__ __launch_bounds__(OVF_LARGE) void ovf_select_large_kernel(
    const float* __restrict__ rewards, const int32_t* __restrict__ offsets, const int32_t* __restrict__ kk,
    int n_groups, const int32_t* __restrict__ new_offsets, int mask_words, uint64_t* __restrict__ masks,
    int32_t* __restrict__ sel_idx, int32_t* __restrict__ status) {
  __shared__ float val[OVF_LARGE];
  __shared__ float sorted[OVF_LARGE];
  __shared__ double sc[4][OVF_LARGE];              // running sums of y, y^2, z, z^2
  __shared__ double red_s[OVF_LARGE / WAVE];
  __shared__ int red_b[OVF_LARGE / WAVE];
  __shared__ int wave_cnt[OVF_LARGE / WAVE];
  const int tid = threadIdx.x, lane = tid & (WAVE - 1), wv = tid / WAVE;
  const int g = blockIdx.x;
  const int b = offsets[g];
  const int n = offsets[g + 1] - b;
  const int k = kk[g];
  const int out0 = new_offsets[g];
  uint64_t* mrow = masks + (int64_t)g * mask_words;
  if (n < 1 || n > OVF_LARGE || n > 64 * mask_words || k < 1 || k > n) {
    if (tid == 0 && !(n == 0 && k == 0)) atomicOr(status, 2);
    if (tid < mask_words) mrow[tid] = 0ull;
    fill_bad_group(sel_idx, out0, b, n, k, tid, OVF_LARGE);
    return;                                          // whole workgroup leaves together
  }
  const bool live = tid < n;
  const float v = live ? rewards[b + tid] + 0.0f : 0.0f;
  const bool bad = live && !(__builtin_fabsf(v) <= 3.4028234663852886e38f);
  const int any_bad = __syncthreads_or(bad ? 1 : 0);
  bool keep;
  if (any_bad || k == n) {
    if (any_bad && tid == 0) atomicOr(status, 1);
    keep = tid < k;
  } else {
    val[tid] = v;
    __syncthreads();
    int rank = 0;
    if (live)
      for (int l = 0; l < n; ++l) {
        const float vl = val[l];
        rank += (vl < v || (vl == v && l < tid)) ? 1 : 0;
      }
    sorted[tid] = 0.0f;
    __syncthreads();
    if (live) sorted[rank] = v;
    __syncthreads();
    int S = WAVE;
    while (S < n) S <<= 1;
    {
      const double y = (double)sorted[tid];
      const double z = live ? (double)sorted[n - 1 - tid] : 0.0;
      sc[0][tid] = y; sc[1][tid] = __dmul_rn(y, y); sc[2][tid] = z; sc[3][tid] = __dmul_rn(z, z);
    }
    __syncthreads();
    for (int dd = 1; dd < S; dd <<= 1) {             // all slots updated from the values of the previous pass
      double t[4] = {0.0, 0.0, 0.0, 0.0};
      if (tid >= dd && tid < S)
#pragma unroll
        for (int q = 0; q < 4; ++q) t[q] = sc[q][tid - dd];
      __syncthreads();
      if (tid >= dd && tid < S)
#pragma unroll
        for (int q = 0; q < 4; ++q) sc[q][tid] = __dadd_rn(sc[q][tid], t[q]);
      __syncthreads();
    }
    // candidate j = tid (0 <= j <= k): j lowest + (k - j) highest
    const int j = tid, m = k - j;
    double score = -__builtin_huge_val();
    int best = j;
    if (j <= k) {
      const double lo = j ? sc[0][j - 1] : 0.0, lo2 = j ? sc[1][j - 1] : 0.0;
      const double hi = m ? sc[2][m - 1] : 0.0, hi2 = m ? sc[3][m - 1] : 0.0;
      const double s1 = __dadd_rn(lo, hi), s2 = __dadd_rn(lo2, hi2);
      score = __dsub_rn(__dmul_rn((double)k, s2), __dmul_rn(s1, s1));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {               // arg-max, ties to the smaller j
      const double os = __shfl_xor(score, o, WAVE);
      const int ob = __shfl_xor(best, o, WAVE);
      if (os > score || (os == score && ob < best)) { score = os; best = ob; }
    }
    if (lane == 0) { red_s[wv] = score; red_b[wv] = best; }
    __syncthreads();
    score = red_s[0]; best = red_b[0];
    for (int w = 1; w < OVF_LARGE / WAVE; ++w)
      if (red_s[w] > score || (red_s[w] == score && red_b[w] < best)) { score = red_s[w]; best = red_b[w]; }
    keep = live && (rank < best || rank >= n - (k - best));
  }
  const uint64_t ballot = __ballot(keep);
  if (lane == 0) {
    wave_cnt[wv] = __popcll(ballot);
    if (wv < mask_words) mrow[wv] = ballot;
  }
  __syncthreads();
  if (keep) {
    int before = 0;
    for (int w = 0; w < wv; ++w) before += wave_cnt[w];
    sel_idx[out0 + before + __popcll(ballot & ((1ull << lane) - 1ull))] = b + tid;
  }
}

// ---- exclusive scan of k over groups (new_offsets[g] = sum of k[0..g)) in three launches ----
__global__ __launch_bounds__(SCAN_THREADS) void scan_block_sums_kernel(const int32_t* __restrict__ kk,
                                                                       int n, int32_t* __restrict__ sums) {
  __shared__ int part[SCAN_THREADS / WAVE];
  int s = 0;
  const int base = blockIdx.x * SCAN_BLOCK + threadIdx.x * SCAN_ITEMS;
  for (int i = 0; i < SCAN_ITEMS; ++i) if (base + i < n) s += counted_k(kk[base + i]);
  for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, WAVE);
  if ((threadIdx.x & (WAVE - 1)) == 0) part[threadIdx.x / WAVE] = s;
  __syncthreads();
  if (threadIdx.x == 0) sums[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

__global__ void scan_sums_kernel(int32_t* __restrict__ sums, int n_blocks) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < n_blocks; ++i) { const int t = sums[i]; sums[i] = run; run += t; }
    sums[n_blocks] = run;
  }
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_write_kernel(const int32_t* __restrict__ kk, int n,
                                                                  const int32_t* __restrict__ sums,
                                                                  int32_t* __restrict__ new_offsets) {
  __shared__ int lane_tot[SCAN_THREADS];
  const int base = blockIdx.x * SCAN_BLOCK + threadIdx.x * SCAN_ITEMS;
  int loc[SCAN_ITEMS];
  int s = 0;
  for (int i = 0; i < SCAN_ITEMS; ++i) { loc[i] = s; if (base + i < n) s += counted_k(kk[base + i]); }
  lane_tot[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = sums[blockIdx.x];
    for (int i = 0; i < SCAN_THREADS; ++i) { const int t = lane_tot[i]; lane_tot[i] = run; run += t; }
  }
  __syncthreads();
  const int off = lane_tot[threadIdx.x];
  for (int i = 0; i < SCAN_ITEMS; ++i) if (base + i < n) new_offsets[base + i] = off + loc[i];
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) new_offsets[n] = sums[gridDim.x];
}

// ---- advantages: one wave per group ----
__device__ __forceinline__ double wave_allsum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}

__global__ __launch_bounds__(OVF_WAVES * WAVE) void group_advantages_kernel(
    const float* __restrict__ rewards, const int32_t* __restrict__ offsets, int n_groups, double eps,
    float* __restrict__ adv) {
  const int wv = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
  const int g = blockIdx.x * OVF_WAVES + wv;
  if (g >= n_groups) return;
  const int b = offsets[g], e = offsets[g + 1];
  const int n = e - b;
  // groups larger than a wave are walked in strides of 64 (not used by the sampling loop)
  double s = 0.0;
  for (int i = b + lane; i < e; i += WAVE) s += (double)rewards[i];
  const double mu = wave_allsum_f64(s) / (double)n;
  double q = 0.0;
  for (int i = b + lane; i < e; i += WAVE) { const double dv = (double)rewards[i] - mu; q += dv * dv; }
  const double sigma = sqrt(wave_allsum_f64(q) / (double)n);
  for (int i = b + lane; i < e; i += WAVE) adv[i] = (float)(((double)rewards[i] - mu) / (sigma + eps));
}

// ---- comparison arm of Sec. 4.1: a uniformly random k-subset per group ----
// Slot j of group g draws one 32-bit key, word 0 of the Philox-4x32-10 block with counter
// (j, draw, g, STREAM_SUBSAMPLE) under the run's seed; the k slots with the smallest (key, slot) stay.
constexpr uint32_t STREAM_SUBSAMPLE = 2u;

__global__ __launch_bounds__(OVF_WAVES * WAVE) void uniform_select_kernel(
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ kk, int n_groups,
    const int32_t* __restrict__ new_offsets, uint32_t k0, uint32_t k1, uint32_t draw,
    uint64_t* __restrict__ masks, int32_t* __restrict__ sel_idx, int32_t* __restrict__ status) {
  const int wv = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
  const int g = blockIdx.x * OVF_WAVES + wv;
  if (g >= n_groups) return;
  const int b = offsets[g];
  const int n = offsets[g + 1] - b;
  const int k = kk[g];
  const int out0 = new_offsets[g];
  if (n < 1 || n > WAVE || k < 1 || k > n) {
    if (lane == 0) {
      if (!(n == 0 && k == 0)) atomicOr(status, 2);
      masks[g] = 0ull;
    }
    fill_bad_group(sel_idx, out0, b, n, k, lane, WAVE);
    return;
  }
  const uint32_t key = philox4x32_10(u32x4{(uint32_t)lane, draw, (uint32_t)g, STREAM_SUBSAMPLE}, k0, k1).x;
  int rank = 0;
  for (int l = 0; l < n; ++l) {
    const uint32_t kl = (uint32_t)__shfl((int)key, l, WAVE);
    rank += (kl < key || (kl == key && l < lane)) ? 1 : 0;
  }
  const bool keep = lane < n && rank < k;
  const uint64_t mask = __ballot(keep);
  if (keep) sel_idx[out0 + __popcll(mask & ((1ull << lane) - 1ull))] = b + lane;
  if (lane == 0) masks[g] = mask;
}

// ---- group diagnostics: sigma_G (population) and the share of members within delta sigma_G of the
// group mean (the clustered region of Eq. 7); one wave per group, any group size ----
__global__ __launch_bounds__(OVF_WAVES * WAVE) void group_stats_kernel(
    const float* __restrict__ rewards, const int32_t* __restrict__ offsets, int n_groups, double delta,
    float* __restrict__ sigma_out, float* __restrict__ share_out) {
  const int wv = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
  const int g = blockIdx.x * OVF_WAVES + wv;
  if (g >= n_groups) return;
  const int b = offsets[g], e = offsets[g + 1];
  const int n = e - b;
  if (n <= 0) {
    if (lane == 0) { if (sigma_out) sigma_out[g] = 0.f; if (share_out) share_out[g] = 0.f; }
    return;
  }
  double s = 0.0;
  for (int i = b + lane; i < e; i += WAVE) s += (double)rewards[i];
  const double mu = wave_allsum_f64(s) / (double)n;
  double q = 0.0;
  for (int i = b + lane; i < e; i += WAVE) { const double dv = (double)rewards[i] - mu; q += dv * dv; }
  const double sigma = sqrt(wave_allsum_f64(q) / (double)n);
  int inside = 0;
  for (int i = b + lane; i < e; i += WAVE) inside += (fabs((double)rewards[i] - mu) <= delta * sigma) ? 1 : 0;
  for (int o = 32; o > 0; o >>= 1) inside += __shfl_xor(inside, o, WAVE);
  if (lane == 0) {
    if (sigma_out) sigma_out[g] = (float)sigma;
    if (share_out) share_out[g] = (float)((double)inside / (double)n);
  }
}

// ---- index bookkeeping around a prune ----
__global__ void gather_ids_kernel(const int32_t* __restrict__ ids_in, const int32_t* __restrict__ sel,
                                  int n_out, int32_t* __restrict__ ids_out) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < n_out) ids_out[r] = ids_in[sel[r]];
}

__global__ void fill_group_of_kernel(const int32_t* __restrict__ offsets, int32_t* __restrict__ group_of) {
  const int g = blockIdx.x;
  for (int i = offsets[g] + threadIdx.x; i < offsets[g + 1]; i += blockDim.x) group_of[i] = g;
}

// survivors imposed from outside: sel_idx from masks (test hook of the sampling loop)
__global__ void masks_to_sel_kernel(const uint64_t* __restrict__ masks, const int32_t* __restrict__ offsets,
                                    const int32_t* __restrict__ new_offsets, int n_groups,
                                    int32_t* __restrict__ sel_idx) {
  const int g = blockIdx.x;
  const int lane = threadIdx.x;
  if (g >= n_groups || lane >= WAVE) return;
  const uint64_t m = masks[g];
  const int n = offsets[g + 1] - offsets[g];
  if (lane < n && ((m >> lane) & 1ull))
    sel_idx[new_offsets[g] + __popcll(m & ((1ull << lane) - 1ull))] = offsets[g] + lane;
}

__global__ void fill_u32_kernel(uint32_t* __restrict__ p, uint32_t v, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

__global__ void iota_kernel(int32_t* __restrict__ p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i;
}

pg_status launch_fill_u32(void* p, uint32_t v, size_t n, hipStream_t s) {
  if (n == 0) return PG_OK;
  const unsigned blocks = (unsigned)((n + 1023) / 1024 > 4096 ? 4096 : (n + 1023) / 1024);
  fill_u32_kernel<<<dim3(blocks), dim3(256), 0, s>>>((uint32_t*)p, v, n);
  PG_LAUNCH_CHECK("fill_u32_kernel");
  return PG_OK;
}

pg_status launch_iota(int32_t* p, int n, hipStream_t s) {
  if (n <= 0) return PG_OK;
  iota_kernel<<<dim3((n + 255) / 256), dim3(256), 0, s>>>(p, n);
  PG_LAUNCH_CHECK("iota_kernel");
  return PG_OK;
}

pg_status launch_gather_ids(const int32_t* in, const int32_t* sel, int n_out, int32_t* out, hipStream_t s) {
  if (n_out <= 0) return PG_OK;
  gather_ids_kernel<<<dim3((n_out + 255) / 256), dim3(256), 0, s>>>(in, sel, n_out, out);
  PG_LAUNCH_CHECK("gather_ids_kernel");
  return PG_OK;
}

pg_status launch_fill_group_of(const int32_t* offsets, int n_groups, int32_t* group_of, hipStream_t s) {
  fill_group_of_kernel<<<dim3(n_groups), dim3(64), 0, s>>>(offsets, group_of);
  PG_LAUNCH_CHECK("fill_group_of_kernel");
  return PG_OK;
}

pg_status launch_masks_to_sel(const uint64_t* masks, const int32_t* offsets, const int32_t* new_offsets,
                              int n_groups, int32_t* sel_idx, hipStream_t s) {
  masks_to_sel_kernel<<<dim3(n_groups), dim3(64), 0, s>>>(masks, offsets, new_offsets, n_groups, sel_idx);
  PG_LAUNCH_CHECK("masks_to_sel_kernel");
  return PG_OK;
}

pg_status launch_uniform_select(const int32_t* offsets, const int32_t* k, int n_groups, const int32_t* new_offsets,
                                uint64_t seed, uint32_t draw, uint64_t* masks, int32_t* sel_idx, int32_t* status,
                                hipStream_t s) {
  uniform_select_kernel<<<dim3((n_groups + OVF_WAVES - 1) / OVF_WAVES), dim3(OVF_WAVES * WAVE), 0, s>>>(
      offsets, k, n_groups, new_offsets, (uint32_t)seed, (uint32_t)(seed >> 32), draw, masks, sel_idx, status);
  PG_LAUNCH_CHECK("uniform_select_kernel");
  return PG_OK;
}

// exclusive scan of k into new_offsets (three launches), shared by the selection entry points
static pg_status scan_k(const int32_t* k, int n_groups, int32_t* scratch, int32_t* new_offsets, hipStream_t s) {
  const int n_blocks = (n_groups + SCAN_BLOCK - 1) / SCAN_BLOCK;
  scan_block_sums_kernel<<<dim3(n_blocks), dim3(SCAN_THREADS), 0, s>>>(k, n_groups, scratch);
  PG_LAUNCH_CHECK("scan_block_sums_kernel");
  scan_sums_kernel<<<dim3(1), dim3(64), 0, s>>>(scratch, n_blocks);
  PG_LAUNCH_CHECK("scan_sums_kernel");
  scan_write_kernel<<<dim3(n_blocks), dim3(SCAN_THREADS), 0, s>>>(k, n_groups, scratch, new_offsets);
  PG_LAUNCH_CHECK("scan_write_kernel");
  return PG_OK;
}

// OVF with new_offsets already known (the sampling loop knows them from its schedule)
pg_status launch_ovf(const float* rewards, const int32_t* offsets, const int32_t* k, int n_groups,
                     const int32_t* new_offsets, uint64_t* masks, int32_t* sel_idx, int32_t* status,
                     hipStream_t s) {
  ovf_select_kernel<<<dim3((n_groups + OVF_WAVES - 1) / OVF_WAVES), dim3(OVF_WAVES * WAVE), 0, s>>>(
      rewards, offsets, k, n_groups, new_offsets, masks, sel_idx, status);
  PG_LAUNCH_CHECK("ovf_select_kernel");
  return PG_OK;
}

}  // namespace pg

using namespace pg;

extern "C" int64_t pg_ovf_scratch_ints(int64_t n_groups) {
  if (n_groups <= 0) return 0;
  return (n_groups + SCAN_BLOCK - 1) / SCAN_BLOCK + 1;
}

extern "C" pg_status pg_ovf_select(const float* rewards, const int32_t* group_offsets, const int32_t* k,
                                   int32_t n_groups, uint64_t* masks, int32_t* sel_idx,
                                   int32_t* new_offsets, int32_t* status, int32_t* scratch, void* stream) {
  if (n_groups < 0) return fail(PG_EINVAL, "pg_ovf_select: n_groups = %d", n_groups);
  if (n_groups == 0) return PG_OK;
  if (!rewards || !group_offsets || !k || !masks || !sel_idx || !new_offsets || !status || !scratch)
    return fail(PG_EINVAL, "pg_ovf_select: null pointer");
  hipStream_t s = (hipStream_t)stream;
  PG_TRY(scan_k(k, n_groups, scratch, new_offsets, s));
  return launch_ovf(rewards, group_offsets, k, n_groups, new_offsets, masks, sel_idx, status, s);
}

// ---- the same selection for callers that cannot allocate: the scan's block sums live in a file-scope device
// array (one copy per GPU, held until the process ends) instead of a buffer the caller brings ----
constexpr int NOALLOC_SCRATCH_INTS = PG_OVF_NOALLOC_MAX_GROUPS / SCAN_BLOCK + 1;
static __device__ __align__(256) int32_t g_ovf_scratch[NOALLOC_SCRATCH_INTS];

// On the host the array's name stands for the symbol, not for device memory: its address on a GPU is looked up
// once per device (with that device current) and kept.
constexpr int MAX_DEVICES = 64;
static int32_t* g_ovf_scratch_ptr[MAX_DEVICES] = {};
static std::mutex g_ovf_scratch_mu;

static pg_status ovf_scratch_on_current_device(hipStream_t s, int32_t** out) {
  int dev = -1;
  PG_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(PG_EHIP, "pg_ovf_select_noalloc: device index %d", dev);
  if (s) {
    int sdev = -1;
    PG_HIP(hipStreamGetDevice(s, &sdev));
    if (sdev != dev)
      return fail(PG_EINVAL, "pg_ovf_select_noalloc: the stream belongs to device %d, the current device is %d", sdev, dev);
  }
  std::lock_guard<std::mutex> lock(g_ovf_scratch_mu);
  if (!g_ovf_scratch_ptr[dev]) {
    void* p = nullptr;
    PG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_ovf_scratch)));
    if (!p) return fail(PG_EHIP, "pg_ovf_select_noalloc: the scratch symbol has no address on device %d", dev);
    g_ovf_scratch_ptr[dev] = static_cast<int32_t*>(p);
  }
  *out = g_ovf_scratch_ptr[dev];
  return PG_OK;
}

extern "C" pg_status pg_ovf_select_noalloc(const float* rewards, const int32_t* group_offsets, const int32_t* k,
                                           int32_t n_groups, uint64_t* masks, int32_t* sel_idx,
                                           int32_t* new_offsets, int32_t* status, void* stream) {
  if (n_groups < 0) return fail(PG_EINVAL, "pg_ovf_select_noalloc: n_groups = %d", n_groups);
  if (n_groups > PG_OVF_NOALLOC_MAX_GROUPS)
    return fail(PG_ESHAPE, "pg_ovf_select_noalloc: %d groups exceed the built-in scratch (at most %d); use pg_ovf_select",
                n_groups, PG_OVF_NOALLOC_MAX_GROUPS);
  if (n_groups == 0) return PG_OK;
  if (!rewards || !group_offsets || !k || !masks || !sel_idx || !new_offsets || !status)
    return fail(PG_EINVAL, "pg_ovf_select_noalloc: null pointer");
  hipStream_t s = (hipStream_t)stream;
  int32_t* sums = nullptr;
  PG_TRY(ovf_scratch_on_current_device(s, &sums));
  PG_TRY(scan_k(k, n_groups, sums, new_offsets, s));          // every word it reads back it has written in this call
  return launch_ovf(rewards, group_offsets, k, n_groups, new_offsets, masks, sel_idx, status, s);
}

extern "C" pg_status pg_group_advantages(const float* rewards, const int32_t* group_offsets,
                                         int32_t n_groups, double eps, float* adv, void* stream) {
  if (n_groups < 0) return fail(PG_EINVAL, "pg_group_advantages: n_groups = %d", n_groups);
  if (!(eps >= 0.0)) return fail(PG_EINVAL, "pg_group_advantages: eps = %g", eps);
  if (n_groups == 0) return PG_OK;
  if (!rewards || !group_offsets || !adv) return fail(PG_EINVAL, "pg_group_advantages: null pointer");
  group_advantages_kernel<<<dim3((n_groups + OVF_WAVES - 1) / OVF_WAVES), dim3(OVF_WAVES * WAVE), 0,
                            (hipStream_t)stream>>>(rewards, group_offsets, n_groups, eps, adv);
  PG_LAUNCH_CHECK("group_advantages_kernel");
  return PG_OK;
}

extern "C" pg_status pg_uniform_select(const int32_t* group_offsets, const int32_t* k, int32_t n_groups,
                                       uint64_t seed, uint32_t draw, uint64_t* masks, int32_t* sel_idx,
                                       int32_t* new_offsets, int32_t* status, int32_t* scratch, void* stream) {
  if (n_groups < 0) return fail(PG_EINVAL, "pg_uniform_select: n_groups = %d", n_groups);
  if (n_groups == 0) return PG_OK;
  if (!group_offsets || !k || !masks || !sel_idx || !new_offsets || !status || !scratch)
    return fail(PG_EINVAL, "pg_uniform_select: null pointer");
  hipStream_t s = (hipStream_t)stream;
  PG_TRY(scan_k(k, n_groups, scratch, new_offsets, s));
  return launch_uniform_select(group_offsets, k, n_groups, new_offsets, seed, draw, masks, sel_idx, status, s);
}

extern "C" pg_status pg_group_stats(const float* rewards, const int32_t* group_offsets, int32_t n_groups,
                                    double delta, float* sigma, float* clustered_share, void* stream) {
  if (n_groups < 0) return fail(PG_EINVAL, "pg_group_stats: n_groups = %d", n_groups);
  if (!(delta >= 0.0)) return fail(PG_EINVAL, "pg_group_stats: delta = %g", delta);
  if (n_groups == 0) return PG_OK;
  if (!rewards || !group_offsets || (!sigma && !clustered_share)) return fail(PG_EINVAL, "pg_group_stats: null pointer");
  group_stats_kernel<<<dim3((n_groups + OVF_WAVES - 1) / OVF_WAVES), dim3(OVF_WAVES * WAVE), 0,
                       (hipStream_t)stream>>>(rewards, group_offsets, n_groups, delta, sigma, clustered_share);
  PG_LAUNCH_CHECK("group_stats_kernel");
  return PG_OK;
}

extern "C" pg_status pg_ovf_select_large(const float* rewards, const int32_t* group_offsets, const int32_t* k,
                                         int32_t n_groups, int32_t mask_words, uint64_t* masks, int32_t* sel_idx,
                                         int32_t* new_offsets, int32_t* status, int32_t* scratch, void* stream) {
  if (n_groups < 0) return fail(PG_EINVAL, "pg_ovf_select_large: n_groups = %d", n_groups);
  if (mask_words < 1 || mask_words > OVF_LARGE / WAVE)
    return fail(PG_EINVAL, "pg_ovf_select_large: mask_words = %d (1..%d)", mask_words, OVF_LARGE / WAVE);
  if (n_groups == 0) return PG_OK;
  if (!rewards || !group_offsets || !k || !masks || !sel_idx || !new_offsets || !status || !scratch)
    return fail(PG_EINVAL, "pg_ovf_select_large: null pointer");
  hipStream_t s = (hipStream_t)stream;
  PG_TRY(scan_k(k, n_groups, scratch, new_offsets, s));
  ovf_select_large_kernel<<<dim3(n_groups), dim3(OVF_LARGE), 0, s>>>(rewards, group_offsets, k, n_groups, new_offsets,
                                                                      mask_words, masks, sel_idx, status);
  PG_LAUNCH_CHECK("ovf_select_large_kernel");
  return PG_OK;
}
