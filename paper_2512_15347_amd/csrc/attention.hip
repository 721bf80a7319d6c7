// Softmax attention of the network on bf16 MFMA (self, joint and cross variants share this kernel).
//
// One workgroup = 4 wavefronts = 128 queries of one (batch, head); each wavefront owns 32 queries and
// walks the keys in tiles of 64 staged through LDS.  The score tile is computed TRANSPOSED,
// S^T = K Q^T, so that in the 32x32 MFMA accumulator layout every lane holds scores of ONE query
// (column) for 16 keys (rows): the online-softmax row statistics are in-lane reductions plus a single
// exchange with the other half-wave.  The probabilities then feed O^T = V^T P^T directly from the
// accumulator registers; the key order inside each 16-key contraction is permuted the same way in the
// V^T operand read from LDS, which is why V is stored transposed ([head dim][key]) by the QKV GEMM.
// The softmax's VALU work, not the MFMAs, sets the pace here, so it is kept minimal: the queries arrive
// pre-multiplied by log2(e)/sqrt(hd) (by the projection GEMM's epilogue), the score accumulators start
// at minus the running reference exponent, so a probability is a bare exp2 of the accumulator; the
// masking of keys past the end exists only in the code for the last, partial tile; a wavefront whose 32
// queries all lie past the end of the sequence (the ragged last query tile) still stages keys and values
// but skips the arithmetic.  (Feeding the reference exponent to the first score MFMA from a register block
// of its own, which saves the per-tile initialisation, measured 6 % slower: the vector ALU is not what
// the waves wait for.)
#include <type_traits>
#include "attention.hpp"

namespace pg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
typedef float f32x2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int ATT_THREADS = 256;
constexpr int QTILE = 128, KTILE = 64;

template <int HD>
__device__ __forceinline__ int k_off(int row, int chunk) {       // K tile [64 keys][HD]
  if (HD == 64) return (row * 8 + (chunk ^ ((row ^ (row >> 3)) & 7))) * 16;
  return (row * 4 + (chunk ^ (((row >> 1) ^ (row >> 3)) & 3))) * 16;
}
__device__ __forceinline__ int v_off(int row, int chunk) {       // V^T tile [HD][64 keys]
  return (row * 8 + (chunk ^ ((row ^ (row >> 3)) & 7))) * 16;
}

template <int HD>
__global__ __launch_bounds__(ATT_THREADS, 2) void attention_kernel(const AttnArgs a) {
  constexpr int KCH = HD / 8;                  // 16-byte chunks per K row
  constexpr int K_PER_THREAD = KTILE * KCH / ATT_THREADS;        // 2 (HD 64) or 1 (HD 32)
  constexpr int V_PER_THREAD = HD * 8 / ATT_THREADS;             // 2 or 1
  constexpr int SLABS = HD / 16;               // k-slabs of the score MFMA
  constexpr int OT = HD / 32;                  // 32-row tiles of O^T
  __shared__ __align__(16) unsigned char sK[KTILE * HD * 2];
  __shared__ __align__(16) unsigned char sV[HD * KTILE * 2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // Workgroups are dealt to the 8 XCDs round-robin by id; the ids are permuted so that each XCD gets a
  // contiguous run of (batch, head, query tile): the query tiles of one head then share its keys and
  // values through one L2 instead of fetching them once per XCD.
  const int nq = (a.Lq + QTILE - 1) / QTILE;
  const int per_xcd = gridDim.x / 8;
  const int wg = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (wg >= nq * a.heads * a.B) return;
  const int b = wg / (nq * a.heads), h = (wg / nq) % a.heads;
  const int q0 = (wg % nq) * QTILE + wave * 32;
  const int kb = a.kv_map ? a.kv_map[b] : b;
  const uint16_t* kbase = a.k + (int64_t)kb * a.k_bstride + h * HD;
  const uint16_t* vbase = a.vt + (int64_t)kb * a.vt_bstride + (int64_t)h * HD * a.Lkpad;

  // Q fragments (B operand: column = query, k = head-dim index), kept in registers
  bf16x8 qf[SLABS];
  {
    const int qr = min(q0 + l32, a.Lq - 1);
    const uint16_t* qp = a.q + ((int64_t)b * a.Lq + qr) * a.ldq + h * HD + 8 * half;
#pragma unroll
    for (int s = 0; s < SLABS; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
    if (!a.q_prescaled) {
#pragma unroll
      for (int s = 0; s < SLABS; ++s)
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[s][e] = (__bf16)((float)qf[s][e] * a.scale_log2);
    }
  }

  f32x16 o[OT];
#pragma unroll
  for (int t = 0; t < OT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
  // Running softmax statistics in the log2 domain.  m_run is a reference exponent, not necessarily the
  // exact running maximum: after the first tile it is only raised (and the accumulators rescaled) when a
  // new score exceeds it by more than 2^8, so most tiles skip the rescale; probabilities stay below 2^8,
  // well inside bf16 / fp32 range, and the final division by l makes the result independent of the
  // reference.
  float m_run = 0.f, l_run = 0.f;
  const bool wave_has_queries = q0 < a.Lq;       // wave-uniform

  const int n_tiles = (a.Lk + KTILE - 1) / KTILE;
  u32x4v rk[K_PER_THREAD], rv[V_PER_THREAD];
  // per-lane staging positions (fixed), advanced by whole tiles
  int k_row[K_PER_THREAD], k_ch[K_PER_THREAD], v_row[V_PER_THREAD], v_ch[V_PER_THREAD];
#pragma unroll
  for (int i = 0; i < K_PER_THREAD; ++i) { const int cc = tid + i * ATT_THREADS; k_row[i] = cc / KCH; k_ch[i] = cc % KCH; }
#pragma unroll
  for (int i = 0; i < V_PER_THREAD; ++i) { const int cc = tid + i * ATT_THREADS; v_row[i] = cc >> 3; v_ch[i] = cc & 7; }

  // staging sources for tile 0; full tiles advance them by whole tiles with wave-uniform offsets
  const uint16_t* k_src[K_PER_THREAD];
  const uint16_t* v_src[V_PER_THREAD];
#pragma unroll
  for (int i = 0; i < K_PER_THREAD; ++i) k_src[i] = kbase + (int64_t)min(k_row[i], a.Lk - 1) * a.ldk + k_ch[i] * 8;
#pragma unroll
  for (int i = 0; i < V_PER_THREAD; ++i) v_src[i] = vbase + (int64_t)v_row[i] * a.Lkpad + v_ch[i] * 8;
  auto load_tile = [&](int kt) {
    const int k0 = kt * KTILE;
    if (k0 + KTILE <= a.Lk) {                    // full tile: no clamping, no masking
      const int64_t koff = (int64_t)k0 * a.ldk;
#pragma unroll
      for (int i = 0; i < K_PER_THREAD; ++i) rk[i] = *reinterpret_cast<const u32x4v*>(k_src[i] + koff);
#pragma unroll
      for (int i = 0; i < V_PER_THREAD; ++i) rv[i] = *reinterpret_cast<const u32x4v*>(v_src[i] + k0);
      return;
    }
#pragma unroll
    for (int i = 0; i < K_PER_THREAD; ++i) {
      const int key = min(k0 + k_row[i], a.Lk - 1);
      rk[i] = *reinterpret_cast<const u32x4v*>(kbase + (int64_t)key * a.ldk + k_ch[i] * 8);
    }
#pragma unroll
    for (int i = 0; i < V_PER_THREAD; ++i) {
      const int kc = k0 + v_ch[i] * 8;
      u32x4v v = *reinterpret_cast<const u32x4v*>(vbase + (int64_t)v_row[i] * a.Lkpad + kc);
      if (kc + 8 > a.Lk) {                       // zero the keys past the end (padding may hold anything)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          uint32_t x = v[w];
          if (kc + 2 * w >= a.Lk) x &= 0xFFFF0000u;
          if (kc + 2 * w + 1 >= a.Lk) x &= 0x0000FFFFu;
          v[w] = x;
        }
      }
      rv[i] = v;
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < K_PER_THREAD; ++i) *reinterpret_cast<u32x4v*>(sK + k_off<HD>(k_row[i], k_ch[i])) = rk[i];
#pragma unroll
    for (int i = 0; i < V_PER_THREAD; ++i) *reinterpret_cast<u32x4v*>(sV + v_off(v_row[i], v_ch[i])) = rv[i];
  };

  // one key tile; MASKED is the variant for a last tile that holds keys past the end
  auto tile = [&](int kt, auto masked_c) {
    constexpr bool MASKED = decltype(masked_c)::value;
    __syncthreads();                             // everyone is done reading the previous tile
    store_tile();
    __syncthreads();
    if (kt + 1 < n_tiles) load_tile(kt + 1);     // overlaps with the math below
    if (!wave_has_queries) return;               // staging and barriers above are the whole workgroup's

    // ---- S^T = K Q^T - m_run : two 32-key tiles ----
    const float neg_m = -m_run;
    f32x16 s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int e = 0; e < 16; ++e) s[t][e] = neg_m;
#pragma unroll
      for (int ks = 0; ks < SLABS; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sK + k_off<HD>(t * 32 + l32, 2 * ks + half));
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[t], 0, 0, 0);
      }
    }
    if (MASKED) {
      const int k0 = kt * KTILE;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (k0 + t * 32 + 8 * (e >> 2) + 4 * half + (e & 3) >= a.Lk) s[t][e] = -__builtin_huge_valf();
    }
    // ---- online softmax for this lane's query; scores are already relative to m_run ----
    float mx = s[0][0];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[t][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
    if (kt == 0 || __builtin_amdgcn_ballot_w64(mx > 8.0f) != 0ull) {   // wave-uniform: rare after the first tile
      const float delta = kt == 0 ? mx : fmaxf(mx, 0.f);               // the first tile sets the reference
      const float alpha = __builtin_amdgcn_exp2f(-delta);
      m_run += delta;
      l_run *= alpha;
#pragma unroll
      for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[t][e] -= delta;
    }
    float psum = 0.f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(s[t][e]);
        const float p1 = __builtin_amdgcn_exp2f(s[t][e + 1]);
        const f32x2v pp = {p0, p1};
        const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
        // the normaliser sums the probabilities as the value product sees them (rounded to bf16)
        psum = __builtin_amdgcn_fdot2_f32_bf16(pb, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, psum, false);
        pf[t][e >> 3][e & 7] = pb[0];
        pf[t][e >> 3][(e & 7) + 1] = pb[1];
      }
    l_run += psum;
    // ---- O^T += V^T P^T : contraction over 16 keys per MFMA, keys permuted as the accumulator holds them ----
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int c0 = 4 * t + 2 * jj;
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
          const int row = ot * 32 + l32;
          const u32x2v lo = *reinterpret_cast<const u32x2v*>(sV + v_off(row, c0) + 8 * half);
          const u32x2v hi = *reinterpret_cast<const u32x2v*>(sV + v_off(row, c0 + 1) + 8 * half);
          const u32x4v packed = {lo[0], lo[1], hi[0], hi[1]};
          const bf16x8 vf = __builtin_bit_cast(bf16x8, packed);
          o[ot] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[t][jj], o[ot], 0, 0, 0);
        }
      }
  };

  load_tile(0);
  const int n_full = a.Lk / KTILE;               // tiles that lie wholly inside the keys
  for (int kt = 0; kt < n_full; ++kt) tile(kt, std::false_type{});
  if (n_full < n_tiles) tile(n_full, std::true_type{});

  // ---- normalise and store: lane holds head-dim rows 8*(e/4) + 4*half + e%4 of its query ----
  const float l_tot = l_run + __shfl_xor(l_run, 32, WAVE);
  const float inv = 1.0f / l_tot;
  const int qr = q0 + l32;
  if (qr < a.Lq) {
    uint16_t* op = (a.split > 0) ? (qr < a.split ? a.out + ((int64_t)b * a.split + qr) * a.ldo + h * HD
                                                 : a.out2 + ((int64_t)b * (a.Lq - a.split) + qr - a.split) * a.ldo + h * HD)
                                 : a.out + ((int64_t)b * a.Lq + qr) * a.ldo + h * HD;
#pragma unroll
    for (int ot = 0; ot < OT; ++ot)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        bf16x4 w;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[t] = (__bf16)(o[ot][4 * q + t] * inv);
        *reinterpret_cast<bf16x4*>(op + ot * 32 + 8 * q + 4 * half) = w;
      }
  }
}

pg_status launch_attention(const AttnArgs& a, int hd, hipStream_t s) {
  if (a.B <= 0 || a.Lq <= 0 || a.heads <= 0) return PG_OK;
  if (a.Lk <= 0) return fail(PG_EINVAL, "attention: no keys");
  if (hd != 32 && hd != 64) return fail(PG_ESHAPE, "attention: head width %d not supported (32 or 64)", hd);
  if (a.Lkpad % 8 || a.Lkpad < a.Lk || a.ldq % 8 || a.ldk % 8 || a.ldo % 4 ||
      ((uintptr_t)a.q & 15) || ((uintptr_t)a.k & 15) || ((uintptr_t)a.vt & 15) || ((uintptr_t)a.out & 7))
    return fail(PG_ESHAPE, "attention: operands need 16-byte aligned rows");
  const int64_t wgs = (int64_t)((a.Lq + QTILE - 1) / QTILE) * a.heads * a.B;
  if (wgs > (1ll << 30)) return fail(PG_ESHAPE, "attention: grid limit");
  const dim3 grid((unsigned)((wgs + 7) / 8 * 8));
  const int rec = prof_open(PROF_ATTENTION, 4.0 * a.B * (double)a.heads * a.Lq * (double)a.Lk * hd, s);
  if (hd == 64) attention_kernel<64><<<grid, dim3(ATT_THREADS), 0, s>>>(a);
  else attention_kernel<32><<<grid, dim3(ATT_THREADS), 0, s>>>(a);
  prof_close(rec, s);
  PG_LAUNCH_CHECK("attention_kernel");
  return PG_OK;
}

}  // namespace pg

using namespace pg;

extern "C" pg_status pg_attention_bf16(const uint16_t* q, const uint16_t* k, const uint16_t* vt, uint16_t* out,
                                       int32_t B, int32_t Lq, int32_t Lk, int32_t heads, int32_t hd,
                                       void* stream) {
  if (B < 0 || Lq < 0 || Lk < 0 || heads < 1) return fail(PG_EINVAL, "pg_attention_bf16: bad sizes");
  if (B == 0 || Lq == 0) return PG_OK;
  if (!q || !k || !vt || !out) return fail(PG_EINVAL, "pg_attention_bf16: null pointer");
  const int D = heads * hd;
  AttnArgs a{};
  a.q = q; a.ldq = D; a.k = k; a.ldk = D; a.k_bstride = (int64_t)Lk * D;
  a.vt = vt; a.Lkpad = (Lk + 63) / 64 * 64; a.vt_bstride = (int64_t)D * a.Lkpad;
  a.out = out; a.ldo = D; a.kv_map = nullptr;
  a.B = B; a.Lq = Lq; a.Lk = Lk; a.heads = heads;
  a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)hd));
  return launch_attention(a, hd, (hipStream_t)stream);
}
