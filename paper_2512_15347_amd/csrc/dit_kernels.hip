// The velocity / noise network evaluated on every active trajectory at every step (the drift input of
// paper Eq. 12): a patch-2 adaLN transformer in four variants (conditioning vector only, extra
// cross-attention over context tokens, context tokens joined to the sequence, and the dual-stream
// form of the latter with per-stream weights and RMS-normalised queries / keys).  This file holds the
// memory-bound glue kernels (patchify, conditioning GEMVs, LayerNorm + modulation, context rows) and
// the orchestration; the contractions live in gemm.hip and attention.hip.
//
// Activation layout: rows r = m * L + token for the M active trajectories (image tokens first, then
// context tokens in the joint variant).  The dual-stream variant keeps two planes instead, image rows
// m * Li + t first and context rows M * Li + m * Lc + j behind them, so that each stream is one contiguous
// GEMM operand; only q | k and V^T use the joint per-trajectory layout that attention reads.
// The residual stream h is fp32; every GEMM operand is bf16.
#include <cmath>
#include "attention.hpp"
#include "ctx.hpp"
#include "gemm.hpp"

namespace pg {

__device__ __forceinline__ float bf2f(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ float silu(float x) { return x / (1.0f + __expf(-x)); }

__device__ __forceinline__ float wave_allsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}

// emb[0:128] = cos(t f_i), emb[128:256] = sin(t f_i), f_i = 10000^(-i/128)
__global__ void timestep_embedding_kernel(double t_in, float* __restrict__ emb) {
  const int i = threadIdx.x;
  if (i < 128) {
    const double f = exp(-9.210340371976184 * (double)i / 128.0);     // fp64: t f reaches 1000 rad
    emb[i] = (float)cos(t_in * f);
    emb[128 + i] = (float)sin(t_in * f);
  }
}

// out[p, n] = act(bias[n] + sum_k W[n, k] in[p, k]); one wave per output n, up to 8 inputs p at a time.
// grid.y walks `blocks` weight sets (w_stride elements apart) writing out + blockIdx.y * out_bstride.
template <bool SILU_OUT>
__global__ __launch_bounds__(256) void gemv_bf16_kernel(const uint16_t* __restrict__ W, int64_t ldw,
                                                        int64_t w_stride, const uint16_t* __restrict__ bias,
                                                        int64_t b_stride, const float* __restrict__ in,
                                                        int64_t in_ld, float* __restrict__ out, int64_t out_ld,
                                                        int64_t out_bstride, int P, int N, int K) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const uint16_t* w = W + blockIdx.y * w_stride + (int64_t)n * ldw;
  const float bv = bf2f(bias[blockIdx.y * b_stride + n]);
  for (int p0 = 0; p0 < P; p0 += 8) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int k = lane * 2; k < K; k += 128) {
      const uint32_t pair = *reinterpret_cast<const uint32_t*>(w + k);
      const float w0 = __builtin_bit_cast(float, pair << 16), w1 = __builtin_bit_cast(float, pair & 0xFFFF0000u);
#pragma unroll
      for (int p = 0; p < 8; ++p)
        if (p0 + p < P) {
          const float2 v = *reinterpret_cast<const float2*>(in + (int64_t)(p0 + p) * in_ld + k);
          acc[p] += w0 * v.x + w1 * v.y;
        }
    }
#pragma unroll
    for (int p = 0; p < 8; ++p)
      if (p0 + p < P) {
        float s = wave_allsum(acc[p]) + bv;
        if (SILU_OUT) s = silu(s);
        if (lane == 0) out[blockIdx.y * out_bstride + (int64_t)(p0 + p) * out_ld + n] = s;
      }
  }
}

// sc[p, n] = silu(c0[n] + y[p, n])
__global__ void cond_silu_kernel(const float* __restrict__ c0, const float* __restrict__ y, float* __restrict__ sc,
                                 int P, int D) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < P * D) sc[i] = silu(c0[i % D] + y[i]);
}

// tok[r, 4c + 2dy + dx] = bf16(x[m, c, 2py + dy, 2px + dx]), r = m * Li + py * Wp + px; columns >= 4C are zero
__global__ void patchify_kernel(const float* __restrict__ x, uint16_t* __restrict__ tok, int M, int C, int H, int Wd,
                                int Kp) {
  const int Wp = Wd / 2, Hp = H / 2;
  const int cq = Kp / 4;                       // 4-column groups per row, channels first then padding
  const int64_t total = (int64_t)M * cq * Hp * Wp;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int px = (int)(i % Wp);
  const int py = (int)((i / Wp) % Hp);
  const int c = (int)((i / ((int64_t)Wp * Hp)) % cq);
  const int m = (int)(i / ((int64_t)Wp * Hp * cq));
  uint32_t lo = 0u, hi = 0u;
  if (c < C) {
    const float* src = x + ((int64_t)m * C + c) * H * Wd + (int64_t)(2 * py) * Wd + 2 * px;
    const float2 r0 = *reinterpret_cast<const float2*>(src);
    const float2 r1 = *reinterpret_cast<const float2*>(src + Wd);
    lo = (uint32_t)f2bf(r0.x) | ((uint32_t)f2bf(r0.y) << 16);
    hi = (uint32_t)f2bf(r1.x) | ((uint32_t)f2bf(r1.y) << 16);
  }
  uint32_t* dst = reinterpret_cast<uint32_t*>(tok + ((int64_t)m * Hp * Wp + (int64_t)py * Wp + px) * Kp + 4 * c);
  dst[0] = lo;
  dst[1] = hi;
}

// out[r', :] = bf16(LN(h[r, :]) * (1 + scale[g]) + shift[g]); one wave per row.  The row lives in
// registers (NV float4 per lane, D = 256 * NV) so h is read once; NV = 0 is the generic route for
// widths that are not a multiple of 256 (three cached passes).
// Rows: r' = m * L_out + t for t < L_out reads h row m * L_in + t (L_out < L_in drops the context rows).
template <int NV>
__global__ __launch_bounds__(256) void ln_modulate_kernel(const float* __restrict__ h, uint16_t* __restrict__ out,
                                                          const float* __restrict__ shift,
                                                          const float* __restrict__ scale, int64_t mod_ld,
                                                          const int32_t* __restrict__ group_of, int rows_out,
                                                          int L_in, int L_out, int D) {
  const int lane = threadIdx.x & 63;
  const int ro = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (ro >= rows_out) return;
  const int m = ro / L_out, t = ro - m * L_out;
  const float* hr = h + ((int64_t)m * L_in + t) * D;
  uint16_t* orow = out + (int64_t)ro * D;
  const float* sh = nullptr;
  const float* sc = nullptr;
  if (shift) {
    const int g = group_of[m];
    sh = shift + (int64_t)g * mod_ld;
    sc = scale + (int64_t)g * mod_ld;
  }
  if (NV > 0) {
    float4 v[NV > 0 ? NV : 1];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      v[i] = reinterpret_cast<const float4*>(hr)[lane + 64 * i];
      s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
    const float mu = wave_allsum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      v[i].x -= mu; v[i].y -= mu; v[i].z -= mu; v[i].w -= mu;
      q += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
    }
    const float rstd = rsqrtf(wave_allsum(q) / (float)D + 1e-6f);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      float4 o = {v[i].x * rstd, v[i].y * rstd, v[i].z * rstd, v[i].w * rstd};
      if (sh) {
        const float4 a = reinterpret_cast<const float4*>(sc)[lane + 64 * i];
        const float4 b = reinterpret_cast<const float4*>(sh)[lane + 64 * i];
        o.x = o.x * (1.0f + a.x) + b.x; o.y = o.y * (1.0f + a.y) + b.y;
        o.z = o.z * (1.0f + a.z) + b.z; o.w = o.w * (1.0f + a.w) + b.w;
      }
      uint2 pk;
      pk.x = (uint32_t)f2bf(o.x) | ((uint32_t)f2bf(o.y) << 16);
      pk.y = (uint32_t)f2bf(o.z) | ((uint32_t)f2bf(o.w) << 16);
      reinterpret_cast<uint2*>(orow)[lane + 64 * i] = pk;
    }
    return;
  }
  float s = 0.f;
  for (int k = lane; k < D; k += WAVE) s += hr[k];
  const float mu = wave_allsum(s) / (float)D;
  float q = 0.f;
  for (int k = lane; k < D; k += WAVE) { const float dv = hr[k] - mu; q += dv * dv; }
  const float rstd = rsqrtf(wave_allsum(q) / (float)D + 1e-6f);
  if (sh) {
    for (int k = lane; k < D; k += WAVE) orow[k] = f2bf((hr[k] - mu) * rstd * (1.0f + sc[k]) + sh[k]);
  } else {
    for (int k = lane; k < D; k += WAVE) orow[k] = f2bf((hr[k] - mu) * rstd);
  }
}

// context rows of trajectory m: h[row_base + m * row_stride + j, :] = ctx_h[group_of[m], j, :]
__global__ void scatter_context_kernel(const float* __restrict__ ctx_h, float* __restrict__ h,
                                       const int32_t* __restrict__ group_of, int M, int64_t row_base,
                                       int row_stride, int Lc, int D4) {
  const int64_t total = (int64_t)M * Lc * D4;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int k = (int)(i % D4);
  const int j = (int)((i / D4) % Lc);
  const int m = (int)(i / ((int64_t)D4 * Lc));
  const float4 v = reinterpret_cast<const float4*>(ctx_h)[((int64_t)group_of[m] * Lc + j) * D4 + k];
  reinterpret_cast<float4*>(h)[(row_base + (int64_t)m * row_stride + j) * D4 + k] = v;
}

// ------------------------------------------------------------------------------------------------

static size_t a256(size_t v) { return (v + 255) & ~(size_t)255; }

pg_status net_plan(pg_ctx* c) {
  c->net = NetPlan{};
  const pg_config& f = c->cfg;
  if (f.net_kind == PG_NET_NONE) return PG_OK;
  const size_t R0 = (size_t)c->M0 * c->L, D = f.D;
  const size_t Lpad = ((size_t)c->L + 63) / 64 * 64, Lcpad = ((size_t)f.Lc + 63) / 64 * 64;
  const size_t Kp = ((size_t)4 * f.C + 63) / 64 * 64;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off = a256(off + bytes); return o; };
  NetPlan& n = c->net;
  n.h = take(R0 * D * 4);
  n.act = take(R0 * D * 2);
  n.qkv = take(R0 * 2 * D * 2);
  n.vt = take((size_t)c->M0 * D * Lpad * 2);
  n.att = take(R0 * D * 2);
  n.hid = take(R0 * 4 * D * 2);
  n.tok = take((size_t)c->M0 * c->Li * Kp * 2);
  n.mod = take(((size_t)f.P * f.blocks * 6 * D * (f.net_kind == PG_NET_MMDIT ? 2 : 1) + (size_t)f.P * 2 * D) * 4);
  n.cond = take((256 + 2 * D + (size_t)f.P * D) * 4);
  if (f.net_kind == PG_NET_JOINT || f.net_kind == PG_NET_MMDIT) n.ctx_h = take((size_t)f.P * f.Lc * D * 4);
  if (f.net_kind == PG_NET_CROSS) {
    n.ckv = take((size_t)f.blocks * f.P * f.Lc * D * 2);
    n.ckvt = take((size_t)f.blocks * f.P * D * Lcpad * 2);
  }
  n.total = off;
  return PG_OK;
}

namespace {
struct Net {
  pg_ctx* c;
  hipStream_t s;
  char* base;
  const uint16_t* wts;
  template <class T> T* at(size_t off) const { return reinterpret_cast<T*>(base + off); }
  const uint16_t* w(int id, int block = 0) const {
    return wts + c->top[id].offset + (id >= PG_W_MOD_W ? c->block_stride * block : 0);
  }
  int ld(int id) const { return c->top[id].ld; }
};
}  // namespace

// Step-independent work: projected context rows (joint) or per-block context keys / values (cross).
pg_status net_prepare(pg_ctx* c, const uint16_t* weights, hipStream_t s) {
  const pg_config& f = c->cfg;
  Net n{c, s, (char*)c->buf.workspace + c->ws_net, weights};
  const int D = f.D;
  if (f.net_kind == PG_NET_JOINT || f.net_kind == PG_NET_MMDIT) {
    GemmArgs g{};
    g.A = c->buf.ctx; g.lda = f.Dc; g.W = n.w(PG_W_CTX_W); g.ldw = n.ld(PG_W_CTX_W); g.bias = n.w(PG_W_CTX_B);
    g.M = f.P * f.Lc; g.N = D; g.K = f.Dc;
    g.outf = n.at<float>(c->net.ctx_h); g.ldo = D;
    PG_TRY(launch_gemm(g, EPI_F32, s));
  } else if (f.net_kind == PG_NET_CROSS) {
    const int Lcpad = (f.Lc + 63) / 64 * 64;
    for (int b = 0; b < f.blocks; ++b) {
      GemmArgs g{};
      g.A = c->buf.ctx; g.lda = f.Dc; g.W = n.w(PG_W_CKV_W, b); g.ldw = n.ld(PG_W_CKV_W); g.bias = n.w(PG_W_CKV_B, b);
      g.M = f.P * f.Lc; g.N = 2 * D; g.K = f.Dc;
      g.outb = n.at<uint16_t>(c->net.ckv) + (size_t)b * f.P * f.Lc * D; g.ldob = D;
      g.vt = n.at<uint16_t>(c->net.ckvt) + (size_t)b * f.P * D * Lcpad; g.v_start = D; g.Lpad = Lcpad; g.L = f.Lc;
      PG_TRY(launch_gemm(g, EPI_QKV, s));
    }
  }
  return PG_OK;
}

pg_status net_forward(pg_ctx* c, int step, const float* x_in, const uint16_t* weights, hipStream_t s) {
  const pg_config& f = c->cfg;
  Net n{c, s, (char*)c->buf.workspace + c->ws_net, weights};
  const NetPlan& pl = c->net;
  const int D = f.D, M = c->M, L = c->L, Li = c->Li, P = f.P, hd = D / f.heads;
  const int R = M * L, Ri = M * Li;
  const int Lpad = (L + 63) / 64 * 64, Lcpad = (f.Lc + 63) / 64 * 64, Kp = (4 * f.C + 63) / 64 * 64;
  if (M == 0) return PG_OK;
  float* h = n.at<float>(pl.h);
  uint16_t* act = n.at<uint16_t>(pl.act);
  uint16_t* qk = n.at<uint16_t>(pl.qkv);
  uint16_t* vt = n.at<uint16_t>(pl.vt);
  uint16_t* att = n.at<uint16_t>(pl.att);
  uint16_t* hid = n.at<uint16_t>(pl.hid);
  uint16_t* tok = n.at<uint16_t>(pl.tok);
  float* mod = n.at<float>(pl.mod);
  float* fmod = mod + (size_t)P * f.blocks * 6 * D;
  float* cmod = fmod + (size_t)P * 2 * D;           // dual-stream variant: the context stream's modulation vectors
  const bool dual = f.net_kind == PG_NET_MMDIT;
  const int Rc = M * f.Lc;                          // context rows (dual-stream planes)
  float* emb = n.at<float>(pl.cond);
  float* t1 = emb + 256;
  float* c0 = t1 + D;
  float* sc = c0 + D;
  const int32_t* group_of = c->buf.group_of;
  const int64_t mod_ld = (int64_t)f.blocks * 6 * D;
  const float scale_log2 = (float)(1.4426950408889634 / std::sqrt((double)hd));

  // ---- conditioning: c = MLP(sincos(t)) + y, modulation vectors of every block ----
  timestep_embedding_kernel<<<dim3(1), dim3(128), 0, s>>>(c->tin[step], emb);
  PG_LAUNCH_CHECK("timestep_embedding_kernel");
  gemv_bf16_kernel<true><<<dim3((D + 3) / 4, 1), dim3(256), 0, s>>>(n.w(PG_W_T_W1), n.ld(PG_W_T_W1), 0, n.w(PG_W_T_B1),
                                                                    0, emb, 256, t1, D, 0, 1, D, 256);
  PG_LAUNCH_CHECK("gemv t1");
  gemv_bf16_kernel<false><<<dim3((D + 3) / 4, 1), dim3(256), 0, s>>>(n.w(PG_W_T_W2), n.ld(PG_W_T_W2), 0,
                                                                     n.w(PG_W_T_B2), 0, t1, D, c0, D, 0, 1, D, D);
  PG_LAUNCH_CHECK("gemv t2");
  cond_silu_kernel<<<dim3((P * D + 255) / 256), dim3(256), 0, s>>>(c0, c->buf.y, sc, P, D);
  PG_LAUNCH_CHECK("cond_silu_kernel");
  gemv_bf16_kernel<false><<<dim3((6 * D + 3) / 4, f.blocks), dim3(256), 0, s>>>(
      n.w(PG_W_MOD_W), n.ld(PG_W_MOD_W), c->block_stride, n.w(PG_W_MOD_B), c->block_stride, sc, D, mod, mod_ld, 6 * D,
      P, 6 * D, D);
  PG_LAUNCH_CHECK("gemv mod");
  if (dual) {
    gemv_bf16_kernel<false><<<dim3((6 * D + 3) / 4, f.blocks), dim3(256), 0, s>>>(
        n.w(PG_W_C_MOD_W), n.ld(PG_W_C_MOD_W), c->block_stride, n.w(PG_W_C_MOD_B), c->block_stride, sc, D, cmod, mod_ld,
        6 * D, P, 6 * D, D);
    PG_LAUNCH_CHECK("gemv cmod");
  }
  gemv_bf16_kernel<false><<<dim3((2 * D + 3) / 4, 1), dim3(256), 0, s>>>(n.w(PG_W_FMOD_W), n.ld(PG_W_FMOD_W), 0,
                                                                         n.w(PG_W_FMOD_B), 0, sc, D, fmod, 2 * D, 0, P,
                                                                         2 * D, D);
  PG_LAUNCH_CHECK("gemv fmod");

  // ---- patch embedding (+ position table), context rows ----
  {
    const int64_t total = (int64_t)M * (Kp / 4) * Li;
    patchify_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(x_in, tok, M, f.C, f.H,
                                                                                f.W, Kp);
    PG_LAUNCH_CHECK("patchify_kernel");
    GemmArgs g{};
    g.A = tok; g.lda = Kp; g.W = n.w(PG_W_PE_W); g.ldw = n.ld(PG_W_PE_W); g.bias = n.w(PG_W_PE_B);
    g.M = Ri; g.N = D; g.K = Kp; g.k_algo = 4 * f.C; g.outf = h; g.ldo = D; g.L = dual ? Li : L; g.Li = Li; g.pos = n.w(PG_W_POS);
    PG_TRY(launch_gemm(g, EPI_EMBED, s));
  }
  if (f.net_kind == PG_NET_JOINT || dual) {
    const int64_t total = (int64_t)M * f.Lc * (D / 4);
    scatter_context_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(
        n.at<float>(pl.ctx_h), h, group_of, M, dual ? (int64_t)Ri : (int64_t)Li, dual ? f.Lc : L, f.Lc, D / 4);
    PG_LAUNCH_CHECK("scatter_context_kernel");
  }

  // out[m * L_out + t, :] = bf16(LN(hin[m * L_in + t, :]) * (1 + scale) + shift), t < L_out
  auto ln = [&](const float* hin, uint16_t* out, const float* shift, const float* scale, int64_t ld, int rows_out,
                int L_in, int L_out) -> pg_status {
    if (rows_out <= 0) return PG_OK;
    const dim3 grid((rows_out + 3) / 4), block(256);
    if (D == 768) ln_modulate_kernel<3><<<grid, block, 0, s>>>(hin, out, shift, scale, ld, group_of, rows_out, L_in, L_out, D);
    else if (D == 1536) ln_modulate_kernel<6><<<grid, block, 0, s>>>(hin, out, shift, scale, ld, group_of, rows_out, L_in, L_out, D);
    else if (D == 1024) ln_modulate_kernel<4><<<grid, block, 0, s>>>(hin, out, shift, scale, ld, group_of, rows_out, L_in, L_out, D);
    else if (D == 256) ln_modulate_kernel<1><<<grid, block, 0, s>>>(hin, out, shift, scale, ld, group_of, rows_out, L_in, L_out, D);
    else ln_modulate_kernel<0><<<grid, block, 0, s>>>(hin, out, shift, scale, ld, group_of, rows_out, L_in, L_out, D);
    PG_LAUNCH_CHECK("ln_modulate_kernel");
    return PG_OK;
  };
  auto layer_norm = [&](const float* shift, const float* scale, int64_t ld, int rows_out, int L_out) -> pg_status {
    return ln(h, act, shift, scale, ld, rows_out, dual ? L_out : L, L_out);
  };

  // ---- dual-stream blocks: two planes (image rows, context rows), joint q | k and V^T ----
  if (dual) {
    float* hs[2] = {h, h + (size_t)Ri * D};
    uint16_t* acts[2] = {act, act + (size_t)Ri * D};
    uint16_t* atts[2] = {att, att + (size_t)Ri * D};
    uint16_t* hids[2] = {hid, hid + (size_t)Ri * 4 * D};
    const int rows[2] = {Ri, Rc}, Ls[2] = {Li, f.Lc}, toff[2] = {0, Li};
    const int W_QN[2] = {PG_W_QN_G, PG_W_C_QN_G}, W_KN[2] = {PG_W_KN_G, PG_W_C_KN_G};
    const int W_QKV[2] = {PG_W_QKV_W, PG_W_C_QKV_W}, B_QKV[2] = {PG_W_QKV_B, PG_W_C_QKV_B};
    const int W_O[2] = {PG_W_O_W, PG_W_C_O_W}, B_O[2] = {PG_W_O_B, PG_W_C_O_B};
    const int W_FC1[2] = {PG_W_FC1_W, PG_W_C_FC1_W}, B_FC1[2] = {PG_W_FC1_B, PG_W_C_FC1_B};
    const int W_FC2[2] = {PG_W_FC2_W, PG_W_C_FC2_W}, B_FC2[2] = {PG_W_FC2_B, PG_W_C_FC2_B};
    for (int b = 0; b < f.blocks; ++b) {
      const float* mbs[2] = {mod + (size_t)b * 6 * D, cmod + (size_t)b * 6 * D};
      for (int st = 0; st < 2; ++st) {
        PG_TRY(ln(hs[st], acts[st], mbs[st], mbs[st] + D, mod_ld, rows[st], Ls[st], Ls[st]));
        GemmArgs g{};
        g.A = acts[st]; g.lda = D; g.W = n.w(W_QKV[st], b); g.ldw = n.ld(W_QKV[st]); g.bias = n.w(B_QKV[st], b);
        g.M = rows[st]; g.N = 3 * D; g.K = D; g.outb = qk; g.ldob = 2 * D; g.vt = vt; g.v_start = 2 * D; g.Lpad = Lpad;
        g.L = Ls[st]; g.Lout = L; g.tok_off = toff[st];
        // queries and keys leave the projection RMS-normalised per head, queries also in the softmax's log2 units
        g.norm_hd = hd; g.qn_g = n.w(W_QN[st], b); g.kn_g = n.w(W_KN[st], b);
        g.out_scale = scale_log2; g.scale_cols = D;
        PG_TRY(launch_gemm(g, EPI_QKV, s));
      }
      AttnArgs a{};
      a.q = qk; a.ldq = 2 * D; a.k = qk + D; a.ldk = 2 * D; a.k_bstride = (int64_t)L * 2 * D;
      a.vt = vt; a.vt_bstride = (int64_t)D * Lpad; a.Lkpad = Lpad; a.out = atts[0]; a.ldo = D;
      a.split = Li; a.out2 = atts[1];
      a.B = M; a.Lq = L; a.Lk = L; a.heads = f.heads; a.scale_log2 = scale_log2; a.q_prescaled = 1;
      PG_TRY(launch_attention(a, hd, s));
      for (int st = 0; st < 2; ++st) {
        GemmArgs o{};
        o.A = atts[st]; o.lda = D; o.W = n.w(W_O[st], b); o.ldw = n.ld(W_O[st]); o.bias = n.w(B_O[st], b);
        o.M = rows[st]; o.N = D; o.K = D; o.outf = hs[st]; o.ldo = D; o.L = Ls[st]; o.gate = mbs[st] + 2 * D;
        o.gate_ld = mod_ld; o.group_of = group_of;
        PG_TRY(launch_gemm(o, EPI_RESID, s));
        PG_TRY(ln(hs[st], acts[st], mbs[st] + 3 * D, mbs[st] + 4 * D, mod_ld, rows[st], Ls[st], Ls[st]));
        GemmArgs g{};
        g.A = acts[st]; g.lda = D; g.W = n.w(W_FC1[st], b); g.ldw = n.ld(W_FC1[st]); g.bias = n.w(B_FC1[st], b);
        g.M = rows[st]; g.N = 4 * D; g.K = D; g.outb = hids[st]; g.ldob = 4 * D;
        PG_TRY(launch_gemm(g, EPI_GELU, s));
        GemmArgs o2{};
        o2.A = hids[st]; o2.lda = 4 * D; o2.W = n.w(W_FC2[st], b); o2.ldw = n.ld(W_FC2[st]); o2.bias = n.w(B_FC2[st], b);
        o2.M = rows[st]; o2.N = D; o2.K = 4 * D; o2.outf = hs[st]; o2.ldo = D; o2.L = Ls[st]; o2.gate = mbs[st] + 5 * D;
        o2.gate_ld = mod_ld; o2.group_of = group_of;
        PG_TRY(launch_gemm(o2, EPI_RESID, s));
      }
    }
  }

  for (int b = 0; b < (dual ? 0 : f.blocks); ++b) {
    const float* mb = mod + (size_t)b * 6 * D;     // shift1, scale1, gate1, shift2, scale2, gate2
    // attention sub-block
    PG_TRY(layer_norm(mb, mb + D, mod_ld, R, L));
    {
      GemmArgs g{};
      g.A = act; g.lda = D; g.W = n.w(PG_W_QKV_W, b); g.ldw = n.ld(PG_W_QKV_W); g.bias = n.w(PG_W_QKV_B, b);
      g.M = R; g.N = 3 * D; g.K = D; g.outb = qk; g.ldob = 2 * D; g.vt = vt; g.v_start = 2 * D; g.Lpad = Lpad; g.L = L;
      g.out_scale = scale_log2; g.scale_cols = D;   // queries leave the projection already in the softmax's log2 units
      PG_TRY(launch_gemm(g, EPI_QKV, s));
      AttnArgs a{};
      a.q = qk; a.ldq = 2 * D; a.k = qk + D; a.ldk = 2 * D; a.k_bstride = (int64_t)L * 2 * D;
      a.vt = vt; a.vt_bstride = (int64_t)D * Lpad; a.Lkpad = Lpad; a.out = att; a.ldo = D;
      a.B = M; a.Lq = L; a.Lk = L; a.heads = f.heads; a.scale_log2 = scale_log2; a.q_prescaled = 1;
      PG_TRY(launch_attention(a, hd, s));
      GemmArgs o{};
      o.A = att; o.lda = D; o.W = n.w(PG_W_O_W, b); o.ldw = n.ld(PG_W_O_W); o.bias = n.w(PG_W_O_B, b);
      o.M = R; o.N = D; o.K = D; o.outf = h; o.ldo = D; o.L = L; o.gate = mb + 2 * D; o.gate_ld = mod_ld;
      o.group_of = group_of;
      PG_TRY(launch_gemm(o, EPI_RESID, s));
    }
    // cross-attention sub-block over the prompt's context tokens
    if (f.net_kind == PG_NET_CROSS) {
      PG_TRY(layer_norm(nullptr, nullptr, 0, R, L));
      GemmArgs g{};
      g.A = act; g.lda = D; g.W = n.w(PG_W_CQ_W, b); g.ldw = n.ld(PG_W_CQ_W); g.bias = n.w(PG_W_CQ_B, b);
      g.M = R; g.N = D; g.K = D; g.outb = qk; g.ldob = D;
      g.out_scale = scale_log2; g.scale_cols = D;
      PG_TRY(launch_gemm(g, EPI_BF16, s));
      AttnArgs a{};
      a.q = qk; a.ldq = D;
      a.k = n.at<uint16_t>(pl.ckv) + (size_t)b * P * f.Lc * D; a.ldk = D; a.k_bstride = (int64_t)f.Lc * D;
      a.vt = n.at<uint16_t>(pl.ckvt) + (size_t)b * P * D * Lcpad; a.vt_bstride = (int64_t)D * Lcpad; a.Lkpad = Lcpad;
      a.out = att; a.ldo = D; a.kv_map = group_of;
      a.B = M; a.Lq = L; a.Lk = f.Lc; a.heads = f.heads; a.scale_log2 = scale_log2; a.q_prescaled = 1;
      PG_TRY(launch_attention(a, hd, s));
      GemmArgs o{};
      o.A = att; o.lda = D; o.W = n.w(PG_W_CO_W, b); o.ldw = n.ld(PG_W_CO_W); o.bias = n.w(PG_W_CO_B, b);
      o.M = R; o.N = D; o.K = D; o.outf = h; o.ldo = D; o.L = L; o.gate = nullptr; o.group_of = group_of;
      PG_TRY(launch_gemm(o, EPI_RESID, s));
    }
    // MLP sub-block
    PG_TRY(layer_norm(mb + 3 * D, mb + 4 * D, mod_ld, R, L));
    {
      GemmArgs g{};
      g.A = act; g.lda = D; g.W = n.w(PG_W_FC1_W, b); g.ldw = n.ld(PG_W_FC1_W); g.bias = n.w(PG_W_FC1_B, b);
      g.M = R; g.N = 4 * D; g.K = D; g.outb = hid; g.ldob = 4 * D;
      PG_TRY(launch_gemm(g, EPI_GELU, s));
      GemmArgs o{};
      o.A = hid; o.lda = 4 * D; o.W = n.w(PG_W_FC2_W, b); o.ldw = n.ld(PG_W_FC2_W); o.bias = n.w(PG_W_FC2_B, b);
      o.M = R; o.N = D; o.K = 4 * D; o.outf = h; o.ldo = D; o.L = L; o.gate = mb + 5 * D; o.gate_ld = mod_ld;
      o.group_of = group_of;
      PG_TRY(launch_gemm(o, EPI_RESID, s));
    }
  }

  // ---- final layer on the image tokens, written straight into the latent layout ----
  PG_TRY(layer_norm(fmod, fmod + D, 2 * D, Ri, Li));
  GemmArgs g{};
  g.A = act; g.lda = D; g.W = n.w(PG_W_F_W); g.ldw = n.ld(PG_W_F_W); g.bias = n.w(PG_W_F_B);
  g.M = Ri; g.N = 4 * f.C; g.K = D; g.outf = c->buf.u; g.Li = Li; g.Wp = f.W / 2; g.HW = f.H * f.W; g.Wimg = f.W;
  return launch_gemm(g, EPI_UNPATCH, s);
}

}  // namespace pg
