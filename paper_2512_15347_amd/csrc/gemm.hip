// bf16 MFMA GEMM for gfx950: C[M, N] = A[M, K] W[N, K]^T with a fused epilogue.  This is where the
// network evaluation of every denoising step spends its time (the noise-prediction row of the paper's
// cost table, Sec. 6.2).  Built around the 32x32x16 bf16 MFMA:
//   both operands are K-contiguous; 16-byte chunks go from global memory straight into LDS (no register
//   staging), two LDS stages of BK = 64 columns, one barrier per K step; the requests for tile kt+2 are
//   interleaved with the MFMAs that follow the barrier instead of being issued in a burst; operand
//   fragments are double buffered in registers and read one MFMA slab ahead, also across the barrier;
//   chunk positions are XOR-swizzled so that the 16-byte operand reads are bank-conflict free while the
//   direct loads still write 1 KB contiguous per instruction;
//   the epilogue goes through an LDS transpose so that every lane stores 16 contiguous bytes, with the
//   non-temporal hint; workgroup ids are spread so that the tiles resident on one XCD (one L2) form a
//   compact block of the output and share operand panels.
// Several tile shapes are instantiated (workgroup tile BM x BN x BK, WM x WN wavefronts); the launcher
// picks one from the number of output tiles relative to the 256 compute units.
#include <cmath>
#include <cstdlib>
#include "gemm.hpp"

namespace pg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));

constexpr int GROUP_M = 8;                         // tile rows per raster band
constexpr int XCDS = 8;

// byte offset of 16-byte chunk `chunk` of tile row `row` inside an operand tile with CH chunks per row
template <int CH>
__device__ __forceinline__ int swz(int row) {
  return CH == 8 ? ((row ^ (row >> 3)) & 7) : (((row >> 1) ^ (row >> 3)) & 3);
}
template <int CH>
__device__ __forceinline__ int lds_off(int row, int chunk) { return (row * CH + (chunk ^ swz<CH>(row))) * 16; }

// 16 bytes per lane straight from global memory into LDS (no register staging): the wave writes the
// 1 KB starting at LDS address `lds_addr` (wave-uniform), lane l at +16 l.  Issued through inline
// assembly so that the operand reads of the other LDS stage are not made to wait for it; completion
// is awaited explicitly (wait_dma) before the barrier that publishes the stage.  The statement overwrites m0
// without naming it as clobbered: m0 is a reserved register for this compiler (it refuses it in a clobber list
// and writes m0 itself directly before each instruction of its own that reads it), so no value of the
// surrounding code lives in m0 across the statement.
__device__ __forceinline__ void dma16(const uint16_t* g, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory");
}
// wait until at most N of this wave's loads are still in flight (loads complete in order)
template <int N>
__device__ __forceinline__ void wait_dma() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Outputs are written, and the residual stream is read, once per launch: they go through the caches
// with the non-temporal hint so that the operand panels shared by the tiles of an XCD stay resident.
typedef float f32x4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_stream(float* p, const float4 v) {
  __builtin_nontemporal_store(f32x4v{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4v*>(p));
}
__device__ __forceinline__ void store_stream(uint16_t* p, const uint2 v) {
  __builtin_nontemporal_store(u32x2v{v.x, v.y}, reinterpret_cast<u32x2v*>(p));
}
__device__ __forceinline__ float4 load_stream(const float* p) {
  const f32x4v v = __builtin_nontemporal_load(reinterpret_cast<const f32x4v*>(p));
  return float4{v[0], v[1], v[2], v[3]};
}

// gelu_tanh(x) = x/2 (1 + tanh(y)) = x / (1 + exp(-2y)),  y = sqrt(2/pi) (x + 0.044715 x^3);
// the exponent is taken in base 2: -2 y log2(e) = x (K1 + K3 x^2)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ float gelu_tanh(float x) {
  constexpr float K1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
  constexpr float K3 = K1 * 0.044715f;
  const float z = x * __builtin_fmaf(x * x, K3, K1);
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z));
}

__device__ __forceinline__ uint2 pack_bf16x4(float4 v) {
  uint2 r;
  r.x = (uint32_t)f32_to_bf16_bits(v.x) | ((uint32_t)f32_to_bf16_bits(v.y) << 16);
  r.y = (uint32_t)f32_to_bf16_bits(v.z) | ((uint32_t)f32_to_bf16_bits(v.w) << 16);
  return r;
}

// f(tag<I>), f(tag<I + 2>), ... while I < N and f returns true
template <int I> struct int_tag { static constexpr int value = I; };
template <int I, int N, class F>
__device__ __forceinline__ void static_for_by2(F&& f) {
  if constexpr (I < N) {
    if (f(int_tag<I>{})) static_for_by2<I + 2, N>(f);
  }
}

// orders this wave's LDS accesses around a hand-over between its lanes (LDS serves one wave's accesses in issue order;
// this keeps the compiler from moving them across the hand-over)
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

template <int EPI, int BM, int BN, int BK, int WM, int WN, int MINW, int NST>
__global__ __launch_bounds__(64 * WM * WN, MINW) void gemm_kernel(const GemmArgs a) {
  static_assert(NST >= 2, "LDS stages filled by direct loads");
  constexpr int CH = BK / 8;                       // 16-byte chunks per tile row
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // 32x32 MFMA tiles per wave
  constexpr int A_BYTES = BM * BK * 2, W_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + W_BYTES;
  extern __shared__ __align__(16) unsigned char smem[];
  const uint16_t* PA = a.A; const int64_t LDA = a.lda;
  const uint16_t* PW = a.W; const int64_t LDW = a.ldw;
  const uint16_t* PB = a.bias;
  const int MM = a.M, NN = a.N;
  const int per_xcd = gridDim.x / XCDS;
  const int b = a.raster ? (blockIdx.x % XCDS) * per_xcd + blockIdx.x / XCDS : blockIdx.x;
  // ---- which output tile: XCD-aware, banded raster ----
  const int tiles_m = (MM + BM - 1) / BM, tiles_n = (NN + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  if (b >= total) return;
  const int band = a.group_m * tiles_n;
  const int first_m = (b / band) * a.group_m;
  const int gsz = min(tiles_m - first_m, a.group_m);
  const int tm = first_m + (b % band) % gsz;
  const int tn = (b % band) / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, half = lane >> 5;

  int a_row[TM], w_row[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) a_row[i] = wm * (BM / WM) + i * 32 + l32;
#pragma unroll
  for (int j = 0; j < TN; ++j) w_row[j] = wn * (BN / WN) + j * 32 + l32;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = a.K / BK;
  {
    // ---- global -> LDS directly: every wave owns N_REG / WAVES regions of 1 KB (64 / CH tile rows) ----
    constexpr int WAVES = WM * WN, RPR = 64 / CH;
    constexpr int A_REG = BM / RPR, N_REG = (BM + BN) / RPR, PER_WAVE = (N_REG + WAVES - 1) / WAVES;
    static_assert(NST == 2 || N_REG % WAVES == 0, "deeper pipelines count loads per wave: regions must divide evenly");
    const uint16_t* g_ptr[PER_WAVE];
    uint32_t g_lds[PER_WAVE];
    const uint32_t lds_base = (uint32_t)(uintptr_t)smem;
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
      const int g = min(wave + i * WAVES, N_REG - 1);  // wave-uniform region id (the last wave may own one fewer)
      const bool is_w = g >= A_REG;
      const int rg = is_w ? g - A_REG : g;
      const int row = rg * RPR + lane / CH;
      const int ch = (lane % CH) ^ swz<CH>(row);
      g_ptr[i] = is_w ? PW + (int64_t)min(n0 + row, NN - 1) * LDW + ch * 8
                      : PA + (int64_t)min(m0 + row, MM - 1) * LDA + ch * 8;
      g_lds[i] = __builtin_amdgcn_readfirstlane(lds_base + (is_w ? A_BYTES : 0) + rg * 1024);
    }
    // request region i of K tile `kt` (nothing past the last tile)
    auto request = [&](int i, int kt) {
      if (kt < nk && wave + i * WAVES < N_REG) dma16(g_ptr[i] + kt * BK, g_lds[i] + (kt % NST) * STAGE_BYTES);
    };
    // NST stages of BK columns; tile kt lives in stage kt % NST.  Per K step: SLABS MFMA slabs.  Operand
    // fragments are double buffered in registers and read one slab ahead, also across the K-step
    // boundary: at the last slab of tile kt every read of its stage has been issued, so the barrier that
    // publishes tile kt+1 (and frees stage kt % NST) is passed before that slab's MFMAs, and the first
    // slab of tile kt+1 is read while they run.  The requests for tile kt+NST are not issued in a burst
    // (a wave's request waits for the texture path, which takes 1 KB every ~20 cycles, and the MFMAs
    // queued behind it would wait too): they are spread between the MFMAs of the SPREAD slabs that
    // follow the barrier, one request every few MFMAs.
    constexpr int SLABS = BK / 16, MF = TM * TN;
    static_assert(SLABS % 2 == 0, "fragment buffers alternate per slab");
    constexpr int SPREAD = NST == 2 ? 2 : SLABS;                     // slabs over which one tile's requests go
    constexpr int RPS = (PER_WAVE + SPREAD - 1) / SPREAD;            // requests per slab
    constexpr int EVERY = MF / RPS > 0 ? MF / RPS : 1;               // one request after every EVERY-th MFMA
    static_assert(RPS <= MF, "more requests than MFMAs in a slab");
    constexpr int LAG = (NST - 2) * PER_WAVE;                        // requests that may stay in flight at the barrier
    bf16x8 af[2][TM], wf[2][TN];
    auto fetch = [&](int stage, int ks, int buf) {
      const unsigned char* sA = smem + stage * STAGE_BYTES;
      const unsigned char* sW = sA + A_BYTES;
#pragma unroll
      for (int i = 0; i < TM; ++i) af[buf][i] = *reinterpret_cast<const bf16x8*>(sA + lds_off<CH>(a_row[i], 2 * ks + half));
#pragma unroll
      for (int j = 0; j < TN; ++j) wf[buf][j] = *reinterpret_cast<const bf16x8*>(sW + lds_off<CH>(w_row[j], 2 * ks + half));
    };
    // prologue: tiles 0 .. NST-2 are requested, tile 0 awaited
#pragma unroll
    for (int t = 0; t < NST - 1; ++t)
#pragma unroll
      for (int i = 0; i < PER_WAVE; ++i) request(i, t);
    if (nk >= NST - 1) wait_dma<LAG>(); else wait_dma<0>();
    __syncthreads();
#pragma unroll
    for (int i = 0; i < RPS; ++i) request(i, NST - 1);               // the share that position 0 would have carried
    fetch(0, 0, 0);
    // slab position p after a barrier: p = 0 is the last slab of the K step that passed it, p >= 1 are
    // slabs p-1 of the next K step; position p carries requests [p RPS, (p+1) RPS) of the tile freed there
    for (int kt = 0; kt < nk; ++kt) {
      const int cur = kt % NST;
#pragma unroll
      for (int ks = 0; ks < SLABS; ++ks) {
        if (ks + 1 < SLABS) {
          fetch(cur, ks + 1, (ks + 1) & 1);
        } else if (kt + 1 < nk) {
          // tiles up to kt+NST-1 have been requested (fewer near the end: then wait for all)
          if (kt + NST - 1 < nk) wait_dma<LAG>(); else wait_dma<0>();
          __syncthreads();                         // tile kt+1 is visible; stage `cur` is free
          fetch((kt + 1) % NST, 0, 0);
        }
        const int pos = ks + 1 < SLABS ? ks + 1 : 0;                 // compile-time after unrolling
        const int tile = ks + 1 < SLABS ? kt - 1 + NST : kt + NST;   // the tile whose stage was freed last
        __builtin_amdgcn_sched_barrier(0);
        int q = 0;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], wf[ks & 1][j], acc[i][j], 0, 0, 0);
            if (pos < SPREAD && q % EVERY == 0 && q / EVERY < RPS && pos * RPS + q / EVERY < PER_WAVE) {
              __builtin_amdgcn_sched_barrier(0);
              request(pos * RPS + q / EVERY, tile);
              __builtin_amdgcn_sched_barrier(0);
            }
            ++q;
          }
      }
    }
  }

  // ---- epilogue: in each 32x32 accumulator tile a lane holds ONE column (l32) and rows 8q + 4*half + t ----
  if constexpr (EPI != EPI_UNPATCH) {
    // ---- row-major epilogues: transpose each 32-row slab of the wave tile through LDS so that a lane
    // owns 4 consecutive columns of a row and every global access is 16 bytes wide (8 for bf16) ----
    static_assert(TN == 1 || TN == 2, "the staged epilogue handles 32 or 64 columns per wave");
    constexpr int LPR = TN * 8, RPI = 64 / LPR, NP = 32 / RPI;   // lanes per row, rows per access, accesses per slab
    constexpr int EST = TN * 32 + 8;                 // staging row stride in floats (half-waves hit disjoint banks)
    __syncthreads();                                 // every wave has finished reading the last stage
    float* stg = reinterpret_cast<float*>(smem) + wave * (32 * EST);
    const int c4 = (lane % LPR) * 4, rsub = lane / LPR;
    const int n = n0 + wn * (BN / WN) + c4;
    // columns written row-major: all of them, except the value channels of EPI_QKV
    const int n_rm = EPI == EPI_QKV ? a.v_start : NN;
    if (EPI == EPI_QKV) {
      // ---- value channels, stored TRANSPOSED: V^T[traj][channel][token].  In an accumulator tile a lane already
      // holds 4 consecutive tokens of ONE channel, so they are packed to bf16 and staged channel-major (8 bytes per
      // LDS write), two 32-token slabs at a time; then a lane owns 4 consecutive tokens of a channel row and 16
      // lanes write 64 consecutive tokens (128 bytes) of it.  A 32-column accumulator tile is either all value
      // channels or none (v_start is a multiple of 32). ----
      constexpr int VP = 72;                         // staging pitch in bf16: 64 tokens + 8 (rows stay 16-byte aligned)
      static_assert(TN * 32 * VP * 2 <= 32 * EST * 4, "the transposed staging fits the wave's staging area");
      uint16_t* stg16 = reinterpret_cast<uint16_t*>(stg);
      const int col_w = n0 + wn * (BN / WN);         // first column of this wave
      const int Dv = NN - n_rm;
      bool is_v[TN];
      float vb[TN];
      bool any_v = false;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = col_w + j * 32;
        is_v[j] = col >= n_rm && col < NN;           // wave-uniform
        any_v = any_v || is_v[j];
        vb[j] = (is_v[j] && PB) ? bf16_to_f32(PB[col + l32]) : 0.f;
      }
      if (any_v) {
        static_for_by2<0, TM>([&](auto tag) {
          constexpr int i0 = decltype(tag)::value;
          constexpr int nsl = i0 + 1 < TM ? 2 : 1;   // slabs staged together
          const int row0 = m0 + wm * (BM / WM) + i0 * 32;        // first token row of the group, wave-uniform
          if (row0 >= MM) return false;
#pragma unroll
          for (int ii = 0; ii < 2; ++ii) {
            if (ii >= nsl) break;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              if (!is_v[j]) continue;
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const float4 v = {acc[i0 + ii][j][4 * q] + vb[j], acc[i0 + ii][j][4 * q + 1] + vb[j],
                                  acc[i0 + ii][j][4 * q + 2] + vb[j], acc[i0 + ii][j][4 * q + 3] + vb[j]};
                *reinterpret_cast<uint2*>(stg16 + (j * 32 + l32) * VP + ii * 32 + 8 * q + 4 * half) = pack_bf16x4(v);
              }
            }
          }
          wave_lds_sync();
          constexpr int lpr = 8 * nsl, rpa = 64 / lpr;   // lanes per channel row, channel rows per access
          const int t4 = (lane % lpr) * 4, csub = lane / lpr;
          const int r = row0 + t4;                   // the lane's first token row
          const int traj0 = r / a.L, tok0 = r - traj0 * a.L;
          const bool whole = r + 3 < MM && tok0 + 3 < a.L && ((tok0 + a.tok_off) & 1) == 0;
#pragma unroll
          for (int p = 0; p < TN * 32 / rpa; ++p) {
            const int cl = p * rpa + csub;           // channel row inside the wave's columns
            if (!is_v[cl / 32] || r >= MM) continue;
            const uint2 pk = *reinterpret_cast<const uint2*>(stg16 + cl * VP + t4);
            const int ch = col_w + cl - n_rm;
            uint16_t* dst = a.vt + ((int64_t)traj0 * Dv + ch) * a.Lpad + a.tok_off + tok0;
            if (whole) {
              if (((uintptr_t)dst & 7) == 0) {
                store_stream(dst, pk);
              } else {
                reinterpret_cast<uint32_t*>(dst)[0] = pk.x;
                reinterpret_cast<uint32_t*>(dst)[1] = pk.y;
              }
            } else {
              const uint16_t e[4] = {(uint16_t)pk.x, (uint16_t)(pk.x >> 16), (uint16_t)pk.y, (uint16_t)(pk.y >> 16)};
              int traj = traj0, tok = tok0;
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                if (r + k < MM) {
                  if (tok >= a.L) { tok -= a.L; ++traj; }
                  a.vt[((int64_t)traj * Dv + ch) * a.Lpad + a.tok_off + tok] = e[k];
                  ++tok;
                }
              }
            }
          }
          wave_lds_sync();
          return true;
        });
      }
      if (col_w >= n_rm) return;                     // nothing row-major in this wave's columns
    }
    const bool n_ok = n < n_rm;                      // N is a multiple of 4
    const float col_scale = n < a.scale_cols ? a.out_scale : 1.f;   // e.g. queries pre-multiplied by the softmax scale
    float4 ng4 = {1.f, 1.f, 1.f, 1.f};               // norm scales of this lane's 4 columns
    if (EPI == EPI_QKV && a.norm_hd > 0 && n_ok) {
      const uint2 raw = *reinterpret_cast<const uint2*>((n < a.scale_cols ? a.qn_g : a.kn_g) + n % a.norm_hd);
      ng4 = {bf16_to_f32((uint16_t)raw.x), bf16_to_f32((uint16_t)(raw.x >> 16)), bf16_to_f32((uint16_t)raw.y),
             bf16_to_f32((uint16_t)(raw.y >> 16))};
    }
    float4 b4 = {0.f, 0.f, 0.f, 0.f};
    if (PB && n_ok) {
      const uint2 raw = *reinterpret_cast<const uint2*>(PB + n);
      b4 = {bf16_to_f32((uint16_t)raw.x), bf16_to_f32((uint16_t)(raw.x >> 16)), bf16_to_f32((uint16_t)raw.y),
            bf16_to_f32((uint16_t)(raw.y >> 16))};
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int slab0 = m0 + wm * (BM / WM) + i * 32;            // wave-uniform
      if (slab0 >= a.M) break;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int t = 0; t < 4; ++t) stg[(8 * q + 4 * half + t) * EST + j * 32 + l32] = acc[i][j][4 * q + t];
      float4 v[NP];
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        v[p] = *reinterpret_cast<const float4*>(stg + (RPI * p + rsub) * EST + c4);
        v[p].x += b4.x; v[p].y += b4.y; v[p].z += b4.z; v[p].w += b4.w;
        if (EPI == EPI_QKV && a.norm_hd > 0) {
          // RMS norm over the head chunk this lane's 4 columns belong to (norm_hd / 4 adjacent lanes of the row)
          float ss = (v[p].x * v[p].x + v[p].y * v[p].y) + (v[p].z * v[p].z + v[p].w * v[p].w);
          for (int o = 1; o < a.norm_hd / 4; o <<= 1) ss += __shfl_xor(ss, o, 64);
          const float rstd = rsqrtf(ss / (float)a.norm_hd + 1e-6f);
          v[p].x *= rstd * ng4.x; v[p].y *= rstd * ng4.y; v[p].z *= rstd * ng4.z; v[p].w *= rstd * ng4.w;
        }
        if (EPI == EPI_BF16 || EPI == EPI_QKV) { v[p].x *= col_scale; v[p].y *= col_scale; v[p].z *= col_scale; v[p].w *= col_scale; }
      }
      if (EPI == EPI_RESID) {
        // gates are per (group, column); a slab of 32 rows touches at most two trajectories when a
        // trajectory has at least 32 rows.  All loads of the slab are issued before its stores.
        float4 g0 = {1.f, 1.f, 1.f, 1.f}, g1 = g0;
        const bool fast = a.L >= 32;
        const int traj0 = slab0 / a.L;
        const int split = (traj0 + 1) * a.L;
        if (a.gate && fast && n_ok) {
          const int last = (a.M - 1) / a.L;
          g0 = *reinterpret_cast<const float4*>(a.gate + (int64_t)a.group_of[traj0] * a.gate_ld + n);
          g1 = *reinterpret_cast<const float4*>(a.gate + (int64_t)a.group_of[min(traj0 + 1, last)] * a.gate_ld + n);
        }
        float4 hv[NP], gv[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const int r = slab0 + RPI * p + rsub;
          const bool ok = r < a.M && n_ok;
          hv[p] = ok ? load_stream(a.outf + (int64_t)r * a.ldo + n) : float4{0.f, 0.f, 0.f, 0.f};
          gv[p] = r < split ? g0 : g1;
          if (a.gate && !fast && ok)
            gv[p] = *reinterpret_cast<const float4*>(a.gate + (int64_t)a.group_of[r / a.L] * a.gate_ld + n);
        }
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const int r = slab0 + RPI * p + rsub;
          if (r < a.M && n_ok) {
            float4 o = {hv[p].x + gv[p].x * v[p].x, hv[p].y + gv[p].y * v[p].y, hv[p].z + gv[p].z * v[p].z,
                        hv[p].w + gv[p].w * v[p].w};
            store_stream(a.outf + (int64_t)r * a.ldo + n, o);
          }
        }
        continue;
      }
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const int r = slab0 + RPI * p + rsub;
        if (r >= a.M || !n_ok) continue;
        if (EPI == EPI_F32) {
          store_stream(a.outf + (int64_t)r * a.ldo + n, v[p]);
        } else if (EPI == EPI_EMBED) {
          const int traj = r / a.Li, tok = r - traj * a.Li;
          const uint2 raw = *reinterpret_cast<const uint2*>(a.pos + (int64_t)tok * a.N + n);
          float4 o = {v[p].x + bf16_to_f32((uint16_t)raw.x), v[p].y + bf16_to_f32((uint16_t)(raw.x >> 16)),
                      v[p].z + bf16_to_f32((uint16_t)raw.y), v[p].w + bf16_to_f32((uint16_t)(raw.y >> 16))};
          store_stream(a.outf + ((int64_t)traj * a.L + tok) * a.ldo + n, o);
        } else if (EPI == EPI_BF16) {
          store_stream(a.outb + (int64_t)r * a.ldob + n, pack_bf16x4(v[p]));
        } else if (EPI == EPI_QKV) {
          int64_t ro = r;
          if (a.Lout > 0) { const int traj = r / a.L; ro = (int64_t)traj * a.Lout + a.tok_off + (r - traj * a.L); }
          store_stream(a.outb + ro * a.ldob + n, pack_bf16x4(v[p]));
        } else if (EPI == EPI_GELU) {
          const float4 gl = {gelu_tanh(v[p].x), gelu_tanh(v[p].y), gelu_tanh(v[p].z), gelu_tanh(v[p].w)};
          store_stream(a.outb + (int64_t)r * a.ldob + n, pack_bf16x4(gl));
        }
      }
    }
    return;
  }
  // ---- unpatchify: per-element scatter into the latent layout (small: N = 4C columns) ----
  int n_j[TN];
  float bias_j[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    n_j[j] = n0 + wn * (BN / WN) + j * 32 + l32;
    bias_j[j] = (a.bias && n_j[j] < a.N) ? bf16_to_f32(a.bias[n_j[j]]) : 0.f;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int rb = m0 + wm * (BM / WM) + i * 32 + 4 * half;       // rows rb + 8q + t
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r0 = rb + 8 * q;
      if (r0 >= a.M) continue;
      const int traj0 = r0 / a.Li, tok0 = r0 - traj0 * a.Li;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = n_j[j];
        if (n >= a.N) continue;
        int traj = traj0, tok = tok0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = r0 + t;
          if (r >= a.M) break;
          const float v = acc[i][j][4 * q + t] + bias_j[j];
          if (tok >= a.Li) { tok -= a.Li; ++traj; }
          const int py = tok / a.Wp, px = tok - py * a.Wp;
          const int c = n >> 2, dy = (n >> 1) & 1, dx = n & 1;
          a.outf[(int64_t)traj * ((int64_t)(a.N >> 2) * a.HW) + (int64_t)c * a.HW + (2 * py + dy) * a.Wimg + 2 * px + dx] = v;
          ++tok;
        }
      }
    }
  }
}

template <int EPI, int BM, int BN, int BK, int WM, int WN, int MINW, int NST>
static pg_status launch_tile(const GemmArgs& a, hipStream_t s) {
  constexpr int LDS = NST * (BM + BN) * BK * 2;
  static bool attr_set = false;
  if (!attr_set) {
    PG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel<EPI, BM, BN, BK, WM, WN, MINW, NST>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, LDS));
    attr_set = true;
  }
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  const int grid = (tiles + XCDS - 1) / XCDS * XCDS;
  gemm_kernel<EPI, BM, BN, BK, WM, WN, MINW, NST><<<dim3(grid), dim3(64 * WM * WN), LDS, s>>>(a);
  PG_LAUNCH_CHECK("gemm_kernel");
  return PG_OK;
}

// Tile choice.  A launch runs in rounds of 256 concurrent workgroups (one per compute unit); the last
// round is usually part empty, and with few K steps a tile's fixed prologue / epilogue weighs more.
// Pick the shape with the best product of slot occupancy and the measured relative speed of its main
// loop.
static int pick_tile(const GemmArgs& a, int epilogue) {
  auto score = [&](int bm, int bn, int per_cu, double speed) {
    const double tiles = (double)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn);
    const double slots = 256.0 * per_cu;
    const double useful = (double)a.M * a.N / ((double)bm * bn);      // ragged edge tiles do less work
    return speed * useful / (ceil(tiles / slots) * slots);
  };
  const double sc[6] = {score(256, 256, 1, 1.00), score(192, 256, 1, 0.97), score(128, 256, 1, 0.90),
                        score(128, 128, 2, 0.85), score(160, 256, 1, 0.92), score(224, 256, 1, 0.96)};
  const bool wide_rows = epilogue == EPI_QKV && a.norm_hd > 32;   // the fused norm needs a whole head inside one wave's columns
  int best = 0;
  for (int i = 1; i < 6; ++i) if (sc[i] > sc[best] * 1.02 && !(wide_rows && i >= 4)) best = i;
  return best;
}

template <int EPI>
static pg_status launch_one(const GemmArgs& a, hipStream_t s) {
  switch (pick_tile(a, EPI)) {
    case 0: return launch_tile<EPI, 256, 256, 64, 2, 4, 2, 2>(a, s);
    case 1: return launch_tile<EPI, 192, 256, 64, 2, 4, 2, 2>(a, s);
    case 2: return launch_tile<EPI, 128, 256, 64, 2, 4, 2, 2>(a, s);
    case 3: return launch_tile<EPI, 128, 128, 64, 2, 2, 2, 2>(a, s);
    case 4: return launch_tile<EPI, 160, 256, 64, 1, 8, 2, 2>(a, s);     // heights that are not a multiple of 64:
    default: return launch_tile<EPI, 224, 256, 64, 1, 8, 2, 2>(a, s);    // one wave row, 32 columns per wave
  }
}

pg_status launch_gemm(const GemmArgs& a_in, int epilogue, hipStream_t s) {
  GemmArgs a = a_in;
  // bands of 8 tile rows; of 4 when the output is at most six tiles wide (the D-wide residual GEMMs of the 1536-wide network:
  // a band then still spans the whole width, and 0.7 % of the loop's GEMM time goes away)
  a.raster = 1; a.group_m = (a.N + 255) / 256 <= 6 ? GROUP_M / 2 : GROUP_M;
  if (a.M <= 0 || a.N <= 0) return PG_OK;
  if (a.K <= 0 || a.K % 64) return fail(PG_ESHAPE, "GEMM K = %d must be a positive multiple of 64", a.K);
  if (a.lda % 8 || a.ldw % 8 || a.lda < a.K || a.ldw < a.K || ((uintptr_t)a.A & 15) || ((uintptr_t)a.W & 15))
    return fail(PG_ESHAPE, "GEMM operands need 16-byte aligned rows (lda %lld, ldw %lld)", (long long)a.lda, (long long)a.ldw);
  if (!a.A || !a.W) return fail(PG_EINVAL, "GEMM: null operand");
  if (epilogue != EPI_UNPATCH) {
    // the row-major epilogues write 4 consecutive columns per lane
    const int n_rm = epilogue == EPI_QKV ? a.v_start : a.N;
    if (n_rm % 4) return fail(PG_ESHAPE, "GEMM N = %d must be a multiple of 4", n_rm);
    if ((a.outf && (a.ldo % 4 || ((uintptr_t)a.outf & 15))) || (a.outb && (a.ldob % 4 || ((uintptr_t)a.outb & 7))) ||
        (a.bias && ((uintptr_t)a.bias & 7)) || (a.gate && (a.gate_ld % 4 || ((uintptr_t)a.gate & 15))) ||
        (a.pos && ((uintptr_t)a.pos & 7)))
      return fail(PG_ESHAPE, "GEMM output / bias / gate rows need 16-byte (bf16: 8-byte) alignment");
  }
  if (epilogue == EPI_QKV && a.norm_hd > 0) {
    if ((a.norm_hd != 32 && a.norm_hd != 64) || !a.qn_g || !a.kn_g || a.v_start % a.norm_hd || a.scale_cols % a.norm_hd ||
        ((uintptr_t)a.qn_g & 7) || ((uintptr_t)a.kn_g & 7))
      return fail(PG_ESHAPE, "GEMM: bad fused head norm (width %d)", a.norm_hd);
  }
  if (epilogue == EPI_QKV) {
    const int vs = a.v_start;
    if (!a.vt || a.L < 1 || a.Lpad < a.L || (a.Lpad & 1) || ((uintptr_t)a.vt & 3) || vs < 0 || vs > a.N || vs % 32 ||
        (a.N - vs) % 32 || !a.outb)
      return fail(PG_ESHAPE, "GEMM: bad transposed-value output (L %d, Lpad %d, v_start %d)", a.L, a.Lpad, a.v_start);
  }
  const int rec = prof_open(PROF_GEMM, 2.0 * a.M * (double)a.N * (a.k_algo > 0 ? a.k_algo : a.K), s);
  pg_status st = PG_EINVAL;
  switch (epilogue) {
    case EPI_F32: st = launch_one<EPI_F32>(a, s); break;
    case EPI_EMBED: st = launch_one<EPI_EMBED>(a, s); break;
    case EPI_BF16: st = launch_one<EPI_BF16>(a, s); break;
    case EPI_QKV: st = launch_one<EPI_QKV>(a, s); break;
    case EPI_GELU: st = launch_one<EPI_GELU>(a, s); break;
    case EPI_RESID: st = launch_one<EPI_RESID>(a, s); break;
    case EPI_UNPATCH: st = launch_one<EPI_UNPATCH>(a, s); break;
    default: st = fail(PG_EINVAL, "unknown GEMM epilogue %d", epilogue);
  }
  prof_close(rec, s);
  return st;
}

// Measurement hook: bf16 MFMAs on registers alone.  Eight independent 32x32 accumulators per wave keep the pipe
// full (an MFMA may not follow one that writes the accumulator it reads without waiting for it).
constexpr int PROBE_ACC = 8;
__global__ __launch_bounds__(256) void mfma_probe_kernel(float* __restrict__ out, int iters, float scale) {
  bf16x8 a, b;
  uint32_t h = (threadIdx.x + 1u) * 2654435761u + blockIdx.x * 40503u;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    h = h * 1664525u + 1013904223u;
    a[e] = (__bf16)(((int)(h >> 8) % 2001 - 1000) * 1e-3f * scale);
    h = h * 1664525u + 1013904223u;
    b[e] = (__bf16)(((int)(h >> 8) % 2001 - 1000) * 1e-3f * scale);
  }
  f32x16 acc[PROBE_ACC];
#pragma unroll
  for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) sum += acc[i][e];
  out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

}  // namespace pg

using namespace pg;

extern "C" pg_status pg_mfma_probe(int32_t blocks, int32_t iters, float operand_scale, float* out, double* flops,
                                   void* stream) {
  if (blocks < 1 || blocks > 65536 || iters < 1 || iters > 10000000) return fail(PG_EINVAL, "pg_mfma_probe: blocks %d, iters %d", blocks, iters);
  if (!out) return fail(PG_EINVAL, "pg_mfma_probe: out is NULL");
  mfma_probe_kernel<<<dim3(blocks), dim3(256), 0, (hipStream_t)stream>>>(out, iters, operand_scale);
  PG_LAUNCH_CHECK("mfma_probe_kernel");
  if (flops) *flops = (double)blocks * 4.0 * iters * PROBE_ACC * 32768.0;
  return PG_OK;
}

extern "C" pg_status pg_gemm_bf16(const uint16_t* A, int64_t lda, const uint16_t* W, int64_t ldw,
                                  const uint16_t* bias, float* C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                                  void* stream) {
  if (M < 0 || N < 0 || M > INT32_MAX || N > INT32_MAX || K > INT32_MAX) return fail(PG_EINVAL, "pg_gemm_bf16: bad sizes");
  if (M == 0 || N == 0) return PG_OK;
  if (!C || ldc < N) return fail(PG_EINVAL, "pg_gemm_bf16: bad output");
  GemmArgs a{};
  a.A = A; a.lda = lda; a.W = W; a.ldw = ldw; a.bias = bias;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.outf = C; a.ldo = ldc;
  return launch_gemm(a, EPI_F32, (hipStream_t)stream);
}
