// bf16 MFMA GEMM for gfx950: C[M, N] = A[M, K] W[N, K]^T with a fused epilogue.  This is where the
// network evaluation of every denoising step spends its time (the noise-prediction row of the paper's
// cost table, Sec. 6.2), so the tile is sized for the 160 KB LDS and the 32x32x16 bf16 MFMA:
//   workgroup tile 256 x 256 x 64, 8 wavefronts as 2 (M) x 4 (N), each owning 128 x 64 = 4 x 2 MFMA tiles;
//   both operands are K-contiguous, staged global -> registers -> LDS in 16-byte chunks, two LDS stages
//   (2 x 64 KB), one barrier per K step; chunk positions are XOR-swizzled so that both the 16-byte
//   staging writes and the 16-byte MFMA operand reads are bank-conflict free;
//   workgroup ids are spread so that the tiles resident on one XCD (one L2) form a compact block of
//   the output and share operand panels.
#include "gemm.hpp"

namespace pg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GEMM_THREADS = 512;
constexpr int TILE_BYTES = BM * BK * 2;            // one operand tile, 32 KB
constexpr int STAGE_BYTES = 2 * TILE_BYTES;        // A + W
constexpr int GEMM_LDS = 2 * STAGE_BYTES;          // 128 KB
constexpr int GROUP_M = 8;                         // tile rows per raster band
constexpr int XCDS = 8;

// byte offset of 16-byte chunk `chunk` (0..7) of tile row `row` inside an operand tile
__device__ __forceinline__ int lds_off(int row, int chunk) {
  return (row * 8 + (chunk ^ ((row ^ (row >> 3)) & 7))) * 16;
}

__device__ __forceinline__ float gelu_tanh(float x) {
  const float y = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  // tanh(y) = 1 - 2 / (exp(2y) + 1)
  const float e = __builtin_amdgcn_exp2f(2.8853900817779268f * y);
  const float t = 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
  return 0.5f * x * (1.0f + t);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

template <int EPI>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(const GemmArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  // ---- which output tile: XCD-aware, banded raster ----
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  const int per_xcd = gridDim.x / XCDS;
  const int b = (blockIdx.x % XCDS) * per_xcd + blockIdx.x / XCDS;
  if (b >= total) return;
  const int band = GROUP_M * tiles_n;
  const int first_m = (b / band) * GROUP_M;
  const int gsz = min(tiles_m - first_m, GROUP_M);
  const int tm = first_m + (b % band) % gsz;
  const int tn = (b % band) / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  // value-channel tiles of the QKV projection are computed transposed (operands swapped) so that
  // V^T can be stored with consecutive lanes on consecutive tokens
  const bool tr = (EPI == EPI_QKV) && (n0 >= a.v_start);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int l32 = lane & 31, half = lane >> 5;

  // ---- staging assignment: 4 chunks of A and 4 of W per lane ----
  const int ld_row = tid >> 3, ld_chunk = tid & 7;
  const uint16_t* a_ptr[4];
  const uint16_t* w_ptr[4];
  int st_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = ld_row + 64 * i;
    a_ptr[i] = a.A + (int64_t)min(m0 + row, a.M - 1) * a.lda + ld_chunk * 8;
    w_ptr[i] = a.W + (int64_t)min(n0 + row, a.N - 1) * a.ldw + ld_chunk * 8;
    st_off[i] = lds_off(row, ld_chunk);
  }
  // operand read offsets inside a tile for k-slab 0; slab ks adds chunk 2*ks (applied under the XOR)
  int a_row[4], w_row[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) a_row[i] = wm * 128 + i * 32 + l32;
#pragma unroll
  for (int j = 0; j < 2; ++j) w_row[j] = wn * 64 + j * 32 + l32;

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4v ra[4], rw[4];
  const int nk = a.K / BK;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ra[i] = *reinterpret_cast<const u32x4v*>(a_ptr[i]);
    rw[i] = *reinterpret_cast<const u32x4v*>(w_ptr[i]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    *reinterpret_cast<u32x4v*>(smem + st_off[i]) = ra[i];
    *reinterpret_cast<u32x4v*>(smem + TILE_BYTES + st_off[i]) = rw[i];
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const unsigned char* sA = smem + (kt & 1) * STAGE_BYTES + (tr ? TILE_BYTES : 0);   // first MFMA operand
    const unsigned char* sW = smem + (kt & 1) * STAGE_BYTES + (tr ? 0 : TILE_BYTES);   // second MFMA operand
    if (kt + 1 < nk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ra[i] = *reinterpret_cast<const u32x4v*>(a_ptr[i] + (kt + 1) * BK);
        rw[i] = *reinterpret_cast<const u32x4v*>(w_ptr[i] + (kt + 1) * BK);
      }
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 af[4], wf[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const bf16x8*>(sA + lds_off(a_row[i], 2 * ks + half));
#pragma unroll
      for (int j = 0; j < 2; ++j) wf[j] = *reinterpret_cast<const bf16x8*>(sW + lds_off(w_row[j], 2 * ks + half));
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      unsigned char* dA = smem + ((kt + 1) & 1) * STAGE_BYTES;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<u32x4v*>(dA + st_off[i]) = ra[i];
        *reinterpret_cast<u32x4v*>(dA + TILE_BYTES + st_off[i]) = rw[i];
      }
    }
    __syncthreads();
  }

  // ---- epilogue: in each 32x32 tile a lane holds ONE column (l32) and rows 8q + 4*half + t ----
  if (EPI == EPI_QKV && tr) {
    // transposed tile: accumulator rows are output columns n (value channels), its columns are tokens,
    // so consecutive lanes write consecutive tokens of one row of V^T
    const int Dv = a.N - a.v_start;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int r = m0 + wn * 64 + j * 32 + l32;
      if (r >= a.M) continue;
      const int traj = r / a.L, tok = r - traj * a.L;
      uint16_t* vcol = a.vt + (int64_t)traj * Dv * a.Lpad + tok;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int n = n0 + wm * 128 + i * 32 + 8 * q + 4 * half + t;
            if (n < a.N) {
              const float bv = a.bias ? bf16_to_f32(a.bias[n]) : 0.f;
              vcol[(int64_t)(n - a.v_start) * a.Lpad] = f32_to_bf16(acc[i][j][4 * q + t] + bv);
            }
          }
    }
    return;
  }
  int n_j[2];
  float bias_j[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    n_j[j] = n0 + wn * 64 + j * 32 + l32;
    bias_j[j] = (a.bias && n_j[j] < a.N) ? bf16_to_f32(a.bias[n_j[j]]) : 0.f;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rb = m0 + wm * 128 + i * 32 + 4 * half;       // rows rb + 8q + t
    if (EPI == EPI_RESID) {
      // phase 1: every load of this 32-row slab (old h, gates) is issued before the first store,
      // so the memory latencies overlap instead of chaining through possible aliasing
      float hv[4][2][4], gv[4][2][4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = rb + 8 * q + t;
          const bool ok = r < a.M;
          int gid = 0;
          if (a.gate && ok) gid = a.group_of[r / a.L];
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const bool okn = ok && n_j[j] < a.N;
            hv[q][j][t] = okn ? a.outf[(int64_t)r * a.ldo + n_j[j]] : 0.f;
            gv[q][j][t] = (a.gate && okn) ? a.gate[(int64_t)gid * a.gate_ld + n_j[j]] : 1.0f;
          }
        }
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = rb + 8 * q + t;
#pragma unroll
          for (int j = 0; j < 2; ++j)
            if (r < a.M && n_j[j] < a.N)
              a.outf[(int64_t)r * a.ldo + n_j[j]] = hv[q][j][t] + gv[q][j][t] * (acc[i][j][4 * q + t] + bias_j[j]);
        }
      continue;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r0 = rb + 8 * q;
      if (r0 >= a.M) continue;
      int traj0 = 0, tok0 = 0;
      if (EPI == EPI_EMBED || EPI == EPI_UNPATCH) { traj0 = r0 / a.Li; tok0 = r0 - traj0 * a.Li; }
      if (EPI == EPI_QKV) { traj0 = r0 / a.L; tok0 = r0 - traj0 * a.L; }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = n_j[j];
        if (n >= a.N) continue;
        int traj = traj0, tok = tok0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = r0 + t;
          if (r >= a.M) break;
          const float v = acc[i][j][4 * q + t] + bias_j[j];
          if (EPI == EPI_F32) {
            a.outf[(int64_t)r * a.ldo + n] = v;
          } else if (EPI == EPI_EMBED) {
            if (tok >= a.Li) { tok -= a.Li; ++traj; }
            a.outf[((int64_t)traj * a.L + tok) * a.ldo + n] = v + bf16_to_f32(a.pos[(int64_t)tok * a.N + n]);
            ++tok;
          } else if (EPI == EPI_BF16) {
            a.outb[(int64_t)r * a.ldob + n] = f32_to_bf16(v);
          } else if (EPI == EPI_QKV) {
            if (tok >= a.L) { tok -= a.L; ++traj; }
            if (n < a.v_start) a.outb[(int64_t)r * a.ldob + n] = f32_to_bf16(v);
            else a.vt[((int64_t)traj * (a.N - a.v_start) + (n - a.v_start)) * a.Lpad + tok] = f32_to_bf16(v);
            ++tok;
          } else if (EPI == EPI_GELU) {
            a.outb[(int64_t)r * a.ldob + n] = f32_to_bf16(gelu_tanh(v));
          } else if (EPI == EPI_UNPATCH) {
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
}

template <int EPI>
static pg_status launch_one(const GemmArgs& a, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    PG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel<EPI>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS));
    attr_set = true;
  }
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  const int grid = (tiles + XCDS - 1) / XCDS * XCDS;
  gemm_kernel<EPI><<<dim3(grid), dim3(GEMM_THREADS), GEMM_LDS, s>>>(a);
  PG_LAUNCH_CHECK("gemm_kernel");
  return PG_OK;
}

pg_status launch_gemm(const GemmArgs& a, int epilogue, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return PG_OK;
  if (a.K <= 0 || a.K % BK) return fail(PG_ESHAPE, "GEMM K = %d must be a positive multiple of %d", a.K, BK);
  if (a.lda % 8 || a.ldw % 8 || a.lda < a.K || a.ldw < a.K || ((uintptr_t)a.A & 15) || ((uintptr_t)a.W & 15))
    return fail(PG_ESHAPE, "GEMM operands need 16-byte aligned rows (lda %lld, ldw %lld)", (long long)a.lda, (long long)a.ldw);
  if (!a.A || !a.W) return fail(PG_EINVAL, "GEMM: null operand");
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

}  // namespace pg

using namespace pg;

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
