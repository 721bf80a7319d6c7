// bf16 MFMA GEMM of the network: C[M, N] = A[M, K] W[N, K]^T (+ fused epilogue), fp32 accumulate.
#pragma once
#include "common.hpp"

namespace pg {

enum GemmEpilogue {
  EPI_F32 = 0,      // outf[r, n] = acc + bias
  EPI_EMBED = 1,    // outf[(r / Li) * L + r % Li, n] = acc + bias + pos[r % Li, n]     (patch embedding)
  EPI_BF16 = 2,     // outb[r, n] = bf16(acc + bias)
  EPI_QKV = 3,      // columns n < v_start as EPI_BF16; value channels n >= v_start are stored transposed:
                    // vt[((r / L) * (N - v_start) + n - v_start) * Lpad + tok_off + r % L] = bf16(acc + bias)
  EPI_GELU = 4,     // outb[r, n] = bf16(gelu_tanh(acc + bias))
  EPI_RESID = 5,    // outf[r, n] += gate[group_of[r / L], n] * (acc + bias)   (gate NULL: plain add)
  EPI_UNPATCH = 6   // u[m, c, 2 py + dy, 2 px + dx] = acc + bias, r = m * Li + py * Wp + px, n = 4 c + 2 dy + dx
};

struct GemmArgs {
  const uint16_t* A; int64_t lda;
  const uint16_t* W; int64_t ldw;
  const uint16_t* bias;            // bf16 [N] or NULL
  int M, N, K;
  int k_algo;                      // unpadded K for flop accounting (0: same as K)
  float* outf; int64_t ldo;
  uint16_t* outb; int64_t ldob;
  // epilogue extras
  int L, Li;                       // rows per trajectory in the output / input
  const uint16_t* pos;             // bf16 [Li, N]
  uint16_t* vt; int v_start, Lpad;
  const float* gate; int64_t gate_ld; const int32_t* group_of;
  int Wp, HW, Wimg;                // unpatchify: patches per row, H*W, W
  int Lout, tok_off;               // EPI_QKV: input row r = traj * L + tok is written as row traj * Lout + tok_off + tok (Lout 0: same row)
  int norm_hd; const uint16_t* qn_g; const uint16_t* kn_g;   // EPI_QKV, norm_hd > 0: every norm_hd-wide head chunk of the row-major columns is RMS-normalised (eps 1e-6) and multiplied by the bf16 scales qn_g (columns < scale_cols) / kn_g [norm_hd]
  float out_scale; int scale_cols; // EPI_BF16 / EPI_QKV: columns n < scale_cols are multiplied by out_scale (after the bias)
  int raster, group_m;             // tile order: XCD-aware remap on/off, tile rows per band (set by the launcher)
};

pg_status launch_gemm(const GemmArgs& a, int epilogue, hipStream_t s);

}  // namespace pg
