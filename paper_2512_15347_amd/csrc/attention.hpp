// Softmax attention on bf16 MFMA (see attention.hip).
#pragma once
#include "common.hpp"

namespace pg {

struct AttnArgs {
  const uint16_t* q; int64_t ldq;                 // [B, Lq, ldq], head h at column h*hd
  const uint16_t* k; int64_t ldk, k_bstride;      // key rows of batch kb at k + kb*k_bstride
  const uint16_t* vt; int64_t vt_bstride; int Lkpad;   // [kb][heads*hd][Lkpad] transposed values
  uint16_t* out; int64_t ldo;                     // [B, Lq, ldo]
  const int32_t* kv_map;                          // batch -> key/value batch (NULL: identity)
  int B, Lq, Lk, heads;
  float scale_log2;                               // log2(e) / sqrt(hd)
  int q_prescaled;
  int split; uint16_t* out2;                      // split > 0: queries >= split go to out2[b * (Lq - split) + q - split, :]                                // the producer of q has already multiplied it by scale_log2
};

pg_status launch_attention(const AttnArgs& a, int hd, hipStream_t s);

}  // namespace pg
