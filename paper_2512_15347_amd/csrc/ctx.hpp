// Host-side state of one sampling context (opaque pg_ctx of the C ABI).
#pragma once
#include <vector>
#include "common.hpp"

struct WeightSlot { int64_t offset; int32_t rows, cols, ld; };

struct NetPlan {             // byte offsets into the workspace for the network's activations
  size_t h, act, qkv, vt, att, hid, tok, mod, cond, ctx_h, ckv, ckvt, total;
};

struct pg_ctx {
  pg_config cfg;
  int d, Li, L, M0;
  std::vector<double> A, B, C, Pv, Qv, tin;
  // schedule[g] = list of (step, k)
  std::vector<std::vector<std::pair<int, int>>> sched;
  std::vector<char> is_checkpoint;        // per step
  // weights
  std::vector<WeightSlot> top;            // PG_W_COUNT entries (per-block ones hold block-0 offsets)
  int64_t block_stride = 0, weights_numel = 0;
  // workspace plan
  size_t ws_partials = 0, ws_k = 0, ws_newoff = 0, ws_forced = 0, ws_sched = 0, ws_off0 = 0, ws_logr = 0, ws_net = 0,
         ws_total = 0;
  NetPlan net{};
  // bound buffers
  pg_buffers buf{};
  bool bound = false;
  // loop state
  uint64_t seed = 0;
  int M = 0, cur_x = 0, cur_id = 0;
  bool pending_gather = false, initialised = false, net_fresh = false;
  std::vector<int> offsets;               // host copy, P+1
  int64_t evals = 0, updates = 0;
  int steps_done = 0;                     // steps taken since pg_init_group
  bool advantages_done = false;
  bool context_ready = false;             // step-independent network precomputation done
  // The funnel as the schedule fixes it: row s = k[P] | new_offsets[P+1] of a prune at step s when every earlier
  // prune followed the schedule.  Uploaded into the workspace once (pg_bind), so a prune needs no host -> device copy.
  std::vector<int32_t> sched_table;       // [T][2P+1]
  // pinned host slot for the counts pg_select_final takes per call (2P+1 ints), and the event that tells when the
  // copy out of it has run (the host waits on it before writing the slot again)
  int32_t* staging = nullptr;
  hipEvent_t staging_read = nullptr;
  bool staging_in_flight = false;
};

namespace pg {
// network (dit_kernels.hip)
pg_status net_plan(pg_ctx* c);                                  // fills c->net, returns bytes in net.total
pg_status net_prepare(pg_ctx* c, const uint16_t* weights, hipStream_t s);   // step-independent precomputation
// u = net(x) for the M active rows of `x` under `weights`
pg_status net_forward(pg_ctx* c, int step, const float* x, const uint16_t* weights, hipStream_t s);
// sampler_kernels.hip
pg_status launch_sde_step(const float* x, const float* u, float* x_out, float* logp, float* logp_hist,
                          float* logp_sum, const int32_t* src, const int32_t* orig_id, int64_t n_traj, int64_t d,
                          double A, double B, double C, uint64_t seed, uint32_t step, float* partials,
                          float* hist_next, hipStream_t s);
pg_status launch_transition_logprob(const float* x, const float* u, const float* x_next_by_id,
                                    const int32_t* orig_id, int64_t n_traj, int64_t d, double A, double B, double C,
                                    uint64_t seed, uint32_t step, float* logp_by_id, double* log_ratio_by_id,
                                    float* partials, hipStream_t s);
pg_status launch_surrogate(const double* log_ratio, const float* adv, const int32_t* offsets,
                           const int32_t* orig_id, int n_groups, int T, int M0, double clip_eps, float* ratio,
                           float* J, hipStream_t s);
// small launches (ovf_kernels.hip)
pg_status launch_fill_u32(void* p, uint32_t v, size_t n, hipStream_t s);
pg_status launch_iota(int32_t* p, int n, hipStream_t s);
pg_status launch_gather_ids(const int32_t* in, const int32_t* sel, int n_out, int32_t* out, hipStream_t s);
pg_status launch_fill_group_of(const int32_t* offsets, int n_groups, int32_t* group_of, hipStream_t s);
pg_status launch_masks_to_sel(const uint64_t* masks, const int32_t* offsets, const int32_t* new_offsets,
                              int n_groups, int32_t* sel_idx, hipStream_t s);
pg_status launch_uniform_select(const int32_t* offsets, const int32_t* k, int n_groups, const int32_t* new_offsets,
                                uint64_t seed, uint32_t draw, uint64_t* masks, int32_t* sel_idx, int32_t* status,
                                hipStream_t s);
pg_status launch_ovf(const float* rewards, const int32_t* offsets, const int32_t* k, int n_groups,
                     const int32_t* new_offsets, uint64_t* masks, int32_t* sel_idx, int32_t* status,
                     hipStream_t s);
}  // namespace pg
