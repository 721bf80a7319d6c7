/*
 * progrpo.h -- C ABI of the MI355X (gfx950) library for the Pro-GRPO sampling hot path:
 * expanded-group sampling with in-loop trajectory pruning (paper Sec. 5.1, Sec. 5.2).
 *
 * Conventions
 *  - Every pointer is tagged [host] or [device].  The library allocates NO device memory and
 *    creates no streams: all device buffers are owned by the caller, and every launch goes to
 *    the HIP stream handle passed in (`void* stream`, a hipStream_t; NULL = default stream).
 *  - Calls return asynchronously (work queued on the stream) unless stated otherwise.
 *  - Every call returns a pg_status.  Argument errors are found on the host before any launch.
 *    pg_last_error() gives a human-readable message for the last failure on this thread.
 *  - Errors that only the device can see (a non-finite proxy reward, a bad count met by a selection
 *    kernel) cannot come back from an asynchronous call: they set a sticky word in pg_buffers.status, the
 *    kernels keep every index they write in bounds, and pg_check() reports them.  CALL pg_check AFTER
 *    pg_sample_group (or after the last call of a hand-written loop) BEFORE USING THE RESULTS: after a
 *    non-finite reward the survivor sets are the first k slots of each group, not Eq. 10's.
 *  - Packed batch layout: the M active trajectories are rows of x[M, d] (fp32, d = C*H*W, NCHW
 *    inside a row), ordered by (group, ascending original slot); group g owns rows
 *    group_offsets[g] .. group_offsets[g+1]-1.  orig_id[row] = g*N + original slot.
 *  - "Step s" is 0-based.  A prune at step s happens after the network evaluation of step s and
 *    before its update, so the survivors' update reuses that evaluation.
 */
#ifndef PROGRPO_H
#define PROGRPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PG_OK = 0,
  PG_EINVAL = 1,     /* bad scalar argument or null pointer */
  PG_ESHAPE = 2,     /* shapes the kernels cannot take (alignment, limits) */
  PG_ENAN = 3,       /* non-finite reward met by the selection */
  PG_ESCHED = 4,     /* pruning schedule not a decreasing funnel, or call out of order */
  PG_EWORKSPACE = 5, /* workspace missing or too small */
  PG_EHIP = 6        /* a HIP runtime call failed */
} pg_status;

enum { PG_SAMPLER_FLOW = 0, PG_SAMPLER_DDIM = 1, PG_SAMPLER_TABLE = 2 };
enum { PG_NET_NONE = 0, PG_NET_ADALN = 1, PG_NET_CROSS = 2, PG_NET_JOINT = 3, PG_NET_MMDIT = 4 };

/* Identifiers of the network tensors inside the flat bf16 weight buffer (see pg_weight_slot). */
enum {
  PG_W_PE_W = 0, PG_W_PE_B, PG_W_POS, PG_W_T_W1, PG_W_T_B1, PG_W_T_W2, PG_W_T_B2,
  PG_W_CTX_W, PG_W_CTX_B, PG_W_FMOD_W, PG_W_FMOD_B, PG_W_F_W, PG_W_F_B,
  /* per block */
  PG_W_MOD_W, PG_W_MOD_B, PG_W_QKV_W, PG_W_QKV_B, PG_W_O_W, PG_W_O_B,
  PG_W_FC1_W, PG_W_FC1_B, PG_W_FC2_W, PG_W_FC2_B,
  PG_W_CQ_W, PG_W_CQ_B, PG_W_CKV_W, PG_W_CKV_B, PG_W_CO_W, PG_W_CO_B,
  /* per block, dual-stream variant: the context stream's own tensors and the query / key norm scales */
  PG_W_C_MOD_W, PG_W_C_MOD_B, PG_W_C_QKV_W, PG_W_C_QKV_B, PG_W_C_O_W, PG_W_C_O_B,
  PG_W_C_FC1_W, PG_W_C_FC1_B, PG_W_C_FC2_W, PG_W_C_FC2_B,
  PG_W_QN_G, PG_W_KN_G, PG_W_C_QN_G, PG_W_C_KN_G,
  PG_W_COUNT
};

/*
 * Problem statement (all arrays [host], read during pg_create only).
 *  P groups (prompts) of N <= 64 trajectories; latent C x H x W (H, W even); T steps.
 *  Sampler: the reverse step is the affine form of the Euler-Maruyama update (Eq. 13)
 *     x' = A_s x + B_s u + C_s xi,   preview (Eq. 15)  x_hat = P_s x + Q_s u,
 *  with per-step scalars built on the host in fp64 from
 *     FLOW : rectified flow (Eq. 3, Eq. 4, RF case of Eq. 12), noise fraction 1 -> 0 in T equal
 *            steps, sigma = noise_level * sqrt(tau / (1 - tau)) (denominator clamped to 1/T);
 *     DDIM : DDIM(eta) posterior step (diffusion case of Eq. 12) on a T_train-entry linear beta
 *            table beta0..beta1, T+1 evenly spread integer timesteps T_train-1 .. 0;
 *     TABLE: the caller's own tables tab_*[T] (tab_tin = network time input per step).
 *  Network: PG_NET_NONE (the caller writes u itself before pg_prune / pg_step) or a patch-2
 *  adaLN transformer of width D (multiple of 64), `blocks` blocks, `heads` heads (head width 32
 *  or 64), with Lc context tokens of width Dc (multiple of 64; CROSS: cross-attention sub-block,
 *  JOINT: context tokens appended to the image tokens; MMDIT: as JOINT, but image and context
 *  tokens keep separate streams with their own modulation, projection and MLP weights in every
 *  block and meet only in the joint attention, whose queries and keys are RMS-normalised per
 *  head (eps 1e-6) with a learnt scale per head channel).
 *  Schedule: n_sched entries (group, step, k): at `step`, group keeps k of its active
 *  trajectories (Sec. 5.2: counts strictly decrease along a group's entries, steps increase).
 *  Reward proxy (stand-in for Eq. 16): R = probe_bias + <probe_w, x_hat>.
 */
typedef struct pg_config {
  int32_t P, N, C, H, W, T;
  int32_t sampler_kind;
  double noise_level;
  double eta, beta0, beta1;
  int32_t T_train;
  const double *tab_A, *tab_B, *tab_C, *tab_P, *tab_Q, *tab_tin;
  int32_t net_kind, D, blocks, heads, Lc, Dc;
  int32_t n_sched;
  const int32_t *sched_group, *sched_step, *sched_k;
  double probe_bias;
  double adv_eps; /* epsilon of Eq. 18, > 0 */
} pg_config;

/*
 * Device buffers, all [device], owned by the caller, sizes with M0 = P*N, d = C*H*W.
 * The library keeps the pointers given to pg_bind until the next pg_bind / pg_destroy.
 */
typedef struct pg_buffers {
  float *x[2];             /* [M0, d] each; ping-pong, pg_state tells which one is current */
  float *u;                /* [M0, d] network output for the current packed batch */
  int32_t *orig_id[2];     /* [M0] each; ping-pong (flips at a prune), pg_state tells which */
  int32_t *group_offsets;  /* [P+1] current offsets (written by the library) */
  int32_t *group_of;       /* [M0] group of each packed row (written by the library) */
  float *rewards;          /* [M0] proxy rewards at a checkpoint / final rewards at the end */
  uint64_t *masks;         /* [P] survivor mask over each group's current slots */
  int32_t *sel_idx;        /* [M0] packed positions of the survivors, (group, slot) order */
  float *logp_hist;        /* [T, M0] per-step log-prob indexed by ORIGINAL id; NaN = not taken */
  float *logp_sum;         /* [M0] sum over executed steps, by original id */
  float *adv;              /* [M0] advantages of the final packed batch (first M_T entries) */
  const float *probe_w;    /* [d] */
  const uint16_t *weights; /* bf16 bit patterns, layout given by pg_weight_slot; NULL if NET_NONE */
  const uint16_t *ctx;     /* bf16 [P, Lc, Dc]; NULL if Lc == 0 */
  const float *y;          /* [P, D] prompt vector added to the timestep embedding */
  int32_t *status;         /* [4] device words: [0] = sticky error bits (1 = non-finite reward, 2 = bad k) */
  void *workspace;         /* pg_workspace_bytes() bytes, 256-byte aligned; the library's from pg_bind (which writes
                              the schedule's tables into it) to the next pg_bind / pg_destroy: do not write it */
  size_t workspace_bytes;
  float *x_hist;           /* optional (NULL: not kept) [T+1, M0, d] latents by ORIGINAL id: slice 0 = x_0,
                              slice s+1 = state after step s (rows of trajectories pruned before step s are not written) */
} pg_buffers;

typedef struct pg_ctx pg_ctx;

const char *pg_last_error(void);

/* Validates the configuration and builds the coefficient tables. *out is NULL on failure. */
pg_status pg_create(const pg_config *cfg, pg_ctx **out);
void pg_destroy(pg_ctx *ctx);

/* Bytes of scratch the caller must provide in pg_buffers.workspace (activations of the network,
 * partial sums of the reductions). */
size_t pg_workspace_bytes(const pg_ctx *ctx);

/* Number of bf16 elements of the flat weight buffer, and where tensor `id` of block `block`
 * (ignored for the tensors above PG_W_MOD_W) lives in it.  A matrix [rows, cols] is stored
 * row-major [out, in] with its row length padded with zeros to *ld elements. */
int64_t pg_weights_numel(const pg_ctx *ctx);
pg_status pg_weight_slot(const pg_ctx *ctx, int32_t id, int32_t block, int64_t *offset,
                         int32_t *rows, int32_t *cols, int32_t *ld);

/* Per-step scalars as the library computed them ([host] out arrays of T doubles, any may be NULL). */
pg_status pg_get_tables(const pg_ctx *ctx, double *A, double *B, double *C, double *P, double *Q,
                        double *t_in);

/* The funnel of Sec. 5.2 as the library will follow it: for a prune at `step`, the number of trajectories
 * each group keeps (k: [host] P ints; a group without an entry at this step keeps what it has) and their
 * exclusive scan (offsets: [host] P+1 ints), given that every earlier checkpoint was followed.  Either may be
 * NULL.  These rows are what pg_bind places in the workspace, so that a prune uploads nothing. */
pg_status pg_get_schedule(const pg_ctx *ctx, int32_t step, int32_t *k, int32_t *offsets);

pg_status pg_bind(pg_ctx *ctx, const pg_buffers *buf);

/* Host-side view of the loop state: active trajectories M, index of the current x buffer and of
 * the current orig_id buffer, and (if not NULL) the current P+1 group offsets, network evaluations and updates
 * counted so far (trajectory-steps; the cost that pruning reduces, Sec. 6.2 efficiency analysis). */
pg_status pg_state(const pg_ctx *ctx, int32_t *M, int32_t *cur_x, int32_t *cur_id,
                   int32_t *offsets /*[host] P+1*/, int64_t *evals, int64_t *updates);

/* Sec. 5.1 "Initialization": x_0 ~ N(0, I) for all P*N trajectories from the Philox stream keyed
 * by (seed, original id); resets offsets, ids, log-prob records, counters. */
pg_status pg_init_group(pg_ctx *ctx, uint64_t seed, void *stream);

/* u = network(x, t_s, prompt) on every active trajectory (the drift input of Eq. 12).  Steps come in order:
 * `step` must be the number of pg_step calls since pg_init_group (PG_ESCHED otherwise; the same holds for
 * pg_prune, pg_prune_forced and pg_step). */
pg_status pg_net_forward(pg_ctx *ctx, int32_t step, void *stream);

/* Checkpoint of Sec. 5.1 "Dynamic latent feature-based pruning": preview (Eq. 14-15), proxy reward
 * (Eq. 16), OVF per group (the arg-max after Eq. 16) with the counts of the schedule; writes rewards,
 * masks, sel_idx, new offsets / ids / group_of.  The latents themselves are compacted by the
 * following pg_step (gather on read).  PG_ESCHED if `step` is not a checkpoint of any group. */
pg_status pg_prune(pg_ctx *ctx, int32_t step, void *stream);

/* Test hook: same as pg_prune but the survivor sets are imposed ([host] masks[P] over current
 * slots; popcounts need not follow the schedule).  The OVF result for the proxy rewards is still
 * written to `ovf_masks_out` ([device] uint64[P]) if not NULL. */
pg_status pg_prune_forced(pg_ctx *ctx, int32_t step, const uint64_t *masks, uint64_t *ovf_masks_out,
                          void *stream);

/* Euler-Maruyama update (Eq. 13) of every active trajectory with Philox noise keyed by
 * (seed, original id, step), plus the Gaussian log-prob of the step (policy of Eq. 19).  PG_ESCHED if the
 * schedule prunes a group at this step and that prune has not been made (Sec. 5.2: the funnel is followed). */
pg_status pg_step(pg_ctx *ctx, int32_t step, void *stream);

/* Final rewards of the survivors and their group-normalised advantages (Eq. 18); after all T steps. */
pg_status pg_advantages(pg_ctx *ctx, void *stream);

/* The whole loop: init, T x (network, prune at checkpoints, step), advantages. */
pg_status pg_sample_group(pg_ctx *ctx, uint64_t seed, void *stream);

/* Comparison arms of Sec. 4.1-4.2 on a finished run (after pg_advantages): select on the FINAL
 * rewards, mode 0 = Optimal Variance Filtering applied once after sampling (Eq. 10), mode 1 = a
 * uniformly random subset (pg_uniform_select with the run's seed and `draw`); k_per_group: [host] P
 * ints, 1 <= k <= current group size.  The kept trajectories are packed (latents into the other
 * x buffer, ids, rewards, group offsets), masks / sel_idx hold the selection, and Eq. 18 is
 * recomputed on the kept members.  Asynchronous on `stream`. */
pg_status pg_select_final(pg_ctx *ctx, int32_t mode, const int32_t *k_per_group, uint32_t draw,
                          void *stream);

/* Forward part of the policy update on the survivors (Sec. 5.1, Eq. 19 and the first term of Eq. 20): the
 * stored transitions (x_s, x_{s+1}) of every surviving trajectory are re-evaluated under another weight set
 * (`weights_new`, [device], same layout as pg_buffers.weights): logp_new[s, id] = log N(x_{s+1}; A_s x_s +
 * B_s u_new(x_s, t_s), C_s^2 I), ratio[s, id] = exp(log pi_new - log pi_old) with the exponent summed in its
 * per-element terms (the noise the sampler drew against the noise the new policy would need, so nothing
 * cancels between two large log-probs), and per group
 * J[g] = mean over survivors and steps of min(r A, clip(r, 1 - clip_eps, 1 + clip_eps) A) with the advantages of
 * pg_advantages.  logp_new, ratio: [device] [T, M0] by original id (NaN off the survivors); J: [device] [P].
 * Needs pg_buffers.x_hist, a finished loop (all T steps and pg_advantages) and a network.  Overwrites the
 * non-current x buffer and u.  The KL term of Eq. 20 (reference policy) is not computed. */
pg_status pg_policy_ratio(pg_ctx *ctx, const uint16_t *weights_new, double clip_eps, float *logp_new,
                          float *ratio, float *J, void *stream);

/* Synchronises the stream and reports sticky device-side errors (PG_ENAN / PG_EINVAL). */
pg_status pg_check(pg_ctx *ctx, void *stream);

/* ---- kernel-level entry points (context-free; all array arguments [device]) ---- */

/* x[n_traj, d] ~ N(0, I): element e of row r is normal (e mod 4) of the Philox-4x32-10 block with
 * counter (e div 4, 0, orig_id[r], 0) and key (seed lo, seed hi); d multiple of 4. */
pg_status pg_init_latents(float *x, const int32_t *orig_id, int64_t n_traj, int64_t d, uint64_t seed,
                          void *stream);

/* Fused Eq. 13 + log-prob: for output row r, source row q = src ? src[r] : r,
 *   x_out[r] = A x[q] + B u[q] + C xi,  xi = Philox(seed; orig_id[r], step),
 *   logp[r] = -1/2 sum xi^2 - d (ln C + 1/2 ln 2 pi)      (needs C > 0).
 * x_out must not alias x.  logp_hist / logp_sum (nullable) are indexed by orig_id[r]:
 * logp_hist[orig_id[r]] = logp, logp_sum[orig_id[r]] += logp.  `partials` is scratch of
 * pg_step_scratch_floats(n_traj, d) floats. */
int64_t pg_step_scratch_floats(int64_t n_traj, int64_t d);
pg_status pg_sde_step_logprob(const float *x, const float *u, float *x_out, float *logp,
                              float *logp_hist, float *logp_sum, const int32_t *src,
                              const int32_t *orig_id, int64_t n_traj, int64_t d, double A, double B,
                              double C, uint64_t seed, uint32_t step, float *partials, void *stream);

/* pg_sde_step_logprob with the latents and the network output stored as bf16 (6 instead of 12 bytes
 * per element; a storage variant, not used by the sampling loop): the arithmetic is fp32 on the
 * bf16 values, x_out is rounded to nearest-even, the noise and the log-prob are those of the fp32
 * call.  d multiple of 8; rows 16-byte aligned. */
pg_status pg_sde_step_logprob_bf16(const uint16_t *x, const uint16_t *u, uint16_t *x_out,
                                   float *logp, float *logp_hist, float *logp_sum,
                                   const int32_t *src, const int32_t *orig_id, int64_t n_traj,
                                   int64_t d, double A, double B, double C, uint64_t seed,
                                   uint32_t step, float *partials, void *stream);

/* rewards[r] = bias + <w, Pc x[r] + Qc u[r]> (Eq. 15-16 with the linear proxy); u may be NULL when
 * Qc == 0.  Same scratch size as pg_step_scratch_floats. */
pg_status pg_preview_reward(const float *x, const float *u, const float *w, float *rewards,
                            int64_t n_traj, int64_t d, double Pc, double Qc, double bias,
                            float *partials, void *stream);

/* OVF (Eq. 10) per ragged group: rewards[group_offsets[n_groups]], group sizes <= 64,
 * 1 <= k[g] <= size.  masks[g]: bit i = slot i kept; sel_idx: packed positions of the kept rows in
 * (group, ascending slot) order; new_offsets[n_groups+1] = exclusive scan of k.  Evaluation order
 * (bit-exact contract): rank by (value, slot); fp64 prefix sums by the 64-slot doubling recurrence;
 * score k*sum(y^2) - (sum y)^2 of "j lowest + k-j highest" without fused multiply-add; largest
 * score wins, ties to the smallest j.  status[0] |= 1 on a non-finite reward, |= 2 on a bad k or
 * size (that group's mask is then 0).  scratch: pg_ovf_scratch_ints(n_groups) int32. */
int64_t pg_ovf_scratch_ints(int64_t n_groups);
pg_status pg_ovf_select(const float *rewards, const int32_t *group_offsets, const int32_t *k,
                        int32_t n_groups, uint64_t *masks, int32_t *sel_idx, int32_t *new_offsets,
                        int32_t *status, int32_t *scratch, void *stream);

/* pg_ovf_select for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments less `scratch`, same results.  The block sums of the
 * offsets scan live in a device array inside the library (PG_OVF_NOALLOC_MAX_GROUPS / 2048 + 1 words, 8 KiB, one
 * copy per GPU for the life of the process), so at most PG_OVF_NOALLOC_MAX_GROUPS groups per call: more is
 * rejected with PG_ESHAPE before anything is launched.  The call allocates and frees nothing.  It runs on the
 * CURRENT device, which must be the stream's (else PG_EINVAL); the first call on a device looks the array's
 * address up (not under stream capture).  Every call on a GPU uses that GPU's one array: calls that overlap in
 * time on one GPU (different streams or threads) race; calls on one stream are ordered and safe. */
#define PG_OVF_NOALLOC_MAX_GROUPS 4194304
pg_status pg_ovf_select_noalloc(const float *rewards, const int32_t *group_offsets, const int32_t *k,
                                int32_t n_groups, uint64_t *masks, int32_t *sel_idx, int32_t *new_offsets,
                                int32_t *status, void *stream);

/* pg_ovf_select for groups of up to 1024 members (a generalisation: the paper's groups have at
 * most 64).  masks: [n_groups, mask_words] uint64, bit i of word w = slot 64 w + i, groups must
 * fit (size <= 64 * mask_words, 1 <= mask_words <= 16).  Same evaluation order, with the prefix
 * sums over 64 zero-padded slots up to 64 members and over the next power of two above that, so
 * groups of at most 64 members get exactly pg_ovf_select's answer. */
pg_status pg_ovf_select_large(const float *rewards, const int32_t *group_offsets, const int32_t *k,
                              int32_t n_groups, int32_t mask_words, uint64_t *masks,
                              int32_t *sel_idx, int32_t *new_offsets, int32_t *status,
                              int32_t *scratch, void *stream);

/* Uniformly random k-subset per ragged group (the subsampling arm of Sec. 4.1), same outputs and
 * status convention as pg_ovf_select.  Slot j of group g draws one 32-bit key, word 0 of the
 * Philox-4x32-10 block with counter (j, draw, g, 2) and key (seed low, seed high); the k[g] slots
 * with the smallest (key, slot) are kept. */
pg_status pg_uniform_select(const int32_t *group_offsets, const int32_t *k, int32_t n_groups,
                            uint64_t seed, uint32_t draw, uint64_t *masks, int32_t *sel_idx,
                            int32_t *new_offsets, int32_t *status, int32_t *scratch, void *stream);

/* Group diagnostics of Sec. 4.1 per ragged group (any size): sigma[g] = population standard
 * deviation of the group's rewards (fp64 inside), clustered_share[g] = share of members with
 * |R - mean| <= delta * sigma (the region C_delta of Eq. 7).  Either output may be NULL; an empty
 * group reports 0, 0. */
pg_status pg_group_stats(const float *rewards, const int32_t *group_offsets, int32_t n_groups,
                         double delta, float *sigma, float *clustered_share, void *stream);

/* out[r, :] = x[src[r], :] for r < n_out (ragged survivor compaction); out must not alias x;
 * d multiple of 4. */
pg_status pg_compact_gather(const float *x, float *out, const int32_t *src, int64_t n_out, int64_t d,
                            void *stream);

/* Eq. 5 / Eq. 18 per ragged group (sizes <= 64): population mean and std in fp64,
 * adv = (R - mu) / (sigma + eps). */
pg_status pg_group_advantages(const float *rewards, const int32_t *group_offsets, int32_t n_groups,
                              double eps, float *adv, void *stream);

/* C[M, N] = A[M, K] W[N, K]^T + bias (bf16 in, fp32 accumulate, fp32 out): the MFMA GEMM used by
 * the network, exposed for unit parity.  K multiple of 64; lda/ldw in elements. */
pg_status pg_gemm_bf16(const uint16_t *A, int64_t lda, const uint16_t *W, int64_t ldw,
                       const uint16_t *bias, float *C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                       void *stream);

/* Softmax attention on MFMA, exposed for unit parity: q [B, Lq, heads*hd], k [B, Lk, heads*hd]
 * row-major bf16; vt [B, heads*hd, Lk_pad] (values transposed, Lk_pad = Lk rounded up to 64);
 * out [B, Lq, heads*hd] bf16; hd 32 or 64; logits scaled by 1/sqrt(hd). */
pg_status pg_attention_bf16(const uint16_t *q, const uint16_t *k, const uint16_t *vt, uint16_t *out,
                            int32_t B, int32_t Lq, int32_t Lk, int32_t heads, int32_t hd,
                            void *stream);

/* ---- measurement hooks (process-wide, not thread-safe) ----
 * Between pg_profile_begin and pg_profile_end every launch of the heavy kernels is bracketed by a
 * pair of HIP events on the stream it is launched on (at most max_records launches are recorded).
 * pg_profile_read waits for the recorded events and returns, for one kind of kernel, the summed
 * durations [ms] (each less the duration an empty event pair reads on that stream, measured once at
 * the first bracket), the summed algorithmic work and the number of launches.
 * kind 0: MFMA GEMM (work = 2 M N K flops), 1: attention (4 B heads Lq Lk hd flops),
 * 2: fused update + log-prob (12 bytes per latent element), 3: preview / reward (8 or 4 bytes per element). */
pg_status pg_profile_begin(int32_t max_records);
pg_status pg_profile_read(int32_t kind, double *total_ms, double *total_work, int64_t *launches);
pg_status pg_profile_end(void);


/* Launches `blocks` workgroups of 256 lanes that each issue iters x 8 bf16 32x32x16 MFMAs per wave on registers
 * alone (no LDS, no memory traffic but one float per lane written to out, [device] blocks * 256 floats): the rate
 * the matrix pipes sustain on this part, the yardstick beside the published peak.  operand_scale 0 gives all-zero
 * operands, 1 gives values spread over [-1, 1].  *flops (nullable, [host]) receives the MFMA flop count. */
pg_status pg_mfma_probe(int32_t blocks, int32_t iters, float operand_scale, float *out, double *flops,
                        void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PROGRPO_H */
