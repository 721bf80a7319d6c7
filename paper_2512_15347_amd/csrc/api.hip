// Host side of the C ABI: configuration checks, per-step coefficient tables, buffer plan and the
// sequencing of the sampling loop (paper Sec. 5.1 and Sec. 5.2).  No device memory is allocated here.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include "ctx.hpp"

namespace pg {

static thread_local char g_err[512] = "";
char* error_buffer() { return g_err; }
pg_status fail(pg_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

struct ProfRec { int kind; double work; hipEvent_t a, b; bool closed; };
static std::vector<ProfRec> g_prof;
static bool g_prof_on = false;
static size_t g_prof_cap = 0;
static double g_prof_empty_ms = -1.0;    // duration an empty bracket reads (event processing), subtracted per record

// Median of a few back-to-back event pairs with nothing between them on this stream.
static void prof_calibrate(hipStream_t s) {
  g_prof_empty_ms = 0.0;
  float v[9];
  int n = 0;
  for (int i = 0; i < 9; ++i) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) break;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); break; }
    (void)hipEventRecord(a, s);
    (void)hipEventRecord(b, s);
    float t = 0.f;
    if (hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(&t, a, b) == hipSuccess) v[n++] = t;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
  }
  if (n > 0) { std::sort(v, v + n); g_prof_empty_ms = v[n / 2]; }
}

int prof_open(int kind, double work, hipStream_t s) {
  if (!g_prof_on || g_prof.size() >= g_prof_cap) return -1;
  if (g_prof_empty_ms < 0.0) prof_calibrate(s);
  ProfRec r{kind, work, nullptr, nullptr, false};
  if (hipEventCreate(&r.a) != hipSuccess) return -1;
  if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return -1; }
  (void)hipEventRecord(r.a, s);
  g_prof.push_back(r);
  return (int)g_prof.size() - 1;
}
void prof_close(int rec, hipStream_t s) {
  if (rec < 0 || rec >= (int)g_prof.size()) return;
  (void)hipEventRecord(g_prof[rec].b, s);
  g_prof[rec].closed = true;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// ---- per-step scalars of x' = A x + B u + C xi and x_hat = P x + Q u ----

// Rectified flow (Eq. 3) read with tau = noise fraction going 1 -> 0 and v = dx/dtau: the marginal
// preserving reverse SDE (Eq. 4, RF case of Eq. 12) has drift v + sigma^2/(2 tau) (x + (1-tau) v).
static void flow_tables(pg_ctx* c) {
  const int T = c->cfg.T;
  const double a = c->cfg.noise_level;
  for (int s = 0; s < T; ++s) {
    const double tau = 1.0 - (double)s / T, tau_next = 1.0 - (double)(s + 1) / T;
    const double dt = tau_next - tau;
    const double sig2 = a * a * tau / std::max(1.0 - tau, 1.0 / T);
    c->A[s] = 1.0 + sig2 * dt / (2.0 * tau);
    c->B[s] = dt * (1.0 + sig2 * (1.0 - tau) / (2.0 * tau));
    c->C[s] = std::sqrt(sig2 * std::fabs(dt));
    c->Pv[s] = 1.0;          // Eq. 15: x + (remaining time) * v with remaining time = -tau
    c->Qv[s] = -tau;
    c->tin[s] = 1000.0 * tau;
  }
}

// DDIM(eta) posterior step on a linear beta table (discretisation of Eq. 2 / diffusion case of Eq. 12).
static void ddim_tables(pg_ctx* c) {
  const int S = c->cfg.T, Tt = c->cfg.T_train;
  std::vector<double> abar(Tt);
  double run = 1.0;
  for (int i = 0; i < Tt; ++i) {
    const double beta = (Tt == 1) ? c->cfg.beta0
                                  : c->cfg.beta0 + (c->cfg.beta1 - c->cfg.beta0) * (double)i / (Tt - 1);
    run *= 1.0 - beta;
    abar[i] = run;
  }
  auto tstep = [&](int i) { return (int)(((int64_t)(S - i) * (Tt - 1) + S / 2) / S); };
  const double eta = c->cfg.eta;
  for (int i = 0; i < S; ++i) {
    const double at = abar[tstep(i)], ap = abar[tstep(i + 1)];
    const double s2 = eta * eta * (1.0 - ap) / (1.0 - at) * (1.0 - at / ap);
    c->A[i] = std::sqrt(ap / at);
    c->B[i] = std::sqrt(1.0 - ap - s2) - std::sqrt(ap * (1.0 - at) / at);
    c->C[i] = std::sqrt(s2);
    c->Pv[i] = 1.0 / std::sqrt(at);               // preview = predicted clean latent
    c->Qv[i] = -std::sqrt((1.0 - at) / at);
    c->tin[i] = (double)tstep(i);
  }
}

static pg_status build_weight_layout(pg_ctx* c) {
  const pg_config& f = c->cfg;
  c->top.assign(PG_W_COUNT, WeightSlot{-1, 0, 0, 0});
  if (f.net_kind == PG_NET_NONE) { c->weights_numel = 0; return PG_OK; }
  const int D = f.D, C4 = 4 * f.C;
  int64_t off = 0;
  auto put = [&](int id, int rows, int cols) {
    const int ld = rows > 1 ? ((cols + 63) / 64) * 64 : cols;
    c->top[id] = WeightSlot{off, rows, cols, ld};
    off += ((int64_t)rows * ld + 127) / 128 * 128;
  };
  put(PG_W_PE_W, D, C4); put(PG_W_PE_B, 1, D); put(PG_W_POS, c->Li, D);
  put(PG_W_T_W1, D, 256); put(PG_W_T_B1, 1, D); put(PG_W_T_W2, D, D); put(PG_W_T_B2, 1, D);
  if (f.net_kind == PG_NET_JOINT || f.net_kind == PG_NET_MMDIT) { put(PG_W_CTX_W, D, f.Dc); put(PG_W_CTX_B, 1, D); }
  put(PG_W_FMOD_W, 2 * D, D); put(PG_W_FMOD_B, 1, 2 * D); put(PG_W_F_W, C4, D); put(PG_W_F_B, 1, C4);
  const int64_t block0 = off;
  put(PG_W_MOD_W, 6 * D, D); put(PG_W_MOD_B, 1, 6 * D); put(PG_W_QKV_W, 3 * D, D); put(PG_W_QKV_B, 1, 3 * D);
  put(PG_W_O_W, D, D); put(PG_W_O_B, 1, D); put(PG_W_FC1_W, 4 * D, D); put(PG_W_FC1_B, 1, 4 * D);
  put(PG_W_FC2_W, D, 4 * D); put(PG_W_FC2_B, 1, D);
  if (f.net_kind == PG_NET_CROSS) {
    put(PG_W_CQ_W, D, D); put(PG_W_CQ_B, 1, D); put(PG_W_CKV_W, 2 * D, f.Dc); put(PG_W_CKV_B, 1, 2 * D);
    put(PG_W_CO_W, D, D); put(PG_W_CO_B, 1, D);
  }
  if (f.net_kind == PG_NET_MMDIT) {
    const int hd = D / f.heads;
    put(PG_W_C_MOD_W, 6 * D, D); put(PG_W_C_MOD_B, 1, 6 * D); put(PG_W_C_QKV_W, 3 * D, D); put(PG_W_C_QKV_B, 1, 3 * D);
    put(PG_W_C_O_W, D, D); put(PG_W_C_O_B, 1, D); put(PG_W_C_FC1_W, 4 * D, D); put(PG_W_C_FC1_B, 1, 4 * D);
    put(PG_W_C_FC2_W, D, 4 * D); put(PG_W_C_FC2_B, 1, D);
    put(PG_W_QN_G, 1, hd); put(PG_W_KN_G, 1, hd); put(PG_W_C_QN_G, 1, hd); put(PG_W_C_KN_G, 1, hd);
  }
  c->block_stride = off - block0;
  c->weights_numel = block0 + c->block_stride * f.blocks;
  return PG_OK;
}

static pg_status validate(const pg_config& f) {
  if (f.P < 1 || f.N < 1 || f.C < 1 || f.H < 2 || f.W < 2 || f.T < 1)
    return fail(PG_EINVAL, "P, N, C, T must be >= 1 and H, W >= 2");
  if (f.N > 64) return fail(PG_ESHAPE, "group size N = %d exceeds 64 (one wavefront per group)", f.N);
  if ((f.H & 1) || (f.W & 1)) return fail(PG_ESHAPE, "H and W must be even (patch size 2)");
  if ((int64_t)f.P * f.N > (1 << 24)) return fail(PG_ESHAPE, "too many trajectories");
  if (!(f.adv_eps > 0.0)) return fail(PG_EINVAL, "adv_eps must be > 0 (Eq. 18)");
  switch (f.sampler_kind) {
    case PG_SAMPLER_FLOW:
      if (!(f.noise_level > 0.0)) return fail(PG_EINVAL, "flow noise level must be > 0: every step needs a log-prob");
      break;
    case PG_SAMPLER_DDIM:
      if (!(f.eta > 0.0)) return fail(PG_EINVAL, "eta must be > 0: every step needs a log-prob");
      if (!(f.beta0 > 0.0 && f.beta0 <= f.beta1 && f.beta1 < 1.0)) return fail(PG_EINVAL, "need 0 < beta0 <= beta1 < 1");
      if (f.T_train < f.T + 1) return fail(PG_EINVAL, "T_train = %d must exceed T = %d", f.T_train, f.T);
      break;
    case PG_SAMPLER_TABLE:
      if (!f.tab_A || !f.tab_B || !f.tab_C || !f.tab_P || !f.tab_Q || !f.tab_tin)
        return fail(PG_EINVAL, "PG_SAMPLER_TABLE needs all six tables");
      for (int s = 0; s < f.T; ++s)
        if (!(f.tab_C[s] > 0.0)) return fail(PG_EINVAL, "tab_C[%d] must be > 0", s);
      break;
    default: return fail(PG_EINVAL, "unknown sampler_kind %d", f.sampler_kind);
  }
  if (f.net_kind != PG_NET_NONE) {
    if (f.net_kind < PG_NET_ADALN || f.net_kind > PG_NET_MMDIT) return fail(PG_EINVAL, "unknown net_kind %d", f.net_kind);
    if (f.D < 64 || f.D % 64) return fail(PG_ESHAPE, "width D = %d must be a positive multiple of 64", f.D);
    if (f.blocks < 1 || f.heads < 1 || f.D % f.heads) return fail(PG_ESHAPE, "heads must divide D, blocks >= 1");
    const int hd = f.D / f.heads;
    if (hd != 32 && hd != 64) return fail(PG_ESHAPE, "head width %d not supported (32 or 64)", hd);
    if (f.net_kind == PG_NET_ADALN) {
      if (f.Lc != 0) return fail(PG_EINVAL, "PG_NET_ADALN takes no context tokens");
    } else {
      if (f.Lc < 1) return fail(PG_EINVAL, "context variants need Lc >= 1");
      if (f.Dc < 64 || f.Dc % 64) return fail(PG_ESHAPE, "context width Dc = %d must be a positive multiple of 64", f.Dc);
    }
  }
  if (f.n_sched < 0 || (f.n_sched > 0 && (!f.sched_group || !f.sched_step || !f.sched_k)))
    return fail(PG_EINVAL, "schedule arrays missing");
  return PG_OK;
}

static pg_status plan_workspace(pg_ctx* c) {
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off = align256(off + bytes); return o; };
  c->ws_partials = take(2 * sizeof(float) * (size_t)c->M0 * chunks_per_traj(c->d));   // two sums per workgroup at most
  c->ws_k = take(sizeof(int32_t) * c->cfg.P);
  c->ws_newoff = take(sizeof(int32_t) * (c->cfg.P + 1));
  c->ws_forced = take(sizeof(uint64_t) * c->cfg.P + sizeof(int32_t) * c->M0);   // masks + sel of the OVF shadow run
  c->ws_sched = take(sizeof(int32_t) * c->sched_table.size());                  // the funnel, uploaded by pg_bind
  c->ws_off0 = take(sizeof(int32_t) * (c->cfg.P + 1));                          // offsets of the full groups
  c->ws_logr = take(sizeof(double) * (size_t)c->cfg.T * c->M0);                 // fp64 log-ratios of pg_policy_ratio
  c->ws_net = off;
  PG_TRY(net_plan(c));
  c->ws_total = align256(off + c->net.total);
  return PG_OK;
}

}  // namespace pg

using namespace pg;

extern "C" const char* pg_last_error(void) { return error_buffer(); }

extern "C" pg_status pg_profile_begin(int32_t max_records) {
  if (max_records < 1) return fail(PG_EINVAL, "pg_profile_begin: max_records = %d", max_records);
  for (auto& r : g_prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  g_prof.clear();
  g_prof.reserve(max_records);
  g_prof_cap = (size_t)max_records;
  g_prof_empty_ms = -1.0;
  g_prof_on = true;
  return PG_OK;
}

extern "C" pg_status pg_profile_read(int32_t kind, double* total_ms, double* total_work, int64_t* launches) {
  if (kind < 0 || kind >= PROF_KINDS) return fail(PG_EINVAL, "pg_profile_read: kind %d", kind);
  double ms = 0.0, work = 0.0;
  int64_t n = 0;
  for (auto& r : g_prof) {
    if (r.kind != kind || !r.closed) continue;
    PG_HIP(hipEventSynchronize(r.b));
    float t = 0.f;
    PG_HIP(hipEventElapsedTime(&t, r.a, r.b));
    ms += std::max(0.0, (double)t - std::max(0.0, g_prof_empty_ms)); work += r.work; ++n;
  }
  if (total_ms) *total_ms = ms;
  if (total_work) *total_work = work;
  if (launches) *launches = n;
  return PG_OK;
}

extern "C" pg_status pg_profile_end(void) {
  g_prof_on = false;
  for (auto& r : g_prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  g_prof.clear();
  g_prof_cap = 0;
  return PG_OK;
}

extern "C" pg_status pg_create(const pg_config* cfg, pg_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) return fail(PG_EINVAL, "pg_create: null argument");
  PG_TRY(validate(*cfg));
  pg_ctx* c = new (std::nothrow) pg_ctx();
  if (!c) return fail(PG_EINVAL, "out of host memory");
  c->cfg = *cfg;
  const pg_config& f = c->cfg;
  c->d = f.C * f.H * f.W;
  c->Li = (f.H / 2) * (f.W / 2);
  c->L = c->Li + (f.net_kind == PG_NET_JOINT || f.net_kind == PG_NET_MMDIT ? f.Lc : 0);
  c->M0 = f.P * f.N;
  const int T = f.T;
  c->A.resize(T); c->B.resize(T); c->C.resize(T); c->Pv.resize(T); c->Qv.resize(T); c->tin.resize(T);
  if (f.sampler_kind == PG_SAMPLER_FLOW) flow_tables(c);
  else if (f.sampler_kind == PG_SAMPLER_DDIM) ddim_tables(c);
  else
    for (int s = 0; s < T; ++s) {
      c->A[s] = f.tab_A[s]; c->B[s] = f.tab_B[s]; c->C[s] = f.tab_C[s];
      c->Pv[s] = f.tab_P[s]; c->Qv[s] = f.tab_Q[s]; c->tin[s] = f.tab_tin[s];
    }
  for (int s = 0; s < T; ++s)
    if (!(c->C[s] > 0.0) || !std::isfinite(c->A[s]) || !std::isfinite(c->B[s])) {
      delete c;
      return fail(PG_EINVAL, "step %d has a non-positive noise scale or non-finite coefficients", s);
    }
  // schedule: per group, steps strictly increasing, counts strictly decreasing below N (Sec. 5.2)
  c->sched.assign(f.P, {});
  c->is_checkpoint.assign(T, 0);
  for (int i = 0; i < f.n_sched; ++i) {
    const int g = f.sched_group[i], s = f.sched_step[i], k = f.sched_k[i];
    if (g < 0 || g >= f.P || s < 0 || s >= T || k < 1) {
      delete c;
      return fail(PG_ESCHED, "schedule entry %d (group %d, step %d, k %d) out of range", i, g, s, k);
    }
    c->sched[g].push_back({s, k});
    c->is_checkpoint[s] = 1;
  }
  for (int g = 0; g < f.P; ++g) {
    std::sort(c->sched[g].begin(), c->sched[g].end());
    int prev_k = f.N, prev_s = -1;
    for (auto& e : c->sched[g]) {
      if (e.first == prev_s || e.second >= prev_k) {
        delete c;
        return fail(PG_ESCHED, "group %d: survivor counts must strictly decrease at distinct steps", g);
      }
      prev_s = e.first; prev_k = e.second;
    }
  }
  // the funnel when every prune follows the schedule: row s = counts kept at step s | their exclusive scan
  {
    const int P = f.P, row = 2 * P + 1;
    c->sched_table.assign((size_t)T * row, 0);
    std::vector<int> size(P, f.N);
    for (int s = 0; s < T; ++s) {
      int32_t* k = c->sched_table.data() + (size_t)s * row;
      int32_t* off = k + P;
      for (int g = 0; g < P; ++g) {
        k[g] = size[g];
        for (auto& e : c->sched[g]) if (e.first == s) k[g] = e.second;
        off[g + 1] = off[g] + k[g];
        size[g] = k[g];
      }
    }
  }
  // nullify host pointers we must not keep
  c->cfg.tab_A = c->cfg.tab_B = c->cfg.tab_C = c->cfg.tab_P = c->cfg.tab_Q = c->cfg.tab_tin = nullptr;
  c->cfg.sched_group = c->cfg.sched_step = c->cfg.sched_k = nullptr;
  pg_status st = build_weight_layout(c);
  if (st == PG_OK) st = plan_workspace(c);
  if (st != PG_OK) { delete c; return st; }
  c->offsets.assign(f.P + 1, 0);
  *out = c;
  return PG_OK;
}

extern "C" void pg_destroy(pg_ctx* c) {
  if (!c) return;
  if (c->staging) (void)hipHostFree(c->staging);
  if (c->staging_read) (void)hipEventDestroy(c->staging_read);
  delete c;
}

extern "C" size_t pg_workspace_bytes(const pg_ctx* c) { return c ? c->ws_total : 0; }
extern "C" int64_t pg_weights_numel(const pg_ctx* c) { return c ? c->weights_numel : 0; }

extern "C" pg_status pg_weight_slot(const pg_ctx* c, int32_t id, int32_t block, int64_t* offset,
                                    int32_t* rows, int32_t* cols, int32_t* ld) {
  if (!c || id < 0 || id >= PG_W_COUNT) return fail(PG_EINVAL, "pg_weight_slot: bad id");
  const WeightSlot& w = c->top[id];
  if (w.offset < 0) return fail(PG_EINVAL, "tensor %d does not exist for this network", id);
  int64_t off = w.offset;
  if (id >= PG_W_MOD_W) {
    if (block < 0 || block >= c->cfg.blocks) return fail(PG_EINVAL, "block %d out of range", block);
    off += c->block_stride * block;
  }
  if (offset) *offset = off;
  if (rows) *rows = w.rows;
  if (cols) *cols = w.cols;
  if (ld) *ld = w.ld;
  return PG_OK;
}

extern "C" pg_status pg_get_tables(const pg_ctx* c, double* A, double* B, double* C, double* P, double* Q,
                                   double* t_in) {
  if (!c) return fail(PG_EINVAL, "pg_get_tables: null context");
  const size_t n = sizeof(double) * c->cfg.T;
  if (A) memcpy(A, c->A.data(), n);
  if (B) memcpy(B, c->B.data(), n);
  if (C) memcpy(C, c->C.data(), n);
  if (P) memcpy(P, c->Pv.data(), n);
  if (Q) memcpy(Q, c->Qv.data(), n);
  if (t_in) memcpy(t_in, c->tin.data(), n);
  return PG_OK;
}

extern "C" pg_status pg_get_schedule(const pg_ctx* c, int32_t step, int32_t* k, int32_t* offsets) {
  if (!c) return fail(PG_EINVAL, "pg_get_schedule: null context");
  if (step < 0 || step >= c->cfg.T) return fail(PG_EINVAL, "step %d out of range", step);
  const int P = c->cfg.P;
  const int32_t* row = c->sched_table.data() + (size_t)step * (2 * P + 1);
  if (k) memcpy(k, row, sizeof(int32_t) * P);
  if (offsets) memcpy(offsets, row + P, sizeof(int32_t) * (P + 1));
  return PG_OK;
}

extern "C" pg_status pg_bind(pg_ctx* c, const pg_buffers* b) {
  if (!c || !b) return fail(PG_EINVAL, "pg_bind: null argument");
  c->bound = false;
  if (!b->x[0] || !b->x[1] || !b->u || !b->orig_id[0] || !b->orig_id[1] || !b->group_offsets ||
      !b->group_of || !b->rewards || !b->masks || !b->sel_idx || !b->logp_hist || !b->logp_sum || !b->adv ||
      !b->probe_w || !b->status)
    return fail(PG_EINVAL, "pg_bind: a required buffer is NULL");
  if (b->x[0] == b->x[1] || b->orig_id[0] == b->orig_id[1]) return fail(PG_EINVAL, "pg_bind: ping-pong buffers alias");
  if (c->cfg.net_kind != PG_NET_NONE && (!b->weights || !b->y)) return fail(PG_EINVAL, "pg_bind: weights / y missing");
  if (c->cfg.net_kind >= PG_NET_CROSS && !b->ctx) return fail(PG_EINVAL, "pg_bind: ctx missing");
  if (!b->workspace || b->workspace_bytes < c->ws_total)
    return fail(PG_EWORKSPACE, "workspace of %zu bytes given, %zu needed", b->workspace_bytes, c->ws_total);
  if (((uintptr_t)b->workspace & 255) || ((uintptr_t)b->x[0] & 15) || ((uintptr_t)b->x[1] & 15) ||
      ((uintptr_t)b->u & 15) || ((uintptr_t)b->probe_w & 15) || ((uintptr_t)b->weights & 15) ||
      ((uintptr_t)b->ctx & 15))
    return fail(PG_ESHAPE, "pg_bind: buffers must be 16-byte aligned (workspace 256)");
  if (!c->staging)
    PG_HIP(hipHostMalloc((void**)&c->staging, (size_t)(2 * c->cfg.P + 1) * sizeof(int32_t), hipHostMallocDefault));
  if (!c->staging_read) PG_HIP(hipEventCreateWithFlags(&c->staging_read, hipEventDisableTiming));
  c->buf = *b;
  // the schedule's counts and offsets live in the workspace from here on (synchronous copies: pg_bind is set-up)
  {
    std::vector<int32_t> off0(c->cfg.P + 1);
    for (int g = 0; g <= c->cfg.P; ++g) off0[g] = g * c->cfg.N;
    PG_HIP(hipMemcpy((char*)b->workspace + c->ws_sched, c->sched_table.data(), sizeof(int32_t) * c->sched_table.size(),
                     hipMemcpyHostToDevice));
    PG_HIP(hipMemcpy((char*)b->workspace + c->ws_off0, off0.data(), sizeof(int32_t) * off0.size(), hipMemcpyHostToDevice));
  }
  c->bound = true;
  c->initialised = false;
  c->context_ready = false;
  return PG_OK;
}

extern "C" pg_status pg_state(const pg_ctx* c, int32_t* M, int32_t* cur_x, int32_t* cur_id,
                              int32_t* offsets, int64_t* evals, int64_t* updates) {
  if (!c) return fail(PG_EINVAL, "pg_state: null context");
  if (M) *M = c->M;
  if (cur_x) *cur_x = c->cur_x;
  if (cur_id) *cur_id = c->cur_id;
  if (offsets) memcpy(offsets, c->offsets.data(), sizeof(int32_t) * (c->cfg.P + 1));
  if (evals) *evals = c->evals;
  if (updates) *updates = c->updates;
  return PG_OK;
}

static char* ws(pg_ctx* c, size_t off) { return (char*)c->buf.workspace + off; }

extern "C" pg_status pg_init_group(pg_ctx* c, uint64_t seed, void* stream) {
  if (!c || !c->bound) return fail(PG_EINVAL, "pg_init_group: context not bound");
  hipStream_t s = (hipStream_t)stream;
  const pg_config& f = c->cfg;
  c->seed = seed;
  c->M = c->M0; c->cur_x = 0; c->cur_id = 0;
  c->pending_gather = false; c->net_fresh = false;
  c->evals = 0; c->updates = 0; c->steps_done = 0; c->advantages_done = false;
  for (int g = 0; g <= f.P; ++g) c->offsets[g] = g * f.N;
  PG_HIP(hipMemcpyAsync(c->buf.group_offsets, ws(c, c->ws_off0), sizeof(int32_t) * (f.P + 1), hipMemcpyDeviceToDevice, s));
  PG_TRY(launch_iota(c->buf.orig_id[0], c->M0, s));
  PG_TRY(launch_fill_group_of(c->buf.group_offsets, f.P, c->buf.group_of, s));
  PG_TRY(launch_fill_u32(c->buf.logp_hist, 0x7FC00000u, (size_t)f.T * c->M0, s));
  PG_TRY(launch_fill_u32(c->buf.logp_sum, 0u, (size_t)c->M0, s));
  PG_TRY(launch_fill_u32(c->buf.status, 0u, 4, s));
  PG_TRY(pg_init_latents(c->buf.x[0], c->buf.orig_id[0], c->M0, c->d, seed, stream));
  if (c->buf.x_hist)
    PG_HIP(hipMemcpyAsync(c->buf.x_hist, c->buf.x[0], sizeof(float) * (size_t)c->M0 * c->d, hipMemcpyDeviceToDevice, s));
  if (f.net_kind != PG_NET_NONE && !c->context_ready) {
    PG_TRY(net_prepare(c, c->buf.weights, s));
    c->context_ready = true;
  }
  c->initialised = true;
  return PG_OK;
}

extern "C" pg_status pg_net_forward(pg_ctx* c, int32_t step, void* stream) {
  if (!c || !c->bound || !c->initialised) return fail(PG_ESCHED, "pg_net_forward: call pg_init_group first");
  if (step < 0 || step >= c->cfg.T) return fail(PG_EINVAL, "step %d out of range", step);
  if (step != c->steps_done) return fail(PG_ESCHED, "pg_net_forward: step %d out of order (next is %d)", step, c->steps_done);
  if (c->pending_gather) return fail(PG_ESCHED, "pg_net_forward: a prune is waiting for its pg_step");
  if (c->cfg.net_kind != PG_NET_NONE)
    PG_TRY(net_forward(c, step, c->buf.x[c->cur_x], c->buf.weights, (hipStream_t)stream));
  c->net_fresh = true;
  c->evals += c->M;
  return PG_OK;
}

// shared tail of pg_prune / pg_prune_forced once sel_idx is on the device; new_off_dev: the new offsets [device]
static pg_status finish_prune(pg_ctx* c, const std::vector<int>& new_off, const int32_t* new_off_dev, hipStream_t s) {
  const int P = c->cfg.P;
  const int M_new = new_off[P];
  PG_TRY(launch_gather_ids(c->buf.orig_id[c->cur_id], c->buf.sel_idx, M_new, c->buf.orig_id[1 - c->cur_id], s));
  c->cur_id = 1 - c->cur_id;
  PG_HIP(hipMemcpyAsync(c->buf.group_offsets, new_off_dev, sizeof(int32_t) * (P + 1), hipMemcpyDeviceToDevice, s));
  PG_TRY(launch_fill_group_of(c->buf.group_offsets, P, c->buf.group_of, s));
  c->offsets = new_off;
  c->M = M_new;
  c->pending_gather = true;
  return PG_OK;
}

static pg_status prune_common(pg_ctx* c, int step, const uint64_t* forced, uint64_t* ovf_masks_out,
                              hipStream_t s) {
  if (!c || !c->bound || !c->initialised) return fail(PG_ESCHED, "pg_prune: call pg_init_group first");
  const pg_config& f = c->cfg;
  if (step < 0 || step >= f.T) return fail(PG_EINVAL, "step %d out of range", step);
  if (step != c->steps_done) return fail(PG_ESCHED, "pg_prune: step %d out of order (next is %d)", step, c->steps_done);
  if (!c->net_fresh) return fail(PG_ESCHED, "pg_prune: no network evaluation for the current latents");
  if (c->pending_gather) return fail(PG_ESCHED, "pg_prune: previous prune not yet consumed by pg_step");
  const int P = f.P;
  std::vector<int> k(P), new_off(P + 1, 0);
  bool any = false;
  for (int g = 0; g < P; ++g) {
    const int n = c->offsets[g + 1] - c->offsets[g];
    k[g] = n;
    for (auto& e : c->sched[g]) if (e.first == step) { k[g] = e.second; any = true; }
    if (k[g] > n) {
      if (!forced) return fail(PG_ESCHED, "group %d holds %d trajectories, schedule asks for %d", g, n, k[g]);
      k[g] = n;
    }
  }
  if (!any && !forced) return fail(PG_ESCHED, "step %d is not a checkpoint of any group", step);
  for (int g = 0; g < P; ++g) new_off[g + 1] = new_off[g] + k[g];
  // Counts and new offsets on the device: the row of the funnel table that pg_bind uploaded, whenever the group
  // sizes are those of the schedule (always, unless a forced prune has departed from it).  Otherwise, and only
  // then, they go up synchronously.
  const int32_t* row = c->sched_table.data() + (size_t)step * (2 * P + 1);
  const bool on_schedule = std::equal(k.begin(), k.end(), row) && std::equal(new_off.begin(), new_off.end(), row + P);
  const int32_t* k_dev = (const int32_t*)ws(c, c->ws_sched) + (size_t)step * (2 * P + 1);
  const int32_t* off_dev = k_dev + P;
  if (!on_schedule) {
    PG_HIP(hipStreamSynchronize(s));
    PG_HIP(hipMemcpy(ws(c, c->ws_k), k.data(), sizeof(int32_t) * P, hipMemcpyHostToDevice));
    PG_HIP(hipMemcpy(ws(c, c->ws_newoff), new_off.data(), sizeof(int32_t) * (P + 1), hipMemcpyHostToDevice));
    k_dev = (const int32_t*)ws(c, c->ws_k);
    off_dev = (const int32_t*)ws(c, c->ws_newoff);
  }
  PG_TRY(pg_preview_reward(c->buf.x[c->cur_x], c->buf.u, c->buf.probe_w, c->buf.rewards, c->M, c->d,
                           c->Pv[step], c->Qv[step], f.probe_bias, (float*)ws(c, c->ws_partials), s));
  if (!forced) {
    PG_TRY(launch_ovf(c->buf.rewards, c->buf.group_offsets, k_dev, P, off_dev, c->buf.masks, c->buf.sel_idx,
                      c->buf.status, s));
    return finish_prune(c, new_off, off_dev, s);
  }
  // forced survivors: run the OVF into shadow buffers (for the record), then impose the masks
  uint64_t* shadow_masks = (uint64_t*)ws(c, c->ws_forced);
  int32_t* shadow_sel = (int32_t*)(ws(c, c->ws_forced) + sizeof(uint64_t) * P);
  PG_TRY(launch_ovf(c->buf.rewards, c->buf.group_offsets, k_dev, P, off_dev, shadow_masks, shadow_sel,
                    c->buf.status, s));
  if (ovf_masks_out)
    PG_HIP(hipMemcpyAsync(ovf_masks_out, shadow_masks, sizeof(uint64_t) * P, hipMemcpyDeviceToDevice, s));
  for (int g = 0; g < P; ++g) {
    const int n = c->offsets[g + 1] - c->offsets[g];
    const uint64_t valid = (n == 64) ? ~0ull : ((1ull << n) - 1ull);
    if (forced[g] & ~valid) return fail(PG_EINVAL, "forced mask of group %d names slots beyond its %d members", g, n);
    const int cnt = __builtin_popcountll(forced[g]);
    if (cnt < 1) return fail(PG_EINVAL, "forced mask of group %d is empty", g);
    new_off[g + 1] = new_off[g] + cnt;
  }
  PG_HIP(hipStreamSynchronize(s));     // test hook: plain synchronous uploads from caller memory
  PG_HIP(hipMemcpy(c->buf.masks, forced, sizeof(uint64_t) * P, hipMemcpyHostToDevice));
  PG_HIP(hipMemcpy(ws(c, c->ws_newoff), new_off.data(), sizeof(int32_t) * (P + 1), hipMemcpyHostToDevice));
  PG_TRY(launch_masks_to_sel(c->buf.masks, c->buf.group_offsets, (int32_t*)ws(c, c->ws_newoff), P,
                             c->buf.sel_idx, s));
  return finish_prune(c, new_off, (const int32_t*)ws(c, c->ws_newoff), s);
}

extern "C" pg_status pg_prune(pg_ctx* c, int32_t step, void* stream) {
  return prune_common(c, step, nullptr, nullptr, (hipStream_t)stream);
}

extern "C" pg_status pg_prune_forced(pg_ctx* c, int32_t step, const uint64_t* masks, uint64_t* ovf_masks_out,
                                     void* stream) {
  if (!masks) return fail(PG_EINVAL, "pg_prune_forced: masks is NULL");
  return prune_common(c, step, masks, ovf_masks_out, (hipStream_t)stream);
}

extern "C" pg_status pg_step(pg_ctx* c, int32_t step, void* stream) {
  if (!c || !c->bound || !c->initialised) return fail(PG_ESCHED, "pg_step: call pg_init_group first");
  if (step < 0 || step >= c->cfg.T) return fail(PG_EINVAL, "step %d out of range", step);
  if (!c->net_fresh) return fail(PG_ESCHED, "pg_step: no network evaluation for the current latents");
  if (step != c->steps_done) return fail(PG_ESCHED, "pg_step: step %d out of order (next is %d)", step, c->steps_done);
  if (c->is_checkpoint[step] && !c->pending_gather) {
    // a group whose schedule has an entry here and that still holds more than that entry keeps must be pruned first
    for (int g = 0; g < c->cfg.P; ++g)
      for (auto& e : c->sched[g])
        if (e.first == step && c->offsets[g + 1] - c->offsets[g] > e.second)
          return fail(PG_ESCHED, "pg_step: step %d is a checkpoint of group %d; call pg_prune first", step, g);
  }
  float* hist_next = c->buf.x_hist ? c->buf.x_hist + (size_t)(step + 1) * c->M0 * c->d : nullptr;
  PG_TRY(launch_sde_step(c->buf.x[c->cur_x], c->buf.u, c->buf.x[1 - c->cur_x], nullptr,
                         c->buf.logp_hist + (size_t)step * c->M0, c->buf.logp_sum,
                         c->pending_gather ? c->buf.sel_idx : nullptr, c->buf.orig_id[c->cur_id], c->M, c->d,
                         c->A[step], c->B[step], c->C[step], c->seed, (uint32_t)step,
                         (float*)ws(c, c->ws_partials), hist_next, (hipStream_t)stream));
  c->steps_done = step + 1;
  c->cur_x = 1 - c->cur_x;
  c->pending_gather = false;
  c->net_fresh = false;
  c->updates += c->M;
  return PG_OK;
}

extern "C" pg_status pg_advantages(pg_ctx* c, void* stream) {
  if (!c || !c->bound || !c->initialised) return fail(PG_ESCHED, "pg_advantages: call pg_init_group first");
  if (c->pending_gather) return fail(PG_ESCHED, "pg_advantages: a prune is waiting for its pg_step");
  if (c->steps_done != c->cfg.T)
    return fail(PG_ESCHED, "pg_advantages: %d of %d steps taken (Eq. 18 is on the final latents)", c->steps_done, c->cfg.T);
  PG_TRY(pg_preview_reward(c->buf.x[c->cur_x], nullptr, c->buf.probe_w, c->buf.rewards, c->M, c->d, 1.0, 0.0,
                           c->cfg.probe_bias, (float*)ws(c, c->ws_partials), stream));
  PG_TRY(pg_group_advantages(c->buf.rewards, c->buf.group_offsets, c->cfg.P, c->cfg.adv_eps, c->buf.adv, stream));
  c->advantages_done = true;
  return PG_OK;
}

// Comparison arms of Sec. 4.1-4.2 on a finished run: select on the FINAL rewards (mode 0: Optimal Variance
// Filtering applied once after sampling, mode 1: a uniformly random k-subset), pack the kept trajectories
// and recompute Eq. 18 on them.
extern "C" pg_status pg_select_final(pg_ctx* c, int32_t mode, const int32_t* k_per_group, uint32_t draw, void* stream) {
  if (!c || !c->bound || !c->initialised) return fail(PG_ESCHED, "pg_select_final: call pg_init_group first");
  if (!c->advantages_done) return fail(PG_ESCHED, "pg_select_final: call pg_advantages first (final rewards)");
  if (mode != 0 && mode != 1) return fail(PG_EINVAL, "pg_select_final: mode %d (0: OVF, 1: uniform)", mode);
  if (!k_per_group) return fail(PG_EINVAL, "pg_select_final: k_per_group is NULL");
  hipStream_t s = (hipStream_t)stream;
  const int P = c->cfg.P;
  std::vector<int> new_off(P + 1, 0);
  for (int g = 0; g < P; ++g) {
    const int n = c->offsets[g + 1] - c->offsets[g];
    if (k_per_group[g] < 1 || k_per_group[g] > n)
      return fail(PG_EINVAL, "pg_select_final: k = %d for group %d of %d trajectories", k_per_group[g], g, n);
    new_off[g + 1] = new_off[g] + k_per_group[g];
  }
  // the counts go up through the pinned slot; a copy of an earlier call that is still queued must have read
  // the slot before it is written again
  if (c->staging_in_flight) PG_HIP(hipEventSynchronize(c->staging_read));
  int32_t* slot = c->staging;
  memcpy(slot, k_per_group, sizeof(int32_t) * P);
  memcpy(slot + P, new_off.data(), sizeof(int32_t) * (P + 1));
  PG_HIP(hipMemcpyAsync(ws(c, c->ws_k), slot, sizeof(int32_t) * P, hipMemcpyHostToDevice, s));
  PG_HIP(hipMemcpyAsync(ws(c, c->ws_newoff), slot + P, sizeof(int32_t) * (P + 1), hipMemcpyHostToDevice, s));
  PG_HIP(hipEventRecord(c->staging_read, s));
  c->staging_in_flight = true;
  if (mode == 0)
    PG_TRY(launch_ovf(c->buf.rewards, c->buf.group_offsets, (int32_t*)ws(c, c->ws_k), P,
                      (int32_t*)ws(c, c->ws_newoff), c->buf.masks, c->buf.sel_idx, c->buf.status, s));
  else
    PG_TRY(launch_uniform_select(c->buf.group_offsets, (int32_t*)ws(c, c->ws_k), P, (int32_t*)ws(c, c->ws_newoff),
                                 c->seed, draw, c->buf.masks, c->buf.sel_idx, c->buf.status, s));
  const int M_new = new_off[P];
  PG_TRY(pg_compact_gather(c->buf.x[c->cur_x], c->buf.x[1 - c->cur_x], c->buf.sel_idx, M_new, c->d, stream));
  c->cur_x = 1 - c->cur_x;
  // rewards are gathered as 32-bit patterns through scratch
  int32_t* tmp = (int32_t*)ws(c, c->ws_partials);
  PG_TRY(launch_gather_ids((const int32_t*)c->buf.rewards, c->buf.sel_idx, M_new, tmp, s));
  PG_HIP(hipMemcpyAsync(c->buf.rewards, tmp, sizeof(float) * M_new, hipMemcpyDeviceToDevice, s));
  PG_TRY(launch_gather_ids(c->buf.orig_id[c->cur_id], c->buf.sel_idx, M_new, c->buf.orig_id[1 - c->cur_id], s));
  c->cur_id = 1 - c->cur_id;
  PG_HIP(hipMemcpyAsync(c->buf.group_offsets, ws(c, c->ws_newoff), sizeof(int32_t) * (P + 1),
                        hipMemcpyDeviceToDevice, s));
  PG_TRY(launch_fill_group_of(c->buf.group_offsets, P, c->buf.group_of, s));
  c->offsets = new_off;
  c->M = M_new;
  PG_TRY(pg_group_advantages(c->buf.rewards, c->buf.group_offsets, P, c->cfg.adv_eps, c->buf.adv, stream));
  return PG_OK;
}

extern "C" pg_status pg_policy_ratio(pg_ctx* c, const uint16_t* weights_new, double clip_eps, float* logp_new,
                                     float* ratio, float* J, void* stream) {
  if (!c || !c->bound || !c->initialised) return fail(PG_ESCHED, "pg_policy_ratio: call pg_init_group first");
  const pg_config& f = c->cfg;
  if (f.net_kind == PG_NET_NONE) return fail(PG_EINVAL, "pg_policy_ratio: the context has no network");
  if (!c->buf.x_hist) return fail(PG_EINVAL, "pg_policy_ratio: pg_buffers.x_hist was not bound");
  if (c->steps_done != f.T || !c->advantages_done || c->pending_gather)
    return fail(PG_ESCHED, "pg_policy_ratio: the sampling loop has not finished (steps %d of %d)", c->steps_done, f.T);
  if (!weights_new || !logp_new || !ratio || !J) return fail(PG_EINVAL, "pg_policy_ratio: null pointer");
  if (((uintptr_t)weights_new & 15)) return fail(PG_ESHAPE, "pg_policy_ratio: weights must be 16-byte aligned");
  if (!(clip_eps >= 0.0 && clip_eps < 1.0)) return fail(PG_EINVAL, "pg_policy_ratio: clip_eps = %g", clip_eps);
  hipStream_t s = (hipStream_t)stream;
  const size_t slice = (size_t)c->M0 * c->d;
  float* xb = c->buf.x[1 - c->cur_x];                 // scratch batch: the survivors' state at step s
  const int32_t* ids = c->buf.orig_id[c->cur_id];
  PG_TRY(launch_fill_u32(logp_new, 0x7FC00000u, (size_t)f.T * c->M0, s));
  PG_TRY(launch_fill_u32(ratio, 0x7FC00000u, (size_t)f.T * c->M0, s));
  PG_TRY(net_prepare(c, weights_new, s));
  c->context_ready = false;                           // the cached context projections now belong to weights_new
  for (int t = 0; t < f.T; ++t) {
    PG_TRY(pg_compact_gather(c->buf.x_hist + (size_t)t * slice, xb, ids, c->M, c->d, stream));
    PG_TRY(net_forward(c, t, xb, weights_new, s));
    PG_TRY(launch_transition_logprob(xb, c->buf.u, c->buf.x_hist + (size_t)(t + 1) * slice, ids, c->M, c->d, c->A[t],
                                     c->B[t], c->C[t], c->seed, (uint32_t)t, logp_new + (size_t)t * c->M0,
                                     (double*)ws(c, c->ws_logr) + (size_t)t * c->M0, (float*)ws(c, c->ws_partials), s));
  }
  c->net_fresh = false;
  return launch_surrogate((const double*)ws(c, c->ws_logr), c->buf.adv, c->buf.group_offsets, ids, f.P, f.T, c->M0,
                          clip_eps, ratio, J, s);
}

extern "C" pg_status pg_sample_group(pg_ctx* c, uint64_t seed, void* stream) {
  PG_TRY(pg_init_group(c, seed, stream));
  for (int s = 0; s < c->cfg.T; ++s) {
    PG_TRY(pg_net_forward(c, s, stream));
    if (c->is_checkpoint[s]) PG_TRY(pg_prune(c, s, stream));
    PG_TRY(pg_step(c, s, stream));
  }
  return pg_advantages(c, stream);
}

extern "C" pg_status pg_check(pg_ctx* c, void* stream) {
  if (!c || !c->bound) return fail(PG_EINVAL, "pg_check: context not bound");
  PG_HIP(hipStreamSynchronize((hipStream_t)stream));
  int32_t st[4] = {0, 0, 0, 0};
  PG_HIP(hipMemcpy(st, c->buf.status, sizeof(st), hipMemcpyDeviceToHost));
  if (st[0] & 1) return fail(PG_ENAN, "a non-finite proxy reward reached the selection");
  if (st[0] & 2) return fail(PG_EINVAL, "the selection met a group with a bad size or count");
  return PG_OK;
}
