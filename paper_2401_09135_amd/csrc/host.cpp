// Host-only parts of the library: error text, configuration checks, the flat parameter
// layout, Dynamic Local Updates (Eq. DyLU) and the event order of the asynchronous loop
// (Alg. 2 with get_worker() from the appendix) on a simulated clock.
#include "common.h"
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <limits>
#include <vector>

namespace als {

static thread_local char g_err[512] = "";

int set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

int head_width(const als_config& c);

int validate_config(const als_config* c) {
  if (!c) return set_error(ALS_ERR_INVALID, "config is null");
  if (c->n_layers < 1 || c->n_layers > 64) return set_error(ALS_ERR_INVALID, "n_layers must be in 1..64");
  if (c->d_model < 64 || c->d_model % 64 || c->d_model > 1024)
    return set_error(ALS_ERR_INVALID, "d_model must be a multiple of 64 in 64..1024");
  if (c->n_heads < 1) return set_error(ALS_ERR_INVALID, "n_heads must be >= 1");
  if (c->head_dim < 0) return set_error(ALS_ERR_INVALID, "head_dim must be >= 0");
  if (c->norm_kind != ALS_NORM_RMS && c->norm_kind != ALS_NORM_LAYER) return set_error(ALS_ERR_INVALID, "unknown norm_kind");
  if (c->head_dim == 0 && c->d_model % c->n_heads) return set_error(ALS_ERR_INVALID, "d_model must be divisible by n_heads");
  int dh = head_width(*c);
  if (dh != 32 && dh != 64) return set_error(ALS_ERR_INVALID, "head width must be 32 or 64");
  if ((c->n_heads * dh) % 64 || c->n_heads * dh > 2048) return set_error(ALS_ERR_INVALID, "attention width h*head width must be a multiple of 64, at most 2048");
  if (c->d_ff < 64 || c->d_ff % 64) return set_error(ALS_ERR_INVALID, "d_ff must be a positive multiple of 64");
  if (c->vocab < 2) return set_error(ALS_ERR_INVALID, "vocab must be >= 2");
  if (c->seq_len < 1 || c->seq_len > 1024) return set_error(ALS_ERR_INVALID, "seq_len must be in 1..1024");
  if (c->batch < 1) return set_error(ALS_ERR_INVALID, "batch must be >= 1");
  if ((int64_t)c->batch * c->seq_len > (1 << 22)) return set_error(ALS_ERR_INVALID, "batch*seq_len too large");
  if (c->dtype != ALS_DTYPE_F32 && c->dtype != ALS_DTYPE_BF16) return set_error(ALS_ERR_INVALID, "unknown dtype");
  if (c->n_workers < 1 || c->n_workers > ALS_MAX_WORKERS) return set_error(ALS_ERR_INVALID, "n_workers out of range");
  if (c->dn_N < 1) return set_error(ALS_ERR_INVALID, "dn_N must be >= 1");
  if (c->max_local_steps < 1) return set_error(ALS_ERR_INVALID, "max_local_steps must be >= 1");
  if (!(c->adam_beta1 >= 0 && c->adam_beta1 < 1) || !(c->adam_beta2 >= 0 && c->adam_beta2 < 1) ||
      !(c->adam_eps > 0) || !(c->weight_decay >= 0))
    return set_error(ALS_ERR_INVALID, "AdamW hyper-parameters out of range");
  if (!(c->outer_beta >= 0 && c->outer_beta < 1) || !isfinite(c->outer_lr))
    return set_error(ALS_ERR_INVALID, "outer optimiser hyper-parameters out of range");
  // momentum activation c of Alg. 3 lies in [0, 1/N]
  if (!(c->dn_c >= 0 && c->dn_c <= 1.0 / c->dn_N + 1e-12))
    return set_error(ALS_ERR_INVALID, "dn_c must lie in [0, 1/N]");
  if (!(c->norm_eps > 0)) return set_error(ALS_ERR_INVALID, "norm_eps must be > 0");
  return ALS_OK;
}

int head_width(const als_config& c) { return c.head_dim ? c.head_dim : c.d_model / c.n_heads; }

void make_layout(const als_config& c, Layout* L) {
  int64_t d = c.d_model, ff = c.d_ff, V = c.vocab, S = c.seq_len, off = 0;
  int64_t da = (int64_t)c.n_heads * head_width(c);  // attention width
  L->E = off; off += V * d;
  L->Ppos = off; off += S * d;
  for (int l = 0; l < c.n_layers; l++) {
    L->Wqkv[l] = off; off += d * 3 * da;
    L->Wo[l] = off; off += da * d;
    L->W1[l] = off; off += d * ff;
    L->W2[l] = off; off += ff * d;
  }
  L->Wout = off; off += d * V;
  L->P_decay = off;
  for (int l = 0; l < c.n_layers; l++) {
    L->g1[l] = off; off += d;
    L->g2[l] = off; off += d;
  }
  L->gf = off; off += d;
  L->P = off;
}

}  // namespace als

using namespace als;

extern "C" const char* als_last_error(void) { return g_err; }

extern "C" int64_t als_param_count(const als_config* cfg) {
  if (validate_config(cfg)) return 0;
  Layout L; make_layout(*cfg, &L);
  return L.P;
}
extern "C" int64_t als_param_count_decayed(const als_config* cfg) {
  if (validate_config(cfg)) return 0;
  Layout L; make_layout(*cfg, &L);
  return L.P_decay;
}
extern "C" int als_param_offsets(const als_config* cfg, int64_t* out, int n_out) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  int n = 6 * cfg->n_layers + 4;
  if (!out || n_out < n) return set_error(ALS_ERR_INVALID, "offsets_out needs room for %d entries", n);
  Layout L; make_layout(*cfg, &L);
  int i = 0;
  out[i++] = L.E; out[i++] = L.Ppos;
  for (int l = 0; l < cfg->n_layers; l++) { out[i++] = L.Wqkv[l]; out[i++] = L.Wo[l]; out[i++] = L.W1[l]; out[i++] = L.W2[l]; }
  out[i++] = L.Wout;
  for (int l = 0; l < cfg->n_layers; l++) { out[i++] = L.g1[l]; out[i++] = L.g2[l]; }
  out[i++] = L.gf;
  return n;
}

// Eq. (DyLU) in fp64: divide, multiply, floor; a zero count is raised to one step.
// Event loop: Alg. 2.  A running worker's completion time is start + H_i / v_i; the earliest
// (time, index) candidate is synchronised when no grace window is open or it falls inside the
// open one; otherwise every synchronised worker restarts at tau_sync + tau_grace.
extern "C" int als_dylu_schedule(const double* speeds, int k, int H_max, double tau_grace,
                                 int n_events, int32_t* H_out, int32_t* ev_worker, double* ev_time,
                                 int32_t* ev_group_end) {
  if (!speeds || !H_out) return set_error(ALS_ERR_INVALID, "speeds and H_out must be non-null");
  if (k <= 0 || k > ALS_MAX_WORKERS) return set_error(ALS_ERR_INVALID, "k out of range");
  if (H_max < 1) return set_error(ALS_ERR_INVALID, "H_max must be >= 1");
  if (!(tau_grace >= 0) || !isfinite(tau_grace)) return set_error(ALS_ERR_INVALID, "tau_grace must be finite and >= 0");
  if (n_events < 0) return set_error(ALS_ERR_INVALID, "n_events must be >= 0");
  double vmax = 0;
  for (int i = 0; i < k; i++) {
    if (!isfinite(speeds[i]) || !(speeds[i] > 0)) return set_error(ALS_ERR_INVALID, "speed %d is not finite and positive", i);
    if (speeds[i] > vmax) vmax = speeds[i];
  }
  for (int i = 0; i < k; i++) {
    double r = speeds[i] / vmax;
    int hi = (int)floor(r * (double)H_max);
    H_out[i] = hi < 1 ? 1 : hi;
  }
  if (!ev_worker || n_events == 0) return ALS_OK;

  const double inf = std::numeric_limits<double>::infinity();
  std::vector<double> done(k);
  std::vector<char> running(k, 1);
  std::vector<int> completed;
  for (int i = 0; i < k; i++) done[i] = 0.0 + (double)H_out[i] / speeds[i];
  double tau_sync = inf;
  int emitted = 0;
  for (;;) {
    int e = -1;
    for (int i = 0; i < k; i++)
      if (running[i] && (e < 0 || done[i] < done[e])) e = i;  // ties keep the smaller index
    bool take = e >= 0 && (tau_sync == inf || done[e] - tau_sync <= tau_grace);
    if (take) {
      if (emitted == n_events) break;  // the open group is cut short: its last flag stays 0
      if (done[e] < tau_sync) tau_sync = done[e];
      ev_worker[emitted] = e;
      if (ev_time) ev_time[emitted] = done[e];
      if (ev_group_end) ev_group_end[emitted] = 0;
      running[e] = 0;
      completed.push_back(e);
      emitted++;
    } else {
      double restart = tau_sync + tau_grace;
      if (ev_group_end && emitted > 0) ev_group_end[emitted - 1] = 1;
      for (int i : completed) {
        done[i] = restart + (double)H_out[i] / speeds[i];
        running[i] = 1;
      }
      completed.clear();
      tau_sync = inf;
      if (emitted == n_events) break;
    }
  }
  return ALS_OK;
}

// Eq. (lr): linear warm-up, then cosine decay to eta_min, per data shard.  ratio = (t - t_warmup)
// / max(T - t_warmup, 0) clamped to [0, 1]; a zero denominator gives ratio 1.
extern "C" int als_lr_schedule(int64_t t0, int n, int64_t t_warmup, int64_t T, double eta_max, double eta_min,
                               float* lr_out) {
  if (n < 0 || t0 < 0 || t_warmup < 0 || T < 0) return set_error(ALS_ERR_INVALID, "als_lr_schedule: negative argument");
  if (n > 0 && !lr_out) return set_error(ALS_ERR_INVALID, "als_lr_schedule: lr_out is null");
  if (!isfinite(eta_max) || !isfinite(eta_min) || eta_min < 0 || eta_max < eta_min)
    return set_error(ALS_ERR_INVALID, "als_lr_schedule: need 0 <= eta_min <= eta_max, finite");
  const double pi = 3.14159265358979323846;
  for (int i = 0; i < n; i++) {
    int64_t t = t0 + i;
    double lr;
    if (t < t_warmup) {
      lr = (double)t * eta_max / (double)t_warmup;
    } else {
      int64_t denom = T - t_warmup > 0 ? T - t_warmup : 0;
      double ratio = denom == 0 ? 1.0 : (double)(t - t_warmup) / (double)denom;
      if (ratio < 0.0) ratio = 0.0;
      if (ratio > 1.0) ratio = 1.0;
      lr = eta_min + 0.5 * (eta_max - eta_min) * (1.0 + cos(ratio * pi));
    }
    lr_out[i] = (float)lr;
  }
  return ALS_OK;
}

// Eq. (data_sample): p_i proportional to max(|D_i| / sum |D_j| - n_i / sum n_j, 0); the progress
// share is 0 while nothing has been learned; if no shard is behind, the size shares are used.
// The shard is drawn by inverse CDF from the caller's uniform number u in [0, 1).
extern "C" int als_shard_sample(const double* sizes, const double* learned, int k, double u, double* p_out,
                                int32_t* shard_out) {
  if (!sizes || !learned || k < 1) return set_error(ALS_ERR_INVALID, "als_shard_sample: null argument or k < 1");
  if (!(u >= 0.0 && u < 1.0)) return set_error(ALS_ERR_INVALID, "als_shard_sample: u must lie in [0, 1)");
  double ssum = 0.0, nsum = 0.0;
  for (int i = 0; i < k; i++) {
    if (!(sizes[i] > 0) || !isfinite(sizes[i]) || !(learned[i] >= 0) || !isfinite(learned[i]))
      return set_error(ALS_ERR_INVALID, "als_shard_sample: sizes must be positive, learned non-negative");
    ssum += sizes[i];
    nsum += learned[i];
  }
  std::vector<double> w(k);
  double wsum = 0.0;
  for (int i = 0; i < k; i++) {
    double d = sizes[i] / ssum - (nsum > 0 ? learned[i] / nsum : 0.0);
    w[i] = d > 0 ? d : 0.0;
    wsum += w[i];
  }
  if (!(wsum > 0.0)) {
    wsum = 0.0;
    for (int i = 0; i < k; i++) { w[i] = sizes[i] / ssum; wsum += w[i]; }
  }
  int pick = -1, last_pos = 0;
  double c = 0.0;
  for (int i = 0; i < k; i++) {
    double p = w[i] / wsum;
    if (p_out) p_out[i] = p;
    if (p > 0) last_pos = i;
    c += p;
    if (pick < 0 && u < c) pick = i;
  }
  if (shard_out) *shard_out = pick >= 0 ? pick : last_pos;
  return ALS_OK;
}
