// Context, arena carve-up and the orchestration of the hot path: a worker's local round
// (inner loop of Alg. 1: forward, backward, AdamW) on that worker's stream, and the server's
// sync() step (pseudo-gradient, Delayed Nesterov of Alg. 3, restart of Alg. 2) ordered
// against the workers with events.
#include "common.h"
#include <math.h>
#include <string.h>
#include <mutex>
#include <new>
#include <vector>

using namespace als;

namespace {

struct Worker {
  float *theta, *start, *adam_m, *adam_v, *grad;
  bf16* lp;
  std::vector<float*> x, xm, rstd1, rstd2, lse;
  std::vector<void*> a, qkv, o, b, u, gl;
  void* xf; float* rstdf; float* logits; void* dlogits; float* loss_row;  // logits: fp32 mode only
  float *dxa, *dxb, *dtmp, *Dbuf, *partial;
  void *dx_lp, *dff, *d_o, *dqkv;
  float* losses_dev; float* losses_host;
  int32_t *sort_offset, *sort_rank, *sort_pos;
  float* splitk_ws; size_t splitk_bytes;
  // Output gradients that the weight-gradient products read (dY), per layer: of the block output
  // (for W2), of the FFN pre-activation (W1), of the attention block output (Wo), of q/k/v (Wqkv).
  // With the grouped launch every layer keeps its own until the end of the backward pass; otherwise
  // all layers point at the same four buffers.
  std::vector<void*> dy2, dy1, dyo, dyqkv;
  DwProblem* dw_probs_dev; DwItem* dw_items_dev; DwSplitTile* dw_split_dev; float* dw_partial;
  std::vector<DwProblem> dw_probs; std::vector<DwItem> dw_items; std::vector<DwSplitTile> dw_split;
  DwPlan dw_plan;
  int64_t adam_n; int last_n;
  int64_t t_restart;  // server event count when this replica last (re)started
  hipStream_t stream; hipEvent_t done_ev, ready_ev;
};

}  // namespace

struct als_ctx {
  als_config cfg;
  Layout L;
  char* arena; size_t arena_bytes;
  float *theta, *m, *delta;
  int64_t t;
  std::vector<Worker> w;
  hipEvent_t server_ev;
  bool bf; bool allow_mfma;
  bool grouped_dw;   // the layers' weight gradients run as one grouped launch at the end of the backward pass
  int T;
};

namespace {

// Walks the arena handing out 256-byte aligned blocks; with base == nullptr it only counts.
struct Carver {
  char* base; size_t off;
  void* take(size_t bytes) {
    size_t a = (off + 255) & ~(size_t)255;
    off = a + bytes;
    return base ? (void*)(base + a) : nullptr;
  }
  float* f32(int64_t n) { return (float*)take((size_t)n * 4); }
  void* act(int64_t n, bool bf) { return take((size_t)n * (bf ? 2 : 4)); }
};

void carve(als_ctx* c, Carver& cv) {
  const als_config& g = c->cfg;
  bool bf = g.dtype == ALS_DTYPE_BF16;
  int64_t P = c->L.P, T = (int64_t)g.batch * g.seq_len, d = g.d_model, ff = g.d_ff, V = g.vocab;
  int64_t da = (int64_t)g.n_heads * head_width(g);  // attention width
  int64_t BhS = (int64_t)g.batch * g.n_heads * g.seq_len;
  c->theta = cv.f32(P); c->m = cv.f32(P); c->delta = cv.f32(P);
  c->w.resize(g.n_workers);
  c->grouped_dw = bf && !(g.flags & 1) && !(g.flags & 2) && g.n_layers > 0 && dw_group_supported((int)d, (int)(3 * da), (int)T, d, 3 * da) &&
                  dw_group_supported((int)da, (int)d, (int)T, da, d) && dw_group_supported((int)d, (int)ff, (int)T, d, ff);
  for (Worker& w : c->w) {
    w.theta = cv.f32(P); w.start = cv.f32(P); w.adam_m = cv.f32(P); w.adam_v = cv.f32(P);
    w.grad = cv.f32(P);
    w.lp = bf ? (bf16*)cv.take((size_t)P * 2) : nullptr;
    int L = g.n_layers;
    w.x.resize(L + 1); w.xm.resize(L); w.rstd1.resize(L); w.rstd2.resize(L); w.lse.resize(L);
    w.a.resize(L); w.qkv.resize(L); w.o.resize(L); w.b.resize(L); w.u.resize(L); w.gl.resize(L);
    for (int l = 0; l <= L; l++) w.x[l] = cv.f32(T * d);
    for (int l = 0; l < L; l++) {
      w.xm[l] = cv.f32(T * d); w.rstd1[l] = cv.f32(T); w.rstd2[l] = cv.f32(T); w.lse[l] = cv.f32(BhS);
      w.a[l] = cv.act(T * d, bf); w.qkv[l] = cv.act(T * 3 * da, bf); w.o[l] = cv.act(T * da, bf);
      w.b[l] = cv.act(T * d, bf); w.u[l] = cv.act(T * ff, bf); w.gl[l] = cv.act(T * ff, bf);
    }
    w.xf = cv.act(T * d, bf); w.rstdf = cv.f32(T);
    // bf16 mode: the output GEMM writes bf16 logits into dlogits and the cross-entropy runs in place
    w.logits = bf ? nullptr : cv.f32(T * V); w.dlogits = cv.act(T * V, bf); w.loss_row = cv.f32(T);
    w.dxa = cv.f32(T * d); w.dxb = cv.f32(T * d); w.dtmp = cv.f32(T * d); w.Dbuf = cv.f32(BhS);
    // one set of gain-gradient partials per norm, in the layout order of the gains (g1, g2 per layer, gf)
    w.partial = cv.f32((int64_t)(2 * g.n_layers + 1) * rmsnorm_bwd_blocks((int)T) * d);
    w.dx_lp = cv.act(T * d, bf); w.dff = cv.act(T * ff, bf); w.d_o = cv.act(T * da, bf);
    w.dqkv = cv.act(T * 3 * da, bf);
    w.losses_dev = cv.f32(g.max_local_steps);
    w.sort_offset = (int32_t*)cv.take((size_t)g.max_local_steps * (V + 1) * 4);
    w.sort_rank = (int32_t*)cv.take((size_t)g.max_local_steps * T * 4);
    w.sort_pos = (int32_t*)cv.take((size_t)g.max_local_steps * T * 4);
    // split-K partials of the weight-gradient GEMMs: up to 16 copies of the largest layer
    // matrix, capped at 64 MiB
    {
      int64_t big = d * (ff > 3 * da ? ff : 3 * da);
      size_t want = (size_t)big * 4 * 16;
      w.splitk_bytes = bf ? (want < ((size_t)64 << 20) ? want : ((size_t)64 << 20)) : 0;
      w.splitk_ws = w.splitk_bytes ? (float*)cv.take(w.splitk_bytes) : nullptr;
    }
    w.dy2.assign(L, w.dx_lp); w.dy1.assign(L, w.dff); w.dyo.assign(L, w.dx_lp); w.dyqkv.assign(L, w.dqkv);
    w.dw_probs_dev = nullptr; w.dw_items_dev = nullptr; w.dw_split_dev = nullptr; w.dw_partial = nullptr;
    w.dw_plan = DwPlan{0, 0, 0, 0.0};
    if (c->grouped_dw) {
      for (int l = 0; l < L; l++) {
        w.dy2[l] = cv.act(T * d, bf); w.dy1[l] = cv.act(T * ff, bf); w.dyo[l] = cv.act(T * d, bf);
        w.dyqkv[l] = cv.act(T * 3 * da, bf);
      }
      // the products, in the order of the flat parameter layout (pointers are null while only counting)
      w.dw_probs.clear();
      int n_tiles = 0;
      auto add = [&](const void* X, int64_t M, const void* dY, int64_t N, int64_t off) {
        w.dw_probs.push_back(DwProblem{(const bf16*)X, (const bf16*)dY, w.grad ? w.grad + off : nullptr, (int)M, (int)N, (int)M, (int)N, {0, 0}});
        n_tiles += (int)(((M + 255) / 256) * ((N + 255) / 256));
      };
      for (int l = 0; l < L; l++) {
        add(w.a[l], d, w.dyqkv[l], 3 * da, c->L.Wqkv[l]);
        add(w.o[l], da, w.dyo[l], d, c->L.Wo[l]);
        add(w.b[l], d, w.dy1[l], ff, c->L.W1[l]);
        add(w.gl[l], ff, w.dy2[l], d, c->L.W2[l]);
      }
      w.dw_items.resize(dw_plan_max_items(n_tiles));
      w.dw_split.resize(dw_plan_max_split(n_tiles) + 1);
      w.dw_plan = dw_group_plan(w.dw_probs.data(), (int)w.dw_probs.size(), (int)T, w.dw_items.data(), w.dw_split.data());
      w.dw_probs_dev = (DwProblem*)cv.take(w.dw_probs.size() * sizeof(DwProblem));
      w.dw_items_dev = (DwItem*)cv.take((size_t)w.dw_plan.n_items * sizeof(DwItem));
      w.dw_split_dev = (DwSplitTile*)cv.take((size_t)(w.dw_plan.n_split + 1) * sizeof(DwSplitTile));
      w.dw_partial = cv.f32((int64_t)w.dw_plan.n_partial_tiles * 65536);
    }
  }
}

GemmDesc desc(const als_ctx* c, const void* A, int a_layout, int64_t lda, const void* B, int b_layout,
              int64_t ldb, int M, int N, int K, void* C, int64_t ldc, bool c_act) {
  GemmDesc g;
  memset(&g, 0, sizeof g);
  g.A = A; g.B = B; g.M = M; g.N = N; g.K = K; g.a_layout = a_layout; g.b_layout = b_layout;
  g.lda = lda; g.ldb = ldb; g.in_bf16 = c->bf; g.C = C; g.ldc = ldc; g.c_bf16 = c_act && c->bf;
  g.epi = EPI_STORE;
  return g;
}

// weight-gradient GEMM: X^T dY into the flat fp32 gradient, with the worker's split-K scratch
GemmDesc desc_dw(const als_ctx* c, const Worker& w, const void* X, int64_t ldx, const void* dY, int64_t ldy,
                 int M, int N, int K, float* out) {
  GemmDesc g = desc(c, X, 1, ldx, dY, 0, ldy, M, N, K, out, N, false);
  g.ws = w.splitk_ws; g.ws_bytes = w.splitk_bytes;
  return g;
}

#define RUN(expr) do { int rc_ = (expr); if (rc_) return rc_; } while (0)

// Weight operand of a GEMM: the bf16 working copy in bf16 mode, the fp32 master otherwise.
inline const void* wptr(const als_ctx* c, const Worker& w, int64_t off) {
  return c->bf ? (const void*)(w.lp + off) : (const void*)(w.theta + off);
}

int forward(als_ctx* c, Worker& w, const int32_t* tok, float* loss_out) {
  const als_config& g = c->cfg;
  const Layout& L = c->L;
  hipStream_t st = w.stream;
  int T = c->T, d = g.d_model, ff = g.d_ff, V = g.vocab, B = g.batch, S = g.seq_len, h = g.n_heads;
  const int dh = head_width(g), da = h * dh;
  const int ln = g.norm_kind == ALS_NORM_LAYER;  // LayerNorm (gain, no bias) instead of RMSNorm
  bool mf = c->allow_mfma;
  float eps = (float)g.norm_eps;
  RUN(embed_fwd(tok, w.theta + L.E, w.theta + L.Ppos, w.x[0], B, S, d, V, st));
  for (int l = 0; l < g.n_layers; l++) {
    RUN(rmsnorm_fwd(w.x[l], w.theta + L.g1[l], w.a[l], w.rstd1[l], T, d, eps, c->bf, ln, st));
    RUN(gemm(desc(c, w.a[l], 0, d, wptr(c, w, L.Wqkv[l]), 0, 3 * da, T, 3 * da, d, w.qkv[l], 3 * da, true), mf, st));
    if (mf && attention_mfma_supported(S, dh, c->bf))
      RUN(attention_fwd_mfma(w.qkv[l], w.o[l], w.lse[l], B, S, h, dh, st));
    else
      RUN(attention_fwd_generic(w.qkv[l], w.o[l], w.lse[l], B, S, h, dh, c->bf, st));
    GemmDesc po = desc(c, w.o[l], 0, da, wptr(c, w, L.Wo[l]), 0, d, T, d, da, w.xm[l], d, false);
    po.epi = EPI_RESID; po.R = w.x[l]; po.ldr = d;
    RUN(gemm(po, mf, st));
    RUN(rmsnorm_fwd(w.xm[l], w.theta + L.g2[l], w.b[l], w.rstd2[l], T, d, eps, c->bf, ln, st));
    GemmDesc f1 = desc(c, w.b[l], 0, d, wptr(c, w, L.W1[l]), 0, ff, T, ff, d, w.u[l], ff, true);
    f1.epi = EPI_GELU; f1.C2 = w.gl[l];
    RUN(gemm(f1, mf, st));
    GemmDesc f2 = desc(c, w.gl[l], 0, ff, wptr(c, w, L.W2[l]), 0, d, T, d, ff, w.x[l + 1], d, false);
    f2.epi = EPI_RESID; f2.R = w.xm[l]; f2.ldr = d;
    RUN(gemm(f2, mf, st));
  }
  RUN(rmsnorm_fwd(w.x[g.n_layers], w.theta + L.gf, w.xf, w.rstdf, T, d, eps, c->bf, ln, st));
  void* logits = c->bf ? w.dlogits : (void*)w.logits;
  RUN(gemm(desc(c, w.xf, 0, d, wptr(c, w, L.Wout), 0, V, T, V, d, logits, V, true), mf, st));
  RUN(cross_entropy(logits, c->bf, tok, w.loss_row, w.dlogits, c->bf, B, S, V, st));
  RUN(mean_rows(w.loss_row, loss_out, T, st));
  return ALS_OK;
}

int backward(als_ctx* c, Worker& w, const int32_t* tok, int slot) {
  const als_config& g = c->cfg;
  const Layout& L = c->L;
  hipStream_t st = w.stream;
  int T = c->T, d = g.d_model, ff = g.d_ff, V = g.vocab, B = g.batch, S = g.seq_len, h = g.n_heads;
  const int dh = head_width(g), da = h * dh;
  const int ln = g.norm_kind == ALS_NORM_LAYER;  // LayerNorm (gain, no bias) instead of RMSNorm
  bool mf = c->allow_mfma;
  int nl = g.n_layers;
  // output matrix and final norm
  RUN(gemm(desc_dw(c, w, w.xf, d, w.dlogits, V, d, V, T, w.grad + L.Wout), mf, st));
  RUN(gemm(desc(c, w.dlogits, 0, V, wptr(c, w, L.Wout), 1, V, T, d, V, w.dtmp, d, false), mf, st));
  // the norms leave their gain-gradient partials; one kernel adds all of them after the last layer
  const int64_t pset = (int64_t)rmsnorm_bwd_blocks(T) * d;
  RUN(rmsnorm_bwd(w.dtmp, w.x[nl], w.rstdf, w.theta + L.gf, nullptr, w.dxa, nl ? w.dy2[nl - 1] : w.dx_lp, c->bf,
                  nullptr, w.partial + 2 * nl * pset, T, d, ln, st));
  // The weight gradient of every matrix is X^T dY.  Either each is a product of its own, issued
  // here next to the input gradient that reads the same dY, or (grouped) every layer keeps its four
  // dY until the loop is over and all of them run as one launch.
  const bool each = !c->grouped_dw;
  for (int l = nl - 1; l >= 0; l--) {
    // feed-forward block: x_next = xm + gelu(b W1) W2
    if (each) RUN(gemm(desc_dw(c, w, w.gl[l], ff, w.dy2[l], d, ff, d, T, w.grad + L.W2[l]), mf, st));
    GemmDesc du = desc(c, w.dy2[l], 0, d, wptr(c, w, L.W2[l]), 1, d, T, ff, d, w.dy1[l], ff, true);
    du.epi = EPI_DGELU; du.U = w.u[l];
    RUN(gemm(du, mf, st));
    if (each) RUN(gemm(desc_dw(c, w, w.b[l], d, w.dy1[l], ff, d, ff, T, w.grad + L.W1[l]), mf, st));
    RUN(gemm(desc(c, w.dy1[l], 0, ff, wptr(c, w, L.W1[l]), 1, ff, T, d, ff, w.dtmp, d, false), mf, st));
    RUN(rmsnorm_bwd(w.dtmp, w.xm[l], w.rstd2[l], w.theta + L.g2[l], w.dxa, w.dxb, w.dyo[l], c->bf,
                    nullptr, w.partial + (2 * l + 1) * pset, T, d, ln, st));
    // attention block: xm = x + attn(a Wqkv) Wo
    if (each) RUN(gemm(desc_dw(c, w, w.o[l], da, w.dyo[l], d, da, d, T, w.grad + L.Wo[l]), mf, st));
    RUN(gemm(desc(c, w.dyo[l], 0, d, wptr(c, w, L.Wo[l]), 1, d, T, da, d, w.d_o, da, true), mf, st));
    if (mf && attention_mfma_supported(S, dh, c->bf))
      RUN(attention_bwd_mfma(w.qkv[l], w.o[l], w.d_o, w.lse[l], w.Dbuf, w.dyqkv[l], B, S, h, dh, st));
    else
      RUN(attention_bwd_generic(w.qkv[l], w.o[l], w.d_o, w.lse[l], w.Dbuf, w.dyqkv[l], B, S, h, dh, c->bf, st));
    if (each) RUN(gemm(desc_dw(c, w, w.a[l], d, w.dyqkv[l], 3 * da, d, 3 * da, T, w.grad + L.Wqkv[l]), mf, st));
    RUN(gemm(desc(c, w.dyqkv[l], 0, 3 * da, wptr(c, w, L.Wqkv[l]), 1, 3 * da, T, d, 3 * da, w.dtmp, d, false), mf, st));
    RUN(rmsnorm_bwd(w.dtmp, w.x[l], w.rstd1[l], w.theta + L.g1[l], w.dxb, w.dxa, l ? w.dy2[l - 1] : w.dx_lp, c->bf,
                    nullptr, w.partial + 2 * l * pset, T, d, ln, st));
  }
  if (!each) RUN(dw_group_launch(w.dw_probs_dev, w.dw_items_dev, w.dw_split_dev, w.dw_plan, w.dw_partial, st));
  RUN(rmsnorm_dg_sum(w.partial, w.grad + L.g1[0], T, d, 2 * nl + 1, st));
  // w.dtmp (T x d floats) is free again here: scratch for the embedding gradient's chunk partials
  RUN(embed_bwd(tok, w.sort_offset + (int64_t)slot * (V + 1), w.sort_pos + (int64_t)slot * T, w.dxa,
                w.grad + L.E, w.grad + L.Ppos, w.dtmp, B, S, d, V, st));
  return ALS_OK;
}

int check_ctx_worker(als_ctx* ctx, int worker) {
  if (!ctx) return set_error(ALS_ERR_INVALID, "context is null");
  if (worker < 0 || worker >= (int)ctx->w.size()) return set_error(ALS_ERR_INVALID, "worker %d out of range", worker);
  return ALS_OK;
}

int sync_all(als_ctx* ctx) {
  for (Worker& w : ctx->w) ALS_HIP(hipStreamSynchronize(w.stream));
  return ALS_OK;
}

}  // namespace

extern "C" size_t als_arena_bytes(const als_config* cfg) {
  if (validate_config(cfg)) return 0;
  als_ctx tmp;
  tmp.cfg = *cfg;
  make_layout(*cfg, &tmp.L);
  Carver cv{nullptr, 0};
  carve(&tmp, cv);
  return cv.off + 256;
}

extern "C" int als_init(const als_config* cfg, void* arena, size_t arena_bytes, const float* theta0,
                        void* const* streams, int n_streams, als_ctx** out) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (!arena || !theta0 || !out || !streams || n_streams < 1)
    return set_error(ALS_ERR_INVALID, "als_init: null argument or no stream");
  if ((uintptr_t)arena % 256) return set_error(ALS_ERR_ARENA, "arena must be 256-byte aligned");
  size_t need = als_arena_bytes(cfg);
  if (arena_bytes < need) return set_error(ALS_ERR_ARENA, "arena too small: %zu bytes given, %zu needed", arena_bytes, need);
  als_ctx* c = new (std::nothrow) als_ctx();
  if (!c) return set_error(ALS_ERR_INVALID, "out of host memory");
  c->cfg = *cfg;
  make_layout(*cfg, &c->L);
  c->arena = (char*)arena; c->arena_bytes = arena_bytes;
  c->bf = cfg->dtype == ALS_DTYPE_BF16;
  c->allow_mfma = c->bf && !(cfg->flags & 1);
  c->T = cfg->batch * cfg->seq_len;
  c->t = 0;
  Carver cv{(char*)arena, 0};
  carve(c, cv);
  if (c->grouped_dw)
    for (Worker& w : c->w) {
      if (hipMemcpy(w.dw_probs_dev, w.dw_probs.data(), w.dw_probs.size() * sizeof(DwProblem), hipMemcpyHostToDevice) != hipSuccess ||
          hipMemcpy(w.dw_items_dev, w.dw_items.data(), (size_t)w.dw_plan.n_items * sizeof(DwItem), hipMemcpyHostToDevice) != hipSuccess ||
          (w.dw_plan.n_split && hipMemcpy(w.dw_split_dev, w.dw_split.data(), (size_t)w.dw_plan.n_split * sizeof(DwSplitTile), hipMemcpyHostToDevice) != hipSuccess)) {
        int code = set_error(ALS_ERR_HIP, "als_init: uploading the weight-gradient work list failed: %s", hipGetErrorString(hipGetLastError()));
        delete c;
        return code;
      }
    }
  int64_t P = c->L.P;
  hipStream_t s0 = (hipStream_t)streams[0];
  c->server_ev = nullptr;
  for (Worker& w : c->w) { w.done_ev = nullptr; w.ready_ev = nullptr; w.losses_host = nullptr; }
  auto fail = [&](int code) { als_destroy(c); return code; };
  if (hipEventCreateWithFlags(&c->server_ev, hipEventDisableTiming) != hipSuccess)
    return fail(set_error(ALS_ERR_HIP, "hipEventCreate failed"));
  if (hipMemcpyAsync(c->theta, theta0, (size_t)P * 4, hipMemcpyHostToDevice, s0) != hipSuccess ||
      hipMemsetAsync(c->m, 0, (size_t)P * 4, s0) != hipSuccess ||
      hipMemsetAsync(c->delta, 0, (size_t)P * 4, s0) != hipSuccess ||
      hipStreamSynchronize(s0) != hipSuccess)
    return fail(set_error(ALS_ERR_HIP, "als_init: copying theta0 failed: %s", hipGetErrorString(hipGetLastError())));
  for (size_t i = 0; i < c->w.size(); i++) {
    Worker& w = c->w[i];
    w.stream = (hipStream_t)streams[i % n_streams];
    w.adam_n = 0; w.last_n = 0; w.t_restart = 0;
    if (hipEventCreateWithFlags(&w.done_ev, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&w.ready_ev, hipEventDisableTiming) != hipSuccess ||
        hipHostMalloc((void**)&w.losses_host, (size_t)cfg->max_local_steps * 4, hipHostMallocDefault) != hipSuccess)
      return fail(set_error(ALS_ERR_HIP, "als_init: event or pinned-buffer creation failed"));
    if (hipMemsetAsync(w.adam_m, 0, (size_t)P * 4, w.stream) != hipSuccess ||
        hipMemsetAsync(w.adam_v, 0, (size_t)P * 4, w.stream) != hipSuccess ||
        hipMemsetAsync(w.grad, 0, (size_t)P * 4, w.stream) != hipSuccess)
      return fail(set_error(ALS_ERR_HIP, "als_init: clearing optimiser state failed"));
    rc = restart_copy(c->theta, w.theta, w.start, w.lp, P, w.stream);
    if (rc) return fail(rc);
    if (hipEventRecord(w.ready_ev, w.stream) != hipSuccess || hipEventRecord(w.done_ev, w.stream) != hipSuccess)
      return fail(set_error(ALS_ERR_HIP, "als_init: hipEventRecord failed"));
  }
  if (hipEventRecord(c->server_ev, s0) != hipSuccess) return fail(set_error(ALS_ERR_HIP, "hipEventRecord failed"));
  rc = sync_all(c);
  if (rc) return fail(rc);
  *out = c;
  return ALS_OK;
}

extern "C" int als_destroy(als_ctx* c) {
  if (!c) return ALS_OK;
  for (Worker& w : c->w) {
    if (w.stream) (void)hipStreamSynchronize(w.stream);
    if (w.done_ev) (void)hipEventDestroy(w.done_ev);
    if (w.ready_ev) (void)hipEventDestroy(w.ready_ev);
    if (w.losses_host) (void)hipHostFree(w.losses_host);
  }
  if (c->server_ev) (void)hipEventDestroy(c->server_ev);
  delete c;
  return ALS_OK;
}

extern "C" int als_worker_local_steps(als_ctx* ctx, int worker, int n_steps, const int32_t* tokens,
                                      const float* lr_host, float* loss_host) {
  int rc = check_ctx_worker(ctx, worker);
  if (rc) return rc;
  const als_config& g = ctx->cfg;
  if (n_steps < 0 || n_steps > g.max_local_steps)
    return set_error(ALS_ERR_INVALID, "n_steps %d outside 0..max_local_steps=%d", n_steps, g.max_local_steps);
  if (n_steps > 0 && (!tokens || !lr_host)) return set_error(ALS_ERR_INVALID, "tokens_dev and lr_host must be non-null");
  Worker& w = ctx->w[worker];
  ALS_HIP(hipStreamWaitEvent(w.stream, w.ready_ev, 0));
  int64_t per = (int64_t)g.batch * (g.seq_len + 1);
  RUN(embed_sort(tokens, n_steps, g.batch, g.seq_len, g.vocab, w.sort_offset, w.sort_rank, w.sort_pos, w.stream));
  for (int s = 0; s < n_steps; s++) {
    const int32_t* tok = tokens + (int64_t)s * per;
    RUN(forward(ctx, w, tok, w.losses_dev + s));
    RUN(backward(ctx, w, tok, s));
    w.adam_n += 1;
    AdamArgs a;
    a.lr = lr_host[s];
    a.beta1 = (float)g.adam_beta1; a.beta2 = (float)g.adam_beta2; a.eps = (float)g.adam_eps;
    a.wd = (float)g.weight_decay;
    a.bc1 = (float)(1.0 - pow(g.adam_beta1, (double)w.adam_n));
    a.bc2 = (float)(1.0 - pow(g.adam_beta2, (double)w.adam_n));
    RUN(adamw(w.theta, w.grad, w.adam_m, w.adam_v, w.lp, ctx->L.P, ctx->L.P_decay, a, w.stream));
  }
  w.last_n = n_steps;
  if (n_steps > 0)
    ALS_HIP(hipMemcpyAsync(w.losses_host, w.losses_dev, (size_t)n_steps * 4, hipMemcpyDeviceToHost, w.stream));
  ALS_HIP(hipEventRecord(w.done_ev, w.stream));
  if (loss_host) {
    ALS_HIP(hipStreamSynchronize(w.stream));
    memcpy(loss_host, w.losses_host, (size_t)n_steps * 4);
  }
  return ALS_OK;
}

extern "C" int als_worker_loss_grad(als_ctx* ctx, int worker, const int32_t* tokens, float* loss_host) {
  int rc = check_ctx_worker(ctx, worker);
  if (rc) return rc;
  if (!tokens || !loss_host) return set_error(ALS_ERR_INVALID, "tokens_dev and loss_host must be non-null");
  Worker& w = ctx->w[worker];
  ALS_HIP(hipStreamWaitEvent(w.stream, w.ready_ev, 0));
  RUN(embed_sort(tokens, 1, ctx->cfg.batch, ctx->cfg.seq_len, ctx->cfg.vocab, w.sort_offset, w.sort_rank,
                 w.sort_pos, w.stream));
  RUN(forward(ctx, w, tokens, w.losses_dev));
  RUN(backward(ctx, w, tokens, 0));
  ALS_HIP(hipMemcpyAsync(w.losses_host, w.losses_dev, 4, hipMemcpyDeviceToHost, w.stream));
  ALS_HIP(hipEventRecord(w.done_ev, w.stream));
  ALS_HIP(hipStreamSynchronize(w.stream));
  *loss_host = w.losses_host[0];
  return ALS_OK;
}

static int outer_apply(als_ctx* ctx, const int32_t* workers, int n_group, int restart_flag, const als_outer_rule& rule) {
  if (!ctx || !workers) return set_error(ALS_ERR_INVALID, "null argument");
  int k = (int)ctx->w.size();
  if (n_group < 1 || n_group > k) return set_error(ALS_ERR_INVALID, "n_group %d outside 1..k", n_group);
  if (rule.kind != ALS_RULE_DN && rule.kind != ALS_RULE_BUFFER) return set_error(ALS_ERR_INVALID, "unknown outer rule %d", rule.kind);
  if (!(rule.poly_exponent >= 0) || !isfinite(rule.poly_exponent) || !isfinite(rule.dc_lambda) || rule.dc_lambda < 0)
    return set_error(ALS_ERR_INVALID, "outer rule: poly_exponent and dc_lambda must be finite and >= 0");
  unsigned long long seen = 0;
  for (int j = 0; j < n_group; j++) {
    if (workers[j] < 0 || workers[j] >= k) return set_error(ALS_ERR_INVALID, "worker %d out of range", workers[j]);
    if (seen >> workers[j] & 1ull) return set_error(ALS_ERR_INVALID, "worker %d listed twice", workers[j]);
    seen |= 1ull << workers[j];
  }
  const als_config& g = ctx->cfg;
  hipStream_t st = ctx->w[workers[0]].stream;
  ALS_HIP(hipStreamWaitEvent(st, ctx->server_ev, 0));
  for (int j = 0; j < n_group; j++) ALS_HIP(hipStreamWaitEvent(st, ctx->w[workers[j]].done_ev, 0));
  int64_t P = ctx->L.P;
  // Which events are applied: a worker whose staleness (server events since it started)
  // exceeds the threshold is discarded -- no server change, no event counted -- but still restarts.
  std::vector<int> applied;
  std::vector<float> weight;
  {
    int64_t t = ctx->t;
    for (int j = 0; j < n_group; j++) {
      int64_t stale = t - ctx->w[workers[j]].t_restart;
      if (rule.staleness_threshold >= 0 && stale > rule.staleness_threshold) continue;
      applied.push_back(workers[j]);
      weight.push_back(rule.poly_exponent > 0 ? (float)pow(1.0 + (double)stale, -rule.poly_exponent) : 1.0f);
      t++;
    }
  }
  int n_app = (int)applied.size();
  bool fused_restart = restart_flag && n_app == n_group && n_group <= ALS_DN_MAX_GROUP;
  for (int j0 = 0; j0 < n_app; j0 += ALS_DN_MAX_GROUP) {
    DnGroup dg;
    memset(&dg, 0, sizeof dg);
    dg.G = n_app - j0 < ALS_DN_MAX_GROUP ? n_app - j0 : ALS_DN_MAX_GROUP;
    dg.restart = fused_restart ? 1 : 0;
    for (int j = 0; j < ALS_DN_MAX_GROUP; j++) dg.weight[j] = 1.0f;
    for (int j = 0; j < dg.G; j++) {
      Worker& w = ctx->w[applied[j0 + j]];
      dg.theta_start[j] = w.start; dg.theta_worker[j] = w.theta; dg.start_out[j] = w.start;
      dg.lp_out[j] = w.lp;
      dg.weight[j] = weight[j0 + j];
      if ((ctx->t + j + 1) % g.dn_N == 0) dg.boundary_mask |= 1u << j;
    }
    dg.lr = (float)g.outer_lr; dg.beta = (float)g.outer_beta;
    dg.c_beta = (float)(g.dn_c * g.outer_beta);
    dg.cb_boundary = (float)((1.0 - g.dn_c * g.dn_N + g.dn_c) * g.outer_beta);
    dg.Nf = (float)g.dn_N;
    dg.dc_lambda = (float)rule.dc_lambda;
    dg.buffered = rule.kind == ALS_RULE_BUFFER;
    RUN(dn_group(ctx->theta, ctx->m, ctx->delta, dg, P, st));
    ctx->t += dg.G;
  }
  if (restart_flag && !fused_restart)
    for (int j = 0; j < n_group; j++) {
      Worker& w = ctx->w[workers[j]];
      RUN(restart_copy(ctx->theta, w.theta, w.start, w.lp, P, st));
    }
  if (restart_flag)
    for (int j = 0; j < n_group; j++) ctx->w[workers[j]].t_restart = ctx->t;
  ALS_HIP(hipEventRecord(ctx->server_ev, st));
  // Whatever touches these replicas next (their local steps, or a later sync) is ordered
  // after this call.
  for (int j = 0; j < n_group; j++) {
    ALS_HIP(hipEventRecord(ctx->w[workers[j]].ready_ev, st));
    ALS_HIP(hipEventRecord(ctx->w[workers[j]].done_ev, st));
  }
  return ALS_OK;
}

extern "C" int als_outer_apply_dn(als_ctx* ctx, const int32_t* workers, int n_group, int restart_flag) {
  als_outer_rule rule;
  memset(&rule, 0, sizeof rule);
  rule.kind = ALS_RULE_DN; rule.staleness_threshold = -1;
  return outer_apply(ctx, workers, n_group, restart_flag, rule);
}

extern "C" int als_outer_apply_rule(als_ctx* ctx, const int32_t* workers, int n_group, int restart_flag,
                                    const als_outer_rule* rule) {
  if (!rule) return set_error(ALS_ERR_INVALID, "rule is null");
  return outer_apply(ctx, workers, n_group, restart_flag, *rule);
}

extern "C" int64_t als_worker_staleness(als_ctx* ctx, int worker) {
  if (check_ctx_worker(ctx, worker)) return -1;
  return ctx->t - ctx->w[worker].t_restart;
}

extern "C" int als_sync(als_ctx* ctx, int worker) {
  if (!ctx) return set_error(ALS_ERR_INVALID, "context is null");
  if (worker < 0) return sync_all(ctx);
  int rc = check_ctx_worker(ctx, worker);
  if (rc) return rc;
  ALS_HIP(hipStreamSynchronize(ctx->w[worker].stream));
  return ALS_OK;
}

static float* vector_ptr(als_ctx* ctx, int which, int worker) {
  switch (which) {
    case ALS_VEC_THETA: return ctx->theta;
    case ALS_VEC_MOMENTUM: return ctx->m;
    case ALS_VEC_DELTA: return ctx->delta;
    default: break;
  }
  if (worker < 0 || worker >= (int)ctx->w.size()) return nullptr;
  Worker& w = ctx->w[worker];
  switch (which) {
    case ALS_VEC_WORKER_THETA: return w.theta;
    case ALS_VEC_WORKER_START: return w.start;
    case ALS_VEC_ADAM_M: return w.adam_m;
    case ALS_VEC_ADAM_V: return w.adam_v;
    case ALS_VEC_GRAD: return w.grad;
    default: return nullptr;
  }
}

extern "C" int als_get_vector(als_ctx* ctx, int which, int worker, float* host_out) {
  if (!ctx || !host_out) return set_error(ALS_ERR_INVALID, "null argument");
  float* p = vector_ptr(ctx, which, worker);
  if (!p) return set_error(ALS_ERR_INVALID, "unknown vector %d / worker %d", which, worker);
  RUN(sync_all(ctx));
  ALS_HIP(hipMemcpy(host_out, p, (size_t)ctx->L.P * 4, hipMemcpyDeviceToHost));
  return ALS_OK;
}

extern "C" int als_set_vector(als_ctx* ctx, int which, int worker, const float* host_in) {
  if (!ctx || !host_in) return set_error(ALS_ERR_INVALID, "null argument");
  float* p = vector_ptr(ctx, which, worker);
  if (!p) return set_error(ALS_ERR_INVALID, "unknown vector %d / worker %d", which, worker);
  RUN(sync_all(ctx));
  ALS_HIP(hipMemcpy(p, host_in, (size_t)ctx->L.P * 4, hipMemcpyHostToDevice));
  if (which == ALS_VEC_WORKER_THETA && ctx->bf) {
    Worker& w = ctx->w[worker];
    RUN(cast_copy(w.theta, w.lp, ctx->L.P, 1, w.stream));
    ALS_HIP(hipStreamSynchronize(w.stream));
  }
  return ALS_OK;
}

extern "C" int als_get_losses(als_ctx* ctx, int worker, float* host_out, int n) {
  int rc = check_ctx_worker(ctx, worker);
  if (rc) return rc;
  Worker& w = ctx->w[worker];
  if (!host_out || n < 0 || n > w.last_n) return set_error(ALS_ERR_INVALID, "n outside 0..%d", w.last_n);
  ALS_HIP(hipStreamSynchronize(w.stream));
  memcpy(host_out, w.losses_host, (size_t)n * 4);
  return ALS_OK;
}

extern "C" int64_t als_server_t(als_ctx* ctx) { return ctx ? ctx->t : -1; }
extern "C" int64_t als_worker_adam_steps(als_ctx* ctx, int worker) {
  if (check_ctx_worker(ctx, worker)) return -1;
  return ctx->w[worker].adam_n;
}

// ---- stand-alone kernel entry points ---------------------------------------------------------
extern "C" int als_k_dn_group(float* theta, float* m, float* delta, float* const* theta_start,
                              float* const* theta_worker, void* const* bf16_worker, int G, int64_t P,
                              int N, int64_t t0, double outer_lr, double beta, double c, int restart,
                              void* stream) {
  if (G < 1 || G > ALS_DN_MAX_GROUP || P < 0 || N < 1 || t0 < 0) return set_error(ALS_ERR_INVALID, "G, P, N or t0 out of range");
  if (!(c >= 0 && c <= 1.0 / N + 1e-12)) return set_error(ALS_ERR_INVALID, "c must lie in [0, 1/N]");
  if (P == 0) return ALS_OK;
  if (!theta || !m || !delta || !theta_start || !theta_worker) return set_error(ALS_ERR_INVALID, "null argument");
  DnGroup dg;
  memset(&dg, 0, sizeof dg);
  dg.G = G; dg.restart = restart ? 1 : 0;
  for (int j = 0; j < ALS_DN_MAX_GROUP; j++) dg.weight[j] = 1.0f;
  for (int j = 0; j < G; j++) {
    if (!theta_start[j] || !theta_worker[j]) return set_error(ALS_ERR_INVALID, "null worker vector");
    dg.theta_start[j] = theta_start[j]; dg.theta_worker[j] = theta_worker[j];
    dg.start_out[j] = theta_start[j];
    dg.lp_out[j] = bf16_worker ? (bf16*)bf16_worker[j] : nullptr;
    if ((t0 + j + 1) % N == 0) dg.boundary_mask |= 1u << j;
  }
  dg.lr = (float)outer_lr; dg.beta = (float)beta; dg.c_beta = (float)(c * beta);
  dg.cb_boundary = (float)((1.0 - c * N + c) * beta); dg.Nf = (float)N;
  return dn_group(theta, m, delta, dg, P, (hipStream_t)stream);
}

extern "C" int als_k_adamw(float* theta, const float* grad, float* m, float* v, void* bf16_out, int64_t P,
                           int64_t P_decay, int64_t step, double lr, double beta1, double beta2,
                           double eps, double wd, void* stream) {
  if (P < 0 || P_decay < 0 || step < 1) return set_error(ALS_ERR_INVALID, "P, P_decay or step out of range");
  if (P == 0) return ALS_OK;
  if (!theta || !grad || !m || !v) return set_error(ALS_ERR_INVALID, "null argument");
  AdamArgs a;
  a.lr = (float)lr; a.beta1 = (float)beta1; a.beta2 = (float)beta2; a.eps = (float)eps; a.wd = (float)wd;
  a.bc1 = (float)(1.0 - pow(beta1, (double)step));
  a.bc2 = (float)(1.0 - pow(beta2, (double)step));
  return adamw(theta, grad, m, v, (bf16*)bf16_out, P, P_decay, a, (hipStream_t)stream);
}

extern "C" int als_k_gemm(const void* A, const void* B, void* C, int M, int N, int K, int a_layout,
                          int b_layout, int in_dtype, int out_dtype, int use_mfma, void* ws_dev,
                          size_t ws_bytes, void* stream) {
  if (!A || !B || !C) return set_error(ALS_ERR_INVALID, "null argument");
  GemmDesc g;
  memset(&g, 0, sizeof g);
  g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K; g.a_layout = a_layout; g.b_layout = b_layout;
  g.lda = a_layout == 0 ? K : M; g.ldb = b_layout == 0 ? N : K; g.ldc = N;
  g.in_bf16 = in_dtype == ALS_DTYPE_BF16; g.c_bf16 = out_dtype == ALS_DTYPE_BF16; g.epi = EPI_STORE;
  g.ws = (float*)ws_dev; g.ws_bytes = ws_dev ? ws_bytes : 0;
  if (use_mfma) {
    if (!gemm_mfma_supported(g)) return set_error(ALS_ERR_INVALID, "shape/dtype not supported by the MFMA GEMM");
    return gemm_mfma(g, (hipStream_t)stream);
  }
  return gemm_generic(g, (hipStream_t)stream);
}

// ---- the entry point that allocates nothing ---------------------------------------------------
// Split-K partials of the stand-alone weight-gradient product live in this file-scope device
// array instead of a caller workspace.  Every GPU the library runs on holds its own copy of the
// array until the process ends; the host only ever uses the address hipGetSymbolAddress() returns
// for the current device (the array's name in host code is a stand-in, not a device address).
static __device__ __align__(256) unsigned char scratch[ALS_STATIC_WS_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];   // per device, filled at the first call on that device

int scratch_for_current_device(void** out) {
  int dev = -1;
  ALS_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return als::set_error(ALS_ERR_INVALID, "device index %d out of range", dev);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    ALS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return als::set_error(ALS_ERR_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return ALS_OK;
}
}  // namespace

extern "C" int als_k_gemm_static_ws(const void* A, const void* B, void* C, int M, int N, int K, int a_layout,
                                    int b_layout, int out_dtype, void* stream) {
  if (!A || !B || !C) return set_error(ALS_ERR_INVALID, "null argument");
  if (M <= 0 || N <= 0 || K <= 0) return set_error(ALS_ERR_INVALID, "M, N, K must be positive");
  // two fp32 partials of the product must fit, so that the split along K has room to happen
  if ((uint64_t)M * (uint64_t)N * sizeof(float) * 2 > (uint64_t)ALS_STATIC_WS_BYTES)
    return set_error(ALS_ERR_INVALID, "als_k_gemm_static_ws: M x N = %d x %d exceeds the static workspace "
                     "(2 fp32 partials must fit %zu bytes, i.e. M*N <= %zu)", M, N, (size_t)ALS_STATIC_WS_BYTES,
                     (size_t)ALS_STATIC_WS_BYTES / 8);
  GemmDesc g;
  memset(&g, 0, sizeof g);
  g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K; g.a_layout = a_layout; g.b_layout = b_layout;
  g.lda = a_layout == 0 ? K : M; g.ldb = b_layout == 0 ? N : K; g.ldc = N;
  g.in_bf16 = 1; g.c_bf16 = out_dtype == ALS_DTYPE_BF16; g.epi = EPI_STORE;
  if (!gemm_mfma_supported(g)) return set_error(ALS_ERR_INVALID, "shape/dtype not supported by the MFMA GEMM");
  void* ws = nullptr;
  int rc = scratch_for_current_device(&ws);
  if (rc) return rc;
  g.ws = (float*)ws; g.ws_bytes = ALS_STATIC_WS_BYTES;
  return gemm_mfma(g, (hipStream_t)stream);
}

namespace {
// workspace of the stand-alone grouped weight-gradient call: tables, then partial tiles
struct DwWsLayout { size_t probs, items, split, partial, total; };
DwWsLayout dw_ws_layout(int n, int n_tiles) {
  auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
  DwWsLayout l;
  l.probs = 0;
  l.items = up(l.probs + (size_t)n * sizeof(DwProblem));
  l.split = up(l.items + (size_t)dw_plan_max_items(n_tiles) * sizeof(DwItem));
  l.partial = up(l.split + (size_t)dw_plan_max_split(n_tiles) * sizeof(DwSplitTile));
  l.total = l.partial + (size_t)DW_PLAN_CUS * 65536 * sizeof(float);
  return l;
}
int dw_tiles(int n, const int* M, const int* N) {
  int t = 0;
  for (int i = 0; i < n; i++) t += ((M[i] + 255) / 256) * ((N[i] + 255) / 256);
  return t;
}
}  // namespace

extern "C" size_t als_k_gemm_dw_grouped_ws_bytes(int n, const int* M, const int* N) {
  if (n <= 0 || !M || !N) return 0;
  for (int i = 0; i < n; i++)
    if (M[i] <= 0 || N[i] <= 0) return 0;
  return dw_ws_layout(n, dw_tiles(n, M, N)).total;
}

extern "C" int als_k_gemm_dw_grouped(int n, const void* const* X, const void* const* dY, float* const* C,
                                     const int* M, const int* N, int K, void* ws_dev, size_t ws_bytes,
                                     void* stream) {
  if (n <= 0 || n > 4096 || !X || !dY || !C || !M || !N || !ws_dev) return set_error(ALS_ERR_INVALID, "null argument or bad count");
  std::vector<DwProblem> probs(n);
  for (int i = 0; i < n; i++) {
    if (!X[i] || !dY[i] || !C[i]) return set_error(ALS_ERR_INVALID, "product %d: null pointer", i);
    if (M[i] <= 0 || N[i] <= 0 || !dw_group_supported(M[i], N[i], K, M[i], N[i]))
      return set_error(ALS_ERR_INVALID, "product %d: %d x %d over %d not supported (M, N multiples of 128, K of 64)", i, M[i], N[i], K);
    if ((uintptr_t)X[i] % 16 || (uintptr_t)dY[i] % 16 || (uintptr_t)C[i] % 16)
      return set_error(ALS_ERR_INVALID, "product %d: pointers must be 16-byte aligned", i);
    probs[i] = DwProblem{(const bf16*)X[i], (const bf16*)dY[i], C[i], M[i], N[i], M[i], N[i], {0, 0}};
  }
  const int n_tiles = dw_tiles(n, M, N);
  const DwWsLayout l = dw_ws_layout(n, n_tiles);
  if ((uintptr_t)ws_dev % 256) return set_error(ALS_ERR_INVALID, "workspace must be 256-byte aligned");
  if (ws_bytes < l.total) return set_error(ALS_ERR_INVALID, "workspace too small: %zu bytes given, %zu needed", ws_bytes, l.total);
  std::vector<DwItem> items(dw_plan_max_items(n_tiles));
  std::vector<DwSplitTile> split(dw_plan_max_split(n_tiles) + 1);
  const DwPlan plan = dw_group_plan(probs.data(), n, K, items.data(), split.data());
  char* ws = (char*)ws_dev;
  hipStream_t st = (hipStream_t)stream;
  ALS_HIP(hipMemcpyAsync(ws + l.probs, probs.data(), (size_t)n * sizeof(DwProblem), hipMemcpyHostToDevice, st));
  ALS_HIP(hipMemcpyAsync(ws + l.items, items.data(), (size_t)plan.n_items * sizeof(DwItem), hipMemcpyHostToDevice, st));
  if (plan.n_split)
    ALS_HIP(hipMemcpyAsync(ws + l.split, split.data(), (size_t)plan.n_split * sizeof(DwSplitTile), hipMemcpyHostToDevice, st));
  ALS_HIP(hipStreamSynchronize(st));   // the tables above are host temporaries
  return dw_group_launch((const DwProblem*)(ws + l.probs), (const DwItem*)(ws + l.items),
                         (const DwSplitTile*)(ws + l.split), plan, (float*)(ws + l.partial), st);
}

// Host only: the work-item list als_k_gemm_dw_grouped would launch for these shapes, for checking
// on the CPU that it covers every tile and every K slice exactly once and stays inside its tables.
extern "C" int als_k_gemm_dw_grouped_plan(int n, const int* M, const int* N, int K, int max_items,
                                          int32_t* items_out, int max_split, int32_t* split_out,
                                          int32_t* counts_out) {
  if (n <= 0 || n > 4096 || !M || !N || !counts_out || (max_items > 0 && !items_out) || (max_split > 0 && !split_out))
    return set_error(ALS_ERR_INVALID, "null argument or bad count");
  std::vector<DwProblem> probs(n);
  for (int i = 0; i < n; i++) {
    if (M[i] <= 0 || N[i] <= 0 || !dw_group_supported(M[i], N[i], K, M[i], N[i]))
      return set_error(ALS_ERR_INVALID, "product %d: %d x %d over %d not supported (M, N multiples of 128, K of 64)", i, M[i], N[i], K);
    probs[i] = DwProblem{nullptr, nullptr, nullptr, M[i], N[i], M[i], N[i], {0, 0}};
  }
  const int n_tiles = dw_tiles(n, M, N);
  std::vector<DwItem> items(dw_plan_max_items(n_tiles));
  std::vector<DwSplitTile> split(dw_plan_max_split(n_tiles) + 1);
  const DwPlan plan = dw_group_plan(probs.data(), n, K, items.data(), split.data());
  counts_out[0] = plan.n_items; counts_out[1] = plan.n_split; counts_out[2] = plan.n_partial_tiles;
  counts_out[3] = dw_plan_max_items(n_tiles); counts_out[4] = dw_plan_max_split(n_tiles); counts_out[5] = DW_PLAN_CUS;
  for (int i = 0; i < plan.n_items && i < max_items; i++) {
    const DwItem& it = items[i];
    int32_t* o = items_out + 6 * (int64_t)i;
    o[0] = it.prob; o[1] = it.tm; o[2] = it.tn; o[3] = it.slot; o[4] = it.slice0; o[5] = it.nk;
  }
  for (int i = 0; i < plan.n_split && i < max_split; i++) {
    const DwSplitTile& t = split[i];
    int32_t* o = split_out + 5 * (int64_t)i;
    o[0] = t.prob; o[1] = t.tm; o[2] = t.tn; o[3] = t.slot0; o[4] = t.nslots;
  }
  return ALS_OK;
}

extern "C" int als_k_gemm_ex(const void* A, const void* B, void* C, int M, int N, int K, int a_layout,
                             int b_layout, int in_dtype, int out_dtype, int use_mfma, int epi, const float* R,
                             void* C2, const void* U, void* ws_dev, size_t ws_bytes, void* stream) {
  if (!A || !B || !C) return set_error(ALS_ERR_INVALID, "null argument");
  if (epi < 0 || epi > 3 || (epi == EPI_RESID && !R) || (epi == EPI_GELU && !C2) || (epi == EPI_DGELU && !U))
    return set_error(ALS_ERR_INVALID, "epilogue %d lacks its operand", epi);
  GemmDesc g;
  memset(&g, 0, sizeof g);
  g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K; g.a_layout = a_layout; g.b_layout = b_layout;
  g.lda = a_layout == 0 ? K : M; g.ldb = b_layout == 0 ? N : K; g.ldc = N;
  g.in_bf16 = in_dtype == ALS_DTYPE_BF16; g.c_bf16 = out_dtype == ALS_DTYPE_BF16; g.epi = epi;
  g.R = R; g.ldr = N; g.C2 = C2; g.U = U;
  g.ws = (float*)ws_dev; g.ws_bytes = ws_dev ? ws_bytes : 0;
  if (use_mfma) {
    if (!gemm_mfma_supported(g)) return set_error(ALS_ERR_INVALID, "shape/dtype/epilogue not supported by the MFMA GEMM");
    return gemm_mfma(g, (hipStream_t)stream);
  }
  return gemm_generic(g, (hipStream_t)stream);
}

extern "C" int als_k_attention_fwd(const void* qkv, void* o, float* lse, int B, int S, int h, int dh,
                                   int dtype, int use_mfma, void* stream) {
  if (!qkv || !o || !lse) return set_error(ALS_ERR_INVALID, "null argument");
  int bf = dtype == ALS_DTYPE_BF16;
  if (use_mfma) {
    if (!attention_mfma_supported(S, dh, bf)) return set_error(ALS_ERR_INVALID, "shape/dtype not supported by the MFMA attention");
    return attention_fwd_mfma(qkv, o, lse, B, S, h, dh, (hipStream_t)stream);
  }
  return attention_fwd_generic(qkv, o, lse, B, S, h, dh, bf, (hipStream_t)stream);
}

extern "C" int als_k_attention_bwd(const void* qkv, const void* o, const void* d_o, const float* lse,
                                   float* dscratch, void* dqkv, int B, int S, int h, int dh, int dtype,
                                   int use_mfma, void* stream) {
  if (!qkv || !o || !d_o || !lse || !dscratch || !dqkv) return set_error(ALS_ERR_INVALID, "null argument");
  int bf = dtype == ALS_DTYPE_BF16;
  if (use_mfma) {
    if (!attention_mfma_supported(S, dh, bf)) return set_error(ALS_ERR_INVALID, "shape/dtype not supported by the MFMA attention");
    return attention_bwd_mfma(qkv, o, d_o, lse, dscratch, dqkv, B, S, h, dh, (hipStream_t)stream);
  }
  return attention_bwd_generic(qkv, o, d_o, lse, dscratch, dqkv, B, S, h, dh, bf, (hipStream_t)stream);
}
