/*
 * als.h -- C ABI of the asynchronous Local-SGD hot path for AMD MI355X (gfx950).
 *
 * What the library computes (citations are to arXiv 2401.09135, "Asynchronous Local-SGD
 * Training for Language Modeling"):
 *   - a worker's local round: the inner loop of Alg. 1 (sample a batch, next-token
 *     cross-entropy loss of a decoder-only transformer, gradient, AdamW update), with the
 *     AdamW state kept on the worker across rounds (appendix, "Inner Optimizer States");
 *   - the server's sync() step of Alg. 2: pseudo-gradient (Alg. 1, delta = theta_start -
 *     theta_worker) fed to the Delayed Nesterov update of Alg. 3, then the restart of the
 *     synchronised workers from the new global parameters (Alg. 2, train(W_completed));
 *   - Dynamic Local Updates (Eq. DyLU) and the deterministic event order of Alg. 2 with
 *     get_worker() from the appendix on a simulated clock.
 *
 * Conventions
 *   - Every function returns an int status: 0 = ALS_OK, negative = error.  Nothing throws
 *     and nothing aborts; als_last_error() returns the text of the calling thread's last
 *     error.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *   - The library never allocates device memory: als_init() carves everything out of one
 *     caller-owned arena, and the als_k_* entry points work on the caller's buffers only.
 *     Streams are borrowed hipStream_t handles passed as void*.
 *   - Flat parameter vector layout (row-major tensors, fp32), P elements in total:
 *       E [V,d], Ppos [S,d], per layer: Wqkv [d,3a] (columns q|k|v, head-major inside each,
 *       a = h * head width = attention width, equal to d unless head_dim is set), Wo [a,d],
 *       W1 [d,ff], W2 [ff,d]; Wout [d,V]; then the RMSNorm gains: per layer g1 [d],
 *       g2 [d]; finally gf [d].  The first P_decay elements (everything but the gains) are
 *       weight-decayed.
 *   - Model (reading of "decoder-only transformer", appendix "Network Architecture"):
 *     pre-norm blocks, RMSNorm (or gain-only LayerNorm, norm_kind), causal softmax attention
 *     scaled by 1/sqrt(head width), tanh-GELU FFN, learned positions, no bias, untied output
 *     matrix, loss averaged over B*S positions.
 */
#ifndef ALS_H
#define ALS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ALS_OK 0
#define ALS_ERR_INVALID (-1) /* bad argument or configuration */
#define ALS_ERR_ARENA (-2)   /* arena too small or misaligned */
#define ALS_ERR_HIP (-3)     /* a HIP runtime call failed */
#define ALS_ERR_STATE (-4)   /* call not valid in the context's current state */

#define ALS_DTYPE_F32 0  /* fp32 everywhere (debug / reference mode) */
#define ALS_DTYPE_BF16 1 /* bf16 GEMM and attention operands and activations between them (logits
                            included), fp32 accumulation, residual stream, master weights, optimiser */
#define ALS_NORM_RMS 0
#define ALS_NORM_LAYER 1

#define ALS_MAX_WORKERS 64

/* Plain-data configuration.  Notation follows the paper: k workers, N = Delayed Nesterov
 * buffer size, c = momentum activation, eps_outer/beta = outer learning rate and decay. */
typedef struct als_config {
  int32_t n_layers;        /* L */
  int32_t d_model;         /* d, multiple of 64 */
  int32_t n_heads;         /* h; head width = head_dim if set, else d/h; must be 32 or 64 */
  int32_t d_ff;            /* ff, multiple of 64 */
  int32_t vocab;           /* V */
  int32_t seq_len;         /* S (tokens carry S+1 per sample), <= 1024 */
  int32_t batch;           /* B samples per worker step */
  int32_t dtype;           /* ALS_DTYPE_* */
  int32_t n_workers;       /* k, 1..ALS_MAX_WORKERS */
  int32_t dn_N;            /* N >= 1 */
  int32_t max_local_steps; /* capacity of the per-worker loss buffer (>= largest n_steps) */
  int32_t flags;           /* bit 0: disable the MFMA kernels (use the generic ones); bit 1: one weight-gradient
                              product per matrix inside the backward loop instead of the grouped launch of all
                              layers' weight gradients at its end (bf16 with widths that are multiples of 128) */
  int32_t head_dim;        /* 0 = d/h; otherwise the attention width h*head_dim may differ from d
                              (the paper's 60M / 150M models: 16 heads of 64 on d = 896) */
  int32_t norm_kind;       /* ALS_NORM_RMS (0): y = x rsqrt(mean x^2 + eps) g ; ALS_NORM_LAYER (1): layer
                              normalisation with a gain and no bias, y = (x - mean x) rsqrt(var x + eps) g */
  double adam_beta1, adam_beta2, adam_eps, weight_decay; /* AdamW (inner optimiser) */
  double outer_lr, outer_beta, dn_c;                     /* Alg. 3: epsilon, beta, c in [0,1/N] */
  double norm_eps;                                       /* RMSNorm epsilon */
} als_config;

typedef struct als_ctx als_ctx;

const char* als_last_error(void);

/* Number of parameters P / decayed parameters for a configuration (0 if invalid). */
int64_t als_param_count(const als_config* cfg);
int64_t als_param_count_decayed(const als_config* cfg);
/* Offsets (in elements) of the tensors of the flat layout, in layout order:
 * E, Ppos, L x (Wqkv, Wo, W1, W2), Wout, L x (g1, g2), gf  ->  4L + 2L + 4 entries.
 * offsets_out has room for n_out int64; returns the number of tensors or a negative error. */
int als_param_offsets(const als_config* cfg, int64_t* offsets_out, int n_out);

/* Device bytes als_init() needs for this configuration (0 if invalid). */
size_t als_arena_bytes(const als_config* cfg);

/* Alg. 2 lines 1-3: theta <- theta0, create the k workers.  Copies theta0_host (P floats,
 * host) into the server parameters and into every worker replica (master, round-start
 * snapshot and, in bf16 mode, the bf16 working copy); zeroes the outer momentum m, the
 * buffer Delta, the event counter t and every worker's AdamW state.
 *   arena_dev/arena_bytes: caller-owned device memory, 256-byte aligned, >= als_arena_bytes;
 *     must outlive the context.  streams: n_streams >= 1 borrowed hipStream_t; worker w runs
 *     on streams[w % n_streams].  *out is owned by the library until als_destroy(). */
int als_init(const als_config* cfg, void* arena_dev, size_t arena_bytes, const float* theta0_host,
             void* const* streams, int n_streams, als_ctx** out);
int als_destroy(als_ctx* ctx);

/* Alg. 1 inner loop for one worker, from its current replica: n_steps times (loss on the
 * next batch, backward, AdamW with this step's learning rate).  AdamW moments and step
 * count persist across calls and restarts.
 *   tokens_dev: int32 [n_steps, B, S+1] on the device, values in [0, V) (ids outside the range
 *     are clamped into it, never dereferenced); position s predicts s+1.  lr_host: n_steps
 *     floats (host), read before the call returns.
 *   loss_host_or_null: if non-null receives the n_steps mean losses and the call waits for
 *     the worker's stream; if null the call only enqueues work (fetch the losses later with
 *     als_get_losses after als_sync).  Does not touch server state. */
int als_worker_local_steps(als_ctx* ctx, int worker, int n_steps, const int32_t* tokens_dev,
                           const float* lr_host, float* loss_host_or_null);

/* sync() of Alg. 2 for a group of workers that completed together, in the given order.
 * For each: g = theta_start - theta_worker (pseudo-gradient), one event of Alg. 3
 * (Delta += g; every N-th event m <- beta m + Delta/N, theta <- theta - eps((1-cN+c) beta m
 * + g/N), Delta <- 0; otherwise theta <- theta - eps(c beta m + g/N)), t <- t+1.  If
 * restart_flag != 0 every listed worker then restarts from the new theta (replica, snapshot,
 * bf16 copy); its AdamW state is kept.  A group call equals n_group single calls followed by
 * the restarts.  Ordered after the listed workers' pending local steps. */
int als_outer_apply_dn(als_ctx* ctx, const int32_t* workers, int n_group, int restart_flag);

/* The comparison rules of the paper's "Existing Fixes" paragraph on the same fused pass.
 *   kind ALS_RULE_DN: Alg. 3 as in als_outer_apply_dn (N = 1 gives asynchronous DiLoCo).
 *   kind ALS_RULE_BUFFER: "Async. Buffer": pseudo-gradients are only added to Delta; every N-th
 *     event applies one Nesterov step (Eq. nesterov) on Delta/N and clears Delta.
 *   poly_exponent a > 0: "Poly": each pseudo-gradient is scaled by (1 + staleness)^-a, staleness =
 *     server events applied since that worker's replica (re)started (the paper uses a = 0.5).
 *   staleness_threshold >= 0: "PolyThres": a worker whose staleness exceeds it is discarded (no
 *     server change, no event counted) but still restarts; -1 = never.
 *   dc_lambda > 0: "Delay Comp.": g <- g + lambda g*g*(theta_now - theta_at_worker_start),
 *     elementwise, before any discount.
 * Everything else (ordering, restart, errors) as als_outer_apply_dn. */
#define ALS_RULE_DN 0
#define ALS_RULE_BUFFER 1
typedef struct als_outer_rule {
  int32_t kind;
  int32_t staleness_threshold;
  double poly_exponent;
  double dc_lambda;
} als_outer_rule;
int als_outer_apply_rule(als_ctx* ctx, const int32_t* workers, int n_group, int restart_flag,
                         const als_outer_rule* rule);
/* Server events applied since the worker's replica (re)started, or -1 on a bad argument. */
int64_t als_worker_staleness(als_ctx* ctx, int worker);

/* Eq. (DyLU) and, optionally, the event order of Alg. 2 on the simulated clock.  Host only.
 *   H_out[k] = max(1, floor(speeds[i] / max(speeds) * H_max)) in fp64.
 *   If ev_worker is non-null, also writes the first n_events sync events: worker index,
 *   completion time (job length = H_i / speeds[i]; all start at 0; restarts at tau_sync +
 *   tau_grace) and a flag that is 1 on the last event of a group whose workers then restart
 *   (ties and arrivals within tau_grace of the group's first event share a group; ties are
 *   ordered by worker index).  ev_time and ev_group_end may be null.
 *   Errors: k <= 0 or > ALS_MAX_WORKERS, non-finite or non-positive speed, H_max < 1,
 *   tau_grace < 0 or non-finite, n_events < 0. */
int als_dylu_schedule(const double* speeds, int k, int H_max, double tau_grace, int n_events,
                      int32_t* H_out, int32_t* ev_worker, double* ev_time, int32_t* ev_group_end);

/* Bookkeeping of train() (appendix pseudocode), host only.
 * als_lr_schedule: Eq. (lr) for the n consecutive steps t0 .. t0+n-1 of one data shard: linear
 *   warm-up t * eta_max / t_warmup while t < t_warmup, then eta_min + (eta_max - eta_min) / 2 *
 *   (1 + cos(pi * ratio)), ratio = (t - t_warmup) / max(T - t_warmup, 0) clamped to [0, 1] (1 if
 *   the denominator is 0).  Computed in fp64, written as float into lr_out[n] (the lr_host
 *   argument of als_worker_local_steps).  Errors: negative counts, eta_min < 0, eta_max < eta_min.
 * als_shard_sample: Eq. (data_sample): p_i proportional to max(sizes_i / sum sizes - learned_i /
 *   sum learned, 0) (progress share 0 while nothing is learned; the size shares if no shard is
 *   behind); writes p into p_out[k] (nullable) and the shard chosen by inverse CDF from the
 *   caller's uniform number u in [0, 1) into *shard_out (nullable). */
int als_lr_schedule(int64_t t0, int n, int64_t t_warmup, int64_t T, double eta_max, double eta_min,
                    float* lr_out);
int als_shard_sample(const double* sizes, const double* learned, int k, double u, double* p_out,
                     int32_t* shard_out);

/* ---- helpers for tests and drivers -------------------------------------------------- */
#define ALS_VEC_THETA 0        /* server parameters              (worker ignored) */
#define ALS_VEC_MOMENTUM 1     /* server momentum m              (worker ignored) */
#define ALS_VEC_DELTA 2        /* server buffer Delta            (worker ignored) */
#define ALS_VEC_WORKER_THETA 3 /* worker replica (fp32 master)   */
#define ALS_VEC_WORKER_START 4 /* worker round-start snapshot    */
#define ALS_VEC_ADAM_M 5
#define ALS_VEC_ADAM_V 6
#define ALS_VEC_GRAD 7         /* worker's last gradient         */
/* Copy a length-P fp32 vector to / from the host; waits for all pending work first. */
int als_get_vector(als_ctx* ctx, int which, int worker, float* host_out);
int als_set_vector(als_ctx* ctx, int which, int worker, const float* host_in);
/* Wait for one worker's stream (worker >= 0) or for everything (worker < 0). */
int als_sync(als_ctx* ctx, int worker);
/* Losses of the worker's most recent als_worker_local_steps call (n <= its n_steps). */
int als_get_losses(als_ctx* ctx, int worker, float* host_out, int n);
/* Number of Alg. 3 events applied so far (t). */
int64_t als_server_t(als_ctx* ctx);
/* AdamW step count of a worker. */
int64_t als_worker_adam_steps(als_ctx* ctx, int worker);
/* Loss and gradient of one batch at the worker's current replica, no update (for parity
 * tests): tokens_dev int32 [B,S+1]; loss_host 1 float; the gradient is left in
 * ALS_VEC_GRAD.  Synchronous. */
int als_worker_loss_grad(als_ctx* ctx, int worker, const int32_t* tokens_dev, float* loss_host);

/* ---- stand-alone kernels on caller-owned device vectors (microbenchmarks, unit tests) -- */
/* One pass of Alg. 3 over G pseudo-gradients g_j = theta_start[j] - theta_worker[j] applied
 * in order to (theta, m, delta), all fp32 device vectors of length P; t0 = number of events
 * applied before the call.  If restart != 0, afterwards writes the new theta into every
 * theta_worker[j], theta_start[j] and (if bf16_worker[j] non-null) a bf16 copy.  G <= 16.
 * Pointer arrays are host arrays of device pointers. */
int als_k_dn_group(float* theta, float* m, float* delta, float* const* theta_start,
                   float* const* theta_worker, void* const* bf16_worker, int G, int64_t P, int N,
                   int64_t t0, double outer_lr, double beta, double c, int restart, void* stream);
/* One fused AdamW step over flat fp32 device vectors of length P (first P_decay decayed);
 * step = 1-based count used for bias correction; bf16_out may be null. */
int als_k_adamw(float* theta, const float* grad, float* m, float* v, void* bf16_out, int64_t P,
                int64_t P_decay, int64_t step, double lr, double beta1, double beta2, double eps,
                double wd, void* stream);
/* C = A.B with fp32 accumulation.  a_layout 0: A is [M,K] row-major, 1: A is stored [K,M];
 * b_layout 0: B is [K,N] row-major, 1: B is stored [N,K].  in_dtype/out_dtype ALS_DTYPE_*;
 * use_mfma != 0 selects the MFMA kernel (bf16 inputs, M,N multiples of 128, K of 64).
 * ws_dev/ws_bytes: optional device scratch for split-K partials (may be null / 0). */
int als_k_gemm(const void* A, const void* B, void* C, int M, int N, int K, int a_layout,
               int b_layout, int in_dtype, int out_dtype, int use_mfma, void* ws_dev,
               size_t ws_bytes, void* stream);
/* Same with an epilogue: epi 0 store, 1 C(fp32) = R + A.B (R fp32 [M,N]), 2 C = gelu'(A.B) and
 * C2 = gelu(A.B) (both bf16), 3 C = (A.B) * U (U bf16 [M,N]).  Unused pointers may be null. */
int als_k_gemm_ex(const void* A, const void* B, void* C, int M, int N, int K, int a_layout,
                  int b_layout, int in_dtype, int out_dtype, int use_mfma, int epi, const float* R,
                  void* C2, const void* U, void* ws_dev, size_t ws_bytes, void* stream);
/* All n weight gradients C_i = X_i^T dY_i of a backward pass (Alg. 1, inner step: the gradient of
 * every weight matrix is a product over the batch's K tokens) as ONE launch of the MFMA kernel:
 * X_i is [K, M_i] and dY_i [K, N_i], both bf16 row-major, C_i [M_i, N_i] fp32; M_i, N_i multiples of
 * 128, K of 64, pointers 16-byte aligned.  Whole rounds of 256 x 256 tiles run over the full K and
 * write C_i directly; the tiles of the last partial round are split along K into partial tiles that
 * are added in a fixed order, so results do not depend on timing.  ws_dev: device scratch (256-byte
 * aligned) of at least als_k_gemm_dw_grouped_ws_bytes(n, M, N) bytes (tables and partial tiles);
 * the call uploads its tables and waits for that upload on the stream before it launches.
 * Errors (ALS_ERR_INVALID): null pointers, unsupported shapes, workspace too small. */
size_t als_k_gemm_dw_grouped_ws_bytes(int n, const int* M, const int* N);
int als_k_gemm_dw_grouped(int n, const void* const* X, const void* const* dY, float* const* C,
                          const int* M, const int* N, int K, void* ws_dev, size_t ws_bytes, void* stream);
/* For callers that cannot allocate device memory and have no workspace to lend (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): als_k_gemm on the MFMA
 * path (bf16 operands, M, N multiples of 128, K of 64) with the split-K partials of the
 * weight-gradient layout (a_layout 1, b_layout 0) kept in a file-scope device array of
 * ALS_STATIC_WS_BYTES that every GPU the library runs on holds until the process ends.  Calls no
 * hipMalloc / hipFree or any allocating routine.  Results equal als_k_gemm with a workspace of
 * ALS_STATIC_WS_BYTES, bit for bit.  Errors (ALS_ERR_INVALID): null pointers, shapes the MFMA
 * kernel does not take, M * N * 8 > ALS_STATIC_WS_BYTES (two fp32 partials must fit).  All calls
 * on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or
 * threads) race on it; calls on one stream are ordered.  Nothing in the array has to start at
 * zero: every partial is written in full before it is read.  The current device must be the
 * stream's device. */
#define ALS_STATIC_WS_BYTES ((size_t)64 << 20)
int als_k_gemm_static_ws(const void* A, const void* B, void* C, int M, int N, int K, int a_layout,
                         int b_layout, int out_dtype, void* stream);
/* Causal attention forward / backward on packed qkv [B*S, 3d] (q|k|v, head-major), dtype
 * ALS_DTYPE_*: o [B*S,d] same dtype, lse fp32 [B,h,S]; backward takes d_o and returns dqkv. */
int als_k_attention_fwd(const void* qkv, void* o, float* lse, int B, int S, int h, int dh,
                        int dtype, int use_mfma, void* stream);
int als_k_attention_bwd(const void* qkv, const void* o, const void* d_o, const float* lse,
                        float* dscratch, void* dqkv, int B, int S, int h, int dh, int dtype,
                        int use_mfma, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ALS_H */
