// HBM-bound kernels of the hot path: fused AdamW (inner optimiser), fused pseudo-gradient +
// Delayed Nesterov event(s) + worker restart (Alg. 3 and the restart of Alg. 2), embedding,
// RMSNorm, softmax cross-entropy and the small reductions around them.
#include "common.h"
#include <math.h>

namespace als {

static inline int blocks_for(int64_t n_items, int per_block, int cap) {
  int64_t b = (n_items + per_block - 1) / per_block;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return (int)b;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

__device__ __forceinline__ void store_bf16x4(bf16* p, float4 v) {
  bf16x4 o;
  o[0] = (bf16)v.x; o[1] = (bf16)v.y; o[2] = (bf16)v.z; o[3] = (bf16)v.w;
  *reinterpret_cast<bf16x4*>(p) = o;
}

// ------------------------------------------------------------------------------------------
// AdamW, one pass over the flat vectors: reads grad, theta, m, v; writes theta, m, v and the
// bf16 working copy.  16 + 12 (+2) bytes per parameter.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float adam_one(float& th, float g, float& m, float& v, bool decay,
                                          const AdamArgs& a) {
  m = a.beta1 * m + (1.0f - a.beta1) * g;
  v = a.beta2 * v + (1.0f - a.beta2) * g * g;
  float mhat = m / a.bc1;
  float vhat = v / a.bc2;
  float upd = mhat / (sqrtf(vhat) + a.eps);
  if (decay) upd += a.wd * th;
  th -= a.lr * upd;
  return th;
}

// Streaming kernels below move 4 float4 per lane and iteration with non-temporal accesses
// (nothing they touch is reused before it leaves the caches): measured 6.0-6.1 TB/s on MI355X
// against 6.35 TB/s for a plain copy.
#define STREAM_U 4
__device__ __forceinline__ f32x4 ldnt(const float* p, int64_t i4) {
  return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p) + i4);
}
__device__ __forceinline__ void stnt(float* p, int64_t i4, f32x4 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p) + i4);
}
__device__ __forceinline__ void stnt_bf16(bf16* p, int64_t i4, f32x4 v) {
  bf16x4 o;
  o[0] = (bf16)v[0]; o[1] = (bf16)v[1]; o[2] = (bf16)v[2]; o[3] = (bf16)v[3];
  __builtin_nontemporal_store(o, reinterpret_cast<bf16x4*>(p) + i4);
}
static inline int stream_blocks(int64_t n4, int u) {
  int64_t b = (n4 + 256 * u - 1) / (256 * u);
  return (int)(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

__global__ __launch_bounds__(256) void adamw_kernel(float* __restrict__ theta,
                                                    const float* __restrict__ grad,
                                                    float* __restrict__ m, float* __restrict__ v,
                                                    bf16* __restrict__ lp, int64_t n4,
                                                    int64_t decay4, AdamArgs a) {
  const int64_t stride = (int64_t)gridDim.x * 256 * STREAM_U;
  for (int64_t i0 = (int64_t)blockIdx.x * 256 * STREAM_U + threadIdx.x; i0 < n4; i0 += stride) {
    f32x4 th[STREAM_U], g[STREAM_U], mm[STREAM_U], vv[STREAM_U];
#pragma unroll
    for (int u = 0; u < STREAM_U; u++) {
      int64_t i = i0 + u * 256;
      if (i < n4) { th[u] = ldnt(theta, i); g[u] = ldnt(grad, i); mm[u] = ldnt(m, i); vv[u] = ldnt(v, i); }
    }
#pragma unroll
    for (int u = 0; u < STREAM_U; u++) {
      int64_t i = i0 + u * 256;
      if (i < n4) {
        bool dec = i < decay4;
#pragma unroll
        for (int e = 0; e < 4; e++) {
          float t = th[u][e], mo = mm[u][e], ve = vv[u][e];
          adam_one(t, g[u][e], mo, ve, dec, a);
          th[u][e] = t; mm[u][e] = mo; vv[u][e] = ve;
        }
        stnt(theta, i, th[u]); stnt(m, i, mm[u]); stnt(v, i, vv[u]);
        if (lp) stnt_bf16(lp, i, th[u]);
      }
    }
  }
}

__global__ void adamw_tail_kernel(float* theta, const float* grad, float* m, float* v, bf16* lp,
                                  int64_t begin, int64_t P, int64_t P_decay, AdamArgs a) {
  int64_t i = begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= P) return;
  float th = theta[i], mm = m[i], vv = v[i];
  adam_one(th, grad[i], mm, vv, i < P_decay, a);
  theta[i] = th; m[i] = mm; v[i] = vv;
  if (lp) lp[i] = (bf16)th;
}

int adamw(float* theta, const float* grad, float* m, float* v, bf16* lp, int64_t P,
          int64_t P_decay, const AdamArgs& a, hipStream_t st) {
  if (P <= 0) return ALS_OK;
  // the vector body covers whole float4 groups that do not straddle the decay boundary
  int64_t n4 = 0, decay4 = 0;
  if (P_decay % 4 == 0 || P_decay >= P) {
    n4 = P / 4;
    decay4 = P_decay >= P ? n4 : P_decay / 4;
  }
  if (n4 > 0) {
    hipLaunchKernelGGL(adamw_kernel, dim3(stream_blocks(n4, STREAM_U)), dim3(256), 0, st, theta, grad, m, v,
                       lp, n4, decay4, a);
    ALS_CHECK_LAUNCH();
  }
  int64_t begin = n4 * 4;
  if (begin < P) {
    int blocks = blocks_for(P - begin, 256, 1 << 30);
    hipLaunchKernelGGL(adamw_tail_kernel, dim3(blocks), dim3(256), 0, st, theta, grad, m, v, lp,
                       begin, P, P_decay, a);
    ALS_CHECK_LAUNCH();
  }
  return ALS_OK;
}

// ------------------------------------------------------------------------------------------
// Pseudo-gradient + Delayed Nesterov for a group of G workers in one pass, optionally fused
// with the restart copy.  Per element, in event order j = 0..G-1:
//   g = theta_start_j - theta_worker_j ; Delta += g
//   N-th event:  m = beta m + Delta/N ; theta -= eps ((1 - cN + c) beta m + g/N) ; Delta = 0
//   otherwise:   theta -= eps (c beta m + g/N)
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void dn_event_scalar(float& th, float& mm, float& de, float ts, float tw,
                                                bool boundary, bool use_m, float wj, const DnGroup& g) {
  float gj = ts - tw;
  // delay compensation: g + lambda g g (theta_now - theta_at_worker_start)
  if (g.dc_lambda != 0.0f) gj = gj + g.dc_lambda * gj * gj * (th - ts);
  if (wj != 1.0f) gj = wj * gj;  // staleness discount
  de += gj;
  if (g.buffered) {  // buffered averaging: Nesterov on Delta/N at every N-th event, nothing in between
    if (boundary) {
      float gbar = de / g.Nf;
      mm = g.beta * mm + gbar;
      th = th - g.lr * (g.beta * mm + gbar);
      de = 0.0f;
    }
    return;
  }
  if (boundary) {
    mm = g.beta * mm + de / g.Nf;
    th = th - g.lr * (g.cb_boundary * mm + gj / g.Nf);
    de = 0.0f;
  } else if (use_m) {
    th = th - g.lr * (g.c_beta * mm + gj / g.Nf);
  } else {
    th = th - g.lr * (gj / g.Nf);
  }
}

// U float4 per lane in flight (4 for one or two events, fewer for larger groups, whose 2 G
// worker vectors already keep many loads in flight).
template <int U>
__global__ __launch_bounds__(256) void dn_group_kernel(float* theta, float* m, float* delta, DnGroup g,
                                                       int64_t n4) {
  const bool use_m = g.c_beta != 0.0f;
  const bool touch_m = use_m || g.boundary_mask != 0u;
  const int64_t stride = (int64_t)gridDim.x * 256 * U;
  for (int64_t i0 = (int64_t)blockIdx.x * 256 * U + threadIdx.x; i0 < n4; i0 += stride) {
    f32x4 th[U], de[U], mm[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
      int64_t i = i0 + u * 256;
      mm[u] = (f32x4){0.f, 0.f, 0.f, 0.f};
      if (i < n4) {
        th[u] = ldnt(theta, i); de[u] = ldnt(delta, i);
        if (touch_m) mm[u] = ldnt(m, i);
      }
    }
    if constexpr (U == 4) {   // one or two events: everything is requested at once
      for (int j = 0; j < g.G; j++) {
        f32x4 ts[U], tw[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
          int64_t i = i0 + u * 256;
          if (i < n4) { ts[u] = ldnt(g.theta_start[j], i); tw[u] = ldnt(g.theta_worker[j], i); }
        }
        const bool boundary = (g.boundary_mask >> j) & 1u;
        const float wj = g.weight[j];
#pragma unroll
        for (int u = 0; u < U; u++)
          if (i0 + u * 256 < n4) {
#pragma unroll
            for (int e = 0; e < 4; e++) {
              float t = th[u][e], mo = mm[u][e], d = de[u][e];
              dn_event_scalar(t, mo, d, ts[u][e], tw[u][e], boundary, use_m, wj, g);
              th[u][e] = t; mm[u][e] = mo; de[u][e] = d;
            }
          }
      }
    } else {
    // Events are taken four at a time, and the worker vectors of the NEXT four are requested
    // before the current four are applied: the loop over events has a run-time trip count, and
    // without this every event would wait for its own two loads with nothing else in flight.
    f32x4 tsA[4][U], twA[4][U], tsB[4][U], twB[4][U];
    auto load4 = [&](int j0, f32x4 (&ts)[4][U], f32x4 (&tw)[4][U]) {
#pragma unroll
      for (int jj = 0; jj < 4; jj++)
        if (j0 + jj < g.G) {
#pragma unroll
          for (int u = 0; u < U; u++) {
            int64_t i = i0 + u * 256;
            if (i < n4) { ts[jj][u] = ldnt(g.theta_start[j0 + jj], i); tw[jj][u] = ldnt(g.theta_worker[j0 + jj], i); }
          }
        }
    };
    auto apply4 = [&](int j0, const f32x4 (&ts)[4][U], const f32x4 (&tw)[4][U]) {
#pragma unroll
      for (int jj = 0; jj < 4; jj++)
        if (j0 + jj < g.G) {
          const bool boundary = (g.boundary_mask >> (j0 + jj)) & 1u;
          const float wj = g.weight[j0 + jj];
#pragma unroll
          for (int u = 0; u < U; u++)
            if (i0 + u * 256 < n4) {
#pragma unroll
              for (int e = 0; e < 4; e++) {
                float t = th[u][e], mo = mm[u][e], d = de[u][e];
                dn_event_scalar(t, mo, d, ts[jj][u][e], tw[jj][u][e], boundary, use_m, wj, g);
                th[u][e] = t; mm[u][e] = mo; de[u][e] = d;
              }
            }
        }
    };
    load4(0, tsA, twA);
    for (int j0 = 0; j0 < g.G; j0 += 8) {
      if (j0 + 4 < g.G) load4(j0 + 4, tsB, twB);
      apply4(j0, tsA, twA);
      if (j0 + 8 < g.G) load4(j0 + 8, tsA, twA);
      if (j0 + 4 < g.G) apply4(j0 + 4, tsB, twB);
    }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
      int64_t i = i0 + u * 256;
      if (i < n4) {
        stnt(theta, i, th[u]); stnt(delta, i, de[u]);
        if (g.boundary_mask != 0u) stnt(m, i, mm[u]);
        if (g.restart)
          for (int j = 0; j < g.G; j++) {
            stnt(g.theta_worker[j], i, th[u]); stnt(g.start_out[j], i, th[u]);
            if (g.lp_out[j]) stnt_bf16(g.lp_out[j], i, th[u]);
          }
      }
    }
  }
}

// scalar tail (P not a multiple of 4)
__global__ void dn_group_tail_kernel(float* theta, float* m, float* delta, DnGroup g, int64_t begin, int64_t P) {
  int64_t i = begin + threadIdx.x;
  if (i >= P) return;
  const bool use_m = g.c_beta != 0.0f;
  float th = theta[i], de = delta[i], mm = (use_m || g.boundary_mask) ? m[i] : 0.0f;
  for (int j = 0; j < g.G; j++)
    dn_event_scalar(th, mm, de, g.theta_start[j][i], g.theta_worker[j][i], (g.boundary_mask >> j) & 1u, use_m, g.weight[j], g);
  theta[i] = th; delta[i] = de;
  if (g.boundary_mask) m[i] = mm;
  if (g.restart)
    for (int j = 0; j < g.G; j++) {
      g.theta_worker[j][i] = th; g.start_out[j][i] = th;
      if (g.lp_out[j]) g.lp_out[j][i] = (bf16)th;
    }
}

// Restart of the G workers of a group from the new theta as a pass of its own: read 4, write 10 G
// bytes per parameter.  A write-dominated pass runs closer to the HBM peak than the same writes
// mixed into the event pass (whose 2 G + 3 read streams and 3 G + 3 write streams together reached
// 61-64 % of the peak; the event pass alone runs at the single-event rate, this one near the
// write-only rate), which more than pays for reading theta once more.
__global__ __launch_bounds__(256) void restart_group_kernel(const float* __restrict__ theta, DnGroup g, int64_t P) {
  const int64_t n4 = P / 4;
  const int64_t stride = (int64_t)gridDim.x * 256 * STREAM_U;
  for (int64_t i0 = (int64_t)blockIdx.x * 256 * STREAM_U + threadIdx.x; i0 < n4; i0 += stride) {
    f32x4 t[STREAM_U];
#pragma unroll
    for (int u = 0; u < STREAM_U; u++)
      if (i0 + u * 256 < n4) t[u] = ldnt(theta, i0 + u * 256);
    for (int j = 0; j < g.G; j++) {
#pragma unroll
      for (int u = 0; u < STREAM_U; u++)
        if (i0 + u * 256 < n4) reinterpret_cast<f32x4*>(g.theta_worker[j])[i0 + u * 256] = t[u];
#pragma unroll
      for (int u = 0; u < STREAM_U; u++)
        if (i0 + u * 256 < n4) reinterpret_cast<f32x4*>(g.start_out[j])[i0 + u * 256] = t[u];
      if (g.lp_out[j]) {
#pragma unroll
        for (int u = 0; u < STREAM_U; u++)
          if (i0 + u * 256 < n4) {
            bf16x4 o;
            o[0] = (bf16)t[u][0]; o[1] = (bf16)t[u][1]; o[2] = (bf16)t[u][2]; o[3] = (bf16)t[u][3];
            reinterpret_cast<bf16x4*>(g.lp_out[j])[i0 + u * 256] = o;
          }
      }
    }
  }
  if (blockIdx.x == 0) {
    for (int64_t i = n4 * 4 + threadIdx.x; i < P; i += blockDim.x) {
      float t = theta[i];
      for (int j = 0; j < g.G; j++) {
        g.theta_worker[j][i] = t; g.start_out[j][i] = t;
        if (g.lp_out[j]) g.lp_out[j][i] = (bf16)t;
      }
    }
  }
}

int dn_group(float* theta, float* m, float* delta, const DnGroup& g_in, int64_t P, hipStream_t st) {
  // groups of more than two workers: events first, then the restart as its own pass
  const bool split_restart = g_in.restart && g_in.G > 2;
  DnGroup g = g_in;
  if (split_restart) g.restart = 0;
  if (g.G < 1 || g.G > ALS_DN_MAX_GROUP) return set_error(ALS_ERR_INVALID, "dn_group: G out of range");
  if (P <= 0) return ALS_OK;
  int64_t n4 = P / 4;
  if (n4 > 0) {
    if (g.G <= 2)
      hipLaunchKernelGGL(dn_group_kernel<4>, dim3(stream_blocks(n4, 4)), dim3(256), 0, st, theta, m, delta, g, n4);
    else
      hipLaunchKernelGGL(dn_group_kernel<2>, dim3(stream_blocks(n4, 2)), dim3(256), 0, st, theta, m, delta, g, n4);
    ALS_CHECK_LAUNCH();
  }
  if (n4 * 4 < P) {
    hipLaunchKernelGGL(dn_group_tail_kernel, dim3(1), dim3(64), 0, st, theta, m, delta, g, n4 * 4, P);
    ALS_CHECK_LAUNCH();
  }
  if (split_restart) {
    hipLaunchKernelGGL(restart_group_kernel, dim3(stream_blocks(n4 > 0 ? n4 : 1, STREAM_U)), dim3(256), 0, st, theta, g, P);
    ALS_CHECK_LAUNCH();
  }
  return ALS_OK;
}

// theta -> worker master, round-start snapshot and bf16 working copy (read 4, write up to 10).
__global__ __launch_bounds__(256) void restart_kernel(const float* __restrict__ theta,
                                                      float* __restrict__ master,
                                                      float* __restrict__ start,
                                                      bf16* __restrict__ lp, int64_t P) {
  const int64_t n4 = P / 4;
  const int64_t stride = (int64_t)gridDim.x * 256 * STREAM_U;
  for (int64_t i0 = (int64_t)blockIdx.x * 256 * STREAM_U + threadIdx.x; i0 < n4; i0 += stride) {
    f32x4 t[STREAM_U];
#pragma unroll
    for (int u = 0; u < STREAM_U; u++)
      if (i0 + u * 256 < n4) t[u] = ldnt(theta, i0 + u * 256);
#pragma unroll
    for (int u = 0; u < STREAM_U; u++) {
      int64_t i = i0 + u * 256;
      if (i < n4) {
        if (master) stnt(master, i, t[u]);
        if (start) stnt(start, i, t[u]);
        if (lp) stnt_bf16(lp, i, t[u]);
      }
    }
  }
  if (blockIdx.x == 0) {
    for (int64_t i = n4 * 4 + threadIdx.x; i < P; i += blockDim.x) {
      float t = theta[i];
      if (master) master[i] = t;
      if (start) start[i] = t;
      if (lp) lp[i] = (bf16)t;
    }
  }
}

int restart_copy(const float* theta, float* master, float* start, bf16* lp, int64_t P,
                 hipStream_t st) {
  if (P <= 0) return ALS_OK;
  hipLaunchKernelGGL(restart_kernel, dim3(stream_blocks(P / 4, STREAM_U)), dim3(256), 0, st, theta, master,
                     start, lp, P);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

int cast_copy(const float* src, void* dst, int64_t n, int dst_bf16, hipStream_t st) {
  if (dst_bf16) return restart_copy(src, nullptr, nullptr, (bf16*)dst, n, st);
  return restart_copy(src, (float*)dst, nullptr, nullptr, n, st);
}

// ------------------------------------------------------------------------------------------
// Embedding: x[b*S+s,:] = E[tok[b,s],:] + Ppos[s,:]   (tokens are [B,S+1]; inputs are s < S)
// ------------------------------------------------------------------------------------------
__global__ void embed_fwd_kernel(const int32_t* __restrict__ tok, const float* __restrict__ E,
                                 const float* __restrict__ Ppos, float* __restrict__ x, int S,
                                 int d, int V) {
  int t = blockIdx.x;
  int b = t / S, s = t % S;
  int id = tok[(int64_t)b * (S + 1) + s];
  id = id < 0 ? 0 : (id >= V ? V - 1 : id);  // out-of-range ids are clamped, never dereferenced
  const float4* e = reinterpret_cast<const float4*>(E + (int64_t)id * d);
  const float4* p = reinterpret_cast<const float4*>(Ppos + (int64_t)s * d);
  float4* o = reinterpret_cast<float4*>(x + (int64_t)t * d);
  for (int c = threadIdx.x; c < d / 4; c += blockDim.x) {
    float4 a = e[c], q = p[c];
    o[c] = make_float4(a.x + q.x, a.y + q.y, a.z + q.z, a.w + q.w);
  }
}

int embed_fwd(const int32_t* tok, const float* E, const float* Ppos, float* x, int B, int S, int d,
              int V, hipStream_t st) {
  int threads = d / 4 < 256 ? (d / 4 < 64 ? 64 : d / 4) : 256;
  hipLaunchKernelGGL(embed_fwd_kernel, dim3(B * S), dim3(threads), 0, st, tok, E, Ppos, x, S, d, V);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

// Embedding gradient without float atomics, so that a step is bit-reproducible.
// (1) embed_sort: one workgroup per step orders the T input positions by token id with a
//     counting sort whose ranks are fixed by position order: offset[v] .. offset[v+1] delimit
//     the positions holding token v inside pos[].  It depends on the tokens only, so one
//     launch prepares every step of a local round.
// (2) embed_bwd: a pass over 32-position chunks of that list and a pass over vocabulary rows
//     (described at the kernels below).
// dPpos[s,:] = sum_b dx[b,s,:] in batch order.
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int n = __shfl_up(v, o, 64);
    if (lane >= o) v += n;
  }
  return v;
}

__global__ __launch_bounds__(1024) void embed_sort_kernel(const int32_t* __restrict__ tok, int B,
                                                          int S, int V, int32_t* offset,
                                                          int32_t* rank, int32_t* pos) {
  __shared__ int ids[1024];
  __shared__ int wsum[16];
  __shared__ int carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int T = B * S;
  const int32_t* tk = tok + (int64_t)blockIdx.x * B * (S + 1);
  int32_t* cnt = offset + (int64_t)blockIdx.x * (V + 1);
  int32_t* rk = rank + (int64_t)blockIdx.x * T;
  int32_t* ps = pos + (int64_t)blockIdx.x * T;
  for (int v = tid; v <= V; v += 1024) cnt[v] = 0;
  __syncthreads();
  for (int c0 = 0; c0 < T; c0 += 1024) {
    int t = c0 + tid;
    bool active = t < T;
    int id = active ? tk[(int64_t)(t / S) * (S + 1) + (t % S)] : -1;
    if (active) id = id < 0 ? 0 : (id >= V ? V - 1 : id);
    ids[tid] = id;
    __syncthreads();
    int before = 0, after = 0;
    int n = T - c0 < 1024 ? T - c0 : 1024;
    if (active)
      for (int j = 0; j < n; j++) {
        int eq = ids[j] == id;
        before += eq & (j < tid);
        after += eq & (j > tid);
      }
    int base = active ? cnt[id] : 0;
    if (active) rk[t] = base + before;
    __syncthreads();
    if (active && after == 0) cnt[id] = base + before + 1;
    __syncthreads();
  }
  // exclusive prefix sum of cnt[0..V] in place
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int v0 = 0; v0 <= V; v0 += 1024) {
    int v = v0 + tid;
    int x = v <= V ? cnt[v] : 0;
    int incl = wave_incl_scan(x, lane);
    if (lane == 63) wsum[wv] = incl;
    __syncthreads();
    int add = carry_s;
    for (int w = 0; w < wv; w++) add += wsum[w];
    if (v <= V) cnt[v] = incl - x + add;
    __syncthreads();
    if (tid == 1023) carry_s = add + incl;
    __syncthreads();
  }
  for (int t = tid; t < T; t += 1024) {
    int id = tk[(int64_t)(t / S) * (S + 1) + (t % S)];
    id = id < 0 ? 0 : (id >= V ? V - 1 : id);
    ps[cnt[id] + rk[t]] = t;
  }
}

int embed_sort(const int32_t* tok, int n_steps, int B, int S, int V, int32_t* offset, int32_t* rank,
               int32_t* pos, hipStream_t st) {
  if (n_steps <= 0) return ALS_OK;
  hipLaunchKernelGGL(embed_sort_kernel, dim3(n_steps), dim3(1024), 0, st, tok, B, S, V, offset, rank, pos);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

// dE from the sorted position list, in two passes that never leave a long list to one block:
//   chunks: block c walks sorted positions [32 c, 32 c + 32), 8 row loads in flight, adding the
//     rows of equal tokens in list order.  A token whose whole list lies in this chunk is written
//     to dE at once; a list that continues into the next chunk leaves its part in scratch slot
//     (c, 1); one that began in an earlier chunk leaves its part in slot (c, 0).
//   rows: one wavefront per vocabulary row: zeros for a token that does not occur, nothing for a
//     list inside one chunk, else slot (first, 1) + slots (first+1 .. last, 0) in chunk order.
// Every sum has a fixed order, so the result does not depend on scheduling.
constexpr int EMB_CH = 32;
#define EMB_MAXD4 4  // float4 slots per lane in the row pass: d <= 1024

__global__ __launch_bounds__(128) void embed_bwd_chunks_kernel(
    const int32_t* __restrict__ tok, const int32_t* __restrict__ offset, const int32_t* __restrict__ pos,
    const float* __restrict__ dx, float* __restrict__ dE, float* __restrict__ scratch, int T, int S, int V, int d) {
  __shared__ int s_pos[EMB_CH], s_tok[EMB_CH];
  const int c = blockIdx.x, i0 = c * EMB_CH, tid = threadIdx.x;
  const int n = T - i0 < EMB_CH ? T - i0 : EMB_CH;
  const int d4 = d / 4;
  if (tid < n) {
    int t = pos[i0 + tid];
    int id = tok[(int64_t)(t / S) * (S + 1) + (t % S)];
    s_pos[tid] = t;
    s_tok[tid] = id < 0 ? 0 : (id >= V ? V - 1 : id);
  }
  __syncthreads();
  const float4* dx4 = reinterpret_cast<const float4*>(dx);
  for (int col = tid; col < d4; col += 128) {   // one pass for d <= 512
    auto flush = [&](int v, float4 acc) {
      int beg = offset[v], end = offset[v + 1];
      int cf = beg / EMB_CH, cl = (end - 1) / EMB_CH;
      float4* dst = cf == cl ? reinterpret_cast<float4*>(dE) + (int64_t)v * d4
                             : reinterpret_cast<float4*>(scratch) + (int64_t)(2 * c + (c == cf ? 1 : 0)) * d4;
      dst[col] = acc;
    };
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    int cur = s_tok[0];
    for (int j0 = 0; j0 < n; j0 += 8) {
      float4 x[8];
#pragma unroll
      for (int u = 0; u < 8; u++) {
        int j = j0 + u;
        x[u] = j < n ? dx4[(int64_t)s_pos[j] * d4 + col] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < 8; u++) {
        int j = j0 + u;
        if (j < n) {
          int tk = s_tok[j];
          if (tk != cur) {  // block-uniform
            flush(cur, acc);
            acc = make_float4(0.f, 0.f, 0.f, 0.f);
            cur = tk;
          }
          acc.x += x[u].x; acc.y += x[u].y; acc.z += x[u].z; acc.w += x[u].w;
        }
      }
    }
    flush(cur, acc);
  }
}

__global__ __launch_bounds__(256) void embed_bwd_rows_kernel(const int32_t* __restrict__ offset,
                                                             const float* __restrict__ scratch,
                                                             float* __restrict__ dE, int V, int d) {
  const int lane = threadIdx.x & 63;
  const int v = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (v >= V) return;
  const int beg = offset[v], end = offset[v + 1];
  const int d4 = d / 4;
  float4* out = reinterpret_cast<float4*>(dE) + (int64_t)v * d4;
  if (beg == end) {
    for (int col = lane; col < d4; col += 64) out[col] = make_float4(0.f, 0.f, 0.f, 0.f);
    return;
  }
  const int cf = beg / EMB_CH, cl = (end - 1) / EMB_CH;
  if (cf == cl) return;  // written by the chunk pass
  const float4* sc = reinterpret_cast<const float4*>(scratch);
#pragma unroll
  for (int s = 0; s < EMB_MAXD4; s++) {
    int col = lane + 64 * s;
    if (col >= d4) break;
    float4 acc = sc[(int64_t)(2 * cf + 1) * d4 + col];
#pragma unroll 8
    for (int c = cf + 1; c <= cl; c++) {
      float4 x = sc[(int64_t)(2 * c) * d4 + col];
      acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    out[col] = acc;
  }
}

__global__ void embed_bwd_pos_kernel(const float* __restrict__ dx, float* __restrict__ dPpos,
                                     int B, int S, int d) {
  int s = blockIdx.x;
  const int d4 = d / 4;
  const float4* dx4 = reinterpret_cast<const float4*>(dx);
  for (int c = threadIdx.x; c < d4; c += blockDim.x) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int b0 = 0; b0 < B; b0 += 8) {  // 8 loads in flight, added in batch order
      float4 x[8];
#pragma unroll
      for (int u = 0; u < 8; u++)
        x[u] = b0 + u < B ? dx4[((int64_t)(b0 + u) * S + s) * d4 + c] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int u = 0; u < 8; u++)
        if (b0 + u < B) { acc.x += x[u].x; acc.y += x[u].y; acc.z += x[u].z; acc.w += x[u].w; }
    }
    reinterpret_cast<float4*>(dPpos)[(int64_t)s * d4 + c] = acc;
  }
}

int embed_bwd(const int32_t* tok, const int32_t* offset, const int32_t* pos, const float* dx, float* dE,
              float* dPpos, float* scratch, int B, int S, int d, int V, hipStream_t st) {
  if (d > 256 * EMB_MAXD4 || d % 4) return set_error(ALS_ERR_INVALID, "embed_bwd: d unsupported");
  const int T = B * S;
  hipLaunchKernelGGL(embed_bwd_chunks_kernel, dim3((T + EMB_CH - 1) / EMB_CH), dim3(128), 0, st, tok, offset,
                     pos, dx, dE, scratch, T, S, V, d);
  ALS_CHECK_LAUNCH();
  hipLaunchKernelGGL(embed_bwd_rows_kernel, dim3((V + 3) / 4), dim3(256), 0, st, offset, scratch, dE, V, d);
  ALS_CHECK_LAUNCH();
  int threads = d / 4 < 256 ? (d / 4 < 64 ? 64 : d / 4) : 256;
  hipLaunchKernelGGL(embed_bwd_pos_kernel, dim3(S), dim3(threads), 0, st, dx, dPpos, B, S, d);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

// ------------------------------------------------------------------------------------------
// Normalisation over the feature dimension, one 64-lane wavefront per row:
//   RMSNorm   (CENTER = false): y = x * rsqrt(mean(x^2) + eps) * g
//   LayerNorm (CENTER = true):  y = (x - mean(x)) * rsqrt(mean((x - mean(x))^2) + eps) * g   (no bias)
// rstd[row] is saved for the backward pass (which recomputes the mean from the row it reads).
// ------------------------------------------------------------------------------------------
#define RMS_MAXD4 4  // float4 slots per lane: d <= 1024
template <typename OT, bool CENTER>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ g,
                                                          OT* __restrict__ y,
                                                          float* __restrict__ rstd, int T, int d,
                                                          float eps) {
  int lane = threadIdx.x & 63;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T) return;
  const int d4 = d / 4;
  const float4* xr = reinterpret_cast<const float4*>(x + (int64_t)row * d);
  const float4* g4 = reinterpret_cast<const float4*>(g);
  float4 v[RMS_MAXD4];  // the row is read once and stays in registers (d <= 1024)
  float sum = 0.0f;
#pragma unroll
  for (int s = 0; s < RMS_MAXD4; s++) {
    int c = lane + 64 * s;
    v[s] = c < d4 ? xr[c] : make_float4(0.f, 0.f, 0.f, 0.f);
    sum += (v[s].x + v[s].y) + (v[s].z + v[s].w);
  }
  const float mean = CENTER ? wave_sum(sum) / (float)d : 0.0f;
  float ss = 0.0f;
#pragma unroll
  for (int s = 0; s < RMS_MAXD4; s++) {
    int c = lane + 64 * s;
    if (CENTER && c < d4) { v[s].x -= mean; v[s].y -= mean; v[s].z -= mean; v[s].w -= mean; }
    ss += v[s].x * v[s].x + v[s].y * v[s].y + v[s].z * v[s].z + v[s].w * v[s].w;
  }
  ss = wave_sum(ss);
  float r = 1.0f / sqrtf(ss / (float)d + eps);
  if (lane == 0) rstd[row] = r;
  OT* yr = y + (int64_t)row * d;
#pragma unroll
  for (int s = 0; s < RMS_MAXD4; s++) {
    int c = lane + 64 * s;
    if (c < d4) {
      float4 gg = g4[c];
      float4 o = make_float4(v[s].x * r * gg.x, v[s].y * r * gg.y, v[s].z * r * gg.z, v[s].w * r * gg.w);
      if (sizeof(OT) == 2) store_bf16x4(reinterpret_cast<bf16*>(yr) + 4 * c, o);
      else reinterpret_cast<float4*>(yr)[c] = o;
    }
  }
}

int rmsnorm_fwd(const float* x, const float* g, void* y, float* rstd, int T, int d, float eps,
                int out_bf16, int center, hipStream_t st) {
  if (d > 256 * RMS_MAXD4 || d % 4) return set_error(ALS_ERR_INVALID, "rmsnorm_fwd: d unsupported");
  dim3 grid((T + 3) / 4), block(256);
  if (out_bf16) {
    if (center) hipLaunchKernelGGL((rmsnorm_fwd_kernel<bf16, true>), grid, block, 0, st, x, g, (bf16*)y, rstd, T, d, eps);
    else hipLaunchKernelGGL((rmsnorm_fwd_kernel<bf16, false>), grid, block, 0, st, x, g, (bf16*)y, rstd, T, d, eps);
  } else {
    if (center) hipLaunchKernelGGL((rmsnorm_fwd_kernel<float, true>), grid, block, 0, st, x, g, (float*)y, rstd, T, d, eps);
    else hipLaunchKernelGGL((rmsnorm_fwd_kernel<float, false>), grid, block, 0, st, x, g, (float*)y, rstd, T, d, eps);
  }
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

// Backward: xhat = x rstd (RMSNorm) or (x - mean x) rstd (LayerNorm) ; dxhat = dy g ;
// dx = rstd (dxhat - xhat mean(dxhat xhat))  [LayerNorm: also - mean(dxhat)] ;
// dg = sum_rows dy xhat.  Each block walks rows with a fixed stride and leaves one partial dg
// row; a second kernel adds the partials in a fixed order.
#define RMS_BWD_MAXD4 4  // per-lane float4 slots: supports d <= 1024
// One wavefront per row, each row read once into registers; a wave keeps two rows in flight.
template <typename LT, bool CENTER>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(
    const float* __restrict__ dy, const float* __restrict__ x, const float* __restrict__ rstd,
    const float* __restrict__ g, const float* dx_in, float* dx_out, LT* __restrict__ dx_lp,
    float* __restrict__ partial, int T, int d) {
  extern __shared__ float smem[];  // [4][d]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int d4 = d / 4;
  const float inv_d = 1.0f / (float)d;
  f32x4 dg[RMS_BWD_MAXD4], gg[RMS_BWD_MAXD4];
#pragma unroll
  for (int s = 0; s < RMS_BWD_MAXD4; s++) {
    dg[s] = (f32x4){0.f, 0.f, 0.f, 0.f};
    int c = lane + 64 * s;
    gg[s] = c < d4 ? reinterpret_cast<const f32x4*>(g)[c] : (f32x4){0.f, 0.f, 0.f, 0.f};
  }
  const int stride = gridDim.x * 4;
  for (int row0 = blockIdx.x * 4 + w; row0 < T; row0 += 2 * stride) {
    f32x4 xv[2][RMS_BWD_MAXD4], dv[2][RMS_BWD_MAXD4], av[2][RMS_BWD_MAXD4];
    float r[2], dot[2], m1[2];
    bool ok[2];
#pragma unroll
    for (int u = 0; u < 2; u++) {
      int row = row0 + u * stride;
      ok[u] = row < T;
      r[u] = ok[u] ? rstd[row] : 0.0f;
#pragma unroll
      for (int s = 0; s < RMS_BWD_MAXD4; s++) {
        int c = lane + 64 * s;
        bool in = ok[u] && c < d4;
        int64_t o = (int64_t)row * d4 + c;
        xv[u][s] = in ? reinterpret_cast<const f32x4*>(x)[o] : (f32x4){0.f, 0.f, 0.f, 0.f};
        dv[u][s] = in ? reinterpret_cast<const f32x4*>(dy)[o] : (f32x4){0.f, 0.f, 0.f, 0.f};
        av[u][s] = (in && dx_in) ? reinterpret_cast<const f32x4*>(dx_in)[o] : (f32x4){0.f, 0.f, 0.f, 0.f};
      }
    }
#pragma unroll
    for (int u = 0; u < 2; u++) {
      if (CENTER) {  // the row's mean, recomputed from the row in registers
        float sx = 0.0f;
#pragma unroll
        for (int s = 0; s < RMS_BWD_MAXD4; s++) sx += (xv[u][s][0] + xv[u][s][1]) + (xv[u][s][2] + xv[u][s][3]);
        const float mean = wave_sum(sx) * inv_d;
#pragma unroll
        for (int s = 0; s < RMS_BWD_MAXD4; s++)
          if (lane + 64 * s < d4) xv[u][s] -= mean;
      }
      float acc = 0.0f, acc1 = 0.0f;
#pragma unroll
      for (int s = 0; s < RMS_BWD_MAXD4; s++) {
        xv[u][s] *= r[u];  // xhat
        f32x4 dh = dv[u][s] * gg[s];
        f32x4 t = dh * xv[u][s];
        acc += (t[0] + t[1]) + (t[2] + t[3]);
        if (CENTER) acc1 += (dh[0] + dh[1]) + (dh[2] + dh[3]);
      }
      dot[u] = wave_sum(acc) * inv_d;
      m1[u] = CENTER ? wave_sum(acc1) * inv_d : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < 2; u++) {
      int row = row0 + u * stride;
      if (!ok[u]) continue;
#pragma unroll
      for (int s = 0; s < RMS_BWD_MAXD4; s++) {
        int c = lane + 64 * s;
        if (c < d4) {
          dg[s] += dv[u][s] * xv[u][s];
          f32x4 o = r[u] * (dv[u][s] * gg[s] - m1[u] - xv[u][s] * dot[u]) + av[u][s];
          int64_t oi = (int64_t)row * d4 + c;
          reinterpret_cast<f32x4*>(dx_out)[oi] = o;
          if (dx_lp) {
            if (sizeof(LT) == 2) store_bf16x4(reinterpret_cast<bf16*>(dx_lp) + 4 * oi, make_float4(o[0], o[1], o[2], o[3]));
            else reinterpret_cast<f32x4*>(dx_lp)[oi] = o;
          }
        }
      }
    }
  }
#pragma unroll
  for (int s = 0; s < RMS_BWD_MAXD4; s++) {
    int c = lane + 64 * s;
    if (c < d4) reinterpret_cast<f32x4*>(smem + w * d)[c] = dg[s];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += 256)
    partial[(int64_t)blockIdx.x * d + c] = smem[c] + smem[d + c] + smem[2 * d + c] + smem[3 * d + c];
}

// out[j][c] = sum_b partial[j][b][c] for nset consecutive sets of partials (blockIdx.y = j; the
// outputs are consecutive rows of d floats): 32 columns per block, 32 row groups each adding
// every 32nd partial (8 independent loads in flight: the kernel is pure load latency), combined
// in a fixed order.
__global__ __launch_bounds__(1024) void sum_partials_kernel(const float* __restrict__ partial,
                                                            float* __restrict__ out, int nblk, int d) {
  __shared__ float sh[32][33];
  partial += (int64_t)blockIdx.y * nblk * d;
  out += (int64_t)blockIdx.y * d;
  int cl = threadIdx.x & 31, rg = threadIdx.x >> 5;
  int c = blockIdx.x * 32 + cl;
  float acc = 0.0f;
  if (c < d)
    for (int b0 = rg; b0 < nblk; b0 += 32 * 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; u++) {
        int b = b0 + 32 * u;
        v[u] = b < nblk ? partial[(int64_t)b * d + c] : 0.0f;
      }
#pragma unroll
      for (int u = 0; u < 8; u++) acc += v[u];
    }
  sh[rg][cl] = acc;
  __syncthreads();
  if (rg == 0 && c < d) {
    float t = sh[0][cl];
#pragma unroll
    for (int r = 1; r < 32; r++) t += sh[r][cl];
    out[c] = t;
  }
}

int rmsnorm_bwd_blocks(int T) {
  int b = (T + 3) / 4;
  return b > 256 ? 256 : b;
}

int rmsnorm_bwd(const float* dy, const float* x, const float* rstd, const float* g,
                const float* dx_in, float* dx_out, void* dx_lp, int lp_bf16, float* dg,
                float* partial, int T, int d, int center, hipStream_t st) {
  if (d > 256 * RMS_BWD_MAXD4 || d % 4) return set_error(ALS_ERR_INVALID, "rmsnorm_bwd: d unsupported");
  int nblk = rmsnorm_bwd_blocks(T);
  size_t sm = (size_t)4 * d * sizeof(float);
#define ALS_NORM_BWD(LT, CEN)                                                                                   \
  hipLaunchKernelGGL((rmsnorm_bwd_kernel<LT, CEN>), dim3(nblk), dim3(256), sm, st, dy, x, rstd, g, dx_in, dx_out, \
                     (LT*)dx_lp, partial, T, d)
  if (lp_bf16) {
    if (center) ALS_NORM_BWD(bf16, true); else ALS_NORM_BWD(bf16, false);
  } else {
    if (center) ALS_NORM_BWD(float, true); else ALS_NORM_BWD(float, false);
  }
#undef ALS_NORM_BWD
  ALS_CHECK_LAUNCH();
  if (dg) return rmsnorm_dg_sum(partial, dg, T, d, 1, st);
  return ALS_OK;
}

int rmsnorm_dg_sum(const float* partial, float* dg, int T, int d, int nset, hipStream_t st) {
  hipLaunchKernelGGL(sum_partials_kernel, dim3((d + 31) / 32, nset), dim3(1024), 0, st, partial, dg,
                     rmsnorm_bwd_blocks(T), d);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

// ------------------------------------------------------------------------------------------
// Softmax cross-entropy, one block per row: loss_row = logsumexp - logit[target];
// dlogits = (softmax - onehot) / T.  Logits are fp32, or bf16 (the bf16 path: the output GEMM
// rounds them like every other activation); dlogits may overwrite the logits (same pointer, same
// element type): every element is read before it is written, by the thread that writes it.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_reduce(float v, bool is_max, float* sh) {
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  v = is_max ? wave_max(v) : wave_sum(v);
  __syncthreads();
  if (lane == 0) sh[w] = v;
  __syncthreads();
  int nw = blockDim.x >> 6;
  float r = sh[0];
  for (int i = 1; i < nw; i++) r = is_max ? fmaxf(r, sh[i]) : r + sh[i];
  return r;
}

template <typename IT, typename OT>
__global__ __launch_bounds__(256) void cross_entropy_kernel(const IT* logits, const int32_t* __restrict__ tok,
                                                            float* __restrict__ loss_row, OT* dl, int S, int V,
                                                            float invT) {
  __shared__ float sh[8];
  int t = blockIdx.x;
  int b = t / S, s = t % S;
  int tgt = tok[(int64_t)b * (S + 1) + s + 1];
  tgt = tgt < 0 ? 0 : (tgt >= V ? V - 1 : tgt);
  const IT* lr = logits + (int64_t)t * V;
  const float ltgt = (float)lr[tgt];
  float mx = -INFINITY;
  for (int c = threadIdx.x; c < V; c += blockDim.x) mx = fmaxf(mx, (float)lr[c]);
  mx = block_reduce(mx, true, sh);
  float sum = 0.0f;
  for (int c = threadIdx.x; c < V; c += blockDim.x) sum += expf((float)lr[c] - mx);
  sum = block_reduce(sum, false, sh);   // its barriers also order the read of lr[tgt] before the writes below
  float lse = mx + logf(sum);
  if (threadIdx.x == 0) loss_row[t] = lse - ltgt;
  OT* dr = dl + (int64_t)t * V;
  for (int c = threadIdx.x; c < V; c += blockDim.x) {
    float p = expf((float)lr[c] - lse);
    if (c == tgt) p -= 1.0f;
    dr[c] = (OT)(p * invT);
  }
}

// Same, reading the row once: each thread keeps up to 32 logits in registers, so a block of BS
// threads covers V <= 32 BS (V a multiple of 8).
template <typename IT, typename OT, int BS>
__global__ __launch_bounds__(BS) void cross_entropy_reg_kernel(const IT* logits, const int32_t* __restrict__ tok,
                                                               float* __restrict__ loss_row, OT* dl, int S, int V,
                                                               float invT) {
  __shared__ float sh[16];
  int t = blockIdx.x;
  int b = t / S, s = t % S;
  int tgt = tok[(int64_t)b * (S + 1) + s + 1];
  tgt = tgt < 0 ? 0 : (tgt >= V ? V - 1 : tgt);
  // a lane owns 8 consecutive columns per slot (16-byte loads, one 16-byte bf16 store)
  const IT* row = logits + (int64_t)t * V;
  const float ltgt = (float)row[tgt];
  const int v8 = V / 8;
  f32x4 x[4][2];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int c = threadIdx.x + i * BS;
    if (c < v8) {
      if (sizeof(IT) == 2) {
        bf16x8 r = reinterpret_cast<const bf16x8*>(row)[c];
#pragma unroll
        for (int e = 0; e < 8; e++) x[i][e >> 2][e & 3] = (float)r[e];
      } else {
        x[i][0] = reinterpret_cast<const f32x4*>(row)[2 * c];
        x[i][1] = reinterpret_cast<const f32x4*>(row)[2 * c + 1];
      }
#pragma unroll
      for (int q = 0; q < 2; q++)
        mx = fmaxf(fmaxf(mx, fmaxf(x[i][q][0], x[i][q][1])), fmaxf(x[i][q][2], x[i][q][3]));
    }
  }
  mx = block_reduce(mx, true, sh);
  float sum = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int c = threadIdx.x + i * BS;
    if (c < v8) {
#pragma unroll
      for (int q = 0; q < 2; q++)
#pragma unroll
        for (int e = 0; e < 4; e++) {
          x[i][q][e] = expf(x[i][q][e] - mx);
          sum += x[i][q][e];
        }
    }
  }
  sum = block_reduce(sum, false, sh);
  float inv = 1.0f / sum;
  if (threadIdx.x == 0) loss_row[t] = mx + logf(sum) - ltgt;
  OT* dr = dl + (int64_t)t * V;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int c = threadIdx.x + i * BS;
    if (c < v8) {
      float p[8];
#pragma unroll
      for (int e = 0; e < 8; e++) {
        p[e] = x[i][e >> 2][e & 3] * inv;
        if (8 * c + e == tgt) p[e] -= 1.0f;
        p[e] *= invT;
      }
      if (sizeof(OT) == 2) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = (bf16)p[e];
        *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(dr) + 8 * c) = o;
      } else {
        reinterpret_cast<float4*>(dr)[2 * c] = make_float4(p[0], p[1], p[2], p[3]);
        reinterpret_cast<float4*>(dr)[2 * c + 1] = make_float4(p[4], p[5], p[6], p[7]);
      }
    }
  }
}

int cross_entropy(const void* logits, int logits_bf16, const int32_t* tok, float* loss_row, void* dlogits,
                  int dl_bf16, int B, int S, int V, hipStream_t st) {
  int T = B * S;
  float invT = 1.0f / (float)T;
  if (logits_bf16 && !dl_bf16) return set_error(ALS_ERR_INVALID, "cross_entropy: bf16 logits need bf16 dlogits");
  if (dl_bf16 && V % 8 == 0 && V <= 32 * 1024) {
    const bool big = V > 32 * 256;
#define ALS_CE_LAUNCH(IT, BS)                                                                               \
  hipLaunchKernelGGL((cross_entropy_reg_kernel<IT, bf16, BS>), dim3(T), dim3(BS), 0, st, (const IT*)logits, \
                     tok, loss_row, (bf16*)dlogits, S, V, invT)
    if (logits_bf16) { if (big) ALS_CE_LAUNCH(bf16, 1024); else ALS_CE_LAUNCH(bf16, 256); }
    else             { if (big) ALS_CE_LAUNCH(float, 1024); else ALS_CE_LAUNCH(float, 256); }
#undef ALS_CE_LAUNCH
    ALS_CHECK_LAUNCH();
    return ALS_OK;
  }
  if (logits_bf16)
    hipLaunchKernelGGL((cross_entropy_kernel<bf16, bf16>), dim3(T), dim3(256), 0, st, (const bf16*)logits, tok,
                       loss_row, (bf16*)dlogits, S, V, invT);
  else if (dl_bf16)
    hipLaunchKernelGGL((cross_entropy_kernel<float, bf16>), dim3(T), dim3(256), 0, st, (const float*)logits, tok,
                       loss_row, (bf16*)dlogits, S, V, invT);
  else
    hipLaunchKernelGGL((cross_entropy_kernel<float, float>), dim3(T), dim3(256), 0, st, (const float*)logits, tok,
                       loss_row, (float*)dlogits, S, V, invT);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

__global__ __launch_bounds__(1024) void mean_rows_kernel(const float* __restrict__ v,
                                                         float* __restrict__ out, int T) {
  __shared__ float sh[16];
  float acc = 0.0f;
  for (int i = threadIdx.x; i < T; i += blockDim.x) acc += v[i];
  acc = block_reduce(acc, false, sh);
  if (threadIdx.x == 0) out[0] = acc / (float)T;
}

int mean_rows(const float* loss_row, float* out, int T, hipStream_t st) {
  hipLaunchKernelGGL(mean_rows_kernel, dim3(1), dim3(1024), 0, st, loss_row, out, T);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

}  // namespace als
