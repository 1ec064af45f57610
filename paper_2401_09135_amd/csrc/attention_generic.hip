// Generic causal attention, one wavefront per query (forward, dq) or per key (dk, dv), fp32
// arithmetic on fp32 or bf16 storage.  Reference-mode path and fallback; the fast path is
// the MFMA kernel.  qkv is [B*S, 3d]: q at column hd*dh, k at d + hd*dh, v at 2d + hd*dh.
#include "common.h"
#include <math.h>

namespace als {

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_generic_kernel(const T* __restrict__ qkv,
                                                               T* __restrict__ o,
                                                               float* __restrict__ lse, int S,
                                                               int h, int dh, float scale) {
  extern __shared__ float sm[];  // [4][S] probabilities, then [4][64] query
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int i = blockIdx.x * 4 + w, hd = blockIdx.y, b = blockIdx.z;
  bool active = i < S;
  int d = h * dh;
  int64_t ld = 3 * (int64_t)d;
  const T* base = qkv + (int64_t)b * S * ld + hd * dh;
  float* p = sm + (size_t)w * S;
  float* qs = sm + (size_t)4 * S + w * 64;
  if (active && lane < dh) qs[lane] = (float)base[(int64_t)i * ld + lane];
  __syncthreads();
  float mx = -INFINITY;
  if (active)
    for (int j = lane; j <= i; j += 64) {
      const T* kr = base + (int64_t)j * ld + d;
      float s = 0.0f;
      for (int c = 0; c < dh; c++) s += qs[c] * (float)kr[c];
      s *= scale;
      p[j] = s;
      mx = fmaxf(mx, s);
    }
  mx = wmax(mx);
  float sum = 0.0f;
  if (active)
    for (int j = lane; j <= i; j += 64) {
      float e = expf(p[j] - mx);
      p[j] = e;
      sum += e;
    }
  sum = wsum(sum);
  __syncthreads();
  if (active) {
    if (lane == 0) lse[((int64_t)b * h + hd) * S + i] = mx + logf(sum);
    if (lane < dh) {
      float acc = 0.0f;
      for (int j = 0; j <= i; j++) acc += p[j] * (float)base[(int64_t)j * ld + 2 * d + lane];
      o[((int64_t)b * S + i) * d + hd * dh + lane] = (T)(acc / sum);
    }
  }
}

// dq_i = scale * sum_{j<=i} ds_ij k_j,  ds_ij = p_ij (do_i.v_j - D_i),  D_i = do_i.o_i
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const T* __restrict__ qkv,
                                                          const T* __restrict__ o,
                                                          const T* __restrict__ d_o,
                                                          const float* __restrict__ lse,
                                                          float* __restrict__ Dbuf,
                                                          T* __restrict__ dqkv, int S, int h,
                                                          int dh, float scale) {
  extern __shared__ float sm[];  // [4][S] ds, [4][64] q, [4][64] do
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int i = blockIdx.x * 4 + w, hd = blockIdx.y, b = blockIdx.z;
  bool active = i < S;
  int d = h * dh;
  int64_t ld = 3 * (int64_t)d;
  const T* base = qkv + (int64_t)b * S * ld + hd * dh;
  float* dsb = sm + (size_t)w * S;
  float* qs = sm + (size_t)4 * S + w * 64;
  float* dos = sm + (size_t)4 * S + 256 + w * 64;
  float Di = 0.0f;
  if (active && lane < dh) {
    int64_t oi = ((int64_t)b * S + i) * d + hd * dh + lane;
    float dv = (float)d_o[oi];
    qs[lane] = (float)base[(int64_t)i * ld + lane];
    dos[lane] = dv;
    Di = dv * (float)o[oi];
  }
  Di = wsum(Di);
  __syncthreads();
  if (active) {
    float l = lse[((int64_t)b * h + hd) * S + i];
    if (lane == 0) Dbuf[((int64_t)b * h + hd) * S + i] = Di;
    for (int j = lane; j <= i; j += 64) {
      const T* kr = base + (int64_t)j * ld + d;
      const T* vr = base + (int64_t)j * ld + 2 * d;
      float s = 0.0f, dp = 0.0f;
      for (int c = 0; c < dh; c++) {
        s += qs[c] * (float)kr[c];
        dp += dos[c] * (float)vr[c];
      }
      float pij = expf(s * scale - l);
      dsb[j] = pij * (dp - Di) * scale;
    }
  }
  __syncthreads();
  if (active && lane < dh) {
    float acc = 0.0f;
    for (int j = 0; j <= i; j++) acc += dsb[j] * (float)base[(int64_t)j * ld + d + lane];
    dqkv[((int64_t)b * S + i) * ld + hd * dh + lane] = (T)acc;
  }
}

// dk_j = scale * sum_{i>=j} ds_ij q_i ; dv_j = sum_{i>=j} p_ij do_i
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const T* __restrict__ qkv,
                                                           const T* __restrict__ d_o,
                                                           const float* __restrict__ lse,
                                                           const float* __restrict__ Dbuf,
                                                           T* __restrict__ dqkv, int S, int h,
                                                           int dh, float scale) {
  extern __shared__ float sm[];  // [4][S] p, [4][S] ds, [4][64] k, [4][64] v
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int j = blockIdx.x * 4 + w, hd = blockIdx.y, b = blockIdx.z;
  bool active = j < S;
  int d = h * dh;
  int64_t ld = 3 * (int64_t)d;
  const T* base = qkv + (int64_t)b * S * ld + hd * dh;
  float* pb = sm + (size_t)w * S;
  float* dsb = sm + (size_t)4 * S + (size_t)w * S;
  float* ks = sm + (size_t)8 * S + w * 64;
  float* vs = sm + (size_t)8 * S + 256 + w * 64;
  if (active && lane < dh) {
    ks[lane] = (float)base[(int64_t)j * ld + d + lane];
    vs[lane] = (float)base[(int64_t)j * ld + 2 * d + lane];
  }
  __syncthreads();
  if (active)
    for (int i = j + lane; i < S; i += 64) {
      const T* qr = base + (int64_t)i * ld;
      const T* dor = d_o + ((int64_t)b * S + i) * d + hd * dh;
      float s = 0.0f, dp = 0.0f;
      for (int c = 0; c < dh; c++) {
        s += (float)qr[c] * ks[c];
        dp += (float)dor[c] * vs[c];
      }
      int64_t li = ((int64_t)b * h + hd) * S + i;
      float pij = expf(s * scale - lse[li]);
      pb[i] = pij;
      dsb[i] = pij * (dp - Dbuf[li]) * scale;
    }
  __syncthreads();
  if (active && lane < dh) {
    float dk = 0.0f, dv = 0.0f;
    for (int i = j; i < S; i++) {
      dv += pb[i] * (float)d_o[((int64_t)b * S + i) * d + hd * dh + lane];
      dk += dsb[i] * (float)base[(int64_t)i * ld + lane];
    }
    dqkv[((int64_t)b * S + j) * ld + d + hd * dh + lane] = (T)dk;
    dqkv[((int64_t)b * S + j) * ld + 2 * d + hd * dh + lane] = (T)dv;
  }
}

static int check_shape(int B, int S, int h, int dh) {
  if (B < 1 || S < 1 || h < 1 || dh < 1 || dh > 64 || S > 1024)
    return set_error(ALS_ERR_INVALID, "attention: unsupported shape B=%d S=%d h=%d dh=%d", B, S, h, dh);
  return ALS_OK;
}

int attention_fwd_generic(const void* qkv, void* o, float* lse, int B, int S, int h, int dh, int bf,
                          hipStream_t st) {
  int rc = check_shape(B, S, h, dh);
  if (rc) return rc;
  dim3 grid((S + 3) / 4, h, B), block(256);
  size_t sm = ((size_t)4 * S + 256) * sizeof(float);
  float scale = 1.0f / sqrtf((float)dh);
  if (bf)
    hipLaunchKernelGGL(attn_fwd_generic_kernel<bf16>, grid, block, sm, st, (const bf16*)qkv, (bf16*)o, lse, S, h, dh, scale);
  else
    hipLaunchKernelGGL(attn_fwd_generic_kernel<float>, grid, block, sm, st, (const float*)qkv, (float*)o, lse, S, h, dh, scale);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

int attention_bwd_generic(const void* qkv, const void* o, const void* d_o, const float* lse,
                          float* dscratch, void* dqkv, int B, int S, int h, int dh, int bf,
                          hipStream_t st) {
  int rc = check_shape(B, S, h, dh);
  if (rc) return rc;
  dim3 grid((S + 3) / 4, h, B), block(256);
  float scale = 1.0f / sqrtf((float)dh);
  size_t sm1 = ((size_t)4 * S + 512) * sizeof(float);
  size_t sm2 = ((size_t)8 * S + 512) * sizeof(float);
  if (bf) {
    hipLaunchKernelGGL(attn_bwd_dq_kernel<bf16>, grid, block, sm1, st, (const bf16*)qkv, (const bf16*)o,
                       (const bf16*)d_o, lse, dscratch, (bf16*)dqkv, S, h, dh, scale);
    ALS_CHECK_LAUNCH();
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<bf16>, grid, block, sm2, st, (const bf16*)qkv,
                       (const bf16*)d_o, lse, dscratch, (bf16*)dqkv, S, h, dh, scale);
  } else {
    hipLaunchKernelGGL(attn_bwd_dq_kernel<float>, grid, block, sm1, st, (const float*)qkv,
                       (const float*)o, (const float*)d_o, lse, dscratch, (float*)dqkv, S, h, dh, scale);
    ALS_CHECK_LAUNCH();
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<float>, grid, block, sm2, st, (const float*)qkv,
                       (const float*)d_o, lse, dscratch, (float*)dqkv, S, h, dh, scale);
  }
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

}  // namespace als
