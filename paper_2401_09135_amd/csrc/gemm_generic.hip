// Generic tiled GEMM with fp32 accumulation: any shape, any of the four operand layouts,
// fp32 or bf16 operands.  This is the reference-mode (fp32) path and the fallback for shapes
// the MFMA kernel does not take; it is not the fast path.
#include "common.h"

namespace als {

__device__ __forceinline__ float gelu_tanh_f(float u) {
  const float a = 0.7978845608028654f, b = 0.044715f;
  return 0.5f * u * (1.0f + tanhf(a * (u + b * u * u * u)));
}
__device__ __forceinline__ float gelu_tanh_grad_f(float u) {
  const float a = 0.7978845608028654f, b = 0.044715f;
  float th = tanhf(a * (u + b * u * u * u));
  float inner = a * (1.0f + 3.0f * b * u * u);
  return 0.5f * (1.0f + th) + 0.5f * u * (1.0f - th * th) * inner;
}

template <typename T>
__device__ __forceinline__ float ld(const void* p, int64_t i) {
  return (float)reinterpret_cast<const T*>(p)[i];
}

template <typename TI, typename TO, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmDesc g) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) acc[i][j] = 0.0f;
  for (int k0 = 0; k0 < g.K; k0 += 16) {
    for (int idx = threadIdx.x; idx < 64 * 16; idx += 256) {
      int mm, kk;
      if (g.a_layout == 0) { kk = idx & 15; mm = idx >> 4; }
      else { mm = idx & 63; kk = idx >> 6; }
      int gm = m0 + mm, gk = k0 + kk;
      float v = 0.0f;
      if (gm < g.M && gk < g.K)
        v = g.a_layout == 0 ? ld<TI>(g.A, (int64_t)gm * g.lda + gk) : ld<TI>(g.A, (int64_t)gk * g.lda + gm);
      As[kk][mm] = v;
      int nn;
      if (g.b_layout == 0) { nn = idx & 63; kk = idx >> 6; }
      else { kk = idx & 15; nn = idx >> 4; }
      int gn = n0 + nn;
      gk = k0 + kk;
      v = 0.0f;
      if (gn < g.N && gk < g.K)
        v = g.b_layout == 0 ? ld<TI>(g.B, (int64_t)gk * g.ldb + gn) : ld<TI>(g.B, (int64_t)gn * g.ldb + gk);
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; kk++) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; j++) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int gm = m0 + ty * 4 + i;
    if (gm >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int gn = n0 + tx * 4 + j;
      if (gn >= g.N) continue;
      int64_t ci = (int64_t)gm * g.ldc + gn;
      float v = acc[i][j];
      if (EPI == EPI_RESID) v += g.R[(int64_t)gm * g.ldr + gn];
      if (EPI == EPI_DGELU) v *= ld<TI>(g.U, ci);
      if (EPI == EPI_GELU) {
        reinterpret_cast<TO*>(g.C2)[ci] = (TO)gelu_tanh_f(v);
        v = gelu_tanh_grad_f(v);
      }
      reinterpret_cast<TO*>(g.C)[ci] = (TO)v;
    }
  }
}

template <typename TI, typename TO>
static int launch_epi(const GemmDesc& g, hipStream_t st) {
  dim3 grid((g.N + 63) / 64, (g.M + 63) / 64), block(256);
  switch (g.epi) {
    case EPI_STORE: hipLaunchKernelGGL((gemm_generic_kernel<TI, TO, EPI_STORE>), grid, block, 0, st, g); break;
    case EPI_RESID: hipLaunchKernelGGL((gemm_generic_kernel<TI, TO, EPI_RESID>), grid, block, 0, st, g); break;
    case EPI_GELU: hipLaunchKernelGGL((gemm_generic_kernel<TI, TO, EPI_GELU>), grid, block, 0, st, g); break;
    case EPI_DGELU: hipLaunchKernelGGL((gemm_generic_kernel<TI, TO, EPI_DGELU>), grid, block, 0, st, g); break;
    default: return set_error(ALS_ERR_INVALID, "gemm: unknown epilogue %d", g.epi);
  }
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

int gemm_generic(const GemmDesc& g, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return set_error(ALS_ERR_INVALID, "gemm: empty shape");
  if (g.epi == EPI_RESID && g.c_bf16) return set_error(ALS_ERR_INVALID, "gemm: residual output must be fp32");
  if (g.in_bf16) return g.c_bf16 ? launch_epi<bf16, bf16>(g, st) : launch_epi<bf16, float>(g, st);
  return g.c_bf16 ? launch_epi<float, bf16>(g, st) : launch_epi<float, float>(g, st);
}

int gemm(const GemmDesc& g, bool allow_mfma, hipStream_t st) {
  if (allow_mfma && gemm_mfma_supported(g)) return gemm_mfma(g, st);
  return gemm_generic(g, st);
}

}  // namespace als
