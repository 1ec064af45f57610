// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/als.h"

namespace als {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

int set_error(int code, const char* fmt, ...);

#define ALS_HIP(expr)                                                                      \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess)                                                                  \
      return als::set_error(ALS_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), \
                            __FILE__, __LINE__);                                           \
  } while (0)

#define ALS_CHECK_LAUNCH() ALS_HIP(hipGetLastError())

// ---- parameter layout -----------------------------------------------------------------
struct Layout {
  int64_t E, Ppos, Wout, gf;
  int64_t Wqkv[64], Wo[64], W1[64], W2[64], g1[64], g2[64];
  int64_t P, P_decay;
};
int validate_config(const als_config* c);
int head_width(const als_config& c);  // head_dim, or d/h when head_dim is 0
void make_layout(const als_config& c, Layout* L);

// ---- GEMM -------------------------------------------------------------------------------
enum Epilogue {
  EPI_STORE = 0,   // C = acc
  EPI_RESID = 1,   // C(fp32) = R(fp32) + acc
  EPI_GELU = 2,    // C = gelu_tanh'(acc) (kept for the backward pass), C2 = gelu_tanh(acc)
  EPI_DGELU = 3,   // C = acc * U, U = the saved gelu_tanh'(pre-activation)
};

struct GemmDesc {
  const void* A; const void* B;
  int M, N, K;
  int a_layout;  // 0: A[m*lda + k] ; 1: A[k*lda + m]
  int b_layout;  // 0: B[k*ldb + n] ; 1: B[n*ldb + k]
  int64_t lda, ldb;
  int in_bf16;   // operands bf16 (else fp32)
  void* C; int64_t ldc; int c_bf16;  // output type
  int epi;
  const float* R; int64_t ldr;       // EPI_RESID
  void* C2;                          // EPI_GELU second output (same type/ld as C)
  const void* U;                     // EPI_DGELU saved derivative (operand type, ld = ldc)
  float* ws; size_t ws_bytes;        // scratch for split-K partials (may be null)
};
int gemm_generic(const GemmDesc& g, hipStream_t st);
bool gemm_mfma_supported(const GemmDesc& g);
int gemm_mfma(const GemmDesc& g, hipStream_t st);
// picks the MFMA kernel when allowed and supported
int gemm(const GemmDesc& g, bool allow_mfma, hipStream_t st);

// All weight gradients of a backward pass (X^T dY over the batch's tokens, bf16 operands, fp32
// results) as ONE launch of the 256 x 256 MFMA kernel.  The host turns the list of products into
// work items: whole rounds of tiles run unsplit over the full contraction and write C directly;
// the tiles of the last, partial round are split along K so that they fill the chip too, into
// 256 x 256 partial tiles that a second small kernel adds in slot order.  The records below are what
// the two kernels read from device memory.
struct DwProblem {
  const bf16* A; const bf16* B; float* C;   // A stored [K, M], B stored [K, N], C [M, N]; M, N multiples of 128
  int M, N, lda, ldb;
  int pad[2];
};
struct DwItem {
  int prob, tm, tn;
  int slot;         // -1: whole tile, result straight into C; else index of the partial tile in the workspace
  int slice0, nk;   // K slices of 64
  int pad[2];
};
struct DwSplitTile { int prob, tm, tn, slot0, nslots, pad[3]; };
static_assert(sizeof(DwProblem) == 48 && sizeof(DwItem) == 32 && sizeof(DwSplitTile) == 32, "table records");
struct DwPlan {
  int n_items, n_split, n_partial_tiles;   // partial tiles are 256 x 256 floats each
  double flops;
};
// Number of CUs the plan fills (MI355X).
constexpr int DW_PLAN_CUS = 256;
// Upper bounds of what dw_group_plan writes for n_tiles tiles in all.
inline int dw_plan_max_items(int n_tiles) { return n_tiles + DW_PLAN_CUS; }
inline int dw_plan_max_split(int n_tiles) { return n_tiles < DW_PLAN_CUS ? n_tiles : DW_PLAN_CUS; }
bool dw_group_supported(int M, int N, int K, int64_t lda, int64_t ldb);
// Shapes only are read from probs (pointers may still be null); items / split receive the tables
// in launch order (room for dw_plan_max_items / dw_plan_max_split records).
DwPlan dw_group_plan(const DwProblem* probs, int n_probs, int K, DwItem* items, DwSplitTile* split);
int dw_group_launch(const DwProblem* d_probs, const DwItem* d_items, const DwSplitTile* d_split, const DwPlan& plan,
                    float* partial_tiles, hipStream_t st);

// ---- attention ----------------------------------------------------------------------------
int attention_fwd_generic(const void* qkv, void* o, float* lse, int B, int S, int h, int dh,
                          int bf, hipStream_t st);
int attention_bwd_generic(const void* qkv, const void* o, const void* d_o, const float* lse,
                          float* dscratch, void* dqkv, int B, int S, int h, int dh, int bf,
                          hipStream_t st);
bool attention_mfma_supported(int S, int dh, int bf);
int attention_fwd_mfma(const void* qkv, void* o, float* lse, int B, int S, int h, int dh,
                       hipStream_t st);
int attention_bwd_mfma(const void* qkv, const void* o, const void* d_o, const float* lse,
                       float* dscratch, void* dqkv, int B, int S, int h, int dh, hipStream_t st);

// ---- elementwise / reductions ----------------------------------------------------------------
int embed_fwd(const int32_t* tok, const float* E, const float* Ppos, float* x, int B, int S, int d,
              int V, hipStream_t st);
// center = 0: RMSNorm ; 1: LayerNorm with gain and no bias
int rmsnorm_fwd(const float* x, const float* g, void* y, float* rstd, int T, int d, float eps,
                int out_bf16, int center, hipStream_t st);
// dx_out = (dx_in ? dx_in : 0) + rmsnorm_backward(dy); optional low-precision copy of dx_out;
// dg = sum over rows of dy * xhat (uses partial[nblk*d] scratch, nblk = rmsnorm_bwd_blocks()).
// With dg == nullptr only the partials are left, for one rmsnorm_dg_sum() over nset consecutive
// sets of partials into nset consecutive gain gradients.
int rmsnorm_bwd_blocks(int T);
int rmsnorm_dg_sum(const float* partial, float* dg, int T, int d, int nset, hipStream_t st);
int rmsnorm_bwd(const float* dy, const float* x, const float* rstd, const float* g,
                const float* dx_in, float* dx_out, void* dx_lp, int lp_bf16, float* dg,
                float* partial, int T, int d, int center, hipStream_t st);
// logits fp32 or bf16; dlogits may be the same buffer as the logits when the two types are equal
int cross_entropy(const void* logits, int logits_bf16, const int32_t* tok, float* loss_row, void* dlogits,
                  int dl_bf16, int B, int S, int V, hipStream_t st);
int mean_rows(const float* loss_row, float* out, int T, hipStream_t st);
// Orders each step's input positions by token id (see elementwise.hip); offset is
// [n_steps][V+1], rank and pos are [n_steps][B*S].
int embed_sort(const int32_t* tok, int n_steps, int B, int S, int V, int32_t* offset, int32_t* rank,
               int32_t* pos, hipStream_t st);
// scratch: 2 * ceil(B*S / 32) * d floats (partial rows of position lists that cross 32-position chunks)
int embed_bwd(const int32_t* tok, const int32_t* offset, const int32_t* pos, const float* dx, float* dE,
              float* dPpos, float* scratch, int B, int S, int d, int V, hipStream_t st);
int cast_copy(const float* src, void* dst, int64_t n, int dst_bf16, hipStream_t st);

struct AdamArgs {
  float lr, beta1, beta2, eps, wd, bc1, bc2;
};
int adamw(float* theta, const float* grad, float* m, float* v, bf16* lp, int64_t P,
          int64_t P_decay, const AdamArgs& a, hipStream_t st);

#define ALS_DN_MAX_GROUP 16
struct DnGroup {
  const float* theta_start[ALS_DN_MAX_GROUP];
  float* theta_worker[ALS_DN_MAX_GROUP];
  float* start_out[ALS_DN_MAX_GROUP];
  bf16* lp_out[ALS_DN_MAX_GROUP];
  int G;
  int restart;
  unsigned boundary_mask;  // bit j set: event j is an N-th event
  float lr, beta, c_beta, cb_boundary, Nf;  // c*beta ; (1 - cN + c)*beta
  // comparison rules of the paper's "Existing Fixes": per-event weight on the pseudo-gradient
  // (polynomial staleness discount; 1 = none), delay-compensation strength lambda (0 = off),
  // buffered mode (no parameter change between N-th events, which apply Nesterov on Delta/N)
  float weight[ALS_DN_MAX_GROUP];
  float dc_lambda;
  int buffered;
};
int dn_group(float* theta, float* m, float* delta, const DnGroup& g, int64_t P, hipStream_t st);
int restart_copy(const float* theta, float* master, float* start, bf16* lp, int64_t P,
                 hipStream_t st);

}  // namespace als
