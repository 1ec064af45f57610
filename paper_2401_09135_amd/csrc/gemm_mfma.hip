// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate) for the
// worker step's projections: C[M,N] = sum_k A(m,k) B(k,n).
//
// One workgroup of 4 wavefronts (2 x 2; 8 wavefronts, 2 x 4, for the 256 x 256 tile) owns a
// BM x BN tile of C and walks K in slices of 64 staged through LDS (one buffer with 2-3
// workgroups per CU, or two buffers); each wavefront owns a sub-tile of 64 x 64 or 128 x 64
// made of 32 x 32 MFMA blocks.  Operands may be stored with the
// contraction index contiguous (tile kept as [row][64 k], read from LDS with 16-byte loads; rows
// padded to 144 bytes, and written in row pairs (r, r+8), so that neither the fragment reads nor
// the staging writes collide on banks) or with the contraction index strided (tile kept as
// [64 k][row], read with the LDS transpose load ds_read_b64_tr_b16; rows padded by 64 bytes), so
// forward (x W), input-gradient (dY W^T) and weight-gradient (X^T dY) products all read the
// tensors as they lie in memory, without transposed copies.
// Weight-gradient products have small M x N and very long K: they are split along K over the
// grid into fp32 partials that a second kernel adds in a fixed order.
//
// Lane layouts of the MFMA (wavefront lane l, 64 lanes):
//   A fragment: row l%32, k = 8*(l/32) .. +7 ; B fragment: column l%32, same k ;
//   accumulator element v (0..15): row 8*(v/4) + 4*(l/32) + v%4, column l%32.
// LDS transpose load: in each group of 16 lanes, lane s supplies 4 consecutive bf16; lane r
// receives element r%4 of lanes r/4, 4 + r/4, 8 + r/4, 12 + r/4.
#include "common.h"
#include "als_bench.h"
#include <hip/hip_ext.h>
#include <stdio.h>

#include <mutex>
#include <string>
#include <vector>

namespace als {

namespace {

constexpr int BK = 64;

// ---- optional per-kernel timing (benchmarks): HIP events around every MFMA GEMM launch, on
// the stream it is launched on, grouped by kernel instantiation -----------------------------
struct ProfRec { hipEvent_t e0, e1; int id; double flops; };
std::mutex g_prof_mu;
bool g_prof_on = false;
int g_prof_every = 1;        // time one launch in g_prof_every
unsigned g_prof_count = 0;
std::vector<ProfRec> g_prof;

int kernel_id(int bm, int bn, int al, int bl, int epi, int to_bf16, int split, int nbuf) {
  return (bm / 128 - 1) | (bn / 128 - 1) << 1 | al << 2 | bl << 3 | epi << 4 | to_bf16 << 6 | split << 7 | (nbuf - 1) << 8;
}

// wavefronts per workgroup: 2 x 2, or 2 x 4 for the 256 x 256 tile (each wavefront then owns a
// 128 x 64 sub-tile, as in the 256 x 128 tile, and two wavefronts share every SIMD)
constexpr int tile_waves(int bm, int bn) { return bm == 256 && bn == 256 ? 8 : 4; }

template <int BM, int BN, int AL, int BL, int NBUF>
struct Tile {
  static constexpr int NT = 64 * tile_waves(BM, BN);  // threads per workgroup
  // AL == 0: A tile kept as [BM rows][64 k] ; AL == 1: as [64 k][BM rows]
  static constexpr int A_STRIDE = AL == 0 ? BK * 2 + 16 : BM * 2 + 64;
  static constexpr int A_BYTES = A_STRIDE * (AL == 0 ? BM : BK);
  // BL == 1: B tile kept as [BN cols][64 k] ; BL == 0: as [64 k][BN cols]
  static constexpr int B_STRIDE = BL == 1 ? BK * 2 + 16 : BN * 2 + 64;
  static constexpr int B_BYTES = B_STRIDE * (BL == 1 ? BN : BK);
  static constexpr int STAGE = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = (NBUF == 2 ? 2 : 1) * STAGE;
  static constexpr int A_CHUNKS = BM * BK * 2 / 16 / NT;  // 16-byte chunks per thread
  static constexpr int B_CHUNKS = BN * BK * 2 / 16 / NT;
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ bf16x8 lds_read_direct(const char* p) {
  return *reinterpret_cast<const bf16x8*>(p);
}

// two transpose loads: k rows kb..kb+3 and kb+4..kb+7 of a [k][row] tile
__device__ __forceinline__ bf16x8 lds_read_tr(const char* p, int stride) {
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * stride));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, r);
}

// gelu_tanh(u) = 0.5 u (1 + tanh y), y = a u (1 + b u^2), equals u sigma(2y) with sigma(z) =
// 1 / (1 + e^-z); its derivative is sigma + u sigma (1 - sigma) 2y', 2y' = 2a (1 + 3b u^2).  One
// hardware exp2 and one reciprocal give sigma (absolute error of a few 1e-7, far below the bf16
// rounding of the stored values); 9 more VALU operations give both outputs.  u -> -inf: e = inf,
// sigma = 0, both outputs 0; u -> +inf: sigma = 1, outputs u and 1.
__device__ __forceinline__ void gelu_both(float u, float& val, float& grad) {
  const float a = 0.7978845608028654f, b = 0.044715f, log2e = 1.4426950408889634f;
  const float k1 = -2.0f * log2e * a, k2 = k1 * b, k3 = 2.0f * a, k4 = 6.0f * a * b;
  float u2 = u * u;
  float e = __builtin_amdgcn_exp2f(u * fmaf(k2, u2, k1));  // e^{-2y}
  float sg = __builtin_amdgcn_rcpf(1.0f + e);
  val = u * sg;
  grad = fmaf(val * (1.0f - sg), fmaf(k4, u2, k3), sg);
}

struct MfmaArgs {
  const bf16* A; const bf16* B;
  int64_t lda, ldb;
  int M, N, K;      // K = length of this launch's K range per split
  int tiles_m, tiles_n, nsplit;
  void* C; int64_t ldc;
  const float* R; int64_t ldr;
  void* C2; const bf16* U;
  int64_t split_stride;  // elements between split partials (split-K only)
};

// NBUF = 2: LDS double buffer, one barrier per K slice, one workgroup per CU for the large
// tiles.  NBUF = 1: single LDS buffer, two barriers per slice, but half the LDS so that OCC
// workgroups share a CU and one's epilogue and barrier stalls hide behind another's MFMAs.
template <int BM, int BN, int AL, int BL, int EPI, typename TO, bool SPLIT, int NBUF, int OCC>
__global__ __launch_bounds__(64 * tile_waves(BM, BN), OCC) void gemm_mfma_kernel(MfmaArgs g) {
  typedef Tile<BM, BN, AL, BL, NBUF> TL;
  constexpr int NW = tile_waves(BM, BN), WGN = NW / 2;   // wavefront grid 2 x WGN
  constexpr int WM = BM / 2, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Without split-K
  // every XCD gets a contiguous run of tiles (n fastest), so tiles sharing an A panel share an
  // L2.  With split-K the K slice is the fastest index: XCD x then owns the slices z = x mod 8
  // for ALL output tiles, and each slice of both operands is fetched from HBM once.
  int ntiles = g.tiles_m * g.tiles_n;
  int id = blockIdx.x, tile, zsplit = 0;
  if (SPLIT) {
    zsplit = id % g.nsplit;
    tile = id / g.nsplit;
  } else {
    int per = ntiles / 8;
    tile = (id < per * 8) ? (id % 8) * per + id / 8 : id;
  }
  const int m0 = (tile / g.tiles_n) * BM, n0 = (tile % g.tiles_n) * BN;
  const int64_t kbase = (int64_t)zsplit * g.K;

  // Global addressing: one 32-bit per-lane byte offset per operand; everything else (tile
  // origin, 16-byte chunk index, K slice) is uniform and lives in scalar registers, so a
  // slice's loads cost no vector address arithmetic.
  const char* Ag = reinterpret_cast<const char*>(AL == 0 ? g.A + (int64_t)m0 * g.lda + kbase : g.A + kbase * g.lda + m0);
  const char* Bg = reinterpret_cast<const char*>(BL == 1 ? g.B + (int64_t)n0 * g.ldb + kbase : g.B + kbase * g.ldb + n0);
  constexpr int A_CPR = AL == 0 ? 8 : BM / 8;   // 16-byte chunks per tile row as it lies in memory
  constexpr int B_CPR = BL == 1 ? 8 : BN / 8;
  constexpr int A_RPC = TL::NT / A_CPR, B_RPC = TL::NT / B_CPR;  // tile rows covered by one pass of the workgroup
  // Lanes 8q..8q+7 move one 128-byte row piece.  For contraction-contiguous tiles (144-byte LDS
  // rows) neighbouring lane groups take rows r and r+8, whose LDS images lie 32 banks apart, so
  // the 16 lanes of one LDS write cycle touch all 64 banks once.
  auto tile_row = [](int q) { return (q & ~15) | ((q & 15) >> 1) | ((q & 1) << 3); };
  const int a_row = AL == 0 ? tile_row(tid / A_CPR) : tid / A_CPR;
  const int b_row = BL == 1 ? tile_row(tid / B_CPR) : tid / B_CPR;
  const uint32_t a_goff = (uint32_t)(((int64_t)a_row * g.lda + (tid % A_CPR) * 8) * 2);
  const uint32_t b_goff = (uint32_t)(((int64_t)b_row * g.ldb + (tid % B_CPR) * 8) * 2);
  const int64_t a_chunk = (int64_t)A_RPC * g.lda * 2, b_chunk = (int64_t)B_RPC * g.ldb * 2;
  const int64_t a_step = AL == 0 ? BK * 2 : (int64_t)BK * g.lda * 2;
  const int64_t b_step = BL == 1 ? BK * 2 : (int64_t)BK * g.ldb * 2;
  const int a_soff = a_row * TL::A_STRIDE + (tid % A_CPR) * 16;
  const int b_soff = b_row * TL::B_STRIDE + (tid % B_CPR) * 16;

  // NBUF == 3: one LDS buffer like NBUF == 1, but two register sets, so that the loads of
  // slice kt+2 are in flight while slice kt is multiplied (memory latency spans two slices).
  constexpr int NSET = NBUF == 3 ? 2 : 1;
  u32x4 ra[NSET][TL::A_CHUNKS], rb[NSET][TL::B_CHUNKS];

  auto load_global = [&](int kt, u32x4 (&ra)[TL::A_CHUNKS], u32x4 (&rb)[TL::B_CHUNKS]) {
    const char* ap = Ag + kt * a_step;
    const char* bp = Bg + kt * b_step;
#pragma unroll
    for (int i = 0; i < TL::A_CHUNKS; i++) ra[i] = *reinterpret_cast<const u32x4*>(ap + i * a_chunk + a_goff);
#pragma unroll
    for (int i = 0; i < TL::B_CHUNKS; i++) rb[i] = *reinterpret_cast<const u32x4*>(bp + i * b_chunk + b_goff);
  };
  auto store_lds = [&](int buf, const u32x4 (&ra)[TL::A_CHUNKS], const u32x4 (&rb)[TL::B_CHUNKS]) {
    char* As = smem + buf * TL::STAGE;
    char* Bs = As + TL::A_BYTES;
#pragma unroll
    for (int i = 0; i < TL::A_CHUNKS; i++) *reinterpret_cast<u32x4*>(As + a_soff + i * (A_RPC * TL::A_STRIDE)) = ra[i];
#pragma unroll
    for (int i = 0; i < TL::B_CHUNKS; i++) *reinterpret_cast<u32x4*>(Bs + b_soff + i * (B_RPC * TL::B_STRIDE)) = rb[i];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

  // per-lane fragment offsets inside a stage
  int a_off, b_off;
  if (AL == 0) a_off = (wm * WM + (lane & 31)) * TL::A_STRIDE + (lane >> 5) * 16;
  else a_off = ((lane >> 5) * 8 + ((lane & 15) >> 2)) * TL::A_STRIDE + (wm * WM + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
  if (BL == 1) b_off = (wn * WN + (lane & 31)) * TL::B_STRIDE + (lane >> 5) * 16;
  else b_off = ((lane >> 5) * 8 + ((lane & 15) >> 2)) * TL::B_STRIDE + (wn * WN + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;

  // The products are formed transposed (B fragment as the MFMA's first operand), so that an
  // accumulator holds, for ONE row m = lane % 32 of C, columns 8 g + 4 (lane / 32) + 0..3:
  // the epilogue then moves 4 consecutive columns per access.
  // Fragments are double-buffered in registers: the LDS reads of 16-wide step kk+1 are issued
  // ahead of the MFMAs of step kk and interleaved with them, one read per few MFMAs.
  auto read_frags = [&](const char* As, const char* Bs, int kk, bf16x8 (&af)[TM], bf16x8 (&bfr)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; i++) {
      if (AL == 0) af[i] = lds_read_direct(As + a_off + i * 32 * TL::A_STRIDE + kk * 32);
      else af[i] = lds_read_tr(As + a_off + kk * 16 * TL::A_STRIDE + i * 64, TL::A_STRIDE);
    }
#pragma unroll
    for (int j = 0; j < TN; j++) {
      if (BL == 1) bfr[j] = lds_read_direct(Bs + b_off + j * 32 * TL::B_STRIDE + kk * 32);
      else bfr[j] = lds_read_tr(Bs + b_off + kk * 16 * TL::B_STRIDE + j * 64, TL::B_STRIDE);
    }
  };
  auto compute = [&](const char* As, const char* Bs) {
    // Scheduling fences and groups keep the order written here: the LDS reads of a 16-wide step
    // are issued DIST steps ahead of its MFMAs, one read behind each MFMA of the current step,
    // so the MFMAs wait (by count) only for reads issued that long ago, the LDS latency hides
    // behind whole steps of MFMAs and the LDS pipe sees a steady trickle instead of bursts
    // (measured: 3 % on the products of the step against all reads ahead of the step's MFMAs).
    constexpr int NS = BK / 16;
    constexpr int DIST = TM * TN <= 4 ? 2 : 1;   // small sub-tiles have short steps: look further ahead
    bf16x8 af[DIST + 1][TM], bfr[DIST + 1][TN];
#pragma unroll
    for (int p = 0; p < DIST; p++) read_frags(As, Bs, p, af[p], bfr[p]);
#pragma unroll
    for (int kk = 0; kk < NS; kk++) {
      __builtin_amdgcn_sched_barrier(0);
      if (kk + DIST < NS) read_frags(As, Bs, kk + DIST, af[(kk + DIST) % (DIST + 1)], bfr[(kk + DIST) % (DIST + 1)]);
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk % (DIST + 1)][j], af[kk % (DIST + 1)][i], acc[i][j], 0, 0, 0);
      // one LDS read (of the step DIST ahead) behind each of the first MFMAs of this step
      if (kk + DIST < NS) {
        constexpr int NR = (AL == 0 ? TM : 2 * TM) + (BL == 1 ? TN : 2 * TN);   // LDS read instructions of a step
        constexpr int PER = (NR + TM * TN - 1) / (TM * TN);
#pragma unroll
        for (int m = 0; m < TM * TN; m++) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, PER, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  const int nk = g.K / BK;
  if (NBUF == 2) {
    load_global(0, ra[0], rb[0]);
    store_lds(0, ra[0], rb[0]);
    __syncthreads();
    for (int kt = 0; kt < nk; kt++) {
      if (kt + 1 < nk) load_global(kt + 1, ra[0], rb[0]);
      const char* As = smem + (kt & 1) * TL::STAGE;
      compute(As, As + TL::A_BYTES);
      if (kt + 1 < nk) store_lds((kt + 1) & 1, ra[0], rb[0]);
      __syncthreads();
    }
  } else {
    auto slice = [&](int kt, u32x4 (&sa)[TL::A_CHUNKS], u32x4 (&sb)[TL::B_CHUNKS]) {
      store_lds(0, sa, sb);
      __syncthreads();
      if (kt + NSET < nk) load_global(kt + NSET, sa, sb);
      compute(smem, smem + TL::A_BYTES);
      __syncthreads();
    };
    load_global(0, ra[0], rb[0]);
    if (NSET == 2) {
      if (nk > 1) load_global(1, ra[1], rb[1]);
      int kt = 0;
      for (; kt + 1 < nk; kt += 2) {
        slice(kt, ra[0], rb[0]);
        slice(kt + 1, ra[NSET - 1], rb[NSET - 1]);
      }
      if (kt < nk) slice(kt, ra[0], rb[0]);
    } else {
      for (int kt = 0; kt < nk; kt++) slice(kt, ra[0], rb[0]);
    }
  }

  // Epilogue.  Each wavefront stages its sub-tile through LDS, 32 rows at a time (fp32, row
  // pitch padded by 16 bytes), and reads it back so that the lanes of one store instruction
  // cover whole row segments, 16 bytes per lane: every global access of the epilogue (residual
  // and saved-derivative reads, outputs) is then fully coalesced.  (Storing straight from the
  // accumulator layout gives 8- or 16-byte pieces in 32 different rows per instruction;
  // measured 8 % slower on the whole step.)
  TO* C = reinterpret_cast<TO*>(g.C);
  if (SPLIT) C += (int64_t)zsplit * g.split_stride;
  constexpr int PITCH = WN * 4 + 16;  // rows 4 banks apart: 16-byte accesses of 16 rows, or of two row halves, never collide
  static_assert(NW * 32 * PITCH <= TL::LDS_BYTES, "epilogue staging must fit the operand buffers");
  char* stg = smem + wave * (32 * PITCH);
  constexpr int CPL = sizeof(TO) == 2 ? 8 : 4;  // consecutive columns per lane
  constexpr int LPR = WN / CPL;                 // lanes per row
  constexpr int RPP = 64 / LPR;                 // rows per pass
  constexpr int NPASS = 32 / RPP;
  // The epilogue's global READS (residual rows, saved derivative) are issued together, ahead of
  // the staging and the stores: loads and stores complete out of order with respect to each
  // other, so a load issued after a store can only be waited for with "everything done", and a
  // load per pass would expose one full memory latency per pass.  All of the sub-tile at once
  // when that fits in 64 registers, else one 32-row block at a time.
  constexpr bool HAS_AUX = EPI == EPI_RESID || EPI == EPI_DGELU;
  constexpr bool AUX_ALL = TM * NPASS * 4 <= 64;
  u32x4 aux[HAS_AUX ? TM : 1][HAS_AUX ? NPASS : 1];
  auto load_aux = [&](int i) {
#pragma unroll
    for (int pass = 0; pass < NPASS; pass++) {
      const int row = m0 + wm * WM + i * 32 + pass * RPP + lane / LPR;
      const int col = n0 + wn * WN + (lane % LPR) * CPL;
      if (EPI == EPI_RESID) aux[i][pass] = *reinterpret_cast<const u32x4*>(g.R + (int64_t)row * g.ldr + col);
      else aux[i][pass] = *reinterpret_cast<const u32x4*>(g.U + (int64_t)row * g.ldc + col);
    }
  };
  if (HAS_AUX && AUX_ALL) {
#pragma unroll
    for (int i = 0; i < TM; i++) load_aux(i);
  }
  __syncthreads();  // every wave is done with the operand tiles
#pragma unroll
  for (int i = 0; i < TM; i++) {
    if (HAS_AUX && !AUX_ALL) load_aux(i);
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int gq = 0; gq < 4; gq++) {
        f32x4 x = {acc[i][j][4 * gq], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]};
        *reinterpret_cast<f32x4*>(stg + (lane & 31) * PITCH + (j * 32 + 8 * gq + 4 * (lane >> 5)) * 4) = x;
      }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // wave-local staging: its own writes have landed
#pragma unroll
    for (int pass = 0; pass < NPASS; pass++) {
      const int rr = pass * RPP + lane / LPR;
      const int cc = (lane % LPR) * CPL;
      const int row = m0 + wm * WM + i * 32 + rr;
      const int col = n0 + wn * WN + cc;
      const int64_t ci = (int64_t)row * g.ldc + col;
      float x[CPL];
#pragma unroll
      for (int q = 0; q < CPL / 4; q++) {
        f32x4 v = *reinterpret_cast<const f32x4*>(stg + rr * PITCH + (cc + 4 * q) * 4);
        x[4 * q] = v[0]; x[4 * q + 1] = v[1]; x[4 * q + 2] = v[2]; x[4 * q + 3] = v[3];
      }
      if (EPI == EPI_RESID) {
        f32x4 r = __builtin_bit_cast(f32x4, aux[HAS_AUX ? i : 0][HAS_AUX ? pass : 0]);
#pragma unroll
        for (int e = 0; e < 4; e++) x[e] += r[e];
      }
      if (EPI == EPI_DGELU) {  // U holds gelu'(pre-activation), saved by the forward pass
        bf16x8 u = __builtin_bit_cast(bf16x8, aux[HAS_AUX ? i : 0][HAS_AUX ? pass : 0]);
#pragma unroll
        for (int e = 0; e < CPL; e++) x[e] *= (float)u[e & 7];
      }
      if (sizeof(TO) == 4) {
        f32x4 o = {x[0], x[1], x[2], x[3]};
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(C) + ci) = o;
      } else {
        bf16x8 o;
        if (EPI == EPI_GELU) {  // C <- gelu'(acc), C2 <- gelu(acc)
          bf16x8 o2;
#pragma unroll
          for (int e = 0; e < CPL; e++) {
            float val, grad;
            gelu_both(x[e], val, grad);
            o[e & 7] = (bf16)grad;
            o2[e & 7] = (bf16)val;
          }
          *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(g.C2) + ci) = o2;
        } else {
#pragma unroll
          for (int e = 0; e < CPL; e++) o[e & 7] = (bf16)x[e];
        }
        *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(C) + ci) = o;
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // reads done before the next block overwrites
  }
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part,
                                                            float* __restrict__ C, int64_t n4,
                                                            int nsplit, int64_t stride4) {
  int64_t step = (int64_t)gridDim.x * blockDim.x;
  const f32x4* p4 = reinterpret_cast<const f32x4*>(part);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += step) {
    f32x4 a = p4[i];
    for (int s0 = 1; s0 < nsplit; s0 += 8) {  // 8 partials in flight, added in split order
      f32x4 b[8];
#pragma unroll
      for (int u = 0; u < 8; u++) b[u] = s0 + u < nsplit ? p4[i + (s0 + u) * stride4] : (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int u = 0; u < 8; u++)
        if (s0 + u < nsplit) a += b[u];
    }
    reinterpret_cast<f32x4*>(C)[i] = a;
  }
}

template <int BM, int BN, int AL, int BL, int EPI, typename TO, bool SPLIT, int NBUF, int OCC>
int launch(const MfmaArgs& a, int nsplit, hipStream_t st) {
  typedef Tile<BM, BN, AL, BL, NBUF> TL;
  auto kern = gemm_mfma_kernel<BM, BN, AL, BL, EPI, TO, SPLIT, NBUF, OCC>;
  static bool attr_set = false;  // idempotent; a race only repeats the call
  if (!attr_set) {
    ALS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES));
    attr_set = true;
  }
  dim3 grid(a.tiles_m * a.tiles_n * nsplit);
  ProfRec rec;
  bool prof = false;
  if (g_prof_on) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (g_prof_on && (g_prof_count++ % (unsigned)g_prof_every) == 0 && hipEventCreate(&rec.e0) == hipSuccess) {
      if (hipEventCreate(&rec.e1) == hipSuccess) prof = true;
      else (void)hipEventDestroy(rec.e0);
    }
  }
  if (prof) {
    // start/stop events attached to the dispatch itself: their difference is the kernel's own
    // execution time, as a profiler reports it
    hipExtLaunchKernelGGL(kern, grid, dim3(TL::NT), TL::LDS_BYTES, st, rec.e0, rec.e1, 0, a);
  } else {
    hipLaunchKernelGGL(kern, grid, dim3(TL::NT), TL::LDS_BYTES, st, a);
  }
  ALS_CHECK_LAUNCH();
  if (prof) {
    rec.id = kernel_id(BM, BN, AL, BL, EPI, sizeof(TO) == 2, SPLIT, NBUF);
    rec.flops = 2.0 * a.M * a.N * (double)a.K * nsplit;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof.push_back(rec);
  }
  return ALS_OK;
}

inline bool fits(int M, int N, int bm, int bn) { return M % bm == 0 && N % bn == 0; }

}  // namespace

bool gemm_mfma_supported(const GemmDesc& g) {
  if (!g.in_bf16) return false;
  // the epilogue moves 16 bytes per lane
  if (g.ldc % 8 || (uintptr_t)g.C % 16) return false;
  if (g.epi == EPI_RESID && (g.ldr % 4 || (uintptr_t)g.R % 16)) return false;
  if (g.epi == EPI_DGELU && (uintptr_t)g.U % 16) return false;
  if (g.epi == EPI_GELU && (uintptr_t)g.C2 % 16) return false;
  if (g.M % 128 || g.N % 128 || g.K % 64 || g.K < 64) return false;
  if (g.lda % 8 || g.ldb % 8) return false;
  if ((uintptr_t)g.A % 16 || (uintptr_t)g.B % 16) return false;
  // operand-layout / epilogue combinations the hot path uses
  if (g.a_layout == 0 && g.b_layout == 0)
    return g.epi == EPI_STORE || (g.epi == EPI_RESID && !g.c_bf16) || (g.epi == EPI_GELU && g.c_bf16);
  if (g.a_layout == 0 && g.b_layout == 1) return g.epi == EPI_STORE || (g.epi == EPI_DGELU && g.c_bf16);
  if (g.a_layout == 1 && g.b_layout == 0) return g.epi == EPI_STORE && !g.c_bf16;
  return false;
}

// tile variants: 256x256 double-buffered (8 wavefronts, 1 workgroup per CU), 256x128 and 128x128 either
// double-buffered or single-buffered with 2 / 3 workgroups per CU
#define ALS_TILE_SWITCH(AL, BL, EPI, TO, SPLIT)                                                            \
  do {                                                                                                     \
    if (bm == 256 && bn == 256) return launch<256, 256, AL, BL, EPI, TO, SPLIT, 2, 1>(a, nsplit, st);      \
    if (bm == 256 && bn == 128 && nbuf == 2) return launch<256, 128, AL, BL, EPI, TO, SPLIT, 2, 1>(a, nsplit, st); \
    if (bm == 256 && bn == 128 && nbuf == 1) return launch<256, 128, AL, BL, EPI, TO, SPLIT, 1, 2>(a, nsplit, st);      \
    if (nbuf == 2) return launch<128, 128, AL, BL, EPI, TO, SPLIT, 2, 2>(a, nsplit, st);                   \
    if (nbuf == 3) return launch<128, 128, AL, BL, EPI, TO, SPLIT, 3, 2>(a, nsplit, st);                   \
    return launch<128, 128, AL, BL, EPI, TO, SPLIT, 1, 3>(a, nsplit, st);                                  \
  } while (0)

static int dispatch(const GemmDesc& g, const MfmaArgs& a, int bm, int bn, int nbuf, int nsplit, hipStream_t st) {
  if (g.a_layout == 0 && g.b_layout == 0) {
    if (g.epi == EPI_RESID) ALS_TILE_SWITCH(0, 0, EPI_RESID, float, false);
    if (g.epi == EPI_GELU) ALS_TILE_SWITCH(0, 0, EPI_GELU, bf16, false);
    if (g.c_bf16) ALS_TILE_SWITCH(0, 0, EPI_STORE, bf16, false);
    ALS_TILE_SWITCH(0, 0, EPI_STORE, float, false);
  }
  if (g.a_layout == 0 && g.b_layout == 1) {
    if (g.epi == EPI_DGELU) ALS_TILE_SWITCH(0, 1, EPI_DGELU, bf16, false);
    if (g.c_bf16) ALS_TILE_SWITCH(0, 1, EPI_STORE, bf16, false);
    ALS_TILE_SWITCH(0, 1, EPI_STORE, float, false);
  }
  if (nsplit > 1) ALS_TILE_SWITCH(1, 0, EPI_STORE, float, true);
  ALS_TILE_SWITCH(1, 0, EPI_STORE, float, false);
}

static int g_force_bm = 0, g_force_bn = 0, g_force_nbuf = 0;  // tuning override, 0 = automatic

int gemm_mfma(const GemmDesc& g, hipStream_t st) {
  if (!gemm_mfma_supported(g)) return set_error(ALS_ERR_INVALID, "gemm_mfma: unsupported shape or layout");
  // Tile choice (measured on MI355X): the single-buffered 128x128 variant, 3 workgroups per CU
  // so that one's prologue/epilogue hides behind another's MFMAs, for short K and few tiles;
  // the double-buffered one once K is long enough to amortise its single resident pair;
  // 256x128 (less operand traffic and fewer LDS bytes per flop) when its tiles fill at least
  // 7/8 of the 512 resident slots (2 per CU).
  int bm = 128, bn = 128, nbuf = 1;
  if (g_force_bm && fits(g.M, g.N, g_force_bm, g_force_bn)) { bm = g_force_bm; bn = g_force_bn; nbuf = g_force_nbuf; }
  else if (g.a_layout == 1) {
    if (fits(g.M, g.N, 256, 256) && (g.M / 256) * (g.N / 256) >= 64) { bm = 256; bn = 256; nbuf = 2; }
    else if (fits(g.M, g.N, 256, 128) && (g.M / 256) * (g.N / 128) >= 128) { bm = 256; bn = 128; nbuf = 1; }
    else nbuf = 2;
  } else if (fits(g.M, g.N, 256, 128) && (g.M / 256) * (g.N / 128) >= 448) { bm = 256; bn = 128; }
  else if (g.K >= 2048) nbuf = 2;
  MfmaArgs a;
  a.A = (const bf16*)g.A; a.B = (const bf16*)g.B; a.lda = g.lda; a.ldb = g.ldb;
  a.M = g.M; a.N = g.N; a.K = g.K; a.tiles_m = g.M / bm; a.tiles_n = g.N / bn;
  a.C = g.C; a.ldc = g.ldc; a.R = g.R; a.ldr = g.ldr; a.C2 = g.C2; a.U = (const bf16*)g.U;
  a.split_stride = 0; a.nsplit = 1;
  int nsplit = 1;
  if (g.a_layout == 1 && g.b_layout == 0 && g.ldc == g.N) {
    // Weight-gradient shape: few tiles, long K.  K is split so that the grid fills the chip in
    // whole rounds of its resident workgroups (2 per CU for the double-buffered 128x128 variant
    // and for 256x128, 3 per CU for the single-buffered 128x128 one).  Candidates are costed in
    // microseconds with measured rates: the product at 700 TFLOP/s times the round-up loss of
    // the last round, plus the fp32 partials written and read back at 4 TB/s; each split keeps
    // at least 512 of K and the partials must fit the workspace.
    const size_t per = (size_t)g.M * g.N * sizeof(float);
    const int maxws = g.ws ? (int)(g.ws_bytes / per) : 1;
    const double t_prod = 2.0 * g.M * g.N * (double)g.K / 700e6;  // us
    double best = 1e30;
    int best_nbuf = nbuf, best_ns = 1;
    for (int cand = 0; cand < (bm == 128 && !g_force_bm ? 2 : 1); cand++) {
      const int nb = cand == 0 ? nbuf : (nbuf == 2 ? 1 : 2);
      const int slots = 256 * (bn == 256 ? 1 : (bm == 128 && nb == 1) ? 3 : 2);  // resident workgroups on the chip
      const int tiles = a.tiles_m * a.tiles_n;
      for (int ns = 1; ns <= 64 && ns <= maxws; ns++) {
        if (g.K % (ns * BK) || (ns > 1 && g.K / ns < 512)) continue;
        const int wgs = tiles * ns;
        const int rounds = (wgs + slots - 1) / slots;
        double cost = t_prod * rounds * slots / wgs + (ns > 1 ? ns * (double)per * 2.0 / 4e6 : 0.0);
        if (cand == 1) cost *= 1.03;  // prefer the first choice on near ties
        if (cost < best) { best = cost; best_nbuf = nb; best_ns = ns; }
      }
    }
    nbuf = best_nbuf;
    nsplit = best_ns;
  }
  if (nsplit > 1) {
    a.K = g.K / nsplit; a.nsplit = nsplit;
    a.C = g.ws; a.ldc = g.N; a.split_stride = (int64_t)g.M * g.N;
    int rc = dispatch(g, a, bm, bn, nbuf, nsplit, st);
    if (rc) return rc;
    int64_t n4 = (int64_t)g.M * g.N / 4;
    int blocks = (int)((n4 + 255) / 256 < 4096 ? (n4 + 255) / 256 : 4096);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, st, g.ws, (float*)g.C, n4,
                       nsplit, n4);
    ALS_CHECK_LAUNCH();
    return ALS_OK;
  }
  return dispatch(g, a, bm, bn, nbuf, 1, st);
}

}  // namespace als

// Benchmark hooks: time every MFMA GEMM launch with HIP events on its own stream.
extern "C" int als_prof_enable(int on) {
  std::lock_guard<std::mutex> lk(als::g_prof_mu);
  als::g_prof_on = on != 0;
  als::g_prof_every = on > 1 ? on : 1;
  als::g_prof_count = 0;
  return ALS_OK;
}

extern "C" int als_prof_collect(int max_entries, int32_t* ids, int64_t* launches, double* ms, double* flops) {
  using namespace als;
  if (max_entries < 0 || (max_entries > 0 && (!ids || !launches || !ms || !flops)))
    return set_error(ALS_ERR_INVALID, "als_prof_collect: null output");
  ALS_HIP(hipDeviceSynchronize());
  std::lock_guard<std::mutex> lk(g_prof_mu);
  int n = 0;
  for (ProfRec& r : g_prof) {
    float t = 0.0f;
    bool ok = hipEventElapsedTime(&t, r.e0, r.e1) == hipSuccess;
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
    if (!ok) continue;
    int k = 0;
    while (k < n && ids[k] != r.id) k++;
    if (k == n) {
      if (n == max_entries) continue;
      ids[n] = r.id; launches[n] = 0; ms[n] = 0.0; flops[n] = 0.0;
      n++;
    }
    launches[k] += 1; ms[k] += t; flops[k] += r.flops;
  }
  g_prof.clear();
  return n;
}

extern "C" int als_prof_kernel_name(int id, char* out, int out_len) {
  if (!out || out_len < 1) return als::set_error(ALS_ERR_INVALID, "als_prof_kernel_name: null output");
  static const char* epi[4] = {"STORE", "RESID", "GELU", "DGELU"};
  int nbuf = ((id >> 8) & 3) + 1, bm = ((id & 1) + 1) * 128, bn = (((id >> 1) & 1) + 1) * 128;
  int occ = nbuf == 2 ? (bm == 128 ? 2 : 1) : nbuf == 3 ? 2 : (bm == 256 ? 2 : 3);
  snprintf(out, out_len, "gemm_mfma_kernel<%d, %d, %d, %d, %s, %s, %s, %d, %d>", bm, bn, (id >> 2) & 1, (id >> 3) & 1,
           epi[(id >> 4) & 3], (id >> 6) & 1 ? "bf16" : "float", (id >> 7) & 1 ? "true" : "false", nbuf, occ);
  return ALS_OK;
}

// Tuning hook: force the MFMA GEMM tile (256x256, 256x128 or 128x128) and its LDS buffering
// (2 = double, 1 = single buffer with more workgroups per CU); 0,0 restores the automatic choice.  Not thread-safe; meant for benchmarks.
extern "C" int als_k_set_gemm_tile(int bm, int bn, int nbuf) {
  bool ok = (bm == 0 && bn == 0) || (bm == 256 && bn == 256) || (bm == 256 && bn == 128) || (bm == 128 && bn == 128);
  if (!ok || (bm && nbuf != 1 && nbuf != 2 && !(nbuf == 3 && bm == 128))) return als::set_error(ALS_ERR_INVALID, "unsupported tile %dx%d/%d", bm, bn, nbuf);
  als::g_force_bm = bm; als::g_force_bn = bn; als::g_force_nbuf = nbuf;
  return ALS_OK;
}
