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

#include <atomic>
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
  int M, N, K;      // K = whole contraction length (split-K: the kernel takes its share of the slices)
  int tiles_m, tiles_n, nsplit;
  void* C; int64_t ldc;
  const float* R; int64_t ldr;
  void* C2; const bf16* U;
  int64_t split_stride;  // elements between split partials (split-K only)
};

// Epilogue of one wavefront's WM x WN sub-tile (TM x TN accumulator blocks of 32 x 32) whose top
// left element is (row0, col0) of C.  The sub-tile is staged through LDS, 32 rows at a time (fp32,
// row pitch padded by 16 bytes), and read back so that the lanes of one store instruction cover
// whole row segments, 16 bytes per lane: every global access of the epilogue (residual and
// saved-derivative reads, outputs) is then fully coalesced.  (Storing straight from the
// accumulator layout gives 8- or 16-byte pieces in 32 different rows per instruction; measured
// 8 % slower on the whole step.)
template <int TM, int TN, int WN, int EPI, typename TO>
struct WaveEpilogue {
  static constexpr int PITCH = WN * 4 + 16;  // rows 4 banks apart: 16-byte accesses of 16 rows, or of two row halves, never collide
  static constexpr int CPL = sizeof(TO) == 2 ? 8 : 4;  // consecutive columns per lane
  static constexpr int LPR = WN / CPL;                 // lanes per row
  static constexpr int RPP = 64 / LPR;                 // rows per pass
  static constexpr int NPASS = 32 / RPP;
  // The epilogue's global READS (residual rows, saved derivative) are issued together, ahead of
  // the staging and the stores: loads and stores complete out of order with respect to each
  // other, so a load issued after a store can only be waited for with "everything done", and a
  // load per pass would expose one full memory latency per pass.  All of the sub-tile at once
  // when that fits in 64 registers, else one 32-row block at a time.
  static constexpr bool HAS_AUX = EPI == EPI_RESID || EPI == EPI_DGELU;
  static constexpr bool AUX_ALL = TM * NPASS * 4 <= 64;
  u32x4 aux[HAS_AUX ? TM : 1][HAS_AUX ? NPASS : 1];
  const MfmaArgs& g;
  const int lane, row0, col0;
  __device__ __forceinline__ WaveEpilogue(const MfmaArgs& g_, int lane_, int row0_, int col0_)
      : g(g_), lane(lane_), row0(row0_), col0(col0_) {}
  __device__ __forceinline__ void load_aux(int i) {
#pragma unroll
    for (int pass = 0; pass < NPASS; pass++) {
      const int row = row0 + i * 32 + pass * RPP + lane / LPR;
      const int col = col0 + (lane % LPR) * CPL;
      if (EPI == EPI_RESID) aux[HAS_AUX ? i : 0][HAS_AUX ? pass : 0] = *reinterpret_cast<const u32x4*>(g.R + (int64_t)row * g.ldr + col);
      else aux[HAS_AUX ? i : 0][HAS_AUX ? pass : 0] = *reinterpret_cast<const u32x4*>(g.U + (int64_t)row * g.ldc + col);
    }
  }
  __device__ __forceinline__ void preload() {
    if (HAS_AUX && AUX_ALL) {
#pragma unroll
      for (int i = 0; i < TM; i++) load_aux(i);
    }
  }
  // stg: this wavefront's 32 x PITCH bytes of LDS; every wavefront that could still read operand
  // tiles there must be done with them
  __device__ __forceinline__ void run(f32x16 (&acc)[TM][TN], char* stg, TO* C) {
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
        const int row = row0 + i * 32 + rr;
        const int col = col0 + cc;
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
  // split-K: the K slices are dealt to the splits as evenly as whole slices allow (the first
  // nk_total % nsplit splits take one slice more)
  const int nk_total = g.K / BK;
  int nk = nk_total, slice0 = 0;
  if (SPLIT) {
    const int q = nk_total / g.nsplit, r = nk_total % g.nsplit;
    nk = q + (zsplit < r ? 1 : 0);
    slice0 = zsplit * q + (zsplit < r ? zsplit : r);
  }
  const int64_t kbase = (int64_t)slice0 * BK;

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

  // Epilogue (WaveEpilogue above): each wavefront stages its sub-tile through the operand buffers.
  TO* C = reinterpret_cast<TO*>(g.C);
  if (SPLIT) C += (int64_t)zsplit * g.split_stride;
  typedef WaveEpilogue<TM, TN, WN, EPI, TO> EP;
  static_assert(NW * 32 * EP::PITCH <= TL::LDS_BYTES, "epilogue staging must fit the operand buffers");
  EP ep(g, lane, m0 + wm * WM, n0 + wn * WN);
  ep.preload();
  __syncthreads();  // every wave is done with the operand tiles
  ep.run(acc, smem + wave * (32 * EP::PITCH), C);
}

// ---- 256 x 256 tile, two wavefront groups in alternating phases ("ping-pong") ----------------
// The vector-memory path feeds a CU about 40 bytes per clock; a 256 x 128 tile at the full MFMA
// rate needs 47, a 256 x 256 tile 32: the larger tile is what the memory path allows.  It leaves
// room for ONE workgroup per CU, so the overlap that two independent workgroups give the smaller
// tiles is built into the workgroup here: 8 wavefronts in two groups of four (group g owns columns
// 128 g .. 128 g + 127 of the tile, each wavefront 128 x 64 of them), every SIMD hosting one
// wavefront of each group.  A group alternates between a MEMORY phase (fragment reads of one
// 32-wide half of the K slice from LDS into registers, LDS stores of its share of the next slice,
// global loads of the slice after that) and a COMPUTE phase (16 MFMAs on those registers, nothing
// else).  The groups run one phase apart, separated by workgroup barriers, so each SIMD's matrix
// pipe always sees exactly one wavefront issuing back-to-back MFMAs while the other wavefront's
// LDS traffic, address arithmetic and waits hide behind them.
//
// Phases (kt = K slice, h = its half; p counts workgroup barriers):
//   group 0: M(kt,h) at p = 4 kt + 2 h, C(kt,h) at p + 1; group 1 the same one phase later.
//   LDS double buffer: slice kt lives in buffer kt & 1.  Slice kt+1 is written into the other
//   buffer during the M phases of slice kt (A chunks in M(kt,0), B chunks in M(kt,1)): the last
//   reads of its previous content (slice kt-1) ended at p = 4 kt - 1 and its first read is at
//   p = 4 kt + 4.  The global loads of a chunk are issued right after the chunk's registers were
//   stored, a whole slice (four phases) before they are needed.
// Rows / columns beyond M / N (M, N multiples of 128, not of 256) are loaded from clamped
// addresses, multiplied, and not stored: a wavefront's 128 x 64 sub-tile is wholly inside or outside.
template <int AL, int BL, int EPI, typename TO, bool SPLIT>
__global__ __launch_bounds__(512, 1) void gemm_pp_kernel(MfmaArgs g) {
  constexpr int BM = 256, BN = 256;
  typedef Tile<BM, BN, AL, BL, 2> TL;
  static_assert(TL::NT == 512 && TL::A_CHUNKS == 4 && TL::B_CHUNKS == 4, "8 wavefronts, 4 + 4 chunks per thread");
  constexpr int WM = 128, WN = 64, TM = 4, TN = 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = wave >> 2, wm = (wave >> 1) & 1, wn = wave & 1;
  const int ncol0 = grp * 128 + wn * WN;   // this wavefront's first column inside the tile

  int ntiles = g.tiles_m * g.tiles_n;
  int id = blockIdx.x, tile, zsplit = 0;
  if (SPLIT) {
    zsplit = id % g.nsplit;
    tile = id / g.nsplit;
  } else {
    int per = ntiles / 8;
    tile = (id < per * 8) ? (id % 8) * per + id / 8 : id;
  }
  // Tiles are numbered down column blocks 8 tiles wide, so that the 32 tiles an XCD works on at
  // a time form a 4 x 8 patch sharing 4 A panels and 8 B panels in its L2 (a row of 32 tiles would
  // share one A panel and stream 32 B panels through it).
  int tm, tn;
  {
    constexpr int GN = 8;
    const int span = GN * g.tiles_m, b = tile / span, r = tile - b * span;
    const int width = g.tiles_n - b * GN < GN ? g.tiles_n - b * GN : GN;
    tm = r / width;
    tn = b * GN + r % width;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  const int nk_total = g.K / BK;   // split-K: slices dealt to the splits as evenly as whole slices allow
  int nk = nk_total, slice0 = 0;
  if (SPLIT) {
    const int q = nk_total / g.nsplit, r = nk_total % g.nsplit;
    nk = q + (zsplit < r ? 1 : 0);
    slice0 = zsplit * q + (zsplit < r ? zsplit : r);
  }
  const int64_t kbase = (int64_t)slice0 * BK;

  // global addressing: scalar tile origin + per-lane, per-chunk 32-bit byte offsets (rows / column
  // runs beyond the matrix are clamped onto its last ones)
  const char* Ag = reinterpret_cast<const char*>(AL == 0 ? g.A + (int64_t)m0 * g.lda + kbase : g.A + kbase * g.lda + m0);
  const char* Bg = reinterpret_cast<const char*>(BL == 1 ? g.B + (int64_t)n0 * g.ldb + kbase : g.B + kbase * g.ldb + n0);
  constexpr int A_CPR = AL == 0 ? 8 : BM / 8, B_CPR = BL == 1 ? 8 : BN / 8;
  constexpr int A_RPC = TL::NT / A_CPR, B_RPC = TL::NT / B_CPR;
  auto tile_row = [](int q) { return (q & ~15) | ((q & 15) >> 1) | ((q & 1) << 3); };
  const int a_row = AL == 0 ? tile_row(tid / A_CPR) : tid / A_CPR;
  const int b_row = BL == 1 ? tile_row(tid / B_CPR) : tid / B_CPR;
  int a_goff[4], b_goff[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    if (AL == 0) {
      int r = a_row + i * A_RPC;
      r = m0 + r < g.M ? r : g.M - 1 - m0;
      a_goff[i] = (int)(((int64_t)r * g.lda + (tid % A_CPR) * 8) * 2);
    } else {
      int c = (tid % A_CPR) * 8;
      c = m0 + c < g.M ? c : g.M - 8 - m0;
      a_goff[i] = (int)(((int64_t)(a_row + i * A_RPC) * g.lda + c) * 2);
    }
    if (BL == 1) {
      int r = b_row + i * B_RPC;
      r = n0 + r < g.N ? r : g.N - 1 - n0;
      b_goff[i] = (int)(((int64_t)r * g.ldb + (tid % B_CPR) * 8) * 2);
    } else {
      int c = (tid % B_CPR) * 8;
      c = n0 + c < g.N ? c : g.N - 8 - n0;
      b_goff[i] = (int)(((int64_t)(b_row + i * B_RPC) * g.ldb + c) * 2);
    }
  }
  const int64_t a_step = AL == 0 ? BK * 2 : (int64_t)BK * g.lda * 2;
  const int64_t b_step = BL == 1 ? BK * 2 : (int64_t)BK * g.ldb * 2;
  const int a_soff = a_row * TL::A_STRIDE + (tid % A_CPR) * 16;
  const int b_soff = b_row * TL::B_STRIDE + (tid % B_CPR) * 16;

  u32x4 ra[4], rb[4];
  auto load_a = [&](int kt) {
    const char* ap = Ag + kt * a_step;
#pragma unroll
    for (int i = 0; i < 4; i++) ra[i] = *reinterpret_cast<const u32x4*>(ap + a_goff[i]);
  };
  auto load_b = [&](int kt) {
    const char* bp = Bg + kt * b_step;
#pragma unroll
    for (int i = 0; i < 4; i++) rb[i] = *reinterpret_cast<const u32x4*>(bp + b_goff[i]);
  };
  auto store_a = [&](int buf) {
    char* As = smem + buf * TL::STAGE;
#pragma unroll
    for (int i = 0; i < 4; i++) *reinterpret_cast<u32x4*>(As + a_soff + i * (A_RPC * TL::A_STRIDE)) = ra[i];
  };
  auto store_b = [&](int buf) {
    char* Bs = smem + buf * TL::STAGE + TL::A_BYTES;
#pragma unroll
    for (int i = 0; i < 4; i++) *reinterpret_cast<u32x4*>(Bs + b_soff + i * (B_RPC * TL::B_STRIDE)) = rb[i];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

  int a_off, b_off;
  if (AL == 0) a_off = (wm * WM + (lane & 31)) * TL::A_STRIDE + (lane >> 5) * 16;
  else a_off = ((lane >> 5) * 8 + ((lane & 15) >> 2)) * TL::A_STRIDE + (wm * WM + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
  if (BL == 1) b_off = (ncol0 + (lane & 31)) * TL::B_STRIDE + (lane >> 5) * 16;
  else b_off = ((lane >> 5) * 8 + ((lane & 15) >> 2)) * TL::B_STRIDE + (ncol0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;

  bf16x8 af[2][TM], bfr[2][TN];   // fragments of one 32-wide half of a K slice
  auto memory_phase = [&](int kt, int h) {
    const char* As = smem + (kt & 1) * TL::STAGE;
    const char* Bs = As + TL::A_BYTES;
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      const int kk = 2 * h + s2;
#pragma unroll
      for (int j = 0; j < TN; j++) {
        if (BL == 1) bfr[s2][j] = lds_read_direct(Bs + b_off + j * 32 * TL::B_STRIDE + kk * 32);
        else bfr[s2][j] = lds_read_tr(Bs + b_off + kk * 16 * TL::B_STRIDE + j * 64, TL::B_STRIDE);
      }
#pragma unroll
      for (int i = 0; i < TM; i++) {
        if (AL == 0) af[s2][i] = lds_read_direct(As + a_off + i * 32 * TL::A_STRIDE + kk * 32);
        else af[s2][i] = lds_read_tr(As + a_off + kk * 16 * TL::A_STRIDE + i * 64, TL::A_STRIDE);
      }
    }
    if (kt + 1 < nk) {
      if (h == 0) store_a((kt + 1) & 1); else store_b((kt + 1) & 1);
    }
    // unconditional (the last slices load the last slice again): with a fixed number of loads in
    // flight the waits before the stores above count exactly, and leave the newer half in flight
    const int kl = kt + 2 < nk ? kt + 2 : nk - 1;
    if (h == 0) load_a(kl); else load_b(kl);
  };
  auto compute_phase = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[s2][j], af[s2][i], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };

  // prologue: slice 0 into buffer 0, slice 1 into the registers
  load_a(0);
  load_b(0);
  store_a(0);
  store_b(0);
  load_a(nk > 1 ? 1 : 0);
  load_b(nk > 1 ? 1 : 0);
  __syncthreads();
  if (grp == 1) __builtin_amdgcn_s_barrier();   // group 1 runs one phase behind group 0
  for (int kt = 0; kt < nk; kt++) {
#pragma unroll
    for (int h = 0; h < 2; h++) {
      memory_phase(kt, h);
      __syncthreads();   // LDS stores visible, fragments in registers
      compute_phase();
      // Both groups execute 4 nk barriers in all: group 1's would-be last one (after its last
      // compute phase) guards nothing.  Group 0's last one is paired with the end of group 1's last
      // memory phase: after it nobody reads operand tiles any more.
      if (!(grp == 1 && kt == nk - 1 && h == 1)) __builtin_amdgcn_s_barrier();
    }
  }

  if (m0 + wm * WM >= g.M || n0 + ncol0 >= g.N) return;   // sub-tile outside the matrix
  TO* C = reinterpret_cast<TO*>(g.C);
  if (SPLIT) C += (int64_t)zsplit * g.split_stride;
  typedef WaveEpilogue<TM, TN, WN, EPI, TO> EP;
  static_assert(8 * 32 * EP::PITCH <= TL::LDS_BYTES, "epilogue staging must fit the operand buffers");
  EP ep(g, lane, m0 + wm * WM, n0 + ncol0);
  ep.preload();
  ep.run(acc, smem + wave * (32 * EP::PITCH), C);
}

// ---- the same ping-pong kernel with operands loaded straight from global memory into LDS ------
// The loads of slice kt + 1 write LDS buffer (kt + 1) & 1 directly (global_load_lds_dwordx4: each
// wavefront instruction fills 1 KB of LDS, lane l supplying bytes 16 l .. 16 l + 15), so the data
// never crosses the vector registers and no LDS store instruction is issued.  Rows cannot be padded
// inside such a 1 KB block, so bank conflicts are avoided by permuting 16-byte chunks inside a tile
// row instead; the permutation is applied on the global side (which chunk a lane fetches) and undone
// in the fragment addresses:
//   contraction-contiguous tile, [256 rows][128 bytes], 8 rows per instruction: row R keeps chunk c
//     at position c ^ ((R >> 1) & 7) (the 16 rows one quarter of a 16-byte fragment read touches
//     then fall into 16 different bank groups);
//   contraction-strided tile, [64 k][512 bytes], 2 k rows per instruction: k row r keeps its 64-byte
//     group q at position q ^ (r & 3) (the 4 k rows that 32 lanes of a transpose read touch then
//     fall into 4 different quarters of the banks).
// These loads are outside the compiler's wait tracking (inline assembly): every wavefront waits
// for its own (vmcnt(0)) before the last barrier that precedes the first read of the buffer.
__device__ __forceinline__ void global_to_lds_16(const void* base, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(base) : "memory");
}

template <int AL, int BL, int EPI, typename TO, bool SPLIT>
__global__ __launch_bounds__(512, 1) void gemm_ppd_kernel(MfmaArgs g) {
  constexpr int BM = 256, BN = 256;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES, LDS_BYTES = 2 * STAGE;
  constexpr int WM = 128, WN = 64, TM = 4, TN = 2;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, wm = (wave >> 1) & 1, wn = wave & 1;
  const int ncol0 = grp * 128 + wn * WN;

  int ntiles = g.tiles_m * g.tiles_n;
  int id = blockIdx.x, tile, zsplit = 0;
  if (SPLIT) {
    zsplit = id % g.nsplit;
    tile = id / g.nsplit;
  } else {
    int per = ntiles / 8;
    tile = (id < per * 8) ? (id % 8) * per + id / 8 : id;
  }
  int tm, tn;
  {
    constexpr int GN = 8;
    const int span = GN * g.tiles_m, b = tile / span, r = tile - b * span;
    const int width = g.tiles_n - b * GN < GN ? g.tiles_n - b * GN : GN;
    tm = r / width;
    tn = b * GN + r % width;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  const int nk_total = g.K / BK;   // split-K: slices dealt to the splits as evenly as whole slices allow
  int nk = nk_total, slice0 = 0;
  if (SPLIT) {
    const int q = nk_total / g.nsplit, r = nk_total % g.nsplit;
    nk = q + (zsplit < r ? 1 : 0);
    slice0 = zsplit * q + (zsplit < r ? zsplit : r);
  }
  const int64_t kbase = (int64_t)slice0 * BK;

  // Wavefront w, instruction i (0..3) moves 1 KB of the A tile and 1 KB of the B tile: tile rows
  // 8 (4 w + i) .. + 7 (contraction-contiguous) or k rows 2 (4 w + i), + 1 (contraction-strided).
  const char* Ag = reinterpret_cast<const char*>(AL == 0 ? g.A + (int64_t)m0 * g.lda + kbase : g.A + kbase * g.lda + m0);
  const char* Bg = reinterpret_cast<const char*>(BL == 1 ? g.B + (int64_t)n0 * g.ldb + kbase : g.B + kbase * g.ldb + n0);
  const int64_t a_step = AL == 0 ? BK * 2 : (int64_t)BK * g.lda * 2;
  const int64_t b_step = BL == 1 ? BK * 2 : (int64_t)BK * g.ldb * 2;
  unsigned a_goff[4], b_goff[4];
  auto chunk_offset = [&](bool kcontig, int i, int origin, int extent, int64_t ld) -> unsigned {
    if (kcontig) {
      const int R = 8 * (4 * wave + i) + (lane >> 3);
      const int chunk = (lane & 7) ^ ((R >> 1) & 7);
      const int r = origin + R < extent ? R : extent - 1 - origin;
      return (unsigned)((int64_t)r * ld * 2 + chunk * 16);
    }
    const int kr = 2 * (4 * wave + i) + (lane >> 5);
    const int chunk = (lane & 31) ^ ((kr & 3) << 2);
    int c = chunk * 8;
    c = origin + c < extent ? c : extent - 8 - origin;
    return (unsigned)(((int64_t)kr * ld + c) * 2);
  };
#pragma unroll
  for (int i = 0; i < 4; i++) {
    a_goff[i] = chunk_offset(AL == 0, i, m0, g.M, g.lda);
    b_goff[i] = chunk_offset(BL == 1, i, n0, g.N, g.ldb);
  }
  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)(smem);
  auto issue_loads = [&](int kt) {   // slice kt into buffer kt & 1
    const char* ap = Ag + kt * a_step;
    const char* bp = Bg + kt * b_step;
    const unsigned dst = lds0 + (kt & 1) * STAGE + (4 * wave) * 1024;
#pragma unroll
    for (int i = 0; i < 4; i++) global_to_lds_16(ap, a_goff[i], dst + i * 1024);
#pragma unroll
    for (int i = 0; i < 4; i++) global_to_lds_16(bp, b_goff[i], dst + A_BYTES + i * 1024);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

  // Fragment addresses.
  // contraction-contiguous: row R = base + (lane & 31), k chunk q = 2 kk + (lane >> 5) sits at
  //   position q ^ f(R), f(R) = ((lane & 31) >> 1) & 7 for every 32-aligned base.
  // contraction-strided (transpose read): k row = 16 kk + 8 (lane >> 5) + ((lane & 15) >> 2) (+ 4 for
  //   the second half), so k row & 3 = (lane >> 2) & 3; the 64-byte group (base * 2) >> 6 of a
  //   32-row block sits at group ^ that.
  const int fx = ((lane >> 5) ^ (((lane & 31) >> 1) & 7));
  const int tx = (lane >> 2) & 3;
  const int tr_row = ((lane >> 5) * 8 + ((lane & 15) >> 2)) * 512 + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;
  const int a_off = AL == 0 ? (wm * WM + (lane & 31)) * 128 : tr_row + wm * 256;
  const int b_off = BL == 1 ? (ncol0 + (lane & 31)) * 128 : tr_row + grp * 256;
  bf16x8 af[2][TM], bfr[2][TN];
  auto memory_phase = [&](int kt, int h) {
    const char* As = smem + (kt & 1) * STAGE;
    const char* Bs = As + A_BYTES;
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      const int kk = 2 * h + s2;
      const int pos = ((kk * 2) ^ fx) * 16;
#pragma unroll
      for (int j = 0; j < TN; j++) {
        if (BL == 1) bfr[s2][j] = lds_read_direct(Bs + b_off + j * 32 * 128 + pos);
        else bfr[s2][j] = lds_read_tr(Bs + b_off + kk * 16 * 512 + (((wn * 2 + j) ^ tx) << 6), 512);
      }
#pragma unroll
      for (int i = 0; i < TM; i++) {
        if (AL == 0) af[s2][i] = lds_read_direct(As + a_off + i * 32 * 128 + pos);
        else af[s2][i] = lds_read_tr(As + a_off + kk * 16 * 512 + ((i ^ tx) << 6), 512);
      }
    }
    if (h == 0 && kt + 1 < nk) issue_loads(kt + 1);
  };
  auto compute_phase = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[s2][j], af[s2][i], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };

  issue_loads(0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (grp == 1) __builtin_amdgcn_s_barrier();   // group 1 runs one phase behind group 0
  for (int kt = 0; kt < nk; kt++) {
#pragma unroll
    for (int h = 0; h < 2; h++) {
      memory_phase(kt, h);
      // Slice kt + 1 is first read in group 0's next memory phase, p = 4 kt + 4.  The last barrier
      // before it is, for group 1, the one that ends this memory phase when h == 1; for group 0
      // the one after its compute phase below.
      if (h == 1 && grp == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      compute_phase();
      if (h == 1 && grp == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (!(grp == 1 && kt == nk - 1 && h == 1)) __builtin_amdgcn_s_barrier();
    }
  }

  if (m0 + wm * WM >= g.M || n0 + ncol0 >= g.N) return;   // sub-tile outside the matrix
  TO* C = reinterpret_cast<TO*>(g.C);
  if (SPLIT) C += (int64_t)zsplit * g.split_stride;
  typedef WaveEpilogue<TM, TN, WN, EPI, TO> EP;
  static_assert(8 * 32 * EP::PITCH <= LDS_BYTES, "epilogue staging must fit the operand buffers");
  EP ep(g, lane, m0 + wm * WM, n0 + ncol0);
  ep.preload();
  ep.run(acc, smem + wave * (32 * EP::PITCH), C);
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
  static std::atomic<bool> attr_set{false};  // the call is idempotent: a race only repeats it
  if (!attr_set.load(std::memory_order_acquire)) {
    ALS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES));
    attr_set.store(true, std::memory_order_release);
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
    rec.flops = 2.0 * a.M * a.N * (double)a.K;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof.push_back(rec);
  }
  return ALS_OK;
}

template <int AL, int BL, int EPI, typename TO, bool SPLIT>
int launch_pp(const MfmaArgs& a, int nsplit, hipStream_t st) {
  typedef Tile<256, 256, AL, BL, 2> TL;
  auto kern = gemm_pp_kernel<AL, BL, EPI, TO, SPLIT>;
  static std::atomic<bool> attr_set{false};  // the call is idempotent: a race only repeats it
  if (!attr_set.load(std::memory_order_acquire)) {
    ALS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES));
    attr_set.store(true, std::memory_order_release);
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
  if (prof) hipExtLaunchKernelGGL(kern, grid, dim3(512), TL::LDS_BYTES, st, rec.e0, rec.e1, 0, a);
  else hipLaunchKernelGGL(kern, grid, dim3(512), TL::LDS_BYTES, st, a);
  ALS_CHECK_LAUNCH();
  if (prof) {
    rec.id = kernel_id(256, 256, AL, BL, EPI, sizeof(TO) == 2, SPLIT, 4);
    rec.flops = 2.0 * a.M * a.N * (double)a.K;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof.push_back(rec);
  }
  return ALS_OK;
}

template <int AL, int BL, int EPI, typename TO, bool SPLIT>
int launch_ppd(const MfmaArgs& a, int nsplit, hipStream_t st) {
  constexpr int LDS = 2 * (256 * 128 + 256 * 128);
  auto kern = gemm_ppd_kernel<AL, BL, EPI, TO, SPLIT>;
  static std::atomic<bool> attr_set{false};  // the call is idempotent: a race only repeats it
  if (!attr_set.load(std::memory_order_acquire)) {
    ALS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS));
    attr_set.store(true, std::memory_order_release);
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
  if (prof) hipExtLaunchKernelGGL(kern, grid, dim3(512), LDS, st, rec.e0, rec.e1, 0, a);
  else hipLaunchKernelGGL(kern, grid, dim3(512), LDS, st, a);
  ALS_CHECK_LAUNCH();
  if (prof) {
    rec.id = kernel_id(256, 256, AL, BL, EPI, sizeof(TO) == 2, SPLIT, 4) | 1 << 10;   // bit 10: direct-to-LDS form
    rec.flops = 2.0 * a.M * a.N * (double)a.K;
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
    if (bm == 256 && bn == 256 && nbuf == 4) return launch_pp<AL, BL, EPI, TO, SPLIT>(a, nsplit, st);      \
    if (bm == 256 && bn == 256 && nbuf == 5) return launch_ppd<AL, BL, EPI, TO, SPLIT>(a, nsplit, st);     \
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

// tuning override, 0 = automatic (set by als_k_set_gemm_tile; atomics so that a launch on another
// thread reads whole values, the three are still not changed as one)
static std::atomic<int> g_force_bm{0}, g_force_bn{0}, g_force_nbuf{0};

int gemm_mfma(const GemmDesc& g, hipStream_t st) {
  if (!gemm_mfma_supported(g)) return set_error(ALS_ERR_INVALID, "gemm_mfma: unsupported shape or layout");
  // Tile choice (measured on MI355X): the single-buffered 128x128 variant, 3 workgroups per CU
  // so that one's prologue/epilogue hides behind another's MFMAs, for short K and few tiles;
  // the double-buffered one once K is long enough to amortise its single resident pair;
  // 256x128 (less operand traffic and fewer LDS bytes per flop) when its tiles fill at least
  // 7/8 of the 512 resident slots (2 per CU).
  // The 256x256 kernel with two wavefront groups in alternating phases (buffering code 4; it
  // masks partial tiles, so M and N need only be multiples of 128) moves a third less operand data
  // per flop than 256x128 and keeps the matrix pipes busy through its LDS traffic.  One product
  // at a time on an idle chip, it loses to the smaller tiles when its tiles fill less than a
  // round of CUs or K is very short (profiles/gemm_mfma_microbench.md); inside worker steps that
  // overlap on several streams it wins there too (20M-class workload: +4 to +5 % tokens/s with
  // it on every product, 150M-class: equal), so it is used whenever the product has at least one
  // whole tile in each direction.  Its direct-to-LDS form (code 5) is 3-6 % faster in the
  // microbenchmark and equal or slightly slower inside a step; the register-staged form is the
  // default.
  int bm = 128, bn = 128, nbuf = 1;
  const bool pp_pays = g.M >= 256 && g.N >= 256;
  if (g_force_bm && g_force_nbuf == 4) { bm = 256; bn = 256; nbuf = 4; }
  else if (g_force_bm && g_force_nbuf == 5) { bm = 256; bn = 256; nbuf = 5; }
  else if (g_force_bm && fits(g.M, g.N, g_force_bm, g_force_bn)) { bm = g_force_bm; bn = g_force_bn; nbuf = g_force_nbuf; }
  else if (!g_force_bm && pp_pays) { bm = 256; bn = 256; nbuf = g_force_nbuf == 5 ? 5 : 4; }
  else if (g.a_layout == 1) {
    if (fits(g.M, g.N, 256, 256) && (g.M / 256) * (g.N / 256) >= 64) { bm = 256; bn = 256; nbuf = 2; }
    else if (fits(g.M, g.N, 256, 128) && (g.M / 256) * (g.N / 128) >= 128) { bm = 256; bn = 128; nbuf = 1; }
    else nbuf = 2;
  } else if (fits(g.M, g.N, 256, 128) && (g.M / 256) * (g.N / 128) >= 448) { bm = 256; bn = 128; }
  else if (g.K >= 2048) nbuf = 2;
  MfmaArgs a;
  a.A = (const bf16*)g.A; a.B = (const bf16*)g.B; a.lda = g.lda; a.ldb = g.ldb;
  a.M = g.M; a.N = g.N; a.K = g.K; a.tiles_m = (g.M + bm - 1) / bm; a.tiles_n = (g.N + bn - 1) / bn;
  a.C = g.C; a.ldc = g.ldc; a.R = g.R; a.ldr = g.ldr; a.C2 = g.C2; a.U = (const bf16*)g.U;
  a.split_stride = 0; a.nsplit = 1;
  int nsplit = 1;
  if (g.a_layout == 1 && g.b_layout == 0 && g.ldc == g.N) {
    // Weight-gradient shape: few tiles, long K.  K is split so that the grid fills the chip in
    // whole rounds of its resident workgroups (2 per CU for the double-buffered 128x128 variant
    // and for 256x128, 3 per CU for the single-buffered 128x128 one).  Candidates are costed in
    // microseconds with measured rates: the product at 700 TFLOP/s times the round-up loss of
    // the last round, plus the fp32 partials written and read back at 4 TB/s; each split keeps
    // at least 512 of K and the partials must fit the workspace.  Splits need not be equal: the K
    // slices are dealt out as evenly as whole slices allow.
    const size_t per = (size_t)g.M * g.N * sizeof(float);
    const int maxws = g.ws ? (int)(g.ws_bytes / per) : 1;
    const double t_prod = 2.0 * g.M * g.N * (double)g.K / 700e6;  // us
    double best = 1e30;
    int best_nbuf = nbuf, best_ns = 1;
    for (int cand = 0; cand < (bm == 128 && !g_force_bm ? 2 : 1); cand++) {
      const int nb = cand == 0 ? nbuf : (nbuf == 2 ? 1 : 2);
      const int slots = 256 * (bn == 256 ? 1 : (bm == 128 && nb == 1) ? 3 : 2);  // resident workgroups on the chip
      const int tiles = a.tiles_m * a.tiles_n;
      const int nk_total = g.K / BK;
      for (int ns = 1; ns <= 64 && ns <= maxws; ns++) {
        const int s_wg = (nk_total + ns - 1) / ns;     // slices of the longest split
        if (ns > 1 && s_wg < 8) continue;
        const int wgs = tiles * ns;
        const int rounds = (wgs + slots - 1) / slots;
        // a round lasts as long as its longest split; ideal = all slices spread over all slots
        double cost = t_prod * ((double)rounds * s_wg * slots) / ((double)tiles * nk_total) +
                      (ns > 1 ? ns * (double)per * 2.0 / 4e6 : 0.0);
        if (cand == 1) cost *= 1.03;  // prefer the first choice on near ties
        if (cost < best) { best = cost; best_nbuf = nb; best_ns = ns; }
      }
    }
    nbuf = best_nbuf;
    nsplit = best_ns;
  }
  if (nsplit > 1) {
    a.nsplit = nsplit;
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
  if (nbuf == 4) {
    snprintf(out, out_len, "gemm_pp%s_kernel<%d, %d, %s, %s, %s>", (id >> 10) & 1 ? "d" : "", (id >> 2) & 1, (id >> 3) & 1, epi[(id >> 4) & 3],
             (id >> 6) & 1 ? "bf16" : "float", (id >> 7) & 1 ? "true" : "false");
    return ALS_OK;
  }
  snprintf(out, out_len, "gemm_mfma_kernel<%d, %d, %d, %d, %s, %s, %s, %d, %d>", bm, bn, (id >> 2) & 1, (id >> 3) & 1,
           epi[(id >> 4) & 3], (id >> 6) & 1 ? "bf16" : "float", (id >> 7) & 1 ? "true" : "false", nbuf, occ);
  return ALS_OK;
}

// Tuning hook: force the MFMA GEMM tile (256x256, 256x128 or 128x128) and its LDS buffering
// (2 = double, 1 = single buffer with more workgroups per CU); 0,0 restores the automatic choice.  Not thread-safe; meant for benchmarks.
extern "C" int als_k_set_gemm_tile(int bm, int bn, int nbuf) {
  // (0, 0, 4) / (0, 0, 5): automatic tile choice, but the register-staged (4) or the direct-to-LDS
  // (5) form of the ping-pong kernel wherever that kernel is chosen
  if (bm == 0 && bn == 0 && (nbuf == 4 || nbuf == 5)) { als::g_force_bm = 0; als::g_force_bn = 0; als::g_force_nbuf = nbuf; return ALS_OK; }
  bool ok = (bm == 0 && bn == 0) || (bm == 256 && bn == 256) || (bm == 256 && bn == 128) || (bm == 128 && bn == 128);
  if (!ok || (bm && nbuf != 1 && nbuf != 2 && !(nbuf == 3 && bm == 128) && !((nbuf == 4 || nbuf == 5) && bm == 256 && bn == 256))) return als::set_error(ALS_ERR_INVALID, "unsupported tile %dx%d/%d", bm, bn, nbuf);
  als::g_force_bm = bm; als::g_force_bn = bn; als::g_force_nbuf = nbuf;
  return ALS_OK;
}
