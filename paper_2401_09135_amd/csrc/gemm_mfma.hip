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
// This file holds that kernel (gemm_mfma_kernel), the launchers, the choice of kernel and split
// for a product, and the measurement hooks.  Products with at least one whole 256 x 256 tile in
// each direction go to the kernels of gemm_pingpong.h (one workgroup of two wavefront groups in
// alternating memory / compute phases per CU); gemm_mfma_common.h has what the kernels share
// (LDS tile geometry, fragment reads, the per-wavefront epilogue).
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

#include "gemm_mfma_common.h"

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

#include "gemm_pingpong.h"

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

bool dw_group_supported(int M, int N, int K, int64_t lda, int64_t ldb) {
  return M >= 128 && N >= 128 && M % 128 == 0 && N % 128 == 0 && K >= 64 && K % 64 == 0 && lda % 8 == 0 && ldb % 8 == 0;
}

DwPlan dw_group_plan(const DwProblem* probs, int n_probs, int K, DwItem* items, DwSplitTile* split) {
  struct T3 { int p, tm, tn; };
  std::vector<T3> all;
  DwPlan plan{0, 0, 0, 0.0};
  for (int p = 0; p < n_probs; p++) {
    const int tms = (probs[p].M + 255) / 256, tns = (probs[p].N + 255) / 256;
    // the shorter tile direction fastest: consecutive tiles then share the panels of the longer one
    if (tms <= tns) { for (int tn = 0; tn < tns; tn++) for (int tm = 0; tm < tms; tm++) all.push_back({p, tm, tn}); }
    else { for (int tm = 0; tm < tms; tm++) for (int tn = 0; tn < tns; tn++) all.push_back({p, tm, tn}); }
    plan.flops += 2.0 * probs[p].M * probs[p].N * (double)K;
  }
  const int nk_total = K / BK, n_all = (int)all.size();
  // the last, partial round of tiles is split along K into as many parts as fill the chip (each at
  // least 4 slices long); a remainder of more than half a round stays whole
  const int r = n_all % DW_PLAN_CUS;
  int S = r ? DW_PLAN_CUS / r : 1;
  if (S > nk_total / 4) S = nk_total / 4;
  if (S < 1) S = 1;
  const int n_split = S > 1 ? r : 0, n_whole = n_all - n_split;
  // Whole tiles, in launch order.  The chip runs DW_PLAN_CUS tiles at a time, the 32 workgroups an XCD
  // holds being ids x, x + 8, ...: each such round takes DW_PLAN_CUS consecutive tiles of the list,
  // XCD x the x-th run of 32 of them.  The tiles of an XCD then share operand panels in its L2, and
  // the runs of one product sit on neighbouring XCDs at the same time, so that a panel one XCD has
  // fetched is still in the last-level cache when the next one asks for it (with a contiguous run of
  // the whole list per XCD instead, every XCD works on layers of its own and each panel comes from
  // HBM once per XCD round that uses it: 2.5 % slower on the 150M-class shapes).  What is left
  // behind the last full round is dealt the same way, XCD x taking the x-th of 8 runs of it.
  const int full = n_whole / DW_PLAN_CUS * DW_PLAN_CUS;
  const int tail_base = (n_whole - full) / 8, tail_rem = (n_whole - full) % 8;
  for (int id = 0; id < n_whole; id++) {
    const int x = id & 7, j = id >> 3;   // full is a multiple of 8: j counts this XCD's workgroups from 0
    const int idx = id < full ? (j / 32) * DW_PLAN_CUS + x * 32 + j % 32
                              : full + x * tail_base + (x < tail_rem ? x : tail_rem) + (j - full / 8);
    const T3& t = all[idx];
    items[id] = DwItem{t.p, t.tm, t.tn, -1, 0, nk_total, {0, 0}};
  }
  int n = n_whole;
  if (n_split) {
    const int q = nk_total / S, rr = nk_total % S;
    for (int s0 = 0; s0 < S; s0++)
      for (int i = 0; i < n_split; i++) {
        const T3& t = all[n_whole + i];
        items[n++] = DwItem{t.p, t.tm, t.tn, i * S + s0, s0 * q + (s0 < rr ? s0 : rr), q + (s0 < rr ? 1 : 0), {0, 0}};
      }
    for (int i = 0; i < n_split; i++) {
      const T3& t = all[n_whole + i];
      split[i] = DwSplitTile{t.p, t.tm, t.tn, i * S, S, {0, 0, 0}};
    }
  }
  plan.n_items = n; plan.n_split = n_split; plan.n_partial_tiles = n_split * S;
  return plan;
}

int dw_group_launch(const DwProblem* d_probs, const DwItem* d_items, const DwSplitTile* d_split, const DwPlan& plan,
                    float* partial_tiles, hipStream_t st) {
  if (plan.n_items <= 0) return ALS_OK;
  typedef Tile<256, 256, 1, 0, 2> TL;
  auto kern = gemm_pp_dw_grouped_kernel;
  static std::atomic<bool> attr_set{false};  // the call is idempotent: a race only repeats it
  if (!attr_set.load(std::memory_order_acquire)) {
    ALS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES));
    attr_set.store(true, std::memory_order_release);
  }
  ProfRec rec;
  bool prof = false;
  if (g_prof_on) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (g_prof_on && (g_prof_count++ % (unsigned)g_prof_every) == 0 && hipEventCreate(&rec.e0) == hipSuccess) {
      if (hipEventCreate(&rec.e1) == hipSuccess) prof = true;
      else (void)hipEventDestroy(rec.e0);
    }
  }
  if (prof) hipExtLaunchKernelGGL(kern, dim3(plan.n_items), dim3(512), TL::LDS_BYTES, st, rec.e0, rec.e1, 0, d_probs, d_items, partial_tiles);
  else hipLaunchKernelGGL(kern, dim3(plan.n_items), dim3(512), TL::LDS_BYTES, st, d_probs, d_items, partial_tiles);
  ALS_CHECK_LAUNCH();
  if (prof) {
    rec.id = 1 << 12;   // bit 12: the grouped weight-gradient kernel
    rec.flops = plan.flops;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof.push_back(rec);
  }
  if (plan.n_split) {
    hipLaunchKernelGGL(dw_tile_reduce_kernel, dim3(plan.n_split * 16), dim3(256), 0, st, d_probs, d_split, partial_tiles);
    ALS_CHECK_LAUNCH();
  }
  return ALS_OK;
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
  if ((id >> 12) & 1) { snprintf(out, out_len, "gemm_pp_dw_grouped_kernel"); return ALS_OK; }
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

