// Device helpers shared by the MFMA GEMM kernels (gemm_mfma.hip, gemm_pingpong.h): tile
// geometry in LDS, fragment reads, the GELU pair, the kernel argument block and the
// per-wavefront epilogue.  Included inside namespace als { namespace { ... } }.
#pragma once

constexpr int BK = 64;

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
// 8 % slower on the whole step.)  Outputs are written with non-temporal stores: a round of tiles
// writes 32-64 MB at once, as much as all L2s hold, and no tile reads them back (3-5 % on the
// products with short K, one product at a time).
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
          __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(reinterpret_cast<float*>(C) + ci));
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
            __builtin_nontemporal_store(__builtin_bit_cast(u32x4, o2), reinterpret_cast<u32x4*>(reinterpret_cast<bf16*>(g.C2) + ci));
          } else {
#pragma unroll
            for (int e = 0; e < CPL; e++) o[e & 7] = (bf16)x[e];
          }
          __builtin_nontemporal_store(__builtin_bit_cast(u32x4, o), reinterpret_cast<u32x4*>(reinterpret_cast<bf16*>(C) + ci));
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // reads done before the next block overwrites
    }
  }
};

