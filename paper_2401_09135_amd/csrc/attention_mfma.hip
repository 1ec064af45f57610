// Causal multi-head attention on the gfx950 matrix cores, head width 64, bf16 operands with
// fp32 accumulation and fp32 online softmax: forward, and backward as two passes (dQ per
// query block; dK and dV per key block) that recompute the probabilities from the saved
// log-sum-exp, so no S x S matrix ever reaches HBM and no atomics are used.
//
// All score products are formed transposed where that helps the softmax: with
// S^T[key, q] = K Q^T the MFMA accumulator gives every lane ONE query column and 16 keys in
// registers, so row maxima and sums are in-register reductions plus a single cross-half
// shuffle, and the probabilities are already in the register layout the next product wants as
// its B operand (contraction index = key, permuted identically on the A side).
//
// MFMA lane layouts (lane l, half hf = l/32):  A fragment: row l%32, contraction 8 hf + e;
// B fragment: column l%32, contraction 8 hf + e;  accumulator element v: row
// 8 (v/4) + 4 hf + v%4, column l%32.  Using accumulator elements v = 8 kk + e of a 32-row
// block as contraction slots (hf, e) of the kk-th following product maps slot (hf, e) to row
// 16 kk + 8 (e/4) + 4 hf + e%4; the transposed A fragments are gathered with that same map by
// two LDS transpose loads (rows +0..3 and +8..11).
#include "common.h"
#include <math.h>

namespace als {

namespace {

constexpr int DH = 64;
constexpr int ROW_D = 144;  // LDS row pitch (bytes) of a [row][64] bf16 tile
constexpr int TILE_BYTES = 64 * ROW_D;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ bf16x8 lds_direct(const char* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ bf16x8 lds_tr2(const char* lo, const char* hi) {
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)lo);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)hi);
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}
__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int v = 0; v < 16; v++) z[v] = 0.0f;
  return z;
}
__device__ __forceinline__ bf16x8 pack8(const f32x16& x, int kk) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; e++) r[e] = (bf16)x[8 * kk + e];
  return r;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)
// A use of fragments that were loaded from global memory before a loop: the compiler then waits
// for those loads HERE.  Without it, it re-checks them inside the loop with a count that also
// covers the loop's own freshly issued tile loads, i.e. every iteration waits for its prefetch.
__device__ __forceinline__ void settle(const bf16x8 (&f)[4]) {
  asm volatile("" ::"v"(f[0]), "v"(f[1]), "v"(f[2]), "v"(f[3]));
}

// byte offset of this lane's source address for a transposed A fragment inside a
// [row][64] tile: block of 32 columns `cb`, 16-row group `rb` (rows rb .. rb+3 and rb+8 .. +11)
__device__ __forceinline__ int tr_off(int lane, int rb, int cb) {
  int hf = lane >> 5;
  return (rb + 4 * hf + ((lane & 15) >> 2)) * ROW_D + (cb + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
}

// Workgroup -> (block along the sequence, head, sample).  Workgroup ids are dealt round-robin to
// the 8 XCDs; with the sequence block as the fastest grid index every XCD would get blocks of
// ONE causal position (all long or all short) and the chip would wait for two XCDs.  Instead
// XCD x takes (head, sample) pairs x, x + 8, ... and runs all sequence blocks of a pair, longest
// first: equal work per XCD, and the blocks that share K and V share an L2.
struct BlockId { int blk, hd, b; };
__device__ __forceinline__ BlockId block_id(int nblk, int h, int B) {
  const int i = blockIdx.x, pairs = h * B;
  int blk, pair;
  if ((pairs & 7) == 0) {
    const int j = i >> 3;
    pair = (i & 7) + 8 * (j / nblk);
    blk = j % nblk;
  } else {
    pair = i / nblk;
    blk = i % nblk;
  }
  return {blk, pair % h, pair / h};
}

// copy a [64 rows][64] bf16 tile from global (row pitch ld elements) to registers / LDS
struct TileRegs { u32x4 r[2]; };
__device__ __forceinline__ void tile_load(TileRegs& t, const bf16* src, int64_t ld, int tid) {
#pragma unroll
  for (int i = 0; i < 2; i++) {
    int c = tid + i * 256;
    t.r[i] = *reinterpret_cast<const u32x4*>(src + (int64_t)(c >> 3) * ld + (c & 7) * 8);
  }
}
__device__ __forceinline__ void tile_store(const TileRegs& t, char* dst, int tid) {
#pragma unroll
  for (int i = 0; i < 2; i++) {
    int c = tid + i * 256;
    *reinterpret_cast<u32x4*>(dst + (c >> 3) * ROW_D + (c & 7) * 16) = t.r[i];
  }
}

// write a transposed accumulator pair (rows = head dim, column = this lane's token) as bf16
__device__ __forceinline__ void store_rows(bf16* dst, const f32x16 (&acc)[2], float mul, int hf) {
#pragma unroll
  for (int dt = 0; dt < 2; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; e++) o[e] = (bf16)(acc[dt][4 * g + e] * mul);
      *reinterpret_cast<bf16x4*>(dst + dt * 32 + 8 * g + 4 * hf) = o;
    }
}

// ------------------------------------------------------------------------------------------
// forward: one workgroup per (128 queries, head, sample); wave w owns 32 queries
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void attn_fwd_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ o,
                                                       float* __restrict__ lse, int S, int h, int B, float scale_log2) {
  __shared__ __attribute__((aligned(16))) char smem[4 * TILE_BYTES];  // 2 stages x (K, V)
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hf = lane >> 5;
  const BlockId id = block_id(S / 128, h, B);
  const int q0 = (S / 128 - 1 - id.blk) * 128, hd = id.hd, b = id.b;
  const int d = h * DH;
  const int64_t ld = 3 * (int64_t)d;
  const bf16* base = qkv + (int64_t)b * S * ld + hd * DH;
  const int qw = q0 + w * 32, q = qw + (lane & 31);

  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; kk++) qf[kk] = *reinterpret_cast<const bf16x8*>(base + (int64_t)q * ld + kk * 16 + hf * 8);

  f32x16 oacc[2] = {zero16(), zero16()};
  float m_run = -INFINITY, l_run = 0.0f;
  const int n_tiles = (q0 + 128) / 64;
  TileRegs kr, vr;
  tile_load(kr, base + d, ld, tid);
  tile_load(vr, base + 2 * d, ld, tid);
  tile_store(kr, smem, tid);
  tile_store(vr, smem + TILE_BYTES, tid);
  settle(qf);
  __syncthreads();
  for (int jt = 0; jt < n_tiles; jt++) {
    const int key0 = jt * 64;
    if (jt + 1 < n_tiles) {
      tile_load(kr, base + (int64_t)(key0 + 64) * ld + d, ld, tid);
      tile_load(vr, base + (int64_t)(key0 + 64) * ld + 2 * d, ld, tid);
    }
    const char* Ks = smem + (jt & 1) * 2 * TILE_BYTES;
    const char* Vs = Ks + TILE_BYTES;
    if (key0 <= qw + 31) {  // wave-uniform: some key of the tile is visible to some query
      // The K fragment reads are issued together ahead of the score MFMAs, the V fragment reads
      // right behind those MFMAs (scheduling fences keep that order): each MFMA waits only for
      // its own operands, by count, and the V fragments arrive while the softmax runs.
      bf16x8 kfr[2][4], vfr[2][2][2];
#pragma unroll
      for (int kk = 0; kk < 4; kk++)
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
          kfr[kt][kk] = lds_direct(Ks + (kt * 32 + (lane & 31)) * ROW_D + kk * 32 + hf * 16);
      __builtin_amdgcn_sched_barrier(0);
      f32x16 s[2] = {zero16(), zero16()};
#pragma unroll
      for (int kk = 0; kk < 4; kk++)
#pragma unroll
        for (int kt = 0; kt < 2; kt++) s[kt] = MFMA(kfr[kt][kk], qf[kk], s[kt]);
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int kk = 0; kk < 2; kk++)
#pragma unroll
          for (int dt = 0; dt < 2; dt++) {
            int off = tr_off(lane, kt * 32 + 16 * kk, dt * 32);
            vfr[kt][kk][dt] = lds_tr2(Vs + off, Vs + off + 8 * ROW_D);
          }
      __builtin_amdgcn_sched_barrier(0);
      // running maximum in raw score units; probabilities are exp2((s - m) * scale_log2) with
      // the scale folded into one fma per element; masking only on tiles that cross the diagonal
      const bool need_mask = key0 + 63 > qw;
      float mx = -INFINITY;
      if (need_mask) {
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
          for (int v = 0; v < 16; v++) {
            int key = key0 + kt * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
            if (key > q) s[kt][v] = -INFINITY;
            mx = fmaxf(mx, s[kt][v]);
          }
      } else {
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
          for (int v = 0; v < 16; v++) mx = fmaxf(mx, s[kt][v]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // The reference point m_run only has to keep the exponentials in range, it need not be the
      // exact running maximum: it moves (and the accumulators are rescaled) only when some row's
      // maximum has grown by more than 2^8 in probability units since it was last set.  The first
      // tile always sets it (m_run = -inf; key 0 is visible to every query, so mx is finite).
      if (__any((mx - m_run) * scale_log2 > 8.0f)) {  // wave-uniform
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2((m_run - m_new) * scale_log2);
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2; dt++)
#pragma unroll
          for (int v = 0; v < 16; v++) oacc[dt][v] *= alpha;
        m_run = m_new;
      }
      const float neg = -m_run * scale_log2;
      float lsum = 0.0f;
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          float p = fast_exp2(fmaf(s[kt][v], scale_log2, neg));
          s[kt][v] = p;
          lsum += p;
        }
      l_run += lsum;
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
          bf16x8 pf = pack8(s[kt], kk);
#pragma unroll
          for (int dt = 0; dt < 2; dt++) oacc[dt] = MFMA(vfr[kt][kk][dt], pf, oacc[dt]);
        }
    }
    if (jt + 1 < n_tiles) {
      char* nxt = smem + ((jt + 1) & 1) * 2 * TILE_BYTES;
      tile_store(kr, nxt, tid);
      tile_store(vr, nxt + TILE_BYTES, tid);
    }
    __syncthreads();
  }
  const float l = l_run + __shfl_xor(l_run, 32, 64);
  store_rows(o + ((int64_t)b * S + q) * d + hd * DH, oacc, 1.0f / l, hf);
  if (hf == 0) lse[((int64_t)b * h + hd) * S + q] = (m_run * scale_log2 + log2f(l)) * LN2;
}

// ------------------------------------------------------------------------------------------
// backward, dQ (and the row dots D = rowsum(dO * O), which it leaves for the dK/dV pass): one
// workgroup per (128 queries, head, sample).  Per 64-key tile:
//   S^T = K Q^T ; dP^T = V dO^T ; dS^T = P^T (dP^T - D) ; dQ^T += K^T dS^T
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 3) void attn_bwd_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ o,
                                                          const bf16* __restrict__ d_o,
                                                          const float* __restrict__ lse, float* __restrict__ D,
                                                          bf16* __restrict__ dqkv, int S, int h, int B, float scale) {
  __shared__ __attribute__((aligned(16))) char smem[4 * TILE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hf = lane >> 5;
  const BlockId id = block_id(S / 128, h, B);
  const int q0 = (S / 128 - 1 - id.blk) * 128, hd = id.hd, b = id.b;
  const int d = h * DH;
  const int64_t ld = 3 * (int64_t)d;
  const bf16* base = qkv + (int64_t)b * S * ld + hd * DH;
  const int qw = q0 + w * 32, q = qw + (lane & 31);
  const float scale_log2 = scale * LOG2E;

  bf16x8 qf[4], gf[4];
  const bf16* dorow = d_o + ((int64_t)b * S + q) * d + hd * DH;
#pragma unroll
  for (int kk = 0; kk < 4; kk++) {
    qf[kk] = *reinterpret_cast<const bf16x8*>(base + (int64_t)q * ld + kk * 16 + hf * 8);
    gf[kk] = *reinterpret_cast<const bf16x8*>(dorow + kk * 16 + hf * 8);
  }
  const float lse2 = lse[((int64_t)b * h + hd) * S + q] * LOG2E;
  // D[q] = sum_c dO[q,c] O[q,c]: each lane holds half of its query's row; kept for the dK/dV pass
  float Dq = 0.0f;
  const bf16* orow = o + ((int64_t)b * S + q) * d + hd * DH;
#pragma unroll
  for (int kk = 0; kk < 4; kk++) {
    bf16x8 of = *reinterpret_cast<const bf16x8*>(orow + kk * 16 + hf * 8);
#pragma unroll
    for (int e = 0; e < 8; e++) Dq += (float)of[e] * (float)gf[kk][e];
  }
  Dq += __shfl_xor(Dq, 32, 64);
  if (hf == 0) D[((int64_t)b * h + hd) * S + q] = Dq;

  f32x16 dq[2] = {zero16(), zero16()};
  const int n_tiles = (q0 + 128) / 64;
  TileRegs kr, vr;
  tile_load(kr, base + d, ld, tid);
  tile_load(vr, base + 2 * d, ld, tid);
  tile_store(kr, smem, tid);
  tile_store(vr, smem + TILE_BYTES, tid);
  settle(qf);
  settle(gf);
  asm volatile("" ::"v"(lse2), "v"(Dq));
  __syncthreads();
  for (int jt = 0; jt < n_tiles; jt++) {
    const int key0 = jt * 64;
    if (jt + 1 < n_tiles) {
      tile_load(kr, base + (int64_t)(key0 + 64) * ld + d, ld, tid);
      tile_load(vr, base + (int64_t)(key0 + 64) * ld + 2 * d, ld, tid);
    }
    const char* Ks = smem + (jt & 1) * 2 * TILE_BYTES;
    const char* Vs = Ks + TILE_BYTES;
    if (key0 <= qw + 31) {
      const bool need_mask = key0 + 63 > qw;
#pragma unroll
      for (int kt = 0; kt < 2; kt++) {
        if (key0 + kt * 32 > qw + 31) continue;  // wave-uniform: every key of this block is masked
        f32x16 s = zero16(), dp = zero16();
        const int roff = (kt * 32 + (lane & 31)) * ROW_D + hf * 16;
        // fragment reads ahead of their MFMAs, the transposed K reads behind the score MFMAs
        // (scheduling fences keep the order; see the forward kernel)
        bf16x8 kfr[4], vfr[4], ktr[2][2];
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
          kfr[kk] = lds_direct(Ks + roff + kk * 32);
          vfr[kk] = lds_direct(Vs + roff + kk * 32);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
          s = MFMA(kfr[kk], qf[kk], s);
          dp = MFMA(vfr[kk], gf[kk], dp);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (need_mask) {
#pragma unroll
          for (int v = 0; v < 16; v++) {
            int key = key0 + kt * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
            float p = fast_exp2(fmaf(s[v], scale_log2, -lse2));
            if (key > q) p = 0.0f;
            s[v] = p * (dp[v] - Dq);
          }
        } else {
#pragma unroll
          for (int v = 0; v < 16; v++) s[v] = fast_exp2(fmaf(s[v], scale_log2, -lse2)) * (dp[v] - Dq);
        }
#pragma unroll
        for (int kk = 0; kk < 2; kk++)
#pragma unroll
          for (int dt = 0; dt < 2; dt++) {
            int off = tr_off(lane, kt * 32 + 16 * kk, dt * 32);
            ktr[kk][dt] = lds_tr2(Ks + off, Ks + off + 8 * ROW_D);
          }
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
          bf16x8 dsf = pack8(s, kk);
#pragma unroll
          for (int dt = 0; dt < 2; dt++) dq[dt] = MFMA(ktr[kk][dt], dsf, dq[dt]);
        }
      }
    }
    if (jt + 1 < n_tiles) {
      char* nxt = smem + ((jt + 1) & 1) * 2 * TILE_BYTES;
      tile_store(kr, nxt, tid);
      tile_store(vr, nxt + TILE_BYTES, tid);
    }
    __syncthreads();
  }
  store_rows(dqkv + ((int64_t)b * S + q) * ld + hd * DH, dq, scale, hf);
}

// ------------------------------------------------------------------------------------------
// backward, dK and dV: one workgroup per (128 KT keys, head, sample); wave w owns 32 KT keys.
// Per 64-query tile, for each 32-query half and 32-key block:
//   S = Q K^T ; dP = dO V^T ; P = exp(S - lse) ; dS = P (dP - D) ;
//   dV^T += dO^T P ; dK^T += Q^T dS
// ------------------------------------------------------------------------------------------
template <int KT>
__global__ __launch_bounds__(256, KT == 1 ? 2 : 1) void attn_bwd_dkv_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ d_o,
                                                           const float* __restrict__ lse, const float* __restrict__ D,
                                                           bf16* __restrict__ dqkv, int S, int h, int B, float scale) {
  // 2 stages x (Q, dO) tiles, then 2 stages x (64 log-sum-exp values, 64 row dots)
  __shared__ __attribute__((aligned(16))) char smem[4 * TILE_BYTES + 2 * 512];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, hf = lane >> 5;
  const BlockId id = block_id(S / (128 * KT), h, B);  // key block 0 (all queries see it) first
  const int kb0 = id.blk * (128 * KT), hd = id.hd, b = id.b;
  const int d = h * DH;
  const int64_t ld = 3 * (int64_t)d;
  const bf16* base = qkv + (int64_t)b * S * ld + hd * DH;
  const bf16* dobase = d_o + (int64_t)b * S * d + hd * DH;
  const float* lse_b = lse + ((int64_t)b * h + hd) * S;
  const float* D_b = D + ((int64_t)b * h + hd) * S;
  const int kw = kb0 + w * 32 * KT;  // this wave's first key
  const float scale_log2 = scale * LOG2E;

  bf16x8 kf[KT][4], vf[KT][4];
#pragma unroll
  for (int kt = 0; kt < KT; kt++) {
    const bf16* row = base + (int64_t)(kw + kt * 32 + (lane & 31)) * ld;
#pragma unroll
    for (int kk = 0; kk < 4; kk++) {
      kf[kt][kk] = *reinterpret_cast<const bf16x8*>(row + d + kk * 16 + hf * 8);
      vf[kt][kk] = *reinterpret_cast<const bf16x8*>(row + 2 * d + kk * 16 + hf * 8);
    }
  }
  f32x16 dk[KT][2], dv[KT][2];
#pragma unroll
  for (int kt = 0; kt < KT; kt++)
#pragma unroll
    for (int dt = 0; dt < 2; dt++) { dk[kt][dt] = zero16(); dv[kt][dt] = zero16(); }

  const int qstart = (kb0 / 64) * 64;
  const int n_tiles = (S - qstart) / 64;
  TileRegs qr, gr;
  float4 st4 = make_float4(0.f, 0.f, 0.f, 0.f);  // lanes 0-15: 4 lse values, lanes 16-31: 4 row dots
  auto stats_load = [&](int q_first) {
    if (tid < 32) st4 = *reinterpret_cast<const float4*>((tid < 16 ? lse_b : D_b) + q_first + 4 * (tid & 15));
    if (tid < 16) { st4.x *= -LOG2E; st4.y *= -LOG2E; st4.z *= -LOG2E; st4.w *= -LOG2E; }  // -lse in log2 units
  };
  auto stats_store = [&](int stage) {
    if (tid < 32) *reinterpret_cast<float4*>(smem + 4 * TILE_BYTES + stage * 512 + tid * 16) = st4;
  };
  tile_load(qr, base + (int64_t)qstart * ld, ld, tid);
  tile_load(gr, dobase + (int64_t)qstart * d, d, tid);
  stats_load(qstart);
  tile_store(qr, smem, tid);
  tile_store(gr, smem + TILE_BYTES, tid);
  stats_store(0);
#pragma unroll
  for (int kt = 0; kt < KT; kt++) { settle(kf[kt]); settle(vf[kt]); }
  __syncthreads();
  for (int it = 0; it < n_tiles; it++) {
    const int qt0 = qstart + it * 64;
    if (it + 1 < n_tiles) {
      tile_load(qr, base + (int64_t)(qt0 + 64) * ld, ld, tid);
      tile_load(gr, dobase + (int64_t)(qt0 + 64) * d, d, tid);
      stats_load(qt0 + 64);
    }
    const char* Qs = smem + (it & 1) * 2 * TILE_BYTES;
    const char* Gs = Qs + TILE_BYTES;
    const char* Ss = smem + 4 * TILE_BYTES + (it & 1) * 512;
#pragma unroll
    for (int qh = 0; qh < 2; qh++) {
      const int qs = qt0 + qh * 32;          // first query of this half tile
      if (qs + 31 < kw) continue;            // wave-uniform: every query precedes every key
      // per-lane row statistics for the 16 accumulator rows: queries qs + 8 g + 4 hf + 0..3
      float4 l4[4], d4[4];
#pragma unroll
      for (int g = 0; g < 4; g++) {
        l4[g] = *reinterpret_cast<const float4*>(Ss + (qh * 32 + 8 * g + 4 * hf) * 4);
        d4[g] = *reinterpret_cast<const float4*>(Ss + 256 + (qh * 32 + 8 * g + 4 * hf) * 4);
      }
      const int roff = (qh * 32 + (lane & 31)) * ROW_D + hf * 16;
      bf16x8 qa[4], ga[4];
#pragma unroll
      for (int kk = 0; kk < 4; kk++) {
        qa[kk] = lds_direct(Qs + roff + kk * 32);
        ga[kk] = lds_direct(Gs + roff + kk * 32);
      }
      bf16x8 qT[2][2], gT[2][2];  // [kk over the 32 queries][head-dim half]
      auto read_transposed = [&]() {
#pragma unroll
        for (int kk = 0; kk < 2; kk++)
#pragma unroll
          for (int dt = 0; dt < 2; dt++) {
            int off = tr_off(lane, qh * 32 + 16 * kk, dt * 32);
            qT[kk][dt] = lds_tr2(Qs + off, Qs + off + 8 * ROW_D);
            gT[kk][dt] = lds_tr2(Gs + off, Gs + off + 8 * ROW_D);
          }
      };
      if (KT != 1) read_transposed();
#pragma unroll
      for (int kt = 0; kt < KT; kt++) {
        const int key = kw + kt * 32 + (lane & 31);
        if (qs + 31 < kw + kt * 32) continue;  // wave-uniform
        f32x16 s = zero16(), dp = zero16();
        if (KT == 1) {
          // the 16 transpose reads for the second pair of products trickle in behind the first
          // pair's 8 MFMAs (two per MFMA)
          __builtin_amdgcn_sched_barrier(0);
          read_transposed();
        }
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
          s = MFMA(qa[kk], kf[kt][kk], s);
          dp = MFMA(ga[kk], vf[kt][kk], dp);
        }
        if (KT == 1) {
#pragma unroll
          for (int m = 0; m < 8; m++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        const bool need_mask = qs < kw + kt * 32 + 31;
        if (need_mask) {  // wave-uniform: only blocks that cross the diagonal pay for the compare
#pragma unroll
          for (int v = 0; v < 16; v++) {
            const float lv = reinterpret_cast<const float*>(&l4[v >> 2])[v & 3];
            const float dvv = reinterpret_cast<const float*>(&d4[v >> 2])[v & 3];
            float p = fast_exp2(fmaf(s[v], scale_log2, lv));
            int qi = qs + 8 * (v >> 2) + 4 * hf + (v & 3);
            if (key > qi) p = 0.0f;
            s[v] = p;
            dp[v] = p * (dp[v] - dvv);
          }
        } else {
#pragma unroll
          for (int v = 0; v < 16; v++) {
            const float lv = reinterpret_cast<const float*>(&l4[v >> 2])[v & 3];
            const float dvv = reinterpret_cast<const float*>(&d4[v >> 2])[v & 3];
            float p = fast_exp2(fmaf(s[v], scale_log2, lv));
            s[v] = p;
            dp[v] = p * (dp[v] - dvv);
          }
        }
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
          bf16x8 pf = pack8(s, kk), dsf = pack8(dp, kk);
#pragma unroll
          for (int dt = 0; dt < 2; dt++) {
            dv[kt][dt] = MFMA(gT[kk][dt], pf, dv[kt][dt]);
            dk[kt][dt] = MFMA(qT[kk][dt], dsf, dk[kt][dt]);
          }
        }
      }
    }
    if (it + 1 < n_tiles) {
      char* nxt = smem + ((it + 1) & 1) * 2 * TILE_BYTES;
      tile_store(qr, nxt, tid);
      tile_store(gr, nxt + TILE_BYTES, tid);
      stats_store((it + 1) & 1);
    }
    __syncthreads();
  }
#pragma unroll
  for (int kt = 0; kt < KT; kt++) {
    bf16* row = dqkv + ((int64_t)b * S + kw + kt * 32 + (lane & 31)) * ld + hd * DH;
    store_rows(row + d, dk[kt], scale, hf);
    store_rows(row + 2 * d, dv[kt], 1.0f, hf);
  }
}

}  // namespace

bool attention_mfma_supported(int S, int dh, int bf) { return bf && dh == 64 && S >= 128 && S % 128 == 0 && S <= 1024; }

int attention_fwd_mfma(const void* qkv, void* o, float* lse, int B, int S, int h, int dh, hipStream_t st) {
  if (!attention_mfma_supported(S, dh, 1) || B < 1 || h < 1) return set_error(ALS_ERR_INVALID, "attention_fwd_mfma: unsupported shape");
  float scale_log2 = (1.0f / sqrtf((float)dh)) * LOG2E;
  hipLaunchKernelGGL(attn_fwd_kernel, dim3(S / 128 * h * B), dim3(256), 0, st, (const bf16*)qkv, (bf16*)o, lse, S, h, B, scale_log2);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

int attention_bwd_mfma(const void* qkv, const void* o, const void* d_o, const float* lse, float* dscratch,
                       void* dqkv, int B, int S, int h, int dh, hipStream_t st) {
  if (!attention_mfma_supported(S, dh, 1) || B < 1 || h < 1) return set_error(ALS_ERR_INVALID, "attention_bwd_mfma: unsupported shape");
  float scale = 1.0f / sqrtf((float)dh);
  hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3(S / 128 * h * B), dim3(256), 0, st, (const bf16*)qkv, (const bf16*)o,
                     (const bf16*)d_o, lse, dscratch, (bf16*)dqkv, S, h, B, scale);
  ALS_CHECK_LAUNCH();
  // one 32-key block per wavefront: two blocks (KT = 2) halve the Q / dO tile traffic but need
  // more than 256 registers, which costs the second resident workgroup and AGPR copies
  hipLaunchKernelGGL(attn_bwd_dkv_kernel<1>, dim3(S / 128 * h * B), dim3(256), 0, st, (const bf16*)qkv,
                     (const bf16*)d_o, lse, dscratch, (bf16*)dqkv, S, h, B, scale);
  ALS_CHECK_LAUNCH();
  return ALS_OK;
}

}  // namespace als
