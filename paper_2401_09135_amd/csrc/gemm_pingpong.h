// The 256 x 256 MFMA GEMM kernels with two wavefront groups in alternating memory / compute
// phases: gemm_pp_kernel (operands staged through registers) and gemm_ppd_kernel (operands
// loaded straight into LDS).  Included by gemm_mfma.hip inside namespace als { namespace { ... } },
// after gemm_mfma_common.h.
#pragma once

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
// addresses and not stored.  A wavefront's 128 x 64 sub-tile is wholly inside or outside the matrix;
// a wavefront outside reads no fragments and issues no MFMAs, and the sub-tiles are dealt to the
// groups (sub_tile below) so that a dead half of the tile is one whole group.
// Workgroup id -> (tile row, tile column, K split).  Workgroup ids are dealt round-robin to the 8
// XCDs, each with its own L2, so what matters is which work items share an XCD.
//   No split: XCD x takes a contiguous run of tiles, numbered down column blocks 8 tiles wide, so
//   that the 32 tiles it works on at a time form a 4 x 8 patch sharing 4 A panels and 8 B panels in
//   its L2 (a row of 32 tiles would share one A panel and stream 32 B panels through it).
//   Split-K: the (split, tile) pairs are ordered split-major, then along the LONGER tile direction,
//   the shorter one fastest, and XCD x takes a contiguous run of them: the tiles it holds at a time
//   share one K range and span the short direction completely, so the panels of the short
//   direction are fetched by the few XCDs that hold that split and the panels of the long direction
//   once each (dealing splits and tiles out by id alone makes every XCD fetch most of both operands).
struct WorkItem { int tm, tn, zsplit; };
template <bool SPLIT>
__device__ __forceinline__ WorkItem work_item(int id, int tiles_m, int tiles_n, int nsplit) {
  const int ntiles = tiles_m * tiles_n;
  if (SPLIT) {
    const int total = ntiles * nsplit, base = total / 8, rem = total % 8;
    const int x = id & 7, j = id >> 3;
    const int p = x * base + (x < rem ? x : rem) + j;   // XCD x holds ids x, x + 8, ...: base (+ 1) of them
    const int z = p / ntiles, t = p - z * ntiles;
    if (tiles_m <= tiles_n) return {t % tiles_m, t / tiles_m, z};
    return {t / tiles_n, t % tiles_n, z};
  }
  const int per = ntiles / 8;
  const int tile = (id < per * 8) ? (id % 8) * per + id / 8 : id;
  constexpr int GN = 8;
  const int span = GN * tiles_m, b = tile / span, r = tile - b * span;
  const int width = tiles_n - b * GN < GN ? tiles_n - b * GN : GN;
  return {r / width, b * GN + r % width, 0};
}

// Which 128 x 64 sub-tile of the 256 x 256 tile a wavefront owns: row half mh, column quarter nq.
// Normally group g (wavefronts 4 g .. 4 g + 3) owns columns 128 g .. 128 g + 127.  In a tile whose
// lower 128 rows lie outside the matrix while its columns do not, the groups own the row halves
// instead: the dead half is then ONE group, whose compute phases are empty, and a K slice of that
// tile costs two MFMA phases instead of four (a dead column half is one group in the normal map).
// Every (mh, nq) pair has exactly one wavefront in both maps, and the four wavefronts of a group sit
// on the four SIMDs either way.
struct SubTile { int mh, nq; };
__device__ __forceinline__ SubTile sub_tile(int wave, int m0, int n0, int M, int N) {
  const int grp = wave >> 2, sub = wave & 3;
  const bool by_rows = m0 + 128 >= M && n0 + 128 < N;   // workgroup-uniform
  return by_rows ? SubTile{grp, sub} : SubTile{sub >> 1, grp * 2 + (sub & 1)};
}

// One 256 x 256 tile: rows m0.., columns n0.., K slices slice0 .. slice0 + nk - 1, results to C
// (leading dimension g.ldc; the caller has added a split's or a partial tile's offset).
template <int AL, int BL, int EPI, typename TO>
__device__ __forceinline__ void pp_tile(const MfmaArgs& g, const int m0, const int n0, const int slice0, const int nk,
                                        TO* C, char* smem) {
  constexpr int BM = 256, BN = 256;
  typedef Tile<BM, BN, AL, BL, 2> TL;
  static_assert(TL::NT == 512 && TL::A_CHUNKS == 4 && TL::B_CHUNKS == 4, "8 wavefronts, 4 + 4 chunks per thread");
  constexpr int WM = 128, WN = 64, TM = 4, TN = 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = wave >> 2;
  const SubTile st = sub_tile(wave, m0, n0, g.M, g.N);
  const int mh = st.mh, ncol0 = st.nq * WN;   // this wavefront's row half and first column inside the tile
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
  if (AL == 0) a_off = (mh * WM + (lane & 31)) * TL::A_STRIDE + (lane >> 5) * 16;
  else a_off = ((lane >> 5) * 8 + ((lane & 15) >> 2)) * TL::A_STRIDE + (mh * WM + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
  if (BL == 1) b_off = (ncol0 + (lane & 31)) * TL::B_STRIDE + (lane >> 5) * 16;
  else b_off = ((lane >> 5) * 8 + ((lane & 15) >> 2)) * TL::B_STRIDE + (ncol0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;

  // A wavefront whose 128 x 64 sub-tile lies outside the matrix (M, N multiples of 128, not of 256)
  // still moves its share of the operand tiles and keeps the barriers, but reads no fragments and
  // issues no MFMAs: the SIMD's matrix pipe and the LDS are left to the live wavefronts.
  const bool live = m0 + mh * WM < g.M && n0 + ncol0 < g.N;   // wavefront-uniform
  bf16x8 af[2][TM], bfr[2][TN];   // fragments of one 32-wide half of a K slice
  auto memory_phase = [&](int kt, int h) {
    const char* As = smem + (kt & 1) * TL::STAGE;
    const char* Bs = As + TL::A_BYTES;
    if (live) {
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
    if (live) {
      __builtin_amdgcn_s_setprio(1);
#pragma unroll
      for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
          for (int j = 0; j < TN; j++)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[s2][j], af[s2][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_s_setprio(0);
    }
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

  if (!live) return;   // sub-tile outside the matrix
  typedef WaveEpilogue<TM, TN, WN, EPI, TO> EP;
  static_assert(8 * 32 * EP::PITCH <= TL::LDS_BYTES, "epilogue staging must fit the operand buffers");
  EP ep(g, lane, m0 + mh * WM, n0 + ncol0);
  ep.preload();
  ep.run(acc, smem + wave * (32 * EP::PITCH), C);
}

template <int AL, int BL, int EPI, typename TO, bool SPLIT>
__global__ __launch_bounds__(512, 1) void gemm_pp_kernel(MfmaArgs g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const WorkItem wi = work_item<SPLIT>(blockIdx.x, g.tiles_m, g.tiles_n, g.nsplit);
  const int nk_total = g.K / BK;   // split-K: slices dealt to the splits as evenly as whole slices allow
  int nk = nk_total, slice0 = 0;
  TO* C = reinterpret_cast<TO*>(g.C);
  if (SPLIT) {
    const int q = nk_total / g.nsplit, r = nk_total % g.nsplit;
    nk = q + (wi.zsplit < r ? 1 : 0);
    slice0 = wi.zsplit * q + (wi.zsplit < r ? wi.zsplit : r);
    C += (int64_t)wi.zsplit * g.split_stride;
  }
  pp_tile<AL, BL, EPI, TO>(g, wi.tm * 256, wi.tn * 256, slice0, nk, C, smem);
}

// ---- all weight gradients of a backward pass in one launch ---------------------------------------
// Every layer's weight gradient is a product X^T dY over the same contraction length (the tokens of
// the batch) with few tiles (16-56 for the 150M-class shapes): one product per launch needs a K
// split of 4-16 to fill the chip, whose fp32 partials cost as much memory traffic as the operands.
// Here the products of ALL layers are one list of work items built on the host (DwItem: product,
// tile, K slice range, where the result goes): whole rounds of tiles run unsplit over the full
// contraction and write the gradient directly; only the tiles of the last, partial round are split
// along K, so that they fill the chip too, into partial tiles that dw_tile_reduce_kernel adds in
// slot order.  Items are stored in launch order; the host lays them out so that the 32 workgroups an
// XCD holds at a time (ids x, x + 8, ...) are consecutive tiles of the same products and the 8 XCDs
// hold consecutive runs of the list.  The kernel
// itself (gemm_pp_dw_grouped_kernel) follows the direct-to-LDS tile body it runs on, further down.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T>
__device__ __forceinline__ T* uniform_ptr(T* p) {
  const uint64_t u = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  return reinterpret_cast<T*>(((uint64_t)hi << 32) | lo);
}

// Adds the partial tiles of the split tiles in slot order and writes the sums into the gradients.
__global__ __launch_bounds__(256) void dw_tile_reduce_kernel(const DwProblem* __restrict__ probs,
                                                             const DwSplitTile* __restrict__ tiles,
                                                             const float* __restrict__ partial_tiles) {
  const DwSplitTile t = tiles[blockIdx.x >> 4];           // 16 workgroups per tile, 16 rows each
  const DwProblem pr = probs[t.prob];
  const int r = (blockIdx.x & 15) * 16 + (threadIdx.x >> 4), c0 = (threadIdx.x & 15) * 4;
  const int row = t.tm * 256 + r;
  if (row >= pr.M) return;
#pragma unroll
  for (int cc = 0; cc < 4; cc++) {
    const int c = c0 + cc * 64, col = t.tn * 256 + c;
    if (col >= pr.N) continue;
    const float* p = partial_tiles + (int64_t)t.slot0 * 65536 + r * 256 + c;
    f32x4 a = *reinterpret_cast<const f32x4*>(p);
    for (int s = 1; s < t.nslots; s++) a += *reinterpret_cast<const f32x4*>(p + (int64_t)s * 65536);
    *reinterpret_cast<f32x4*>(pr.C + (int64_t)row * pr.N + col) = a;
  }
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

template <int AL, int BL, int EPI, typename TO>
__device__ __forceinline__ void ppd_tile(const MfmaArgs& g, const int m0, const int n0, const int slice0, const int nk,
                                         TO* C, char* smem) {
  constexpr int BM = 256, BN = 256;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES, LDS_BYTES = 2 * STAGE;
  constexpr int WM = 128, WN = 64, TM = 4, TN = 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;
  const SubTile st = sub_tile(wave, m0, n0, g.M, g.N);
  const int mh = st.mh, nq = st.nq, ncol0 = nq * WN;
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
  const int a_off = AL == 0 ? (mh * WM + (lane & 31)) * 128 : tr_row + mh * 256;
  const int b_off = BL == 1 ? (ncol0 + (lane & 31)) * 128 : tr_row + (nq >> 1) * 256;
  const bool live = m0 + mh * WM < g.M && n0 + ncol0 < g.N;   // as in gemm_pp_kernel
  bf16x8 af[2][TM], bfr[2][TN];
  auto memory_phase = [&](int kt, int h) {
    const char* As = smem + (kt & 1) * STAGE;
    const char* Bs = As + A_BYTES;
    if (live) {
#pragma unroll
      for (int s2 = 0; s2 < 2; s2++) {
        const int kk = 2 * h + s2;
        const int pos = ((kk * 2) ^ fx) * 16;
#pragma unroll
        for (int j = 0; j < TN; j++) {
          if (BL == 1) bfr[s2][j] = lds_read_direct(Bs + b_off + j * 32 * 128 + pos);
          else bfr[s2][j] = lds_read_tr(Bs + b_off + kk * 16 * 512 + ((((nq & 1) * 2 + j) ^ tx) << 6), 512);
        }
#pragma unroll
        for (int i = 0; i < TM; i++) {
          if (AL == 0) af[s2][i] = lds_read_direct(As + a_off + i * 32 * 128 + pos);
          else af[s2][i] = lds_read_tr(As + a_off + kk * 16 * 512 + ((i ^ tx) << 6), 512);
        }
      }
    }
    if (h == 0 && kt + 1 < nk) issue_loads(kt + 1);
  };
  auto compute_phase = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    if (live) {
      __builtin_amdgcn_s_setprio(1);
#pragma unroll
      for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
          for (int j = 0; j < TN; j++)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[s2][j], af[s2][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_s_setprio(0);
    }
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

  if (!live) return;   // sub-tile outside the matrix
  typedef WaveEpilogue<TM, TN, WN, EPI, TO> EP;
  static_assert(8 * 32 * EP::PITCH <= LDS_BYTES, "epilogue staging must fit the operand buffers");
  EP ep(g, lane, m0 + mh * WM, n0 + ncol0);
  ep.preload();
  ep.run(acc, smem + wave * (32 * EP::PITCH), C);
}

template <int AL, int BL, int EPI, typename TO, bool SPLIT>
__global__ __launch_bounds__(512, 1) void gemm_ppd_kernel(MfmaArgs g) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const WorkItem wi = work_item<SPLIT>(blockIdx.x, g.tiles_m, g.tiles_n, g.nsplit);
  const int nk_total = g.K / BK;   // split-K: slices dealt to the splits as evenly as whole slices allow
  int nk = nk_total, slice0 = 0;
  TO* C = reinterpret_cast<TO*>(g.C);
  if (SPLIT) {
    const int q = nk_total / g.nsplit, r = nk_total % g.nsplit;
    nk = q + (wi.zsplit < r ? 1 : 0);
    slice0 = wi.zsplit * q + (wi.zsplit < r ? wi.zsplit : r);
    C += (int64_t)wi.zsplit * g.split_stride;
  }
  ppd_tile<AL, BL, EPI, TO>(g, wi.tm * 256, wi.tn * 256, slice0, nk, C, smem);
}

// The grouped weight-gradient launch (its work items and tables are described above, next to
// dw_tile_reduce_kernel).  It runs on the direct-to-LDS tile body: on these long contractions with both operands contraction-strided
// that form is 2-3 % faster also inside overlapped worker steps (150M workload +1.2 % tokens/s).
__global__ __launch_bounds__(512, 1) void gemm_pp_dw_grouped_kernel(const DwProblem* __restrict__ probs,
                                                                     const DwItem* __restrict__ items,
                                                                     float* __restrict__ partial_tiles) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const DwItem it = items[blockIdx.x];
  const DwProblem pr = probs[uniform(it.prob)];
  MfmaArgs g;
  g.A = uniform_ptr(pr.A); g.B = uniform_ptr(pr.B);
  g.lda = uniform(pr.lda); g.ldb = uniform(pr.ldb);
  g.M = uniform(pr.M); g.N = uniform(pr.N); g.K = 0;
  g.tiles_m = 0; g.tiles_n = 0; g.nsplit = 1;
  g.R = nullptr; g.ldr = 0; g.C2 = nullptr; g.U = nullptr; g.split_stride = 0;
  const int m0 = uniform(it.tm) * 256, n0 = uniform(it.tn) * 256, slot = uniform(it.slot);
  float* C;
  if (slot < 0) { C = uniform_ptr(pr.C); g.ldc = g.N; }
  else { C = partial_tiles + (int64_t)slot * 65536 - ((int64_t)m0 * 256 + n0); g.ldc = 256; }
  g.C = C;
  ppd_tile<1, 0, EPI_STORE, float>(g, m0, n0, uniform(it.slice0), uniform(it.nk), C, smem);
}

