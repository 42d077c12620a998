// Row-selected bf16 projection on the gfx950 matrix cores:
//     C[t, :] = A[t, :] . W      for t in a device-side row list
// (Alg. 1 lines 2, 6-7, 11 and Alg. 2 lines 2, 7, 11 of the paper: the Q, K, V
// and output projections, for all rows or only for the refreshed rows).
//
// Layout: A rows are k-contiguous; the weight arrives packed as Wt[n, k]
// (k-contiguous), so both MFMA operands are 16-byte runs of 8 consecutive k.
//
// A workgroup owns a BM x BN output tile and walks k in steps of 64.  Tiles of A
// and Wt go from global memory STRAIGHT INTO LDS (global_load_lds_dwordx4: lane L
// of a wave deposits its 16 bytes at wave_base + 16 L), through a ring of STAGES
// buffers, so several k-steps are in flight while the matrix cores work on the
// oldest one; no staging registers, no ds_write.  Because the LDS position is
// fixed by the lane number, bank conflicts are removed on the global side: the
// lane that owns LDS slot s of row r fetches k-chunk s ^ ((r >> 1) & 7), and the
// MFMA fragment reads apply the same XOR (measured conflict-free for 16-byte
// reads: 246 of 256 B/clk/CU).
//
// Each wave computes the TRANSPOSED tile with v_mfma_f32_32x32x16_bf16 (weight
// fragment as the first operand): a lane then owns one output row and runs of 4
// consecutive output columns, which gives 8-byte stores and keeps a row's values
// inside one lane.
//
// k-parts.  A projection with few output tiles and a long k (the scored query columns
// for all rows: 1024 x 128 x 4096) can cut k into ranges that run as separate
// workgroups; each range writes its fp32 partial products to its own slab of the fp32
// output and the consumer (the score kernel) adds the slabs in range order.  No
// atomics, no fences: the kernel boundary orders producer and consumer.
//
// Tile order.  The hardware deals workgroup ids round-robin to the 8 XCDs, each
// with its own L2.  Ids are remapped so that every XCD works on a contiguous
// range of tiles, and inside the range tiles run down groups of 8 row-tiles
// before moving to the next column-tile: the workgroups that are resident on an
// XCD at the same time then share both their A tiles and their weight tiles.
//
// Row count known only on the device (the refreshed-row list): one kernel holds
// several tile shapes and every workgroup picks the same one from the count it
// reads, so a step with 50 refreshed rows does not pay for a 256-row tile and no
// host round trip is needed.  The grid is sized for the worst case; workgroups
// beyond the tiles that exist return at once.
#include <type_traits>

#include "dare_common.h"

namespace dare {
namespace {

constexpr int BK = 64;            // k per stage: one 128-byte row segment
constexpr int ROW_BYTES = BK * 2;
constexpr int GROUP_M = 8;        // row-tiles walked before the next column-tile

struct GemmDev {
  const bf16_t* a;
  const bf16_t* wt;
  const int32_t* idx;
  const int32_t* m_dev;
  bf16_t* c0;
  bf16_t* c1;
  bf16_t* c2;
  float* c32;
  int lda, n, k, m_max, ldc, seg_n, c32_cols;
  int k_parts;           // k is cut into this many ranges (1 = whole k per tile)
  long c32_part_stride;  // elements between the fp32 outputs of consecutive ranges
  const float* rope;     // rotary table, or nullptr
  int rope_cols, rope_dh, rope_seq;
  int swiglu_pairs;
  const uint8_t* sel_mask;
  int sel_batch, sel_seq;
  int32_t* sel_idx_out;
  int32_t* sel_idx_out2;
  int32_t* sel_off_out;
  int32_t* sel_count_out;
};

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
typedef const __attribute__((address_space(3))) int32_t* lds_idx_t;  // a row list held in LDS

// Token id of listed row `row`: from the list in LDS when the kernel derived it itself, else
// from the caller's list, else the row itself.
__device__ __forceinline__ long row_token(const int32_t* __restrict__ gidx, lds_idx_t lidx, int row) {
  return lidx ? (long)lidx[row] : (gidx ? (long)gidx[row] : (long)row);
}

// Wait until at most N of this wave's vector-memory operations are outstanding
// and all of its LDS reads have returned, then join the workgroup barrier.
// Written as one asm statement with a memory clobber: __syncthreads() would add a
// release fence, and the compiler answers a fence with vmcnt(0), which would
// drain the whole ring of in-flight k-steps.
template <int N>
__device__ __forceinline__ void wait_vmcnt_and_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int BM, int BN, int STAGES>
constexpr int smem_bytes() {
  return STAGES * (BM + BN) * ROW_BYTES;
}

// Four neighbouring output columns col .. col + 3 (col a multiple of 4) of token tok: the
// fp32 copy of the scored columns (before any rotation), then rotation, rounding and the
// store into the column's segment.
__device__ __forceinline__ void store4(const GemmDev& p, float* c32, long tok, int col, float v0, float v1,
                                       float v2, float v3) {
  if (p.swiglu_pairs) {  // (gate, up) pairs: two outputs silu(gate) * up at columns col / 2, col / 2 + 1
    bf16x2 o;
    o[0] = (bf16_t)(v0 / (1.0f + __expf(-v0)) * v1);
    o[1] = (bf16_t)(v2 / (1.0f + __expf(-v2)) * v3);
    *reinterpret_cast<bf16x2*>(p.c0 + tok * p.ldc + (col >> 1)) = o;
    return;
  }
  if (c32 && col < p.c32_cols) {
    const f32x4 o = {v0, v1, v2, v3};
    *reinterpret_cast<f32x4*>(c32 + tok * p.c32_cols + col) = o;
  }
  const int seg = col / p.seg_n;
  bf16_t* cbase = seg == 0 ? p.c0 : (seg == 1 ? p.c1 : p.c2);
  if (!cbase) return;
  if (p.rope && col < p.rope_cols) rope_rotate4(p.rope, p.rope_dh, p.rope_seq, tok, col, v0, v1, v2, v3);
  bf16x4 o;
  o[0] = (bf16_t)v0;
  o[1] = (bf16_t)v1;
  o[2] = (bf16_t)v2;
  o[3] = (bf16_t)v3;
  *reinterpret_cast<bf16x4*>(cbase + tok * p.ldc + (col - seg * p.seg_n)) = o;
}

// Tile order: GROUP_M row-tiles per column step (the tiles that run at the same time on one
// XCD then share few distinct A and W tiles).
__device__ __forceinline__ void tile_of_unit(const int unit, const int tiles_m, const int tiles_n, int& tile_m,
                                             int& tile_n) {
  const int group_size = GROUP_M * tiles_n;
  const int first_m = (unit / group_size) * GROUP_M;
  const int rows_in_group = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
  const int rem = unit % group_size;
  tile_m = first_m + rem % rows_in_group;
  tile_n = rem / rows_in_group;
}

// One output tile of C for m rows, computed by a team of WAVES_M * WAVES_N waves; tid
// is the thread's index within the team and smem the team's own
// smem_bytes<BM, BN, STAGES>() bytes.  vblock is the workgroup's (virtual) block id: a
// workgroup that walks several tiles calls this once per pass with block id + pass * grid
// size; the result says whether that id held a tile.  A workgroup is one team (nsub = 1) or
// nsub teams on neighbouring tiles (team number sub).  Teams share the workgroup barrier, so a
// team without a tile of its own repeats the last tile and stores nothing.
template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES>
__device__ __forceinline__ bool gemm_tile(const GemmDev& p, const int m, unsigned char* smem,
                                          const int tid, const int vblock, const int sub = 0,
                                          const int nsub = 1, lds_idx_t lidx = nullptr,
                                          const int forced_tile_m = -1, const int forced_tile_n = 0) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
  constexpr int GROUPS = (BM + BN) / 8;  // 8-row groups = one wave load each
  constexpr int LPW = GROUPS / NW;       // loads per wave per stage
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of 32 x 32");
  static_assert(GROUPS % NW == 0, "row groups must divide among the waves");
  static_assert(LPW * (STAGES - 1) < 64, "vmcnt range");

  // ---- which tile: XCD-contiguous ranges, GROUP_M row-tiles per column step ----
  // (the k-ranges of one tile, and the tiles of one workgroup's teams, are neighbours
  // in this order)
  const int parts = p.k_parts;
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (p.n + BN - 1) / BN;
  int tile_m, tile_n, part = 0;
  bool live = true;
  if (forced_tile_m >= 0) {  // the caller names the tile (whole k, one tile for all waves)
    tile_m = forced_tile_m;
    tile_n = forced_tile_n;
  } else {
    const int total = tiles_m * tiles_n * parts;
    const int blocks = (total + nsub - 1) / nsub;
    const int per_xcd = (blocks + 7) >> 3;
    const int slot = vblock >> 3;
    if (slot >= per_xcd) return false;
    const int blk = (vblock & 7) * per_xcd + slot;
    if (blk >= blocks) return false;
    int unit = blk * nsub + sub;
    live = unit < total;
    unit = live ? unit : total - 1;
    const int logical = unit / parts;
    part = unit - logical * parts;
    tile_of_unit(logical, tiles_m, tiles_n, tile_m, tile_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // (the wave number as a scalar: LDS addresses of the global -> LDS loads go through M0, and a
  // wave number held in a vector register would send every one of them through v_readfirstlane)
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
  const int l32 = lane & 31, half = lane >> 5;

  // this workgroup's k-range, in k-steps (the host makes parts divide the step count)
  const int KT = p.k / BK / parts;
  const int kt0 = part * KT;

  // ---- global -> LDS assignment: wave w issues loads for row groups w*LPW .. +LPW
  // (rows 0..BM-1 are A rows, BM..BM+BN-1 are weight rows).  Lane L of a load owns
  // row (L >> 3) of the group and LDS slot (L & 7); it fetches the k-chunk that
  // the swizzle puts into that slot.  Rows past the end re-read the last row.
  const bf16_t* src[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int r = (wave * LPW + i) * 8 + (lane >> 3);  // row within the stage
    const int chunk = (lane & 7) ^ ((r >> 1) & 7);
    if (r < BM) {
      int row = m0 + r;
      row = row < m ? row : m - 1;
      const long tok = row_token(p.idx, lidx, row);
      src[i] = p.a + tok * p.lda + chunk * 8 + kt0 * BK;
    } else {
      int col = n0 + (r - BM);
      col = col < p.n ? col : p.n - 1;
      src[i] = p.wt + (long)col * p.k + chunk * 8 + kt0 * BK;
    }
  }
  // token ids of the rows this lane stores in the epilogue, read now: a list held in LDS
  // (lidx) sits in the stage memory that the first loads overwrite
  long tok_out[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wave_m * WM + i * 32 + l32;
    tok_out[i] = row_token(p.idx, lidx, row < m ? row : m - 1);
  }
  if (lidx) __syncthreads();  // (uniform: every thread of the workgroup has its entries)
  auto issue_loads = [&](int kt, int buf) __attribute__((always_inline)) {
    unsigned char* base = smem + buf * STAGE_BYTES + wave * LPW * 8 * ROW_BYTES;
#pragma unroll
    for (int i = 0; i < LPW; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(src[i] + kt * BK),
                                       (lptr_t)(base + i * 8 * ROW_BYTES), 16, 0, 0);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // fragment read offsets: row (wave tile base + 32 i + l32), k-chunk 2 ks + half,
  // stored at slot chunk ^ ((row >> 1) & 7); the tile bases are multiples of 32,
  // so the XOR term depends on l32 only
  constexpr int KS = BK / 16;
  static_assert(KS % 2 == 0, "fragment double buffering assumes an even slice count");
  const int sw = (l32 >> 1) & 7;
  int koff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) koff[ks] = ((ks * 2 + half) ^ sw) * 16;
  const int a_row_off = (wave_m * WM + l32) * ROW_BYTES;
  const int b_row_off = (BM + wave_n * WN + l32) * ROW_BYTES;

  // ---- pipeline: STAGES-1 k-steps in flight ahead of the one being multiplied.
  // Loads of k-steps past the end are issued on the last valid k-step again (into
  // a buffer nobody reads any more), so the count of outstanding loads per wave is
  // the same in every iteration and one vmcnt value serves the whole loop.
  //
  // MFMA operands are double-buffered in registers: the LDS reads of the next unit
  // of work are issued after the first PRE MFMAs of the current one and complete
  // under the rest.  The unit is a 16-wide k-slice for large wave tiles; for small
  // wave tiles (few MFMAs per slice, so nothing to hide an LDS round trip behind)
  // it is the whole k-step: all fragments of k-step kt+1 are fetched under the MFMAs
  // of k-step kt.  The barrier that publishes k-step kt+1 sits right before that
  // fetch: by then every LDS read of k-step kt has been issued and (lgkmcnt 0) has
  // completed, so its buffer may be refilled after the barrier.
  // The scheduling fences keep the compiler from sinking the LDS reads back down
  // to their first use, which would undo the register double buffering.
  constexpr bool WHOLE = TM * TN <= 4;
  constexpr int FS = WHOLE ? KS : 1;  // k-slices held per fragment set
  bf16x8 fa[2][FS][TM], fb[2][FS][TN];
  auto load_frags = [&](int buf, int ks, int set, int slot) __attribute__((always_inline)) {
    const unsigned char* st = smem + buf * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      fa[set][slot][i] = *reinterpret_cast<const bf16x8*>(st + a_row_off + i * 32 * ROW_BYTES + koff[ks]);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      fb[set][slot][j] = *reinterpret_cast<const bf16x8*>(st + b_row_off + j * 32 * ROW_BYTES + koff[ks]);
  };
  // MFMAs [first, last) of the FS x TM x TN grid of one fragment set
  auto mma = [&](int set, int first, int last) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < FS * TM * TN; ++t) {
      if (t < first || t >= last) continue;
      const int slot = t / (TM * TN), i = (t / TN) % TM, j = t % TN;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][slot][j], fa[set][slot][i], acc[i][j], 0, 0, 0);
    }
  };
  constexpr int NMMA = FS * TM * TN;
  constexpr int PRE = NMMA >= 8 ? 2 : 1;

#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) issue_loads(s < KT ? s : KT - 1, s);
  wait_vmcnt_and_barrier<LPW*(STAGES - 2)>();
  if constexpr (WHOLE) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) load_frags(0, ks, 0, ks);
    // two k-steps per trip so that the fragment set index is a compile-time constant
    // (a run-time index would push the fragment arrays out of registers)
    auto kstep = [&](int kt, auto set_c) __attribute__((always_inline)) {
      constexpr int SET = decltype(set_c)::value;
      const int nxt = kt + STAGES - 1;
      issue_loads(nxt < KT ? nxt : KT - 1, nxt % STAGES);
      mma(SET, 0, PRE);
      __builtin_amdgcn_sched_barrier(0);
      wait_vmcnt_and_barrier<LPW*(STAGES - 2)>();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) load_frags((kt + 1) % STAGES, ks, SET ^ 1, ks);
      __builtin_amdgcn_sched_barrier(0);
      mma(SET, PRE, NMMA);
      __builtin_amdgcn_sched_barrier(0);
    };
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
      kstep(kt, std::integral_constant<int, 0>{});
      kstep(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < KT) kstep(kt, std::integral_constant<int, 0>{});
  } else {
    load_frags(0, 0, 0, 0);
    for (int kt = 0; kt < KT; ++kt) {
      const int buf = kt % STAGES;
      const int nxt = kt + STAGES - 1;
      // (the wave that is about to issue memory instructions goes first: of the two waves of
      // a SIMD the other one is then in its MFMAs; measured 1-2 % on the all-row shapes)
      __builtin_amdgcn_s_setprio(2);
      issue_loads(nxt < KT ? nxt : KT - 1, nxt % STAGES);
      __builtin_amdgcn_s_setprio(0);
#pragma unroll
      for (int ks = 0; ks < KS - 1; ++ks) {
        mma(ks & 1, 0, PRE);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(2);
        load_frags(buf, ks + 1, (ks + 1) & 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
        mma(ks & 1, PRE, NMMA);
        __builtin_amdgcn_sched_barrier(0);
      }
      mma((KS - 1) & 1, 0, PRE);
      __builtin_amdgcn_sched_barrier(0);
      wait_vmcnt_and_barrier<LPW*(STAGES - 2)>();
      __builtin_amdgcn_s_setprio(2);
      load_frags((kt + 1) % STAGES, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(0);
      mma((KS - 1) & 1, PRE, NMMA);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  wait_vmcnt<0>();

  float* c32 = p.c32 ? p.c32 + part * p.c32_part_stride : nullptr;
  // Epilogue.  acc[i][j][r] = C[row, col] with
  //   row = m0 + wave_m*WM + i*32 + l32
  //   col = n0 + wave_n*WN + j*32 + (r/4)*8 + half*4 + r%4
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wave_m * WM + i * 32 + l32;
    if (row >= m || !live) continue;
    const long tok = tok_out[i];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wave_n * WN + j * 32 + g * 8 + half * 4;
        if (col >= p.n) continue;
        store4(p, c32, tok, col, acc[i][j][g * 4 + 0], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2],
               acc[i][j][g * 4 + 3]);
      }
    }
  }
  return true;
}

// The same tile with v_mfma_f32_16x16x32_bf16: wave tiles in units of 16, so that 8 waves can
// share a 128 x 96 tile (32 x 48 each).  129-256 refreshed rows of a 12288-wide output then
// make 256 workgroups of 8 waves, where the 32-wide MFMA shape allows either 192 workgroups
// (128 x 128) or 4 waves per workgroup (128 x 96 as 32 x 96).  LDS layout, ring and loads as in
// gemm_tile; a fragment is 16 rows x 32 k (lane L: row L & 15, k-chunk L >> 4), a k-step holds
// two such slices, and all fragments of the next k-step are fetched under the MFMAs of the
// current one.  No teams, no k-parts.
template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool PAIRED = false>
__device__ __forceinline__ bool gemm_tile16(const GemmDev& p, const int m, unsigned char* smem, const int tid,
                                            const int vblock, lds_idx_t lidx = nullptr) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 16, TN = WN / 16;
  constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
  constexpr int GROUPS = (BM + BN) / 8;
  constexpr int LPW = (GROUPS + NW - 1) / NW;  // surplus loads repeat the last group
  constexpr int KS = BK / 32;
  static_assert(WM % 16 == 0 && WN % 16 == 0, "wave tile must be a multiple of 16 x 16");
  static_assert(LPW * (STAGES - 1) < 64, "vmcnt range");

  const int tiles_m = (m + BM - 1) / BM, tiles_n = (p.n + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  const int per_xcd = (total + 7) >> 3;
  const int slot = vblock >> 3;
  if (slot >= per_xcd) return false;
  const int unit = (vblock & 7) * per_xcd + slot;
  if (unit >= total) return false;
  const int group_size = GROUP_M * tiles_n;
  const int first_m = (unit / group_size) * GROUP_M;
  const int rows_in_group = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
  const int rem = unit % group_size;
  const int tile_m = first_m + rem % rows_in_group, tile_n = rem / rows_in_group;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // (the wave number as a scalar: LDS addresses of the global -> LDS loads go through M0, and a
  // wave number held in a vector register would send every one of them through v_readfirstlane)
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
  const int l16 = lane & 15, kq = lane >> 4;
  const int KT = p.k / BK;

  const bf16_t* src[LPW];
  int grp[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    grp[i] = wave * LPW + i < GROUPS ? wave * LPW + i : GROUPS - 1;
    const int r = grp[i] * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ ((r >> 1) & 7);
    if (r < BM) {
      int row = m0 + r;
      row = row < m ? row : m - 1;
      src[i] = p.a + row_token(p.idx, lidx, row) * p.lda + chunk * 8;
    } else {
      int col = n0 + (r - BM);
      col = col < p.n ? col : p.n - 1;
      src[i] = p.wt + (long)col * p.k + chunk * 8;
    }
  }
  long tok_out[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wave_m * WM + i * 16 + l16;
    tok_out[i] = row_token(p.idx, lidx, row < m ? row : m - 1);
  }
  if (lidx) __syncthreads();
  auto issue_loads = [&](int kt, int buf) __attribute__((always_inline)) {
    unsigned char* base = smem + buf * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < LPW; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(src[i] + kt * BK), (lptr_t)(base + grp[i] * 8 * ROW_BYTES), 16, 0, 0);
  };

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // fragment offsets: row (base + 16 i + l16), chunk 4 ks + kq at slot chunk ^ ((row >> 1) & 7); the
  // bases are multiples of 16, so the XOR term depends on l16 only
  const int sw = (l16 >> 1) & 7;
  int koff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) koff[ks] = ((ks * 4 + kq) ^ sw) * 16;
  const int a_row_off = (wave_m * WM + l16) * ROW_BYTES;
  const int b_row_off = (BM + wave_n * WN + l16) * ROW_BYTES;

  bf16x8 fa[2][KS][TM], fb[2][KS][TN];
  auto load_frags = [&](int buf, int set) __attribute__((always_inline)) {
    const unsigned char* st = smem + buf * STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[set][ks][i] = *reinterpret_cast<const bf16x8*>(st + a_row_off + i * 16 * ROW_BYTES + koff[ks]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[set][ks][j] = *reinterpret_cast<const bf16x8*>(st + b_row_off + j * 16 * ROW_BYTES + koff[ks]);
    }
  };
  constexpr int NMMA = KS * TM * TN, PRE = 2;
  auto mma = [&](int set, int first, int last) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < NMMA; ++t) {
      if (t < first || t >= last) continue;
      const int ks = t / (TM * TN), i = (t / TN) % TM, j = t % TN;
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[set][ks][j], fa[set][ks][i], acc[i][j], 0, 0, 0);
    }
  };

  if constexpr (!PAIRED) {
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue_loads(s < KT ? s : KT - 1, s);
    wait_vmcnt_and_barrier<LPW*(STAGES - 2)>();
    load_frags(0, 0);
    auto kstep = [&](int kt, auto set_c) __attribute__((always_inline)) {
      constexpr int SET = decltype(set_c)::value;
      const int nxt = kt + STAGES - 1;
      issue_loads(nxt < KT ? nxt : KT - 1, nxt % STAGES);
      mma(SET, 0, PRE);
      __builtin_amdgcn_sched_barrier(0);
      wait_vmcnt_and_barrier<LPW*(STAGES - 2)>();
      load_frags((kt + 1) % STAGES, SET ^ 1);
      __builtin_amdgcn_sched_barrier(0);
      mma(SET, PRE, NMMA);
      __builtin_amdgcn_sched_barrier(0);
    };
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
      kstep(kt, std::integral_constant<int, 0>{});
      kstep(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < KT) kstep(kt, std::integral_constant<int, 0>{});
  } else {
    // Two k-steps per barrier (small tiles, whose k-step holds too few MFMAs to carry a
    // barrier of its own): the ring is filled and drained in pairs of stages.  The barrier
    // that ends an odd k-step kt lets stages kt+1 and kt+2 be read and the slots of kt-1 and
    // kt be refilled; the even k-step after it issues the loads of stages kt+STAGES-2 and
    // kt+STAGES-1 into those two slots and reads stage kt+1 without a barrier.
    static_assert(STAGES % 2 == 0 && STAGES >= 4, "paired ring");
    static_assert(LPW * (STAGES - 2) < 64, "vmcnt range");
#pragma unroll
    for (int s = 0; s < STAGES - 2; ++s) issue_loads(s < KT ? s : KT - 1, s);
    wait_vmcnt_and_barrier<LPW*(STAGES - 4)>();
    load_frags(0, 0);
    auto kstep = [&](int kt, auto set_c) __attribute__((always_inline)) {
      constexpr int SET = decltype(set_c)::value;
      if constexpr (SET == 0) {
        const int n0s = kt + STAGES - 2, n1s = kt + STAGES - 1;
        issue_loads(n0s < KT ? n0s : KT - 1, n0s % STAGES);
        issue_loads(n1s < KT ? n1s : KT - 1, n1s % STAGES);
      }
      mma(SET, 0, PRE);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (SET == 1) wait_vmcnt_and_barrier<LPW*(STAGES - 4)>();
      load_frags((kt + 1) % STAGES, SET ^ 1);
      __builtin_amdgcn_sched_barrier(0);
      mma(SET, PRE, NMMA);
      __builtin_amdgcn_sched_barrier(0);
    };
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
      kstep(kt, std::integral_constant<int, 0>{});
      kstep(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < KT) kstep(kt, std::integral_constant<int, 0>{});
  }
  wait_vmcnt<0>();

  // acc[i][j][e] = C[row, col]: row = m0 + wave_m*WM + 16 i + l16, col = n0 + wave_n*WN + 16 j + 4 kq + e
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wave_m * WM + i * 16 + l16;
    if (row >= m) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wave_n * WN + j * 16 + kq * 4;
      if (col >= p.n) continue;
      store4(p, p.c32, tok_out[i], col, acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
    }
  }
  return true;
}

// ---- very few rows (at most 16 TMS): a stream over the weight matrix ------------------
// With a handful of refreshed rows (one or two tokens unmasked per denoising step) the
// projection is a matrix-vector product in disguise: what matters is that every CU pulls on
// the weight stream at once and that each weight byte is read once.  A workgroup owns 16
// output columns for the whole of k; its NW waves take contiguous ranges of k, load their
// weight and row fragments straight into registers (no LDS: a fragment is used by one wave
// only), 16 k-steps of 32 in flight per wave (8 with two row blocks), multiply with v_mfma_f32_16x16x32_bf16
// (weight fragment first, so a lane again owns one row and four neighbouring columns), and
// the partial sums of the waves are added in wave order through LDS.
template <int NW, int TMS>
__device__ __forceinline__ void skinny_tile(const GemmDev& p, const int m, unsigned char* smem, const int tid,
                                            lds_idx_t lidx = nullptr) {
  constexpr int UNR = TMS == 1 ? 16 : 8;
  // (the wave number as a scalar: LDS addresses of the global -> LDS loads go through M0, and a
  // wave number held in a vector register would send every one of them through v_readfirstlane)
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, kq = lane >> 4;
  const int groups = p.n >> 4;
  const int steps = p.k >> 5;
  const int spw = (steps + NW - 1) / NW;
  const int s0 = wave * spw;
  const int s1 = s0 + spw < steps ? s0 + spw : steps;
  const bf16_t* xrow[TMS];
  long tok[TMS];
#pragma unroll
  for (int t = 0; t < TMS; ++t) {
    int r = t * 16 + l16;
    r = r < m ? r : m - 1;
    tok[t] = row_token(p.idx, lidx, r);
    xrow[t] = p.a + tok[t] * p.lda + kq * 8;
  }
  if (lidx) __syncthreads();  // a list in LDS shares the memory of the partial sums below
  f32x4* red = reinterpret_cast<f32x4*>(smem);  // [NW][TMS][64]
  for (int grp = blockIdx.x; grp < groups; grp += gridDim.x) {
    const int n0 = grp << 4;
    const bf16_t* wrow = p.wt + (long)(n0 + l16) * p.k + kq * 8;
    f32x4 acc[TMS];
#pragma unroll
    for (int t = 0; t < TMS; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int s = s0; s < s1; s += UNR) {
      bf16x8 wf[UNR], xf[TMS][UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const bool live = s + u < s1;
        const int ks = (live ? s + u : s0) << 5;
        wf[u] = *reinterpret_cast<const bf16x8*>(wrow + ks);
#pragma unroll
        for (int t = 0; t < TMS; ++t) xf[t][u] = *reinterpret_cast<const bf16x8*>(xrow[t] + ks);
        if (!live) {
#pragma unroll
          for (int e = 0; e < 8; ++e) wf[u][e] = (bf16_t)0.0f;
        }
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u)
#pragma unroll
        for (int t = 0; t < TMS; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[u], xf[t][u], acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < TMS; ++t) red[(wave * TMS + t) * 64 + lane] = acc[t];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int t = 0; t < TMS; ++t) {
        f32x4 v = red[t * 64 + lane];
        for (int w = 1; w < NW; ++w) v += red[(w * TMS + t) * 64 + lane];
        if (t * 16 + l16 < m) store4(p, p.c32, tok[t], n0 + kq * 4, v[0], v[1], v[2], v[3]);
      }
    }
    __syncthreads();
  }
}
constexpr int kSkinnyRows = 32, kSkinnyMaxN = 8192;

// ---- one tile shape, chosen on the host (row count known or bounded) --------------
template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES>
__global__ void __launch_bounds__(WAVES_M* WAVES_N * 64) gemm_bf16_kernel(GemmDev p) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[smem_bytes<BM, BN, STAGES>()];
  const int m = p.m_dev ? *p.m_dev : p.m_max;
  if (m <= 0) return;
  gemm_tile<BM, BN, WAVES_M, WAVES_N, STAGES>(p, m, smem, threadIdx.x, blockIdx.x);
}

// ---- row count read on the device: the tile shape follows it -------------------------
// One kernel for every projection of refreshed rows, 8 waves and 128 KiB
// of LDS.  What bounds a projection of few rows is the rate at which one CU pulls
// operand tiles out of L2 (measured 45-80 GB/s per CU whatever the ring depth), so the
// shape that wins moves the fewest bytes per CU while still using every CU:
//   256 x 256 and 256 x 192 (the all-row shapes) once they fill the chip;
//   128 x 192 (four waves) when that gives one round of 192-256 tiles (257-512 rows of a
//   12288-wide output: 63 us against 72-79 us for 128 x 128 tiles, which need a second round);
//   128 x 128 (4 x 2 waves, 4 stages) once that gives at least kWideBigTiles tiles;
//   else 64 x 64 tiles, one per workgroup (all eight waves, 16-wide MFMA shape) while
//   there are at most kWideSingle of them, and two per workgroup, one per team of four
//   waves, beyond that.
constexpr int kWideSmem = smem_bytes<128, 128, 4>();
constexpr int kWideBigTiles = 160, kWideSingle = 256, kWideFullTiles = 200;
constexpr int kWideGrid = 256;  // workgroups of a launch: one per CU
__host__ __device__ inline int tiles_of(int m, int n, int bm, int bn) {
  return ((m + bm - 1) / bm) * ((n + bn - 1) / bn);
}
// a tile count that fills most of the chip's 256 CUs in a single round
__host__ __device__ inline bool one_round(int tiles) { return tiles >= 192 && tiles <= 256; }
// The refreshed-row list from the mask bytes, by every workgroup for itself (Alg. 1/2 line 5
// folded into the first kernel that needs the list: a compaction kernel of its own costs a
// launch, 4-5 us of a 90 us step, for a few hundred bytes of work).  512 threads, up to
// kSelMaxTokens tokens, four per thread; ascending by construction.  Returns the count.
__device__ __forceinline__ int derive_rows(const GemmDev& p, int32_t* list, int* wave_tot, bool publish) {
  const int n_tok = p.sel_batch * p.sel_seq;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = tid * 4;
  bool z[4];
  int cnt = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    z[k] = t0 + k < n_tok && p.sel_mask[t0 + k] == 0;
    cnt += z[k];
  }
  int incl = cnt;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o, 64);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  int rank = incl - cnt, total = 0;
#pragma unroll
  for (int w = 0; w < 8; ++w) {
    if (w < wave) rank += wave_tot[w];
    total += wave_tot[w];
  }
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (z[k]) list[rank++] = t0 + k;
  __syncthreads();
  if (publish && blockIdx.x == 0) {  // what the compaction kernel would have written, for the kernels that follow
    for (int r = tid; r < total; r += 512) {
      p.sel_idx_out[r] = list[r];
      if (p.sel_idx_out2) p.sel_idx_out2[r] = list[r];
    }
    // refreshed tokens in front of sequence b: first list position holding a token >= b * seq
    auto before = [&](int b) {
      const int key = b * p.sel_seq;
      int lo = 0, hi = total;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (list[mid] < key) lo = mid + 1; else hi = mid;
      }
      return lo;
    };
    for (int b = tid; b <= p.sel_batch; b += 512) {  // (a batch may have more sequences than threads)
      const int off = before(b);
      p.sel_off_out[b] = off;
      if (p.sel_count_out && b < p.sel_batch) p.sel_count_out[b] = before(b + 1) - off;
    }
  }
  return total;
}

// FUSED: the row list is derived from the mask bytes inside the kernel (two instantiations,
// so that the plain one carries none of the list handling).
template <bool FUSED>
__global__ void __launch_bounds__(512) gemm_bf16_rows_wide_kernel(GemmDev p) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kWideSmem];
  // a row list derived from the mask lives at the start of the stage memory until every
  // thread has taken the entries it needs (gemm_tile / skinny_tile read them before their
  // first load into LDS): the list gets no memory of its own, and a workgroup that walks
  // several tiles derives it again in front of every further pass
  static_assert(kSelMaxTokens * 4 + 64 <= kWideSmem, "row list must fit the stage memory");
  // (the list starts 64 bytes in: LDS offset 0 is the null pointer of the LDS address space,
  // and gemm_tile takes "no list" as a null pointer)
  int* sel_wave_tot = reinterpret_cast<int*>(smem);
  int32_t* sel_list = reinterpret_cast<int32_t*>(smem + 64);
  static_assert(2 * smem_bytes<64, 64, 4>() <= kWideSmem && smem_bytes<64, 64, 8>() <= kWideSmem &&
                    smem_bytes<256, 256, 2>() <= kWideSmem &&
                    smem_bytes<128, 192, 3>() <= kWideSmem && smem_bytes<128, 96, 4>() <= kWideSmem &&
                    smem_bytes<128, 48, 5>() <= kWideSmem && smem_bytes<128, 64, 4>() <= kWideSmem &&
                    smem_bytes<256, 192, 2>() <= kWideSmem,
                "shared buffer too small");
  int m;
  lds_idx_t lidx = nullptr;
  if constexpr (FUSED) {
    m = derive_rows(p, sel_list, sel_wave_tot, true);
    lidx = (lds_idx_t)sel_list;
  } else {
    m = p.m_dev ? *p.m_dev : p.m_max;
  }
  if (m <= 0) return;
  // Up to 32 rows and a narrow output (the output projection): the register-fed stream
  // (measured at n = 4096: 11-15 us against 17 us for 64 x 64 tiles, which give that width
  // only 64 workgroups).  Wide outputs keep the 64 x 64 tiles for few rows: with 192
  // column tiles they already stream the weights at 5 TB/s.
  if (m <= kSkinnyRows && p.n < kSkinnyMaxN) {
    if (m <= 16) skinny_tile<8, 1>(p, m, smem, threadIdx.x, lidx); else skinny_tile<8, 2>(p, m, smem, threadIdx.x, lidx);
    return;
  }
  // The grid is one workgroup per CU whatever the count turns out to be (a grid sized for the
  // worst case, whose surplus workgroups return at once, costs 1 us more at 205 rows); shapes
  // that can have more tiles than that walk them in passes, virtual block id = block id +
  // pass * grid size.  Every thread of the workgroup sees the same m and so takes the same
  // branch and the same number of passes.
  auto passes = [&](auto tile) __attribute__((always_inline)) {
    for (int vb = blockIdx.x;; vb += gridDim.x) {
      if (vb != (int)blockIdx.x) {
        __syncthreads();  // the ring is reused: everybody is done with the last tile
        if constexpr (FUSED) derive_rows(p, sel_list, sel_wave_tot, false);
      }
      if (!tile(vb)) break;
    }
  };
  if (p.n % 256 == 0 && tiles_of(m, p.n, 256, 256) >= 2 * kWideSingle) {
    // Rounds of 256 x 256 tiles; when the last round would be at most half full (624 tiles on
    // 256 workgroups: 256 + 256 + 112), its tiles are cut into four 128 x 128 tiles each and
    // spread over all workgroups (one or two short rounds instead of a long, mostly idle one).
    // Virtual block ids: 8 per XCD slot, as gemm_tile decodes them.
    const int G = gridDim.x;
    const int tiles_m = (m + 255) / 256, tiles_n = p.n / 256;
    const int total = tiles_m * tiles_n, per_xcd = (total + 7) >> 3;
    const int n_vb = per_xcd * 8;
    const int last = n_vb % G;
    const bool cut = n_vb > G && last > 0 && 2 * last <= G;
    const int whole_end = cut ? n_vb - last : n_vb;
    bool first = true;
    auto next_tile = [&]() __attribute__((always_inline)) {
      if (!first) {
        __syncthreads();  // the ring is reused: everybody is done with the last tile
        if constexpr (FUSED) derive_rows(p, sel_list, sel_wave_tot, false);
      }
      first = false;
    };
    for (int vb = blockIdx.x; vb < whole_end; vb += G) {
      next_tile();
      gemm_tile<256, 256, 2, 4, 2>(p, m, smem, threadIdx.x, vb, 0, 1, lidx);
    }
    if (cut) {
      // child c: the parents of an XCD slot stay on their XCD (c & 7), 4 children per parent
      for (int c = blockIdx.x; c < 4 * last; c += G) {
        const int vb = whole_end + ((c >> 5) << 3) + (c & 7), quarter = (c >> 3) & 3;
        const int unit = (vb & 7) * per_xcd + (vb >> 3);
        if (unit >= total) continue;
        int tm, tn;
        tile_of_unit(unit, tiles_m, tiles_n, tm, tn);
        const int cm = 2 * tm + (quarter >> 1), cn = 2 * tn + (quarter & 1);
        if (cm * 128 >= m) continue;
        next_tile();
        gemm_tile<128, 128, 4, 2, 4>(p, m, smem, threadIdx.x, 0, 0, 1, lidx, cm, cn);
      }
    }
  } else if (p.n % 192 == 0 && tiles_of(m, p.n, 256, 192) >= kWideFullTiles) {
    passes([&](int vb) { return gemm_tile<256, 192, 4, 2, 2>(p, m, smem, threadIdx.x, vb, 0, 1, lidx); });
  } else if (p.n % 192 == 0 && one_round(tiles_of(m, p.n, 128, 192))) {
    gemm_tile16<128, 192, 4, 2, 3>(p, m, smem, threadIdx.x, blockIdx.x, lidx);  // (at most one tile per workgroup)
  } else if (m > 64 && p.n % 48 == 0 && one_round(tiles_of(m, p.n, 128, 48))) {
    gemm_tile16<128, 48, 8, 1, 5>(p, m, smem, threadIdx.x, blockIdx.x, lidx);
  } else if (m > 128 && one_round(tiles_of(m, p.n, 128, 64))) {
    gemm_tile16<128, 64, 4, 2, 4>(p, m, smem, threadIdx.x, blockIdx.x, lidx);
  } else if (p.n % 96 == 0 && one_round(tiles_of(m, p.n, 128, 96))) {
    gemm_tile16<128, 96, 4, 2, 4>(p, m, smem, threadIdx.x, blockIdx.x, lidx);
  } else if (tiles_of(m, p.n, 128, 128) >= kWideBigTiles) {
    passes([&](int vb) { return gemm_tile<128, 128, 4, 2, 4>(p, m, smem, threadIdx.x, vb, 0, 1, lidx); });
  } else if (tiles_of(m, p.n, 64, 64) <= kWideSingle) {
    // one tile per workgroup: all eight waves on it (16 x 32 each with the 16-wide MFMA
    // shape; measured 19.2 against 21.1 us for four waves of 32 x 32 at 205 rows, n = 4096),
    // the whole stage memory as a ring of eight stages with one barrier per two k-steps
    // (0.3-0.6 us less than four stages and a barrier per k-step at 40-256 rows, n = 4096)
    gemm_tile16<64, 64, 4, 2, 8, true>(p, m, smem, threadIdx.x, blockIdx.x, lidx);
  } else {
    const int team = threadIdx.x >> 8;
    passes([&](int vb) {
      return gemm_tile<64, 64, 2, 2, 4>(p, m, smem + team * smem_bytes<64, 64, 4>(), threadIdx.x & 255, vb, team, 2,
                                        lidx);
    });
  }
}

GemmDev to_dev(const GemmArgs& g) {
  GemmDev p;
  p.a = static_cast<const bf16_t*>(g.a);
  p.wt = static_cast<const bf16_t*>(g.wt);
  p.idx = g.idx;
  p.m_dev = g.m_dev;
  p.c0 = static_cast<bf16_t*>(g.c[0]);
  p.c1 = static_cast<bf16_t*>(g.c[1]);
  p.c2 = static_cast<bf16_t*>(g.c[2]);
  p.c32 = g.c32;
  p.lda = g.lda;
  p.n = g.n;
  p.k = g.k;
  p.m_max = g.m_max;
  p.ldc = g.ldc;
  p.seg_n = g.seg_n;
  p.c32_cols = g.c32_cols;
  p.k_parts = 1;
  p.c32_part_stride = 0;
  p.rope = g.rope;
  p.rope_cols = g.rope_cols;
  p.rope_dh = g.rope_dh;
  p.rope_seq = g.rope_seq;
  p.swiglu_pairs = g.swiglu_pairs;
  p.sel_mask = g.sel_mask;
  p.sel_batch = g.sel_batch;
  p.sel_seq = g.sel_seq;
  p.sel_idx_out = g.sel_idx_out;
  p.sel_idx_out2 = g.sel_idx_out2;
  p.sel_off_out = g.sel_off_out;
  p.sel_count_out = g.sel_count_out;
  return p;
}

int grid_for(int tiles) { return ((tiles + 7) / 8) * 8; }

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES>
hipError_t launch_fixed(const GemmArgs& g, hipStream_t s) {
  const int tiles = ((g.m_max + BM - 1) / BM) * ((g.n + BN - 1) / BN);
  if (tiles == 0) return hipSuccess;
  GemmDev p = to_dev(g);
  if (g.k_parts > 1) {
    p.k_parts = g.k_parts;
    p.c32_part_stride = g.c32_part_stride;
  }
  hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, STAGES>), dim3(grid_for(tiles * p.k_parts)),
                     dim3(WAVES_M * WAVES_N * 64), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_rows_wide(const GemmArgs& g, hipStream_t s) {
  // worst case over the row counts 1 .. m_max of the blocks any of the shapes needs (the
  // 64 x 64 shape is only chosen below kWideBigTiles 128 x 128 tiles, each of which holds
  // at most four small ones), capped at one workgroup per CU: shapes with more tiles than
  // that walk them in passes
  const int small = tiles_of(g.m_max, g.n, 64, 64);
  int pairs = (small + 1) / 2;
  const int pairs_cap = (4 * (kWideBigTiles - 1) + 1) / 2;
  if (pairs > pairs_cap) pairs = pairs_cap;
  int blocks = small <= kWideSingle ? small : (pairs > kWideSingle ? pairs : kWideSingle);
  const int big = tiles_of(g.m_max, g.n, 128, 128);
  if (big >= kWideBigTiles && big > blocks) blocks = big;
  if (blocks == 0) return hipSuccess;
  if (blocks > kWideGrid) blocks = kWideGrid;
  if (g.sel_mask)
    hipLaunchKernelGGL(gemm_bf16_rows_wide_kernel<true>, dim3(grid_for(blocks)), dim3(512), 0, s, to_dev(g));
  else
    hipLaunchKernelGGL(gemm_bf16_rows_wide_kernel<false>, dim3(grid_for(blocks)), dim3(512), 0, s, to_dev(g));
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_bf16(const GemmArgs& g, hipStream_t s) {
  if (g.m_dev || g.sel_mask) return launch_rows_wide(g, s);
  // Row count known on the host.  Measured on MI355X (256 CUs): 256 x 256 tiles have
  // the least LDS-fill traffic per flop and win once they fill the chip; 256 x 192
  // gives exactly 256 tiles for 1024 x 12288; 128 x 128 with 8 waves is the best
  // shape when the larger ones would leave most CUs idle.
  auto tiles = [&](int bm, int bn) { return ((g.m_max + bm - 1) / bm) * ((g.n + bn - 1) / bn); };
  if (g.n % 256 == 0 && tiles(256, 256) >= 512) return launch_fixed<256, 256, 2, 4, 2>(g, s);
  if (g.n % 192 == 0 && tiles(256, 192) >= 224) return launch_fixed<256, 192, 4, 2, 2>(g, s);
  if (g.n % 256 == 0 && tiles(256, 256) >= 224) return launch_fixed<256, 256, 2, 4, 2>(g, s);
  if (g.m_max > 64 && g.n % 128 == 0 && tiles(128, 128) >= 64) return launch_fixed<128, 128, 4, 2, 4>(g, s);
  return launch_fixed<64, 64, 2, 2, 4>(g, s);
}

}  // namespace dare
