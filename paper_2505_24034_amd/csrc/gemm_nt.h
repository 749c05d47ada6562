// gemm_nt.h -- the one MFMA main loop every contraction of the path runs on.
//
// C[m,n] = sum_k A[m,k] * B[n,k]   ("NT": both operands are K-contiguous), fp32 accumulate.
//   forward / recompute : A = W [V,d] tile       B = H rows (gathered)   K = d
//   dW = dz^T H         : A = dz^T [V,N]         B = H^T [d,N]           K = N
//   (fp32 only) dH      : A = dz [N,V]           B = W^T [d,V]           K = V
//
// gfx950 mapping
//   - one workgroup = 8 wavefronts (2 x 4) = one 256 x 256 output tile; a wavefront owns 128 x 64 of it as
//     8 x 4 blocks of v_mfma_f32_16x16x32_bf16 (128 fp32 accumulator registers per lane).  The 16x16x32 shape is
//     the one to use on this chip: in an MFMA-only loop it sustains 2.0 PFLOP/s where 32x32x16 sustains 1.75 --
//     the chip is power-limited and the smaller shape lets it clock higher.
//   - K advances in slabs of 128 bytes per row (64 bf16 / 32 fp32) = two k-steps of one MFMA depth.  A slab of
//     both operands is 64 KB of LDS; two slabs are resident (128 of the CU's 160 KB).
//   - slabs go HBM/L2 -> LDS with buffer loads that write LDS directly (16 bytes per lane, no VGPR staging).
//     The hardware puts lane i's 16 bytes at LDS base + 16 i, so the bank-conflict swizzle is applied on the
//     global side: physical 16-byte slot p of row r holds logical chunk p ^ ((r >> 1) & 7), which spreads the
//     16 rows that 16 lanes of a ds_read_b128 touch over all 64 LDS banks.
//   - the loop is software-pipelined by hand (see TileGemm::run): every ds_read_b128 and every slab load is
//     issued in the shadow of an MFMA, far ahead of its use, and scheduling fences pin that interleave.
//   - out-of-range rows and the K tail use the buffer descriptor's bounds check: such lanes read zeros.
//   - kernels are persistent (one workgroup per CU walks a list of tiles) and fetch the first slabs of their next
//     tile before the epilogue of the current one, so the epilogue's VALU work overlaps that latency.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace llamarl {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

constexpr int BM = 256;       // tile rows (A rows)
constexpr int BN = 256;       // tile cols (B rows)
constexpr int NTHREADS = 512;
constexpr int WAVES_N = 4;    // wave grid 2 (M) x 4 (N)
constexpr int MB = 8;         // 16 x 16 MFMA blocks per wave along M  (128 rows)
constexpr int NB = 4;         // ... along N                            (64 cols)
constexpr int WAVE_M = MB * 16;
constexpr int WAVE_N = NB * 16;
constexpr int SLAB_ROW_BYTES = 128;
constexpr int BLOCK_BYTES = 16 * SLAB_ROW_BYTES;                  // 16 slab rows: one MFMA block of an operand
constexpr int SLAB_A_BYTES = BM * SLAB_ROW_BYTES;                 // 32 KB
constexpr int STAGE_BYTES = (BM + BN) * SLAB_ROW_BYTES;           // 64 KB
constexpr int MAINLOOP_LDS_BYTES = 2 * STAGE_BYTES;               // 128 KB
constexpr uint32_t OOB_OFFSET = 0x80000000u;                      // beyond any descriptor range used here

struct BF16 {
  typedef uint16_t store_t;
  typedef bf16x8_t frag_t;
  static constexpr int EPC = 8;  // elements per 16-byte chunk
};
struct F32 {
  typedef float store_t;
  typedef f32x4_t frag_t;
  static constexpr int EPC = 4;
};

// A fragment is the 16 bytes a lane reads from its row: row = lane % 16 of the block, chunk = lane / 16 of the
// k-step.  bf16: that is the operand layout of the 16x16x32 MFMA (8 consecutive k per lane).
__device__ __forceinline__ void mma(const bf16x8_t& a, const bf16x8_t& b, f32x4_t& c) {
  c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// fp32: the 16x16x4 MFMA takes one float per lane (k = lane / 16); four of them consume the lane's chunk.  Which
// k lands in which MFMA does not matter as long as both operands agree, and they do.
__device__ __forceinline__ void mma(const f32x4_t& a, const f32x4_t& b, f32x4_t& c) {
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], c, 0, 0, 0);
}

__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Where the accumulator element (ib, jb, r) of this lane sits inside the 256 x 256 tile.
// MFMA 16x16 output layout: register r of lane l holds row 4 (l / 16) + r, column l % 16.
struct LanePos {
  int wm, wn, lane;
  __device__ __forceinline__ int row(int ib, int r) const { return wm * WAVE_M + ib * 16 + (lane >> 4) * 4 + r; }
  __device__ __forceinline__ int col(int jb) const { return wn * WAVE_N + jb * 16 + (lane & 15); }
  // Quad-interleaved columns (see tile_row_of): the lane's four column blocks hold NEIGHBOURING columns
  // col_quad() + jb, so 16 lanes own 64 consecutive columns of one row.
  __device__ __forceinline__ int col_quad() const { return wn * WAVE_N + 4 * (lane & 15); }
};

// Which row of an operand tile the loader puts into LDS row `r`.  A wave's 64 LDS rows of the column operand feed
// its four 16-column MFMA blocks (block jb = bits 5:4, MFMA column n = low 4 bits); with QUAD, block jb / column n
// is tile row 4 n + jb of those 64, so that acc[.][0..3] of a lane are four neighbouring output columns and an
// epilogue can store them as one unit.  Only the global side changes: LDS layout, swizzle and fragment reads stay.
template <bool QUAD>
__device__ __forceinline__ int tile_row_of(int r) {
  static_assert(NB == 4 && WAVE_N == 64, "the interleave covers exactly four column blocks");
  return QUAD ? ((r & ~63) | ((r & 15) << 2) | ((r >> 4) & 3)) : r;
}

// Persistent tile schedule.  The grid has one workgroup per CU (any size works); the hardware deals workgroups
// round-robin to the 8 XCDs, each with a private L2.  Tile ids are ordered so that 32 consecutive ones form a patch
// (group_m x 32/group_m tiles) that shares A and B panels; the workgroups of one XCD take one patch at a time, so
// those panels are shared in its L2, and the eight patches in flight on the chip are consecutive in id order, so
// they share panels through the Infinity Cache (against giving every XCD a contiguous eighth of the ids: -3.5 %
// step time, -6.5 % for the dH contraction whose two operands both stream from HBM).  tiles_m x tiles_n is the
// number of tiles that exist once the device-side active-row count is known.
struct TileSchedule {
  int tiles_m, tiles_n, group_m;
  int next_id, end_id, stride;
  // group_m_: rows of a patch.  The 32 workgroups of an XCD work on 32 consecutive ids = group_m x (32 / group_m)
  // tiles, which load group_m A panels and 32 / group_m B panels: a B panel is shared by group_m tiles, an A panel
  // by 32 / group_m.  Give the larger share to the operand that has to come from HBM.
  __device__ __forceinline__ void init(int tiles_m_, int tiles_n_, int group_m_ = 8) {
    tiles_m = tiles_m_;
    tiles_n = tiles_n_;
    group_m = group_m_;
    const int ntiles = tiles_m * tiles_n;
    const int bid = blockIdx.x, nblk = gridDim.x;
    const int xcd = bid & 7, local = bid >> 3;
    if ((nblk & 7) == 0) {
      // Patches dealt round-robin over the XCDs: in round k XCD x works on patch 8 k + x, so the eight patches in
      // flight are neighbours in id order and share operand panels through the Infinity Cache.
      const int per = nblk >> 3;                            // workgroups per XCD = tiles per patch
      next_id = xcd * per + local;
      stride = nblk;
      end_id = ntiles;
      return;
    }
    const int base = ntiles >> 3, rem = ntiles & 7;
    const int start = xcd * base + min(xcd, rem);
    end_id = start + base + (xcd < rem ? 1 : 0);
    next_id = start + local;
    stride = (nblk >> 3) + ((nblk & 7) > xcd ? 1 : 0);      // workgroups of this grid that sit on my XCD
  }
  __device__ __forceinline__ bool has_tile() const { return next_id < end_id; }
  __device__ __forceinline__ int take() {                   // id of the next tile; advance
    const int id = next_id;
    next_id += stride;
    return id;
  }
  __device__ __forceinline__ void coords(int id, int& tm, int& tn) const {
    const int per_group = group_m * tiles_n;
    const int g = id / per_group;
    const int first_m = g * group_m;
    const int gsize = min(tiles_m - first_m, group_m);
    const int in_g = id - g * per_group;
    tm = first_m + in_g % gsize;
    tn = in_g / gsize;
  }
};

__device__ __forceinline__ int swizzle(int row) { return (row >> 1) & 7; }

// One operand slab stream: 256 rows x 128 bytes per step; this thread moves four 16-byte chunks of it.
// Wave-instruction `it` of wave w fills rows (it*8 + w)*8 .. +7 of the slab; lane l takes row +l/8 and the
// physical 16-byte slot l%8.  Because it*64 rows is a multiple of 16, the swizzle (and so the logical chunk this
// lane fetches) is the same for all four instructions.
template <typename TT>
struct SlabLoader {
  // The buffer descriptor is rebuilt from these at every use; readfirstlane pins them to scalar registers, so
  // the compiler never has to guess that the descriptor is wave-uniform (a guess it loses across loops).
  uint32_t base_lo, base_hi, records;
  uint32_t voff[4];       // per-lane byte offset of (row, logical chunk) inside the panel at k = 0

  __device__ __forceinline__ void set_base(const void* base, uint32_t bytes) {
    const uint64_t p = reinterpret_cast<uint64_t>(base);
    base_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)p);
    base_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));
    records = (uint32_t)__builtin_amdgcn_readfirstlane((int)bytes);
  }
  __device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc() const {
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)base_hi << 32) | base_lo), 0,
                                             (int)records, 0x00020000);
  }

  __device__ __forceinline__ static int lane_chunk(int wave, int lane) {
    return (lane & 7) ^ swizzle(wave * 8 + (lane >> 3));
  }
  // base: first row of the tile; ld in elements; rows_valid <= 256 rows exist from base on.
  template <bool QUAD = false>
  __device__ __forceinline__ void init(const void* base, int64_t ld, int rows_valid, int wave, int lane) {
    const uint32_t row_bytes = (uint32_t)(ld * (int64_t)sizeof(typename TT::store_t));
    set_base(base, row_bytes * (uint32_t)rows_valid);
    const uint32_t c16 = (uint32_t)lane_chunk(wave, lane) * 16u;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = tile_row_of<QUAD>((it * 8 + wave) * 8 + (lane >> 3));
      voff[it] = (row < rows_valid) ? (uint32_t)row * row_bytes + c16 : OOB_OFFSET;
    }
  }
  // Gathered panel: tile row r is row rows[r] of the whole matrix `base` (total_rows rows, < 2^31 bytes).
  // Free with per-lane buffer offsets: this is how masked tokens are skipped without a packed copy of H.
  template <bool QUAD = false>
  __device__ __forceinline__ void init_gather(const void* base, int64_t ld, int64_t total_rows, const int32_t* rows,
                                              int rows_valid, int wave, int lane) {
    const uint32_t row_bytes = (uint32_t)(ld * (int64_t)sizeof(typename TT::store_t));
    set_base(base, (uint32_t)total_rows * row_bytes);
    const uint32_t c16 = (uint32_t)lane_chunk(wave, lane) * 16u;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = tile_row_of<QUAD>((it * 8 + wave) * 8 + (lane >> 3));
      voff[it] = (row < rows_valid) ? (uint32_t)rows[row] * row_bytes + c16 : OOB_OFFSET;
    }
  }
  // The four tile rows this lane fetches (one per wave-instruction), for callers that load the gather list
  // themselves -- in one batch, ahead of time -- and hand the result to init_gathered().
  template <bool QUAD = false>
  __device__ __forceinline__ static int lane_tile_row(int it, int wave, int lane) {
    return tile_row_of<QUAD>((it * 8 + wave) * 8 + (lane >> 3));
  }
  // grow[it] = row of the whole matrix that tile row lane_tile_row(it) maps to (any valid row where the tile row
  // is >= rows_valid: it is not fetched).
  template <bool QUAD = false>
  __device__ __forceinline__ void init_gathered(const void* base, int64_t ld, int64_t total_rows, const int (&grow)[4],
                                                int rows_valid, int wave, int lane) {
    const uint32_t row_bytes = (uint32_t)(ld * (int64_t)sizeof(typename TT::store_t));
    set_base(base, (uint32_t)total_rows * row_bytes);
    const uint32_t c16 = (uint32_t)lane_chunk(wave, lane) * 16u;
#pragma unroll
    for (int it = 0; it < 4; ++it)
      voff[it] = (lane_tile_row<QUAD>(it, wave, lane) < rows_valid) ? (uint32_t)grow[it] * row_bytes + c16 : OOB_OFFSET;
  }
  // k0: first k of the slab (elements); K: contraction length.  lds: start of this operand's slab in LDS.
  // tail: the slab may reach past K (only the last slab of a contraction whose K is not a multiple of the slab
  // depth): lanes whose chunk lies past K fetch nothing.
  __device__ __forceinline__ void issue_one(char* lds, int it, int k0, int K, int wave, int lane, bool tail) const {
    const int soff = k0 * (int)sizeof(typename TT::store_t);
    uint32_t v = voff[it];
    if (tail) v = (k0 + lane_chunk(wave, lane) * TT::EPC >= K) ? OOB_OFFSET : v;   // `tail` is a constant once inlined
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc(), (lds_void_ptr)(lds + (it * 8 + wave) * 8 * SLAB_ROW_BYTES), 16,
                                             (int)v, soff, 0, 0);
  }
  __device__ __forceinline__ void issue(char* lds, int k0, int K, int wave, int lane) const {
#pragma unroll
    for (int it = 0; it < 4; ++it) issue_one(lds, it, k0, K, wave, lane, true);
  }
};

__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

#define LLAMARL_FENCE() __builtin_amdgcn_sched_barrier(0)

// The loads of one K slab, issued one per MFMA slot after the barrier of a k-step.
template <typename TT>
struct SlabFetch {
  const SlabLoader<TT>* la;
  const SlabLoader<TT>* lb;
  char* dst;      // stage that receives the slab
  int k0, K, wave, lane;
};

// Column block of MFMA slot t: rows of blocks are walked alternately left-to-right and right-to-left, so the column
// operand stays the same across a row change (the row operand changes there).  The chip is power-limited under
// MFMA load and operand switching costs energy: this order measured 0.5 % faster on every contraction kernel than
// restarting each row at column block 0.
__device__ __forceinline__ constexpr int snake_col(int t) { return ((t >> 2) & 1) ? 3 - (t & 3) : (t & 3); }

// One k-step = one MFMA depth (two per slab): 32 slots, slot t runs block (ib, jb) = (t / 4, snake_col(t)).
//   a[8]   : the A fragments of this k-step, one register set each.  Block ib is done after slot 4 ib + 3 and its
//            registers take the NEXT k-step's fragment right away (slot 4 ib + 4): 28 slots ahead of its use.
//            a[7] of a k-step is read at its own slot 0.
//   bc, bn : B fragments of this / the next k-step (all four are used by every ib, so they are double-buffered).
//   BAR    : this is the last k-step of a slab that has a successor.  By slot 0 every read of the slab has been
//            issued, so the barrier can sit as early as slot TB = 8: it waits for this thread's share of the next
//            slab (vmcnt) and for its own reads (lgkmcnt), then the 24 MFMAs left run from registers while the
//            next slab's fragments are read and, with FETCH, the slab after that is requested (one load every
//            other slot from slot LS on, into the stage this barrier just freed).  LS = 11 for the logits kernels;
//            the store contraction (dW) asks two slots earlier, which measured 1 - 1.5 % faster for it at three of
//            four shapes and the same at the fourth, while the logits kernels lose 0.5 % with it at the longest
//            batch.  Slots of the same parity as the fragment reads (even) are 4 - 6 % slower.
//   NEXT   : there is a next k-step (pa_nxt / pb_nxt: lane's fragment address of its blocks 0).
//   LS     : a template parameter although only its value matters: every specialisation of this template must be
//            called from ONE function instantiation only -- the host pass of hipcc (ROCm 7.2) rejects a second
//            caller of the same specialisation ("substitution failure", no reason given; the device pass accepts it).
template <typename TT, bool BAR, bool NEXT, bool FETCH, int LS>
__device__ __forceinline__ void k_step(typename TT::frag_t (&a)[MB], const typename TT::frag_t (&bc)[NB],
                                       typename TT::frag_t (&bn)[NB], f32x4_t (&acc)[MB][NB], const char* pa_cur,
                                       const char* pa_nxt, const char* pb_nxt, const SlabFetch<TT>* sf) {
  typedef typename TT::frag_t frag_t;
  constexpr int TB = 8;
  static_assert(MB == 8 && NB == 4, "slot table written for an 8 x 4 wave tile");
#pragma unroll
  for (int t = 0; t < MB * NB; ++t) {
    const int ib = t >> 2, jb = snake_col(t);
    if (BAR && t == TB) {
      wait_vmcnt0();      // this thread's share of the next slab has landed in LDS
      __syncthreads();    // everyone's has, and everyone is done reading this slab
      LLAMARL_FENCE();
    }
    mma(a[ib], bc[jb], acc[ib][jb]);
    LLAMARL_FENCE();
    if (t == 0) {
      a[7] = *reinterpret_cast<const frag_t*>(pa_cur + 7 * BLOCK_BYTES);
      LLAMARL_FENCE();
    }
    if (NEXT) {
      if (t == TB) a[0] = *reinterpret_cast<const frag_t*>(pa_nxt);
      if (t == TB + 1) a[1] = *reinterpret_cast<const frag_t*>(pa_nxt + BLOCK_BYTES);
      if (t >= 12 && (t & 3) == 0) a[ib - 1] = *reinterpret_cast<const frag_t*>(pa_nxt + (ib - 1) * BLOCK_BYTES);
      if (t == 10) bn[0] = *reinterpret_cast<const frag_t*>(pb_nxt);
      if (t == 14) bn[1] = *reinterpret_cast<const frag_t*>(pb_nxt + BLOCK_BYTES);
      if (t == 18) bn[2] = *reinterpret_cast<const frag_t*>(pb_nxt + 2 * BLOCK_BYTES);
      if (t == 22) bn[3] = *reinterpret_cast<const frag_t*>(pb_nxt + 3 * BLOCK_BYTES);
      LLAMARL_FENCE();
    }
    if (FETCH && t >= LS && t <= LS + 14 && ((t - LS) & 1) == 0) {
      const int n = (t - LS) >> 1;
      if (n < 4) sf->la->issue_one(sf->dst, n, sf->k0, sf->K, sf->wave, sf->lane, true);
      else sf->lb->issue_one(sf->dst + SLAB_A_BYTES, n - 4, sf->k0, sf->K, sf->wave, sf->lane, true);
      LLAMARL_FENCE();
    }
  }
}

// The main loop, split in two so that a persistent workgroup can start fetching its NEXT tile before it runs the
// epilogue of the current one:
//   prefetch(): set up both operand streams of a tile and issue its first two K slabs.  Only legal once every
//               wave of the workgroup is done reading LDS (a __syncthreads() after the previous run()).
//   run():      the K loop.  Waves leave it at different times: __syncthreads() before reusing LDS.
// smem must hold MAINLOOP_LDS_BYTES.
//
// GATHER_B: the B panel is gathered -- B_tile is then the base of the whole matrix with b_total rows and
// tile row r is its row b_rows[r].  QUAD_B: output columns are quad-interleaved over the lane's four column blocks
// (tile_row_of); the epilogue must then take its columns from LanePos::col_quad().
template <typename TT, int LOAD_SLOT = 11>
struct TileGemm {
  typedef typename TT::frag_t frag_t;
  static constexpr int BK = 8 * TT::EPC;
  SlabLoader<TT> la, lb;
  int K;

  template <bool GATHER_B, bool QUAD_B = false>
  __device__ __forceinline__ void prefetch(const void* A_tile, int64_t lda, int rowsA, const void* B_tile, int64_t ldb,
                                           int rowsB, int64_t K_, char* smem, const int32_t* b_rows = nullptr,
                                           int64_t b_total = 0) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    K = (int)K_;
    la.init(A_tile, lda, rowsA, wave, lane);
    if constexpr (GATHER_B) lb.template init_gather<QUAD_B>(B_tile, ldb, b_total, b_rows, rowsB, wave, lane);
    else lb.template init<QUAD_B>(B_tile, ldb, rowsB, wave, lane);
    la.issue(smem, 0, K, wave, lane);
    lb.issue(smem + SLAB_A_BYTES, 0, K, wave, lane);
    if (K > BK) {
      la.issue(smem + STAGE_BYTES, BK, K, wave, lane);
      lb.issue(smem + STAGE_BYTES + SLAB_A_BYTES, BK, K, wave, lane);
    }
  }

  // as prefetch<true, QUAD_B>, with the gather list entries of this lane already in registers (SlabLoader::
  // init_gathered): no global load stands between the caller's barrier and the first slab request
  template <bool QUAD_B>
  __device__ __forceinline__ void prefetch_gathered(const void* A_tile, int64_t lda, int rowsA, const void* B_base,
                                                    int64_t ldb, int rowsB, int64_t K_, char* smem, const int (&grow)[4],
                                                    int64_t b_total) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    K = (int)K_;
    la.init(A_tile, lda, rowsA, wave, lane);
    lb.template init_gathered<QUAD_B>(B_base, ldb, b_total, grow, rowsB, wave, lane);
    la.issue(smem, 0, K, wave, lane);
    lb.issue(smem + SLAB_A_BYTES, 0, K, wave, lane);
    if (K > BK) {
      la.issue(smem + STAGE_BYTES, BK, K, wave, lane);
      lb.issue(smem + STAGE_BYTES + SLAB_A_BYTES, BK, K, wave, lane);
    }
  }

  __device__ __forceinline__ void run(char* smem, f32x4_t (&acc)[MB][NB]) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

    const int nk = (K + BK - 1) / BK;
    // per-lane read addresses of block 0: row = lane % 16, chunk 4 ks + lane / 16 of k-step ks, swizzled.  The
    // swizzle depends on the low four row bits only, so block ib is the same address + ib * BLOCK_BYTES.
    const int g = lane >> 4, l16 = lane & 15;
    const int sw = swizzle(l16);
    int a_addr[2], b_addr[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      a_addr[ks] = (wm * WAVE_M + l16) * SLAB_ROW_BYTES + (((4 * ks + g) ^ sw) * 16);
      b_addr[ks] = SLAB_A_BYTES + (wn * WAVE_N + l16) * SLAB_ROW_BYTES + (((4 * ks + g) ^ sw) * 16);
    }
    // Slabs 0 and 1 were issued by prefetch(); stores of a previous epilogue may sit between them and now in the
    // vmcnt queue, so wait for everything rather than count.
    wait_vmcnt0();
    __syncthreads();
    frag_t a[MB], b0[NB], b1[NB];
    a[0] = *reinterpret_cast<const frag_t*>(smem + a_addr[0]);
#pragma unroll
    for (int j = 0; j < NB; ++j) b0[j] = *reinterpret_cast<const frag_t*>(smem + b_addr[0] + j * BLOCK_BYTES);
#pragma unroll
    for (int i = 1; i < MB - 1; ++i) a[i] = *reinterpret_cast<const frag_t*>(smem + a_addr[0] + i * BLOCK_BYTES);

    // slabs 0 .. nk-3 fetch slab kt+2 after their barrier; slab nk-2 (nothing left to fetch) and the last slab
    // follow, written out one after the other (a branch inside one loop body makes the compiler copy accumulators)
    for (int kt = 0; kt < nk - 2; ++kt) {
      char* cur = smem + (kt & 1) * STAGE_BYTES;
      const char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      k_step<TT, false, true, false, LOAD_SLOT>(a, b0, b1, acc, cur + a_addr[0], cur + a_addr[1], cur + b_addr[1],
                                                nullptr);
      const SlabFetch<TT> sf{&la, &lb, cur, (kt + 2) * BK, K, wave, lane};
      k_step<TT, true, true, true, LOAD_SLOT>(a, b1, b0, acc, cur + a_addr[1], nxt + a_addr[0], nxt + b_addr[0],
                                              &sf);
    }
    if (nk >= 2) {
      const char* cur = smem + ((nk - 2) & 1) * STAGE_BYTES;
      const char* nxt = smem + ((nk - 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      k_step<TT, false, true, false, LOAD_SLOT>(a, b0, b1, acc, cur + a_addr[0], cur + a_addr[1], cur + b_addr[1],
                                                nullptr);
      k_step<TT, true, true, false, LOAD_SLOT>(a, b1, b0, acc, cur + a_addr[1], nxt + a_addr[0], nxt + b_addr[0],
                                               nullptr);
    }
    {
      const char* cur = smem + ((nk - 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      k_step<TT, false, true, false, LOAD_SLOT>(a, b0, b1, acc, cur + a_addr[0], cur + a_addr[1], cur + b_addr[1],
                                                nullptr);
      k_step<TT, false, false, false, LOAD_SLOT>(a, b1, b0, acc, cur + a_addr[1], nullptr, nullptr, nullptr);
    }
  }
};

}  // namespace llamarl
