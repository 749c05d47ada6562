// gemm_nt.h -- the one MFMA main loop every contraction of the path runs on.
//
// C[m,n] = sum_k A[m,k] * B[n,k]   ("NT": both operands are K-contiguous), fp32 accumulate.
//   forward / recompute : A = H [N,d]        B = W   [V,d]     K = d
//   dH = dz W           : A = dz [N,V]       B = W^T [d,V]     K = V
//   dW = dz^T H         : A = dz^T [V,N]     B = H^T [d,N]     K = N
//
// gfx950 mapping
//   - one workgroup = 8 wavefronts (2 x 4) = one 256 x 256 output tile; a wavefront owns 128 x 64 of it
//     as 4 x 2 MFMA 32x32 blocks (128 fp32 accumulator registers per lane).
//   - K advances in slabs of 128 bytes per row (64 bf16 / 32 fp32).  A slab of both operands is 64 KB of LDS;
//     two slabs are resident (128 of the CU's 160 KB) so the next slab streams in while this one is multiplied.
//   - slabs go HBM/L2 -> LDS with buffer loads that write LDS directly (16 bytes per lane, no VGPR staging).
//     The hardware puts lane i's 16 bytes at LDS base + 16 i, so the bank-conflict swizzle is applied on the
//     global side: physical 16-byte slot p of row r holds logical chunk p ^ ((r >> 1) & 7), which spreads the
//     16 rows a ds_read_b128 serves per pass over all 64 LDS banks.
//   - the loop is software-pipelined by hand: MFMA fragments are double-buffered in registers, every
//     ds_read_b128 is issued in the shadow of an MFMA one k-substep ahead of its use, and scheduling fences
//     pin that interleave (the compiler's own schedule exposes the LDS latency).
//   - out-of-range rows and the K tail use the buffer descriptor's bounds check: such lanes read zeros.
//   - kernels are persistent (one workgroup per CU walks a list of tiles) and fetch the first slabs of their next
//     tile before the epilogue of the current one, so the epilogue's VALU work overlaps that latency.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace llamarl {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

constexpr int BM = 256;       // tile rows (A rows)
constexpr int BN = 256;       // tile cols (B rows)
constexpr int NTHREADS = 512;
constexpr int WAVES_N = 4;    // wave grid 2 (M) x 4 (N)
constexpr int TM = 4;         // 32x32 MFMA blocks per wave along M  (128 rows)
constexpr int TN = 2;         // ... along N                          (64 cols)
constexpr int WAVE_M = TM * 32;
constexpr int WAVE_N = TN * 32;
constexpr int SLAB_ROW_BYTES = 128;
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

__device__ __forceinline__ void mma(const bf16x8_t& a, const bf16x8_t& b, f32x16_t& c) {
  c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// fp32: the 32x32x2 MFMA takes one float per lane (k = lane / 32).  A lane holds 4 consecutive k of one chunk;
// the two half-waves hold different chunks, so four MFMAs cover the 8 k values of a chunk pair.
__device__ __forceinline__ void mma(const f32x4_t& a, const f32x4_t& b, f32x16_t& c) {
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], c, 0, 0, 0);
}

__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Where the accumulator element (i, j, r) of this lane sits inside the 256 x 256 tile.
// MFMA 32x32 output layout: register r of lane l holds row (r/4)*8 + (l/32)*4 + r%4, column l%32.
struct LanePos {
  int wm, wn, lane;
  __device__ __forceinline__ int row(int i, int r) const {
    return wm * WAVE_M + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
  }
  __device__ __forceinline__ int col(int j) const { return wn * WAVE_N + j * 32 + (lane & 31); }
  // Pair-interleaved columns (see paired_row): the lane's two column blocks hold NEIGHBOURING columns, so a lane
  // owns a contiguous pair and 32 lanes own 64 consecutive columns of one row.
  __device__ __forceinline__ int col_pair() const { return wn * WAVE_N + 2 * (lane & 31); }
};

// Which row of an operand tile the loader puts into LDS row `r`.  A wave's 64 LDS rows of the column operand feed
// its two 32-column MFMA blocks (block j = bit 5, MFMA column n = low 5 bits); with pairing, block j / column n is
// tile row 2n + j of those 64, so that accumulator registers acc[.][0] and acc[.][1] of a lane are neighbouring
// output columns.  Only the global side changes: LDS layout, swizzle and fragment reads stay as they are.
template <bool PAIR>
__device__ __forceinline__ int tile_row_of(int r) {
  static_assert(TN == 2 && WAVE_N == 64, "pairing interleaves exactly two column blocks");
  return PAIR ? ((r & ~63) | ((r & 31) << 1) | ((r >> 5) & 1)) : r;
}

// Persistent tile schedule.  The grid has one workgroup per CU (any size works); workgroups are dealt round-robin
// to the 8 XCDs, each with a private L2.  Every XCD owns a contiguous run of tile ids and its workgroups walk it
// in lock-step, so the tiles an XCD works on at any time are consecutive ids; ids are ordered so that 32
// consecutive ones form an 8 x 4 patch that shares A and B panels.  tiles_m x tiles_n is the number of tiles that
// exist once the device-side active-row count is known.
struct TileSchedule {
  int tiles_m, tiles_n;
  int next_id, end_id, stride;
  __device__ __forceinline__ void init(int tiles_m_, int tiles_n_) {
    tiles_m = tiles_m_;
    tiles_n = tiles_n_;
    const int ntiles = tiles_m * tiles_n;
    const int bid = blockIdx.x, nblk = gridDim.x;
    const int xcd = bid & 7, local = bid >> 3;
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
    constexpr int GROUP_M = 8;
    const int per_group = GROUP_M * tiles_n;
    const int g = id / per_group;
    const int first_m = g * GROUP_M;
    const int gsize = min(tiles_m - first_m, GROUP_M);
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
  template <bool PAIR = false>
  __device__ __forceinline__ void init(const void* base, int64_t ld, int rows_valid, int wave, int lane) {
    const uint32_t row_bytes = (uint32_t)(ld * (int64_t)sizeof(typename TT::store_t));
    set_base(base, row_bytes * (uint32_t)rows_valid);
    const uint32_t c16 = (uint32_t)lane_chunk(wave, lane) * 16u;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = tile_row_of<PAIR>((it * 8 + wave) * 8 + (lane >> 3));
      voff[it] = (row < rows_valid) ? (uint32_t)row * row_bytes + c16 : OOB_OFFSET;
    }
  }
  // Gathered panel: tile row r is row rows[r] of the whole matrix `base` (total_rows rows, < 2^31 bytes).
  // Free with per-lane buffer offsets: this is how masked tokens are skipped without a packed copy of H.
  template <bool PAIR = false>
  __device__ __forceinline__ void init_gather(const void* base, int64_t ld, int64_t total_rows, const int32_t* rows,
                                              int rows_valid, int wave, int lane) {
    const uint32_t row_bytes = (uint32_t)(ld * (int64_t)sizeof(typename TT::store_t));
    set_base(base, (uint32_t)total_rows * row_bytes);
    const uint32_t c16 = (uint32_t)lane_chunk(wave, lane) * 16u;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = tile_row_of<PAIR>((it * 8 + wave) * 8 + (lane >> 3));
      voff[it] = (row < rows_valid) ? (uint32_t)rows[row] * row_bytes + c16 : OOB_OFFSET;
    }
  }
  // k0: first k of the slab (elements); K: contraction length.  lds: start of this operand's slab in LDS.
  // TAIL: the slab may reach past K (only the last slab of a contraction whose K is not a multiple of the slab
  // depth): lanes whose chunk lies past K fetch nothing.  Callers pick TAIL = false wherever they can, it saves a
  // select per load.
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

template <typename TT>
struct Frags {
  typename TT::frag_t a[TM];
  typename TT::frag_t b[TN];
};

// Loads of one K slab handed to a k-substep, which issues one after each of its MFMAs (8 loads, 8 MFMAs): spread
// out like this they cost the matrix pipe less than as a burst after the barrier (-4 % time on the bare loop).
template <typename TT>
struct SlabFetch {
  const SlabLoader<TT>* la;
  const SlabLoader<TT>* lb;
  char* dst;      // stage that receives the slab
  int k0, K, wave, lane;
};

// One k-substep: TM x TN MFMA blocks on `cur`; in the shadow of MFMA q the q-th fragment of the next substep is
// read into `nxt` (A0 B0 A1 B1 ... then the rest of the longer operand).  FETCH: 0 none, 1 slab loads without a K
// tail, 2 with.
template <typename TT, int FETCH = 0>
__device__ __forceinline__ void k_substep(const Frags<TT>& cur, Frags<TT>& nxt, const char* rd, int a_addr, int b_addr,
                                          f32x16_t (&acc)[TM][TN], bool read, const SlabFetch<TT>* sf = nullptr) {
  typedef typename TT::frag_t frag_t;
  constexpr int NR = TM + TN;
  constexpr int MINAB = TM < TN ? TM : TN;
  static_assert(TM * TN == 8, "one slab load per MFMA slot");
#pragma unroll
  for (int q = 0; q < TM * TN; ++q) {
    const int i = q / TN, j = q % TN;
    mma(cur.a[i], cur.b[j], acc[i][j]);
    LLAMARL_FENCE();
    if (q < NR && read) {
      if (q < 2 * MINAB) {
        if ((q & 1) == 0) nxt.a[q >> 1] = *reinterpret_cast<const frag_t*>(rd + a_addr + (q >> 1) * 32 * SLAB_ROW_BYTES);
        else nxt.b[q >> 1] = *reinterpret_cast<const frag_t*>(rd + b_addr + (q >> 1) * 32 * SLAB_ROW_BYTES);
      } else {
        const int r = q - MINAB;
        if (TM > TN) nxt.a[r] = *reinterpret_cast<const frag_t*>(rd + a_addr + r * 32 * SLAB_ROW_BYTES);
        else nxt.b[r] = *reinterpret_cast<const frag_t*>(rd + b_addr + r * 32 * SLAB_ROW_BYTES);
      }
      LLAMARL_FENCE();
    }
    if constexpr (FETCH != 0) {
      if (q < 4) sf->la->issue_one(sf->dst, q, sf->k0, sf->K, sf->wave, sf->lane, FETCH == 2);
      else sf->lb->issue_one(sf->dst + SLAB_A_BYTES, q - 4, sf->k0, sf->K, sf->wave, sf->lane, FETCH == 2);
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
// Per slab kt (4 k-substeps s = 0..3, fragment sets f0/f1 alternate):
//   s=0..2 : MFMAs of substep s, reads of substep s+1 from slab kt
//   sync   : wait for this thread's share of slab kt+1, barrier (slab kt+1 visible, slab kt no longer read)
//   s=3    : MFMAs of substep 3 (already in registers), reads of substep 0 of slab kt+1, and one load of slab
//            kt+2 after each MFMA, into the buffer slab kt just vacated
//
// GATHER_B: the B panel is gathered -- B_tile is then the base of the whole matrix with b_total rows and
// tile row r is its row b_rows[r].  PAIR_B: output columns are pair-interleaved over the lane's two column blocks
// (tile_row_of); the epilogue must then take its columns from LanePos::col_pair().
template <typename TT>
struct TileGemm {
  typedef typename TT::frag_t frag_t;
  static constexpr int BK = 8 * TT::EPC;
  SlabLoader<TT> la, lb;
  int K;

  template <bool GATHER_B, bool PAIR_B = false>
  __device__ __forceinline__ void prefetch(const void* A_tile, int64_t lda, int rowsA, const void* B_tile, int64_t ldb,
                                           int rowsB, int64_t K_, char* smem, const int32_t* b_rows = nullptr,
                                           int64_t b_total = 0) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    K = (int)K_;
    la.init(A_tile, lda, rowsA, wave, lane);
    if constexpr (GATHER_B) lb.template init_gather<PAIR_B>(B_tile, ldb, b_total, b_rows, rowsB, wave, lane);
    else lb.template init<PAIR_B>(B_tile, ldb, rowsB, wave, lane);
    la.issue(smem, 0, K, wave, lane);
    lb.issue(smem + SLAB_A_BYTES, 0, K, wave, lane);
    if (K > BK) {
      la.issue(smem + STAGE_BYTES, BK, K, wave, lane);
      lb.issue(smem + STAGE_BYTES + SLAB_A_BYTES, BK, K, wave, lane);
    }
  }

  __device__ __forceinline__ void run(char* smem, f32x16_t (&acc)[TM][TN]) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = (K + BK - 1) / BK;
    // per-lane read addresses: row = lane % 32 inside a 32-row block, chunk pair (2s, 2s+1) split over half-waves
    const int half = lane >> 5;
    const int arow = wm * WAVE_M + (lane & 31), brow = wn * WAVE_N + (lane & 31);
    int a_addr[4], b_addr[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      a_addr[s] = arow * SLAB_ROW_BYTES + (((2 * s + half) ^ swizzle(arow)) * 16);
      b_addr[s] = SLAB_A_BYTES + brow * SLAB_ROW_BYTES + (((2 * s + half) ^ swizzle(brow)) * 16);
    }
    // Slabs 0 and 1 were issued by prefetch(); stores of a previous epilogue may sit between them and now in the
    // vmcnt queue, so wait for everything rather than count.
    wait_vmcnt0();
    __syncthreads();
    Frags<TT> f0, f1;
    // same order as the reads of a k-substep (A0 B0 A1 B1 A2 A3), so that the wait counts the compiler derives for
    // the loop head agree on both ways into it
    static_assert(TM == 4 && TN == 2, "read order written out for a 4 x 2 wave tile");
    f0.a[0] = *reinterpret_cast<const frag_t*>(smem + a_addr[0]);
    f0.b[0] = *reinterpret_cast<const frag_t*>(smem + b_addr[0]);
    f0.a[1] = *reinterpret_cast<const frag_t*>(smem + a_addr[0] + 32 * SLAB_ROW_BYTES);
    f0.b[1] = *reinterpret_cast<const frag_t*>(smem + b_addr[0] + 32 * SLAB_ROW_BYTES);
    f0.a[2] = *reinterpret_cast<const frag_t*>(smem + a_addr[0] + 2 * 32 * SLAB_ROW_BYTES);
    f0.a[3] = *reinterpret_cast<const frag_t*>(smem + a_addr[0] + 3 * 32 * SLAB_ROW_BYTES);

    // slabs 0 .. nk-3: each fetches slab kt+2.  Then slab nk-2 (nothing left to fetch) and the last slab, written
    // out one after the other: a branch inside one loop body made the compiler copy the accumulators around.
    for (int kt = 0; kt < nk - 2; ++kt) {
      char* cur = smem + (kt & 1) * STAGE_BYTES;
      char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      k_substep<TT>(f0, f1, cur, a_addr[1], b_addr[1], acc, true);
      k_substep<TT>(f1, f0, cur, a_addr[2], b_addr[2], acc, true);
      k_substep<TT>(f0, f1, cur, a_addr[3], b_addr[3], acc, true);
      wait_vmcnt0();      // this thread's share of slab kt+1 has landed in LDS
      __syncthreads();    // everyone's has, and everyone is done reading slab kt
      LLAMARL_FENCE();
      const SlabFetch<TT> sf{&la, &lb, cur, (kt + 2) * BK, K, wave, lane};
      k_substep<TT, 2>(f1, f0, nxt, a_addr[0], b_addr[0], acc, true, &sf);
    }
    if (nk >= 2) {
      const char* cur = smem + ((nk - 2) & 1) * STAGE_BYTES;
      const char* nxt = smem + ((nk - 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      k_substep<TT>(f0, f1, cur, a_addr[1], b_addr[1], acc, true);
      k_substep<TT>(f1, f0, cur, a_addr[2], b_addr[2], acc, true);
      k_substep<TT>(f0, f1, cur, a_addr[3], b_addr[3], acc, true);
      wait_vmcnt0();
      __syncthreads();
      LLAMARL_FENCE();
      k_substep<TT>(f1, f0, nxt, a_addr[0], b_addr[0], acc, true);
    }
    {
      const char* cur = smem + ((nk - 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      k_substep<TT>(f0, f1, cur, a_addr[1], b_addr[1], acc, true);
      k_substep<TT>(f1, f0, cur, a_addr[2], b_addr[2], acc, true);
      k_substep<TT>(f0, f1, cur, a_addr[3], b_addr[3], acc, true);
      k_substep<TT>(f1, f0, cur, 0, 0, acc, false);
    }
  }
};

}  // namespace llamarl
