// gemm_tn.h -- the same main loop for operands that are K-MAJOR in memory (bf16 only):
//
//   C[m,n] = sum_k At[k,m] * Bt[k,n]        At [K][lda], Bt [K][ldb], rows are k, m / n contiguous
//
// Used for dH = dz W with At = dz^T [V][tokens] (the one orientation the recompute kernel writes) and Bt = W [V][d]
// as the caller holds it: no transposed copy of W and no second orientation of dz are ever made.
//
// gfx950 mapping: a K slab of an operand is 64 k-rows x 256 columns x bf16 = 64 rows of 512 bytes in LDS (32 KB,
// same footprint as the K-contiguous slab).  The 16x16x32 MFMA wants, per lane, 8 consecutive k of ONE column
// (column = lane % 16, k group = lane / 16); in this layout they sit 512 bytes apart.  ds_read_b64_tr_b16 does the
// transposition in the LDS pipe: inside each group of 16 lanes, lane 4j+q loads 8 bytes (4 columns) of k-row j,
// and lane i receives column i of the resulting 4 x 16 block, i.e. 4 consecutive k of its own column.  Two such
// reads (k-rows 8g .. 8g+3 and 8g+4 .. 8g+7 for lane group g) make one MFMA fragment.
//
// Bank conflicts: the 32 lanes served together are two lane groups, i.e. k-rows 8g + 0..3 for two values of g, 32
// bytes of each.  Rows are 512 bytes apart (same banks), so 16-byte slot p of row k holds logical chunk
// p ^ (2 (k & 3) | 8 ((k >> 3) & 1)): the four rows of a group land in four different 32-byte positions and the
// two groups in different bank halves.  As in gemm_nt.h the permutation is applied on the global-address side of
// the LDS-direct loads.
#pragma once
#include "gemm_nt.h"

namespace llamarl {

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
constexpr int KM_ROW_BYTES = 512;        // one k-row of a slab: 256 columns of bf16

typedef int i32x4_t __attribute__((ext_vector_type(4)));
// buffer_load_dwordx4 ... lds, written out by hand.  The compiler's wait-count pass cannot tell which LDS bytes
// an LDS-direct load will fill, and ds_read_b64_tr_b16 carries no memory operand, so with the builtin it makes
// every transposing read wait for ALL loads in flight -- which serialises the loop.  Issued from inline asm the
// loads are invisible to that pass; the loop's own s_waitcnt vmcnt(0) + barrier order them against the reads.
__device__ __forceinline__ void lds_dma16(uint32_t lds_addr, uint32_t voff, i32x4_t rsrc, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory", "m0");
}

// XOR applied to the 16-byte chunk index of k-row k (see the header)
__device__ __forceinline__ int km_swz(int k) { return 2 * (k & 3) | 8 * ((k >> 3) & 1); }

// One k-major operand stream.  The descriptor is re-based at every slab (a K range can span many GiB) and covers
// exactly the k-rows that are left, so the K tail reads zeros.
struct KMajorLoader {
  uint32_t base_lo, base_hi;   // first k-row of the K range, first column of the tile
  uint32_t row_bytes, col0_bytes;
  uint32_t voff;               // this lane's (k-row inside a 16-row group, logical chunk) byte offset

  // origin = element (first k-row of the range, column col0) of a matrix with ld columns
  __device__ __forceinline__ void init(const void* origin, int64_t ld, int64_t col0, int wave, int lane) {
    const uint64_t p = reinterpret_cast<uint64_t>(origin);
    base_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)p);
    base_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));
    row_bytes = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(ld * 2));
    col0_bytes = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(col0 * 2));
    // wave-instruction `it` of wave w fills k-rows 2(it*8 + w), +1; lane l: row +l/32, physical slot l%32.
    // Bits 0, 1 and 3 of the row do not depend on `it`, so one offset serves all four instructions.
    const int r = 2 * wave + (lane >> 5);
    const int c = (lane & 31) ^ km_swz(r);
    voff = (uint32_t)r * row_bytes + (uint32_t)c * 16u;
  }
  // slab kt of a K range of k_len rows -> lds: the descriptor (uniform) once, then four loads
  struct Slab {
    i32x4_t rs;
    uint32_t lds0;
  };
  __device__ __forceinline__ Slab slab(char* lds, int kt, int k_len) const {
    const int rows_left = k_len - kt * 64;
    // the range ends with the last k-row that is left: counted from column col0, that is col0 bytes short of
    // rows * row_bytes (a tile that overhangs the right edge wraps into the next row, never past the matrix)
    const uint32_t rows = (uint32_t)(rows_left <= 0 ? 0 : (rows_left < 64 ? rows_left : 64));
    const uint32_t records = rows ? rows * row_bytes - col0_bytes : 0u;
    const uint64_t b = (((uint64_t)base_hi << 32) | base_lo) + (uint64_t)kt * 64u * row_bytes;
    Slab sl;
    sl.rs = i32x4_t{(int)(uint32_t)b, (int)((uint32_t)(b >> 32) & 0xffffu), (int)records, 0x00020000};
    sl.lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    return sl;
  }
  __device__ __forceinline__ void issue_one(const Slab& sl, int it, int wave) const {
    lds_dma16(sl.lds0 + (uint32_t)((it * 8 + wave) * 2 * KM_ROW_BYTES), voff, sl.rs, it * 16u * row_bytes);
  }
  __device__ __forceinline__ void issue(char* lds, int kt, int k_len, int wave) const {
    const Slab sl = slab(lds, kt, k_len);
#pragma unroll
    for (int it = 0; it < 4; ++it) issue_one(sl, it, wave);
  }
};

struct TileGemmTN {
  typedef BF16 TT;
  typedef bf16x8_t frag_t;
  KMajorLoader la, lb;
  int k_len;

  // At_origin / Bt_origin: element (first k-row of the range, first column of the tile).  Columns past the
  // matrix edge read the neighbouring row's finite values: they only reach output rows / columns nobody stores.
  __device__ __forceinline__ void prefetch(const uint16_t* At_origin, int64_t lda, int64_t a_col0,
                                           const uint16_t* Bt_origin, int64_t ldb, int64_t b_col0, int k_len_,
                                           char* smem) {
    const int lane = threadIdx.x & 63, wave = wave_id();
    k_len = k_len_;
    la.init(At_origin, lda, a_col0, wave, lane);
    lb.init(Bt_origin, ldb, b_col0, wave, lane);
    la.issue(smem, 0, k_len, wave);
    lb.issue(smem + SLAB_A_BYTES, 0, k_len, wave);
    if (k_len > 64) {
      la.issue(smem + STAGE_BYTES, 1, k_len, wave);
      lb.issue(smem + STAGE_BYTES + SLAB_A_BYTES, 1, k_len, wave);
    }
  }

  // one fragment = 8 k-values of this lane's column: two transposing 8-byte reads, 4 k-rows apart
  __device__ __forceinline__ static frag_t read_frag(const char* p) {
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4_ptr)(__attribute__((address_space(3))) void*)const_cast<char*>(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4_ptr)(__attribute__((address_space(3))) void*)const_cast<char*>(p + 4 * KM_ROW_BYTES));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8_t;
    const s16x8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(frag_t, v);
  }

  struct Fetch {     // the eight loads of one slab, issued one per MFMA slot after the barrier
    const KMajorLoader* la;
    const KMajorLoader* lb;
    KMajorLoader::Slab sa, sb;
    int wave;
  };

  // Address of block b's fragment: blocks are 32 bytes (two chunks) apart before the chunk swizzle, which XORs bits
  // 1..3 of the chunk index -- bits the block index occupies too -- so it is an XOR, not an add.  A: the 8 blocks
  // of a wave span bits 1..3 (fx = the whole swizzle).  B: the 4 blocks span bits 1..2 and the wave's position
  // bits 3..4, so bit 3 of the swizzle is folded into the base and fx carries bits 1..2 only.
  __device__ __forceinline__ static const char* blk(const char* base, int b, int fx) { return base + ((b * 32) ^ fx); }

  // One k-step (32 k-rows); the slot table of k_step in gemm_nt.h with the barrier of a slab's last k-step moved up
  // to slot 4 and the slab loads to the odd slots 5 .. 19.  Every fragment is two LDS instructions here, so the 24
  // reads of the next slab need the room: barrier at slot 8 / loads from slot 11 measured 3.4 % slower for the dH
  // contraction, barrier at slot 6: 0.8 % slower, at slot 2: 0.5 % slower; loads on even slots (where the fragment
  // reads sit): 4 - 6 % slower.  (The K-contiguous loop does not care: +-0.5 % for the same moves.)
  // pa / pb: slab base + this lane's row and byte offset for the k-step; fx: the lane's chunk swizzle in bytes.
  template <bool BAR, bool NEXT, bool FETCH>
  __device__ __forceinline__ static void k_step(frag_t (&a)[MB], const frag_t (&bc)[NB], frag_t (&bn)[NB],
                                                f32x4_t (&acc)[MB][NB], const char* pa_cur, const char* pa_nxt,
                                                const char* pb_nxt, int fx, int fxb, const Fetch* f) {
    constexpr int TB = 4;      // barrier slot: a[7], the last read of the slab, was issued at slot 0
    constexpr int LS = 5;      // first of the eight load slots (every other slot from here)
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
        a[7] = read_frag(blk(pa_cur, 7, fx));
        LLAMARL_FENCE();
      }
      if (NEXT) {
        if (t == 4) a[0] = read_frag(blk(pa_nxt, 0, fx));        // block 0 is done after slot 3, block 1 after slot 7
        if (t == 8) a[1] = read_frag(blk(pa_nxt, 1, fx));
        if (t >= 12 && (t & 3) == 0) a[ib - 1] = read_frag(blk(pa_nxt, ib - 1, fx));
        if (t == 10) bn[0] = read_frag(blk(pb_nxt, 0, fxb));
        if (t == 14) bn[1] = read_frag(blk(pb_nxt, 1, fxb));
        if (t == 18) bn[2] = read_frag(blk(pb_nxt, 2, fxb));
        if (t == 22) bn[3] = read_frag(blk(pb_nxt, 3, fxb));
        LLAMARL_FENCE();
      }
      if (FETCH && t >= LS && t <= LS + 14 && ((t - LS) & 1) == 0) {
        const int n = (t - LS) >> 1;
        if (n < 4) f->la->issue_one(f->sa, n, f->wave);
        else f->lb->issue_one(f->sb, n - 4, f->wave);
        LLAMARL_FENCE();
      }
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
    const int nk = (k_len + 63) / 64;

    // lane -> what it LOADS for the transposing read: lane group g = lane / 16 serves k-rows 8g .. 8g+7 of a k-step;
    // inside the group lane 4j+q loads k-row j (the second read: j + 4), columns 4q .. 4q+3 of the 16-column block.
    const int g = lane >> 4, jrow = (lane >> 2) & 3, q4 = lane & 3;
    const int krow = 8 * g + jrow;
    const int fx = km_swz(krow) * 16;                  // same for krow + 4; bit 3 of the k-row is g & 1 in both k-steps
    // block 0 of this wave: chunk (column / 8) before the swizzle, + the 8-byte half the lane's 4 columns sit in
    const int a_off = krow * KM_ROW_BYTES + (wm * WAVE_M / 8 + (q4 >> 1)) * 16 + (q4 & 1) * 8;
    const int fxb = fx & 0x60;
    const int b_off = SLAB_A_BYTES + krow * KM_ROW_BYTES + ((wn * WAVE_N * 2) ^ (fx & 0x80)) + (q4 >> 1) * 16 + (q4 & 1) * 8;
    constexpr int KS = 32 * KM_ROW_BYTES;              // bytes between the two k-steps of a slab

    wait_vmcnt0();
    __syncthreads();
    frag_t a[MB], b0[NB], b1[NB];
    a[0] = read_frag(blk(smem + a_off, 0, fx));
#pragma unroll
    for (int j = 0; j < NB; ++j) b0[j] = read_frag(blk(smem + b_off, j, fxb));
#pragma unroll
    for (int i = 1; i < MB - 1; ++i) a[i] = read_frag(blk(smem + a_off, i, fx));

    // slabs 0 .. nk-3 fetch slab kt+2 after their barrier; slab nk-2 and the last slab follow, written out
    for (int kt = 0; kt < nk - 2; ++kt) {
      char* cur = smem + (kt & 1) * STAGE_BYTES;
      const char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      k_step<false, true, false>(a, b0, b1, acc, cur + a_off, cur + a_off + KS, cur + b_off + KS, fx, fxb, nullptr);
      const Fetch f{&la, &lb, la.slab(cur, kt + 2, k_len), lb.slab(cur + SLAB_A_BYTES, kt + 2, k_len), wave};
      k_step<true, true, true>(a, b1, b0, acc, cur + a_off + KS, nxt + a_off, nxt + b_off, fx, fxb, &f);
    }
    if (nk >= 2) {
      const char* cur = smem + ((nk - 2) & 1) * STAGE_BYTES;
      const char* nxt = smem + ((nk - 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      k_step<false, true, false>(a, b0, b1, acc, cur + a_off, cur + a_off + KS, cur + b_off + KS, fx, fxb, nullptr);
      k_step<true, true, false>(a, b1, b0, acc, cur + a_off + KS, nxt + a_off, nxt + b_off, fx, fxb, nullptr);
    }
    {
      const char* cur = smem + ((nk - 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      k_step<false, true, false>(a, b0, b1, acc, cur + a_off, cur + a_off + KS, cur + b_off + KS, fx, fxb, nullptr);
      k_step<false, false, false>(a, b1, b0, acc, cur + a_off + KS, nullptr, nullptr, fx, fxb, nullptr);
    }
  }
};

}  // namespace llamarl
