// gemm_tn.h -- the same main loop for operands that are K-MAJOR in memory (bf16 only):
//
//   C[m,n] = sum_k At[k,m] * Bt[k,n]        At [K][lda], Bt [K][ldb], rows are k, m / n contiguous
//
// Used for dH = dz W with At = dz^T [V][tokens] (the one orientation the recompute kernel writes) and Bt = W [V][d]
// as the caller holds it: no transposed copy of W and no second orientation of dz are ever made.
//
// gfx950 mapping: a K slab of an operand is 64 k-rows x 256 columns x bf16 = 64 rows of 512 bytes in LDS (32 KB,
// same footprint as the K-contiguous slab).  MFMA wants, per lane, 8 k-values of ONE column; in this layout they
// sit 512 bytes apart.  ds_read_b64_tr_b16 does the transposition in the LDS pipe: inside each group of 16 lanes,
// lane 4j+q loads 8 bytes (4 columns) of k-row j, and lane i receives column i of the resulting 4 x 16 block, i.e.
// 4 consecutive k of its own column.  Two such reads make one MFMA fragment.  Any assignment of k-values to
// fragment slots is correct as long as both operands use the same one, and they do.
//
// Bank conflicts: the 32 lanes served together touch 4 k-rows x 2 column halves x 32 bytes.  Rows are 512 bytes
// apart (same banks), so 16-byte slot p of row k holds logical chunk  pi(p ^ 2(k & 3)), where pi swaps bits 1 and
// 3 of the chunk index: the 4 rows land in 4 different slot pairs and the two column halves in different
// bank halves.  As in gemm_nt.h the permutation is applied on the global-address side of the LDS-direct loads.
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

__device__ __forceinline__ int km_pi(int c) {   // swap bits 1 and 3 (an involution)
  const int b1 = (c >> 1) & 1, b3 = (c >> 3) & 1;
  return (c & ~0xA) | (b1 << 3) | (b3 << 1);
}

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
    // (row & 3) = 2(w & 1) + l/32 whatever `it` is, so one offset serves all four instructions.
    const int r = 2 * wave + (lane >> 5);
    const int c = km_pi((lane & 31) ^ (2 * (r & 3)));
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

  struct Fetch {     // the eight loads of one slab, issued one after each MFMA of a substep
    const KMajorLoader* la;
    const KMajorLoader* lb;
    KMajorLoader::Slab sa, sb;
    int wave;
  };

  // substep: TM x TN MFMAs on `cur`; the fragments of the next substep are read in their shadow
  template <bool FETCH = false>
  __device__ __forceinline__ static void substep(const Frags<TT>& cur, Frags<TT>& nxt, const char* rd, const int (&a_off)[TM],
                                                 const int (&b_off)[TN], int s_bytes, f32x16_t (&acc)[TM][TN], bool read,
                                                 const Fetch* f = nullptr) {
    static_assert(TM * TN == 8, "one slab load per MFMA slot");
    constexpr int NR = TM + TN;
    constexpr int MINAB = TM < TN ? TM : TN;
#pragma unroll
    for (int q = 0; q < TM * TN; ++q) {
      const int i = q / TN, j = q % TN;
      mma(cur.a[i], cur.b[j], acc[i][j]);
      LLAMARL_FENCE();
      if (q < NR && read) {
        if (q < 2 * MINAB) {
          if ((q & 1) == 0) nxt.a[q >> 1] = read_frag(rd + a_off[q >> 1] + s_bytes);
          else nxt.b[q >> 1] = read_frag(rd + b_off[q >> 1] + s_bytes);
        } else {
          const int r = q - MINAB;
          if (TM > TN) nxt.a[r] = read_frag(rd + a_off[r] + s_bytes);
          else nxt.b[r] = read_frag(rd + b_off[r] + s_bytes);
        }
        LLAMARL_FENCE();
      }
      if constexpr (FETCH) {
        if (q < 4) f->la->issue_one(f->sa, q, f->wave);
        else f->lb->issue_one(f->sb, q - 4, f->wave);
        LLAMARL_FENCE();
      }
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
    const int nk = (k_len + 63) / 64;

    // lane -> what it LOADS for the transposing read: group g = lane/16 serves columns (g&1)*16 .. +15 of a 32-column
    // block and k-rows 8(g>>1) .. +7 of a 16-row substep; inside the group lane 4j+q loads k-row j, columns 4q .. 4q+3.
    const int g = lane >> 4, jrow = (lane >> 2) & 3, q4 = lane & 3;
    const int krow = 8 * (g >> 1) + jrow;                                  // first of the two reads; second is +4
    int a_off[TM], b_off[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = wm * WAVE_M + i * 32 + (g & 1) * 16 + 4 * q4;
      a_off[i] = krow * KM_ROW_BYTES + ((km_pi(m >> 3) ^ (2 * jrow)) * 16) + ((m >> 2) & 1) * 8;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = wn * WAVE_N + j * 32 + (g & 1) * 16 + 4 * q4;
      b_off[j] = SLAB_A_BYTES + krow * KM_ROW_BYTES + ((km_pi(n >> 3) ^ (2 * jrow)) * 16) + ((n >> 2) & 1) * 8;
    }
    constexpr int SUB = 16 * KM_ROW_BYTES;                                 // bytes between k-substeps

    wait_vmcnt0();
    __syncthreads();
    Frags<TT> f0, f1;
    // same order as the reads of a substep (A0 B0 A1 B1 A2 A3)
    static_assert(TM == 4 && TN == 2, "read order written out for a 4 x 2 wave tile");
    f0.a[0] = read_frag(smem + a_off[0]);
    f0.b[0] = read_frag(smem + b_off[0]);
    f0.a[1] = read_frag(smem + a_off[1]);
    f0.b[1] = read_frag(smem + b_off[1]);
    f0.a[2] = read_frag(smem + a_off[2]);
    f0.a[3] = read_frag(smem + a_off[3]);

    // slabs 0 .. nk-3 fetch slab kt+2 under their last substep; slab nk-2 and the last slab follow, written out
    for (int kt = 0; kt < nk - 2; ++kt) {
      char* cur = smem + (kt & 1) * STAGE_BYTES;
      char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      substep(f0, f1, cur, a_off, b_off, 1 * SUB, acc, true);
      substep(f1, f0, cur, a_off, b_off, 2 * SUB, acc, true);
      substep(f0, f1, cur, a_off, b_off, 3 * SUB, acc, true);
      wait_vmcnt0();      // this thread's share of slab kt+1 has landed in LDS
      __syncthreads();    // everyone's has, and everyone is done reading slab kt
      LLAMARL_FENCE();
      const Fetch f{&la, &lb, la.slab(cur, kt + 2, k_len), lb.slab(cur + SLAB_A_BYTES, kt + 2, k_len), wave};
      substep<true>(f1, f0, nxt, a_off, b_off, 0, acc, true, &f);
    }
    if (nk >= 2) {
      const char* cur = smem + ((nk - 2) & 1) * STAGE_BYTES;
      const char* nxt = smem + ((nk - 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      substep(f0, f1, cur, a_off, b_off, 1 * SUB, acc, true);
      substep(f1, f0, cur, a_off, b_off, 2 * SUB, acc, true);
      substep(f0, f1, cur, a_off, b_off, 3 * SUB, acc, true);
      wait_vmcnt0();
      __syncthreads();
      LLAMARL_FENCE();
      substep(f1, f0, nxt, a_off, b_off, 0, acc, true);
    }
    {
      const char* cur = smem + ((nk - 1) & 1) * STAGE_BYTES;
      LLAMARL_FENCE();
      substep(f0, f1, cur, a_off, b_off, 1 * SUB, acc, true);
      substep(f1, f0, cur, a_off, b_off, 2 * SUB, acc, true);
      substep(f0, f1, cur, a_off, b_off, 3 * SUB, acc, true);
      substep(f1, f0, cur, a_off, b_off, 0, acc, false);
    }
  }
};

}  // namespace llamarl
