// llamarl.hip -- host side of the C ABI declared in include/llamarl.h: argument validation, workspace
// layout and kernel launches.  No allocation, no synchronisation, no state between calls.
#include "../../include/llamarl.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "ceiling_kernel.h"
#include "head_kernels.h"
#include "loss_kernels.h"

using namespace llamarl;

namespace {

thread_local char g_err[512] = "";

llamarl_status fail(llamarl_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t esize(llamarl_dtype dt) { return dt == LLAMARL_BF16 ? 2 : 4; }

// ---- workspace layouts (every block 256-byte aligned) ----------------------------------------------------
struct FwdWs {
  int tiles_v, tiles_t;
  int64_t n_pad;
  size_t off_m, off_s, off_zt, off_rows, off_nact, total;
};
FwdWs fwd_ws(int64_t N, int64_t V) {
  FwdWs w;
  w.tiles_v = (int)((V + BM - 1) / BM);
  w.tiles_t = (int)((N + BN - 1) / BN);
  w.n_pad = round_up(N, BN);
  const size_t plane = (size_t)w.tiles_v * (size_t)w.n_pad * sizeof(float);
  w.off_m = 0;
  w.off_s = round_up((int64_t)plane, 256);
  w.off_zt = w.off_s + round_up((int64_t)plane, 256);
  w.off_rows = w.off_zt + (size_t)round_up(w.n_pad * (int64_t)sizeof(float), 256);
  w.off_nact = w.off_rows + (size_t)round_up(w.n_pad * (int64_t)sizeof(int32_t), 256);
  w.total = w.off_nact + 256;
  return w;
}

struct LossWs {
  int nblocks;
  size_t off_len, off_bad, off_part, off_ticket, total;
};
LossWs loss_ws(int64_t N, int64_t B) {  // B generations, N = B * T tokens
  LossWs w;
  w.nblocks = (int)std::min<int64_t>((N + LOSS_BLOCK_TOKENS - 1) / LOSS_BLOCK_TOKENS, LOSS_MAX_BLOCKS);
  w.off_len = 0;
  w.off_bad = (size_t)round_up(B * 4, 256);
  w.off_part = w.off_bad + (size_t)round_up(B * 4, 256);
  w.off_ticket = w.off_part + (size_t)round_up((int64_t)w.nblocks * LOSS_NSUM * 8, 256);
  w.total = w.off_ticket + 256;
  return w;
}


// Scratch of llamarl_offpolicy_loss_fwd_static: room for the LossWs layout at the entry point's stated maximum
// (2 x 65536 per-generation counters, LOSS_MAX_BLOCKS x LOSS_NSUM partial sums, the ticket): about 0.5 MB that every
// GPU the library runs on holds until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress(); kernels get the device address that call returns.
constexpr int64_t STATIC_MAX_TOKENS = (int64_t)1 << 22;
constexpr int64_t STATIC_MAX_GENERATIONS = (int64_t)1 << 16;
constexpr size_t STATIC_SCRATCH_BYTES =
    2 * (size_t)STATIC_MAX_GENERATIONS * 4 + ((size_t)LOSS_MAX_BLOCKS * LOSS_NSUM * 8 + 255) / 256 * 256 + 256;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int STATIC_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[STATIC_MAX_DEVICES] = {};      // device address of `scratch` on each GPU, looked up once

struct BwdWs {
  int64_t R;          // active rows one pass takes (a multiple of 256, or N): dz, the operand panels and the split
                      // partials are sized for R rows; more active rows than that are taken in further passes
  int n_pass;         // passes the host enqueues = ceil(N / R); passes past the active rows find nothing to do
  int64_t ldz, ldzt;  // padded leading dimensions (elements): V rounded up to 64; packed_pitch(R)
  size_t off_dz, off_dzt, off_wt, off_ht, off_rows, off_nact, off_plan, off_part, total;
};
// Most workgroups a persistent grid has (one per CU of an MI355X); also the most split items the last round of a
// store contraction can hold, each leaving one BM x BN fp32 block in the workspace.
constexpr int MAX_GRID = 256;
constexpr int STORE_MAX_SPLITS = 8;
BwdWs bwd_ws(int64_t N, int64_t d, int64_t V, llamarl_dtype dt, int64_t max_rows_per_pass) {
  BwdWs w;
  const size_t es = esize(dt);
  w.R = (max_rows_per_pass <= 0 || max_rows_per_pass >= N) ? N : std::min(N, round_up(max_rows_per_pass, BN));
  w.n_pass = (int)((N + w.R - 1) / w.R);
  w.ldz = round_up(V, 64);
  w.ldzt = packed_pitch(w.R);        // the kernels use packed_pitch(active rows of the pass) <= this
  // bf16: dz exists in the vocab-major orientation only and W is read as it is (k-major dH contraction);
  // fp32 keeps a token-major dz and a transposed copy of W as well
  const bool both = dt == LLAMARL_F32;
  w.off_dz = 0;
  w.off_dzt = w.off_dz + (both ? (size_t)round_up(w.R * w.ldz * (int64_t)es, 256) : 0);
  w.off_wt = w.off_dzt + (size_t)round_up(V * w.ldzt * (int64_t)es, 256);
  w.off_ht = w.off_wt + (both ? (size_t)round_up(d * w.ldz * (int64_t)es, 256) : 0);
  w.off_rows = w.off_ht + (size_t)round_up(d * w.ldzt * (int64_t)es, 256);
  w.off_nact = w.off_rows + (size_t)round_up(round_up(N, 64) * (int64_t)sizeof(int32_t), 256);
  w.off_plan = w.off_nact + (size_t)round_up((int64_t)(1 + w.n_pass) * (int64_t)sizeof(int32_t), 256);
  w.off_part = w.off_plan + 256;
  // fp32 partial blocks of the split tiles at the end of a store contraction (see StorePlan): at most
  // STORE_TAIL_ROUNDS per workgroup of the grid, and never more than eight per tile
  const int64_t tiles_dh = ((w.R + BM - 1) / BM) * ((d + BN - 1) / BN), tiles_dw = ((V + BM - 1) / BM) * ((d + BN - 1) / BN);
  const int64_t blocks = std::min<int64_t>((int64_t)STORE_TAIL_ROUNDS * MAX_GRID, std::max(tiles_dh, tiles_dw) * STORE_MAX_SPLITS);
  w.total = w.off_part + (size_t)(blocks * BM * BN * 4);
  return w;
}

llamarl_status check_head_shape(int64_t N, int64_t d, int64_t V, llamarl_dtype dt) {
  if (dt != LLAMARL_F32 && dt != LLAMARL_BF16) return fail(LLAMARL_ERR_INVALID_ARG, "unknown dtype %d", (int)dt);
  if (N <= 0 || d <= 0 || V <= 0)
    return fail(LLAMARL_ERR_INVALID_ARG, "N, d, V must be positive (got %lld, %lld, %lld)", (long long)N,
                (long long)d, (long long)V);
  const int epc = dt == LLAMARL_BF16 ? 8 : 4;
  if (d % epc != 0)
    return fail(LLAMARL_ERR_UNSUPPORTED, "d = %lld must be a multiple of %d for this dtype (16-byte rows)",
                (long long)d, epc);
  // one 256-row operand panel must stay below 2^31 bytes (32-bit buffer offsets)
  const int64_t widest = (d > V ? d : V) > N ? (d > V ? d : V) : N;
  if (round_up(widest, 64) * (int64_t)esize(dt) * 256 >= (int64_t)1 << 31)
    return fail(LLAMARL_ERR_UNSUPPORTED, "a 256-row panel of %lld elements per row exceeds 2 GiB", (long long)widest);
  if (N * d * (int64_t)esize(dt) >= (int64_t)1 << 31)
    return fail(LLAMARL_ERR_UNSUPPORTED, "H must be smaller than 2 GiB (its rows are gathered with 32-bit offsets)");
  if ((N + BM - 1) / BM * ((V + BN - 1) / BN) >= (int64_t)1 << 31 || V >= (int64_t)1 << 31)
    return fail(LLAMARL_ERR_UNSUPPORTED, "too many tiles");
  return LLAMARL_OK;
}

template <typename K>
hipError_t set_lds(K kernel, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             bytes);
}

// One persistent workgroup per CU (256 on MI355X); a smaller problem gets one workgroup per tile.
int persistent_grid(int64_t tiles) {
  static int cus = 0;   // a device property, not call state: read once
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = MAX_GRID;
    if (cus > MAX_GRID) cus = MAX_GRID;
  }
  return (int)(tiles < (int64_t)cus ? tiles : (int64_t)cus);
}

#define HIP_TRY(expr)                                                                              \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) return fail(LLAMARL_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

template <typename TT, bool KMAJOR, int MODE>
llamarl_status launch_store_mode(const StoreArgs& a, int64_t work_items, int tiles_worst, hipStream_t st) {
  HIP_TRY(set_lds(k_gemm_store<TT, KMAJOR, MODE>, MAINLOOP_LDS_BYTES));
  const int grid = persistent_grid(work_items);
  k_gemm_store<TT, KMAJOR, MODE><<<dim3((unsigned)grid), dim3(NTHREADS), MAINLOOP_LDS_BYTES, st>>>(a);
  HIP_TRY(hipGetLastError());
  if (a.max_splits > 1) {
    // the split tiles of the last round, if the device-side sizes left any: fewer than `grid` of them
    const int tail = std::min(grid - 1, tiles_worst);
    if (tail > 0) {
      k_reduce_tail<MODE><<<dim3((unsigned)tail, BM / TAIL_STRIPE_ROWS), dim3(256), 0, st>>>(a);
      HIP_TRY(hipGetLastError());
    }
  }
  return LLAMARL_OK;
}

// C [M,Nn] (+)= A B^T on the persistent grid; ws_part / ws_plan: workspace of the last round's split tiles
template <typename TT, bool KMAJOR = false>
llamarl_status launch_store_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t M, int64_t Nn,
                                 int64_t K, void* C, int64_t ldc, int c_is_f32, int accumulate, const int32_t* m_count,
                                 const int32_t* k_count, const int32_t* c_rows, float* ws_part, int32_t* ws_plan,
                                 const int32_t* pitch_count, int packed_a, int packed_b, hipStream_t st) {
  // the store epilogue of the K-contiguous loop writes four neighbouring columns per lane as one unit, and so
  // does the tail reduction
  if (Nn % 4 != 0 || ldc % 4 != 0)
    return fail(LLAMARL_ERR_UNSUPPORTED, "output columns and row stride must be multiples of 4");
  StoreArgs a;
  a.m_count = m_count; a.k_count = k_count; a.c_rows = c_rows;
  a.max_splits = STORE_MAX_SPLITS; a.part = ws_part; a.plan_out = ws_plan;

  a.pitch_count = pitch_count; a.packed_a = packed_a; a.packed_b = packed_b;
  a.A = A; a.lda = lda; a.B = B; a.ldb = ldb; a.M = M; a.Nn = Nn; a.K = K;
  const int tiles_m = (int)((M + BM - 1) / BM);      // worst case: every row active
  a.tiles_n = (int)((Nn + BN - 1) / BN);
  a.group_m = (KMAJOR && a.tiles_n <= 16) ? PATCH_ROWS_KMAJOR : PATCH_ROWS_STORE;
  a.C = C; a.ldc = ldc; a.c_is_f32 = c_is_f32; a.accumulate = accumulate;
  const int tiles = tiles_m * a.tiles_n;
  const int64_t items = (int64_t)tiles * STORE_MAX_SPLITS;   // a small contraction still gets a workgroup per split
  if (c_is_f32) return accumulate ? launch_store_mode<TT, KMAJOR, 2>(a, items, tiles, st)
                                  : launch_store_mode<TT, KMAJOR, 1>(a, items, tiles, st);
  if constexpr (sizeof(typename TT::store_t) == 2) {
    return accumulate ? launch_store_mode<TT, KMAJOR, 4>(a, items, tiles, st)
                      : launch_store_mode<TT, KMAJOR, 3>(a, items, tiles, st);
  } else {
    return fail(LLAMARL_ERR_INVALID_ARG, "a 16-bit output needs a 16-bit input type");
  }
}

// W holds the vocabulary rows [v_off, v_off + V) of a head with V_total rows (the whole head: v_off = 0, V = V_total).
// partial == 0: out0 = logp, out1 = lse.  partial != 0: (out0, out1, out2) = the shard's (m, s, zt).
template <typename TT>
llamarl_status run_logprobs(const void* H, const void* W, const int32_t* targets, const uint8_t* mask, int64_t N,
                            int64_t d, int64_t V, int64_t v_off, int64_t V_total, int partial, float* out0,
                            float* out1, float* out2, char* ws, hipStream_t st) {
  const FwdWs w = fwd_ws(N, V);
  FwdArgs a;
  a.H = H; a.W = W; a.targets = targets; a.N = N; a.d = d; a.V = V; a.v_off = v_off;
  a.tiles_v = w.tiles_v; a.tiles_t = w.tiles_t; a.n_pad = w.n_pad;
  a.part_m = reinterpret_cast<float*>(ws + w.off_m);
  a.part_s = reinterpret_cast<float*>(ws + w.off_s);
  a.zt = reinterpret_cast<float*>(ws + w.off_zt);
  int32_t* rows = reinterpret_cast<int32_t*>(ws + w.off_rows);
  int32_t* n_act = reinterpret_cast<int32_t*>(ws + w.off_nact);
  a.rows = rows; a.n_act = n_act;
  // active-token list (mask and target range); inactive rows get their outputs here
  k_compact_rows<<<dim3((unsigned)((N + COMPACT_BLOCK_ROWS - 1) / COMPACT_BLOCK_ROWS)), dim3(COMPACT_THREADS), 0, st>>>(
      partial ? 2 : 0, mask, targets, V_total, nullptr, N, rows, n_act, out0, out1, out2);
  HIP_TRY(hipGetLastError());
  HIP_TRY(set_lds(k_fwd_partials<TT>, FWD_LDS_BYTES));
  k_fwd_partials<TT><<<dim3((unsigned)persistent_grid((int64_t)w.tiles_v * w.tiles_t)), dim3(NTHREADS), FWD_LDS_BYTES,
                       st>>>(a);
  HIP_TRY(hipGetLastError());
  MergeArgs m;
  m.part_m = a.part_m; m.part_s = a.part_s; m.zt = a.zt; m.rows = rows; m.n_act = n_act; m.tiles_v = w.tiles_v;
  m.n_pad = w.n_pad; m.out0 = out0; m.out1 = out1; m.out2 = out2; m.targets = targets; m.v_off = v_off; m.V = V;
  const dim3 mgrid((unsigned)((N + MERGE_TOKENS - 1) / MERGE_TOKENS)), mblock(MERGE_TOKENS * MERGE_SLICES);
  if (partial) k_merge_logp<true><<<mgrid, mblock, 0, st>>>(m);
  else k_merge_logp<false><<<mgrid, mblock, 0, st>>>(m);
  HIP_TRY(hipGetLastError());
  return LLAMARL_OK;
}

// active rows of each pass: cnt[c] = clamp(n_act - c * R, 0, R)
__global__ void k_pass_counts(const int32_t* n_act, int64_t R, int n_pass, int32_t* cnt) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= n_pass) return;
  const int64_t left = (int64_t)*n_act - (int64_t)c * R;
  cnt[c] = (int32_t)(left < 0 ? 0 : (left > R ? R : left));
}

template <typename TT>
llamarl_status run_bwd(const void* H, const void* W, const int32_t* targets, const float* lse, const float* coef,
                       float g, int64_t N, int64_t d, int64_t V, int64_t v_off, llamarl_dtype dt, void* dH, void* dW,
                       llamarl_dtype dW_dt, int accumulate_dW, int64_t max_rows_per_pass, char* ws, hipStream_t st,
                       void* const* ev) {
  typedef typename TT::store_t stt;
  const BwdWs w = bwd_ws(N, d, V, dt, max_rows_per_pass);
  // ev (optional, 6 caller-owned hipEvent_t): recorded on the stream at the phase boundaries of a one-pass backward
#define PHASE_EVENT(i) \
  do { if (ev) HIP_TRY(hipEventRecord(reinterpret_cast<hipEvent_t>(ev[i]), st)); } while (0)
  PHASE_EVENT(0);
  stt* dz = reinterpret_cast<stt*>(ws + w.off_dz);
  stt* dzt = reinterpret_cast<stt*>(ws + w.off_dzt);
  stt* wt = reinterpret_cast<stt*>(ws + w.off_wt);
  stt* ht = reinterpret_cast<stt*>(ws + w.off_ht);
  int32_t* all_rows = reinterpret_cast<int32_t*>(ws + w.off_rows);
  int32_t* n_act_all = reinterpret_cast<int32_t*>(ws + w.off_nact);
  int32_t* pass_cnt = n_act_all + 1;

  // tokens that carry gradient (coef != 0), and exact zeros for the dH rows of all the others
  k_compact_rows<<<dim3((unsigned)((N + COMPACT_BLOCK_ROWS - 1) / COMPACT_BLOCK_ROWS)), dim3(COMPACT_THREADS), 0, st>>>(
      1, nullptr, nullptr, V, coef, N, all_rows, n_act_all, nullptr, nullptr, nullptr);
  HIP_TRY(hipGetLastError());
  k_zero_inactive_rows<stt><<<dim3((unsigned)N), dim3(256), 0, st>>>(reinterpret_cast<stt*>(dH), coef, N, d);
  HIP_TRY(hipGetLastError());
  if (w.n_pass > 1) {
    k_pass_counts<<<dim3((unsigned)((w.n_pass + 255) / 256)), dim3(256), 0, st>>>(n_act_all, w.R, w.n_pass, pass_cnt);
    HIP_TRY(hipGetLastError());
  }
  constexpr bool kBf16 = sizeof(stt) == 2;
  if (!kBf16) {   // fp32 only: W^T [d][ldz] for the K-contiguous dH contraction
    k_transpose<stt><<<dim3((unsigned)(w.ldz / 64), (unsigned)((d + 63) / 64)), dim3(256), 0, st>>>(
        reinterpret_cast<const stt*>(W), V, d, d, wt, w.ldz, nullptr, nullptr);
    HIP_TRY(hipGetLastError());
  }

  for (int c = 0; c < w.n_pass; ++c) {
    // this pass: list positions [c R, c R + n_act), n_act = the pass's own count (device scalar)
    const int32_t* rows = all_rows + (int64_t)c * w.R;
    const int32_t* n_act = w.n_pass > 1 ? pass_cnt + c : n_act_all;
    const int64_t Rc = std::min(w.R, N - (int64_t)c * w.R);       // rows the pass can hold at most
    // operand panel H^T [d][pitch] of the pass's tokens (dW contraction)
    k_transpose<stt><<<dim3((unsigned)(w.ldzt / 64), (unsigned)((d + 63) / 64)), dim3(256), 0, st>>>(
        reinterpret_cast<const stt*>(H), N, d, d, ht, w.ldzt, rows, n_act);
    HIP_TRY(hipGetLastError());
    if (c == 0) PHASE_EVENT(1);

    // recompute logits tile by tile, turn them into dz (rows / columns = list positions of the pass)
    DzArgs a;
    a.H = H; a.W = W; a.targets = targets; a.lse = lse; a.coef = coef; a.g = g; a.N = N; a.d = d; a.V = V;
    a.v_off = v_off;
    a.tiles_v = (int)((V + BM - 1) / BM);
    a.tiles_t = (int)((Rc + BN - 1) / BN);
    a.dz = dz; a.ldz = w.ldz; a.dzt = dzt; a.rows = rows; a.n_act = n_act;
    const int dz_lds = MAINLOOP_LDS_BYTES;
    HIP_TRY(set_lds(k_bwd_dz<TT>, dz_lds));
    k_bwd_dz<TT><<<dim3((unsigned)persistent_grid((int64_t)a.tiles_v * a.tiles_t)), dim3(NTHREADS), dz_lds, st>>>(a);
    HIP_TRY(hipGetLastError());
    if (c == 0) PHASE_EVENT(2);

    // dH [active rows, d] = dz [n_act,V] . W [V,d], scattered to the token rows.
    //   bf16: k-major operands dz^T [V][n_act] and W [V][d], K = V exactly
    //   fp32: K-contiguous operands dz [n_act][ldz] and W^T [d][ldz], K zero-padded to ldz
    llamarl_status s;
    float* part = reinterpret_cast<float*>(ws + w.off_part);
    int32_t* plan = reinterpret_cast<int32_t*>(ws + w.off_plan);
    if constexpr (kBf16) {
      s = launch_store_gemm<TT, true>(dzt, w.ldzt, W, d, Rc, d, V, dH, d, 0, 0, n_act, nullptr, rows, part, plan, n_act,
                                      1, 0, st);
    } else {
      s = launch_store_gemm<TT>(dz, w.ldz, wt, w.ldz, Rc, d, w.ldz, dH, d, 1, 0, n_act, nullptr, rows, part, plan,
                                nullptr, 0, 0, st);
    }
    if (s != LLAMARL_OK) return s;
    if (c == 0) PHASE_EVENT(3);
    if (c == 0) PHASE_EVENT(4);
    // dW [V,d] (+)= dz^T [V,n_act] . H^T[d,n_act]^T      (K = n_act, zero-padded to a multiple of 64); passes after
    // the first add to what the earlier ones stored
    s = launch_store_gemm<TT>(dzt, w.ldzt, ht, w.ldzt, V, d, w.ldzt, dW, d, dW_dt == LLAMARL_F32,
                              c == 0 ? accumulate_dW : 1, nullptr, n_act, nullptr, part, plan, n_act, 1, 1, st);
    if (s != LLAMARL_OK) return s;
    if (c == 0) PHASE_EVENT(5);
  }
#undef PHASE_EVENT
  return LLAMARL_OK;
}

typedef void (*ceiling_traffic_kernel_t)(int, float*, const void*);
llamarl_status launch_ceiling_traffic(ceiling_traffic_kernel_t kernel, int grid, int iters, float* sink,
                                      const void* panels, hipStream_t st) {
  HIP_TRY(set_lds(kernel, MAINLOOP_LDS_BYTES));
  kernel<<<dim3((unsigned)grid), dim3(NTHREADS), MAINLOOP_LDS_BYTES, st>>>(iters, sink, panels);
  HIP_TRY(hipGetLastError());
  return LLAMARL_OK;
}

}  // namespace

extern "C" {

const char* llamarl_last_error(void) { return g_err; }
const char* llamarl_version(void) { return "llamarl-mi355x 0.1 (gfx950)"; }

size_t llamarl_workspace_bytes(int64_t N, int64_t d, int64_t V, llamarl_dtype dt, llamarl_pass pass) {
  if (N <= 0) return 0;
  switch (pass) {
    case LLAMARL_PASS_LOGPROBS:
      if (V <= 0) return 0;
      return fwd_ws(N, V).total;
    case LLAMARL_PASS_LOSS_FWD:
      return loss_ws(N, N).total;     // sized for the worst case B = N
    case LLAMARL_PASS_LOSS_BWD:
      if (V <= 0 || d <= 0 || (dt != LLAMARL_F32 && dt != LLAMARL_BF16)) return 0;
      return bwd_ws(N, d, V, dt, 0).total;
    default:
      return 0;
  }
}

static llamarl_status logprobs_entry(const void* H, const void* W, const int32_t* targets, const uint8_t* mask, int64_t N,
                                     int64_t d, int64_t V, int64_t v_off, int64_t V_total, llamarl_dtype dt, int partial,
                                     float* out0, float* out1, float* out2, void* ws, size_t ws_bytes, void* stream) {
  if (!H || !W || !targets || !out0 || !out1 || (partial && !out2))
    return fail(LLAMARL_ERR_INVALID_ARG, "null pointer argument");
  llamarl_status s = check_head_shape(N, d, V, dt);
  if (s != LLAMARL_OK) return s;
  if (v_off < 0 || V_total >= ((int64_t)1 << 31) || v_off + V > V_total)
    return fail(LLAMARL_ERR_INVALID_ARG, "vocabulary slice [%lld, %lld) does not lie inside [0, %lld)", (long long)v_off,
                (long long)(v_off + V), (long long)V_total);
  if (!aligned16(H) || !aligned16(W)) return fail(LLAMARL_ERR_INVALID_ARG, "H and W must be 16-byte aligned");
  const size_t need = fwd_ws(N, V).total;
  if (!ws || ws_bytes < need)
    return fail(LLAMARL_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed", ws ? ws_bytes : (size_t)0, need);
  if (!aligned16(ws)) return fail(LLAMARL_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (dt == LLAMARL_BF16)
    return run_logprobs<BF16>(H, W, targets, mask, N, d, V, v_off, V_total, partial, out0, out1, out2,
                              reinterpret_cast<char*>(ws), st);
  return run_logprobs<F32>(H, W, targets, mask, N, d, V, v_off, V_total, partial, out0, out1, out2,
                           reinterpret_cast<char*>(ws), st);
}

llamarl_status llamarl_token_logprobs(const void* H, const void* W, const int32_t* targets, const uint8_t* mask,
                                      int64_t N, int64_t d, int64_t V, llamarl_dtype dt, float* logp, float* lse,
                                      void* ws, size_t ws_bytes, void* stream) {
  return logprobs_entry(H, W, targets, mask, N, d, V, 0, V, dt, 0, logp, lse, nullptr, ws, ws_bytes, stream);
}

llamarl_status llamarl_token_logprobs_partial(const void* H, const void* W_slice, const int32_t* targets,
                                              const uint8_t* mask, int64_t N, int64_t d, int64_t V_slice, int64_t v0,
                                              int64_t V_total, llamarl_dtype dt, float* m, float* s, float* zt,
                                              void* ws, size_t ws_bytes, void* stream) {
  return logprobs_entry(H, W_slice, targets, mask, N, d, V_slice, v0, V_total, dt, 1, m, s, zt, ws, ws_bytes, stream);
}

llamarl_status llamarl_merge_partials(const float* m, const float* s, const float* zt, int shards, int64_t N,
                                      float* logp, float* lse, void* stream) {
  if (!m || !s || !zt || !logp || !lse) return fail(LLAMARL_ERR_INVALID_ARG, "null pointer argument");
  if (shards <= 0 || N <= 0) return fail(LLAMARL_ERR_INVALID_ARG, "shards and N must be positive");
  if (N >= ((int64_t)1 << 39)) return fail(LLAMARL_ERR_UNSUPPORTED, "too many tokens");
  k_merge_shards<<<dim3((unsigned)((N + 255) / 256)), dim3(256), 0, reinterpret_cast<hipStream_t>(stream)>>>(
      m, s, zt, shards, N, logp, lse);
  HIP_TRY(hipGetLastError());
  return LLAMARL_OK;
}

static llamarl_status check_loss_args(const float* logp, const float* mu_logp, const float* adv, const uint8_t* mask,
                                      const int32_t* targets, int64_t V, int64_t B, int64_t T,
                                      const llamarl_loss_params* p, const float* loss, const float* coef,
                                      const float* stats) {
  if (!logp || !mu_logp || !adv || !p || !loss || !coef || !stats)
    return fail(LLAMARL_ERR_INVALID_ARG, "null pointer argument");
  if (B <= 0 || T <= 0) return fail(LLAMARL_ERR_INVALID_ARG, "B and T must be positive");
  if (B >= ((int64_t)1 << 31) || T >= ((int64_t)1 << 31) || B * T >= ((int64_t)1 << 40))
    return fail(LLAMARL_ERR_UNSUPPORTED, "batch too large");
  if (p->clip_mode != LLAMARL_CLIP_AIPO && p->clip_mode != LLAMARL_CLIP_PPO)
    return fail(LLAMARL_ERR_INVALID_ARG, "unknown clip_mode %d", p->clip_mode);
  if (p->norm_mode < 0 || p->norm_mode > 2) return fail(LLAMARL_ERR_INVALID_ARG, "unknown norm_mode %d", p->norm_mode);
  if (p->clip_mode == LLAMARL_CLIP_AIPO && !(p->rho > 0.f))
    return fail(LLAMARL_ERR_INVALID_ARG, "rho must be positive (got %g)", (double)p->rho);
  if (p->clip_mode == LLAMARL_CLIP_PPO && (!(p->eps_lo >= 0.f) || !(p->eps_hi >= 0.f) || p->eps_lo > 1.f))
    return fail(LLAMARL_ERR_INVALID_ARG, "PPO mode needs 0 <= eps_lo <= 1 and eps_hi >= 0");
  if (targets && V <= 0) return fail(LLAMARL_ERR_INVALID_ARG, "targets given but V <= 0");
  if (!aligned16(logp) || !aligned16(mu_logp) || !aligned16(coef) || !aligned16(adv) || !aligned16(targets) ||
      (reinterpret_cast<uintptr_t>(mask) & 3u) != 0)
    return fail(LLAMARL_ERR_INVALID_ARG, "logp, mu_logp, adv, targets and coef must be 16-byte aligned, mask 4-byte");
  return LLAMARL_OK;
}

// the two launches of the loss forward; wsb holds a LossWs layout for (B*T, B)
static llamarl_status launch_loss_fwd(const float* logp, const float* mu_logp, const float* adv, int adv_per_token,
                                      const uint8_t* mask, const int32_t* targets, int64_t V, int64_t B, int64_t T,
                                      const llamarl_loss_params* p, float* loss, float* coef, float* stats, char* wsb,
                                      const LossWs& w, hipStream_t st) {
  LossArgs a;
  a.logp = logp; a.mu_logp = mu_logp; a.adv = adv; a.mask = mask; a.targets = targets; a.V = V; a.B = B; a.T = T;
  a.adv_per_token = adv_per_token; a.rho = p->rho; a.clip_mode = p->clip_mode; a.eps_lo = p->eps_lo;
  a.eps_hi = p->eps_hi; a.norm_mode = p->norm_mode;
  a.seq_len = reinterpret_cast<int32_t*>(wsb + w.off_len);
  a.seq_bad = reinterpret_cast<int32_t*>(wsb + w.off_bad);
  a.partials = reinterpret_cast<double*>(wsb + w.off_part);
  a.ticket = reinterpret_cast<unsigned int*>(wsb + w.off_ticket);
  a.nblocks = w.nblocks; a.coef = coef; a.loss = loss; a.stats = stats;
  k_seq_lengths<<<dim3((unsigned)B), dim3(SEQ_THREADS), 0, st>>>(a);          // also clears the ticket
  HIP_TRY(hipGetLastError());
  k_loss_tokens<<<dim3((unsigned)w.nblocks), dim3(LOSS_THREADS), 0, st>>>(a);   // its last block writes loss, stats
  HIP_TRY(hipGetLastError());
  return LLAMARL_OK;
}

llamarl_status llamarl_offpolicy_loss_fwd(const float* logp, const float* mu_logp, const float* adv,
                                          int adv_per_token, const uint8_t* mask, const int32_t* targets, int64_t V,
                                          int64_t B, int64_t T, const llamarl_loss_params* p, float* loss,
                                          float* coef, float* stats, void* ws, size_t ws_bytes, void* stream) {
  llamarl_status s = check_loss_args(logp, mu_logp, adv, mask, targets, V, B, T, p, loss, coef, stats);
  if (s != LLAMARL_OK) return s;
  const LossWs w = loss_ws(B * T, B);
  if (!ws || ws_bytes < w.total)
    return fail(LLAMARL_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed", ws ? ws_bytes : (size_t)0, w.total);
  if (!aligned16(ws)) return fail(LLAMARL_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
  return launch_loss_fwd(logp, mu_logp, adv, adv_per_token, mask, targets, V, B, T, p, loss, coef, stats,
                         reinterpret_cast<char*>(ws), w, reinterpret_cast<hipStream_t>(stream));
}

// Device address of this GPU's copy of `scratch` (each GPU has its own, at its own address).
static llamarl_status scratch_of_current_device(char** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(LLAMARL_ERR_UNSUPPORTED, "device ordinal %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return fail(LLAMARL_ERR_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = static_cast<char*>(g_scratch_ptr[dev]);
  return LLAMARL_OK;
}

llamarl_status llamarl_offpolicy_loss_fwd_static(const float* logp, const float* mu_logp, const float* adv,
                                                 int adv_per_token, const uint8_t* mask, const int32_t* targets,
                                                 int64_t V, int64_t B, int64_t T, const llamarl_loss_params* p,
                                                 float* loss, float* coef, float* stats, void* stream) {
  llamarl_status s = check_loss_args(logp, mu_logp, adv, mask, targets, V, B, T, p, loss, coef, stats);
  if (s != LLAMARL_OK) return s;
  if (B > STATIC_MAX_GENERATIONS || B * T > STATIC_MAX_TOKENS)
    return fail(LLAMARL_ERR_UNSUPPORTED,
                "B = %lld, B*T = %lld exceed the static scratch of this entry point (at most %lld generations, %lld "
                "tokens): use llamarl_offpolicy_loss_fwd with a workspace",
                (long long)B, (long long)(B * T), (long long)STATIC_MAX_GENERATIONS, (long long)STATIC_MAX_TOKENS);
  const LossWs w = loss_ws(B * T, B);
  if (w.total > STATIC_SCRATCH_BYTES) return fail(LLAMARL_ERR_UNSUPPORTED, "static scratch too small for this batch");
  char* base = nullptr;
  s = scratch_of_current_device(&base);
  if (s != LLAMARL_OK) return s;
  // nothing in the scratch has to start at zero: k_seq_lengths overwrites the counters and clears the ticket
  return launch_loss_fwd(logp, mu_logp, adv, adv_per_token, mask, targets, V, B, T, p, loss, coef, stats, base, w,
                         reinterpret_cast<hipStream_t>(stream));
}

static llamarl_status bwd_entry(const void* H, const void* W, const int32_t* targets, const float* lse,
                                const float* coef, float grad_loss, int64_t N, int64_t d, int64_t V, int64_t v_off,
                                llamarl_dtype dt, void* dH, void* dW, llamarl_dtype dW_dt, int accumulate_dW,
                                int64_t max_rows_per_pass, void* ws, size_t ws_bytes, void* stream, void* const* ev) {
  if (!H || !W || !targets || !lse || !coef || !dH || !dW) return fail(LLAMARL_ERR_INVALID_ARG, "null pointer argument");
  llamarl_status s = check_head_shape(N, d, V, dt);
  if (s != LLAMARL_OK) return s;
  if (dW_dt != LLAMARL_F32 && dW_dt != dt)
    return fail(LLAMARL_ERR_INVALID_ARG, "dW_dt must be LLAMARL_F32 or equal to dt");
  if (!aligned16(H) || !aligned16(W) || !aligned16(dH) || !aligned16(dW))
    return fail(LLAMARL_ERR_INVALID_ARG, "H, W, dH, dW must be 16-byte aligned");
  if (!std::isfinite(grad_loss)) return fail(LLAMARL_ERR_INVALID_ARG, "grad_loss must be finite");
  if (v_off < 0 || v_off + V >= ((int64_t)1 << 31)) return fail(LLAMARL_ERR_INVALID_ARG, "bad vocabulary offset");
  if (max_rows_per_pass < 0) return fail(LLAMARL_ERR_INVALID_ARG, "max_rows_per_pass must not be negative");
  const size_t need = bwd_ws(N, d, V, dt, max_rows_per_pass).total;
  if (!ws || ws_bytes < need)
    return fail(LLAMARL_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed", ws ? ws_bytes : (size_t)0, need);
  if (!aligned16(ws)) return fail(LLAMARL_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (dt == LLAMARL_BF16)
    return run_bwd<BF16>(H, W, targets, lse, coef, grad_loss, N, d, V, v_off, dt, dH, dW, dW_dt, accumulate_dW,
                         max_rows_per_pass,
                         reinterpret_cast<char*>(ws), st, ev);
  return run_bwd<F32>(H, W, targets, lse, coef, grad_loss, N, d, V, v_off, dt, dH, dW, dW_dt, accumulate_dW,
                      max_rows_per_pass,
                      reinterpret_cast<char*>(ws), st, ev);
}

llamarl_status llamarl_offpolicy_loss_bwd(const void* H, const void* W, const int32_t* targets, const float* lse,
                                          const float* coef, float grad_loss, int64_t N, int64_t d, int64_t V,
                                          llamarl_dtype dt, void* dH, void* dW, llamarl_dtype dW_dt,
                                          int accumulate_dW, void* ws, size_t ws_bytes, void* stream) {
  return bwd_entry(H, W, targets, lse, coef, grad_loss, N, d, V, 0, dt, dH, dW, dW_dt, accumulate_dW, 0, ws, ws_bytes,
                   stream, nullptr);
}

size_t llamarl_bwd_workspace_bytes(int64_t N, int64_t d, int64_t V, llamarl_dtype dt, int64_t max_rows_per_pass) {
  if (N <= 0 || V <= 0 || d <= 0 || max_rows_per_pass < 0 || (dt != LLAMARL_F32 && dt != LLAMARL_BF16)) return 0;
  return bwd_ws(N, d, V, dt, max_rows_per_pass).total;
}

llamarl_status llamarl_offpolicy_loss_bwd_chunked(const void* H, const void* W, const int32_t* targets,
                                                  const float* lse, const float* coef, float grad_loss, int64_t N,
                                                  int64_t d, int64_t V, llamarl_dtype dt, void* dH, void* dW,
                                                  llamarl_dtype dW_dt, int accumulate_dW, int64_t max_rows_per_pass,
                                                  void* ws, size_t ws_bytes, void* stream) {
  return bwd_entry(H, W, targets, lse, coef, grad_loss, N, d, V, 0, dt, dH, dW, dW_dt, accumulate_dW, max_rows_per_pass,
                   ws, ws_bytes, stream, nullptr);
}

llamarl_status llamarl_offpolicy_loss_bwd_slice(const void* H, const void* W_slice, const int32_t* targets,
                                                const float* lse, const float* coef, float grad_loss, int64_t N,
                                                int64_t d, int64_t V_slice, int64_t v0, llamarl_dtype dt,
                                                void* dH_partial, void* dW_slice, llamarl_dtype dW_dt,
                                                int accumulate_dW, void* ws, size_t ws_bytes, void* stream) {
  return bwd_entry(H, W_slice, targets, lse, coef, grad_loss, N, d, V_slice, v0, dt, dH_partial, dW_slice, dW_dt,
                   accumulate_dW, 0, ws, ws_bytes, stream, nullptr);
}

llamarl_status llamarl_offpolicy_loss_bwd_phases(const void* H, const void* W, const int32_t* targets,
                                                 const float* lse, const float* coef, float grad_loss, int64_t N,
                                                 int64_t d, int64_t V, llamarl_dtype dt, void* dH, void* dW,
                                                 llamarl_dtype dW_dt, int accumulate_dW, void* ws, size_t ws_bytes,
                                                 void* stream, void* const* phase_events) {
  if (!phase_events) return fail(LLAMARL_ERR_INVALID_ARG, "phase_events is null");
  for (int i = 0; i < 6; ++i)
    if (!phase_events[i]) return fail(LLAMARL_ERR_INVALID_ARG, "phase_events[%d] is null", i);
  return bwd_entry(H, W, targets, lse, coef, grad_loss, N, d, V, 0, dt, dH, dW, dW_dt, accumulate_dW, 0, ws, ws_bytes,
                   stream, phase_events);
}

llamarl_status llamarl_mfma_ceiling(int iters, float* sink, double* flops, void* stream) {
  if (!sink || !flops) return fail(LLAMARL_ERR_INVALID_ARG, "null pointer argument");
  if (iters <= 0) return fail(LLAMARL_ERR_INVALID_ARG, "iters must be positive");
  const int grid = persistent_grid((int64_t)1 << 30);      // one workgroup per CU
  k_mfma_ceiling<<<dim3((unsigned)grid), dim3(NTHREADS), 0, reinterpret_cast<hipStream_t>(stream)>>>(iters, sink);
  HIP_TRY(hipGetLastError());
  // 16x16x32 MFMA = 2 * 16 * 16 * 32 flop; MB x NB of them per k-step and wavefront
  *flops = (double)grid * (NTHREADS / 64) * (double)iters * CEILING_KSTEPS_PER_ITER * (MB * NB) * (2.0 * 16 * 16 * 32);
  return LLAMARL_OK;
}

llamarl_status llamarl_mfma_ceiling_traffic(int traffic, int iters, const void* panels, size_t panel_bytes,
                                            float* sink, double* flops, void* stream) {
  if (!sink || !flops || !panels) return fail(LLAMARL_ERR_INVALID_ARG, "null pointer argument");
  if (iters <= 0) return fail(LLAMARL_ERR_INVALID_ARG, "iters must be positive");
  if (traffic < 0 || traffic > 3) return fail(LLAMARL_ERR_INVALID_ARG, "traffic must be 0 .. 3");
  if (panel_bytes < CEILING_PANEL_BYTES || !aligned16(panels))
    return fail(LLAMARL_ERR_INVALID_ARG, "panels must be 16-byte aligned and hold %zu bytes (got %zu)",
                CEILING_PANEL_BYTES, panel_bytes);
  const int grid = persistent_grid((int64_t)1 << 30);      // one workgroup per CU
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  static const ceiling_traffic_kernel_t kernels[4] = {k_mfma_ceiling_schedule, k_mfma_ceiling_lds_reads,
                                                      k_mfma_ceiling_slab_loads, k_mfma_ceiling_reads_and_loads};
  const llamarl_status s = launch_ceiling_traffic(kernels[traffic], grid, iters, sink, panels, st);
  if (s != LLAMARL_OK) return s;
  *flops = (double)grid * (NTHREADS / 64) * (double)iters * CEILING_KSTEPS_PER_ITER * (MB * NB) * (2.0 * 16 * 16 * 32);
  return LLAMARL_OK;
}

llamarl_status llamarl_group_advantages(const float* rewards, int64_t P, int64_t n, int normalise_std, float eps,
                                        float* adv, void* stream) {
  if (!rewards || !adv) return fail(LLAMARL_ERR_INVALID_ARG, "null pointer argument");
  if (P <= 0 || n <= 0) return fail(LLAMARL_ERR_INVALID_ARG, "P and n must be positive");
  if (P >= ((int64_t)1 << 31) * 4) return fail(LLAMARL_ERR_UNSUPPORTED, "too many prompts");
  if (normalise_std && !(eps >= 0.f)) return fail(LLAMARL_ERR_INVALID_ARG, "eps must be non-negative");
  k_group_advantages<<<dim3((unsigned)((P + 3) / 4)), dim3(256), 0, reinterpret_cast<hipStream_t>(stream)>>>(
      rewards, P, n, normalise_std, eps, adv);
  HIP_TRY(hipGetLastError());
  return LLAMARL_OK;
}

llamarl_status llamarl_kl_shaped_rewards(const float* rewards, const float* logp, const float* base_logp,
                                         const uint8_t* mask, int64_t B, int64_t T, float lambda_kl, float* shaped,
                                         float* kl, void* stream) {
  if (!rewards || !logp || !base_logp || !shaped) return fail(LLAMARL_ERR_INVALID_ARG, "null pointer argument");
  if (B <= 0 || T <= 0) return fail(LLAMARL_ERR_INVALID_ARG, "B and T must be positive");
  if (B >= (int64_t)1 << 31) return fail(LLAMARL_ERR_UNSUPPORTED, "too many generations");
  if (!(lambda_kl == lambda_kl)) return fail(LLAMARL_ERR_INVALID_ARG, "lambda_kl is NaN");
  k_kl_shaped_rewards<<<dim3((unsigned)B), dim3(LOSS_THREADS), 0, reinterpret_cast<hipStream_t>(stream)>>>(
      rewards, logp, base_logp, mask, T, lambda_kl, shaped, kl);
  HIP_TRY(hipGetLastError());
  return LLAMARL_OK;
}

}  // extern "C"
