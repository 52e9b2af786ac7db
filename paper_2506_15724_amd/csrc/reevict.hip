// Re-eviction during generation (the long-generation outlook of the paper's Sec. 6; the method itself,
// Sec. 3.3, evicts once after the prefill).  After T decode steps a head's segment of the reduced cache
// holds its kept rows, the W window rows and T appended rows.  Re-eviction brings it back to the size
// the prompt eviction gave it: the last W rows become the new proxy set (their queries are the caller's
// most recent W queries), every earlier row is a candidate again, scored against the new proxies
// (Eq. 7 over the rows of the cache), the head's total of Eq. 9-11 stays what it was, its split over
// the modalities follows the current masses (Eq. 6, Eq. 8; generated tokens are text), and the
// best-scored candidates per modality survive (ties: lower row).  Everything is per head: nothing
// couples heads or layers here.
//
//   restats_kernel   per head: modality of every row (from the row's original position: a prompt
//                    position looks up the modality mask, a generated token is text), masses and counts
//                    over the candidates, pooled scores, then the Eq. 8 split of the unchanged total
//   (the one-sweep scoring kernel and the selection kernel run on the ragged segments in between)
//   compact_kernel   per head: rows sel[0] < sel[1] < ... move down to rows 0, 1, ... inside the
//                    head's own segment, K, V and the original positions alike; sel[j] >= j, so
//                    batches of rows, read completely before any is written, never overwrite a row
//                    that is still to be read
#include "common.h"

#include <algorithm>
#include "mpa_split.h"

namespace madakv {

constexpr int RE_THREADS = 256;
constexpr float RE_FX_SCALE = 17592186044416.0f;    // 2^44, the fixed-point unit of the statistics kernel
constexpr float RE_PSI_MAX = 256.0f;

struct RestatsArgs {
  const float* psi; const int32_t* kept_idx; const uint8_t* mask; const int64_t* seg_off; const int32_t* seg_len;
  float* psi_pool; uint8_t* rowmod; void* stats; int32_t* budgets;
  int B, H, L, W, M, appended, pool_r, pool_mode, share_mode, mpa_mode;
};

__device__ __forceinline__ unsigned long long re_to_fx(float v) {
  v = fminf(fmaxf(v, 0.f), RE_PSI_MAX);
  return __float2ull_rn(v * RE_FX_SCALE);
}

__global__ __launch_bounds__(RE_THREADS) void restats_kernel(RestatsArgs a) {
  __shared__ unsigned long long s_w[4];
  __shared__ unsigned int s_n[4];
  const int tid = threadIdx.x;
  const int head = blockIdx.x;
  const int b = (head / a.H) % a.B;
  const int len = a.seg_len[head];
  if (len <= 0) return;                                     // an empty segment stays empty
  const long long off = a.seg_off[head];
  const int len0 = len - a.appended;                        // rows before the appended ones: they have original positions
  const int nc = len - a.W;                                 // candidates: everything before the new window
  if (tid < 4) { s_w[tid] = 0ULL; s_n[tid] = 0u; }
  __syncthreads();
  unsigned long long wl[4] = {0ULL, 0ULL, 0ULL, 0ULL};
  unsigned int nl[4] = {0u, 0u, 0u, 0u};
  for (int i = tid; i < len; i += RE_THREADS) {
    int m = 0;                                              // generated tokens are text
    if (i < len0) {
      const int origin = a.kept_idx[off + i];
      if (origin < a.L) m = min((int)a.mask[(long long)b * a.L + origin], a.M - 1);
    }
    a.rowmod[off + i] = (uint8_t)m;
    const float v = a.psi[off + i];
    if (i < nc || a.share_mode) {
      const unsigned long long fx = re_to_fx(v);
#pragma unroll
      for (int j = 0; j < 4; ++j) wl[j] += (m == j) ? fx : 0ULL;
    }
    if (i < nc) {
#pragma unroll
      for (int j = 0; j < 4; ++j) nl[j] += (m == j) ? 1u : 0u;
      // pooled score over the neighbouring rows of the cache, clipped at the candidate range
      const int lo = max(i - a.pool_r, 0), hi = min(i + a.pool_r, nc - 1);
      float acc = a.pool_mode ? 0.f : v;
      for (int j = lo; j <= hi; ++j) acc = a.pool_mode ? acc + a.psi[off + j] : fmaxf(acc, a.psi[off + j]);
      a.psi_pool[off + i] = a.pool_mode ? acc / (float)(hi - lo + 1) : acc;
    }
  }
  // integer sums: the order of the additions does not matter
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const unsigned long long ws = (unsigned long long)wave_sum_i64((long long)wl[j]);
    const unsigned int ns = (unsigned int)wave_sum_i64((long long)nl[j]);
    if ((tid & 63) == 0) { atomicAdd(&s_w[j], ws); atomicAdd(&s_n[j], ns); }
  }
  __syncthreads();
  if (tid == 0) {
    float wm[4]; long long nm[4], bm[4];
    for (int j = 0; j < 4; ++j) {
      wm[j] = j < a.M ? (float)((double)s_w[j] * (1.0 / (double)RE_FX_SCALE)) : 0.f;
      nm[j] = j < a.M ? (long long)s_n[j] : 0;
    }
    float* rec = reinterpret_cast<float*>(a.stats) + (long long)head * 2 * a.M;   // {float w[M]; int32 n[M]}
    for (int j = 0; j < a.M; ++j) { rec[j] = wm[j]; reinterpret_cast<int32_t*>(rec)[a.M + j] = (int32_t)nm[j]; }
    const long long ah = min((long long)(len0 - a.W), (long long)nc);   // the head's total of the prompt eviction
    mpa_split_device(ah, wm, nm, a.M, a.mpa_mode, bm);
    for (int j = 0; j < a.M; ++j) a.budgets[(long long)head * a.M + j] = (int32_t)bm[j];
  }
}

typedef __attribute__((ext_vector_type(4))) unsigned int ru32x4_t;

struct CompactArgs {
  void* k_c; void* v_c; int32_t* kept_idx; const int32_t* sel; const int64_t* seg_off; int32_t* kv_len; const int32_t* budgets;
  int W, M, L, appended, gen_base;
};

template <int LPR>   // 16-byte pieces per row
__global__ __launch_bounds__(RE_THREADS) void compact_kernel(CompactArgs a) {
  constexpr int RPI = RE_THREADS / LPR;          // rows the workgroup moves per instruction
  constexpr int UN = 4;
  constexpr int BATCH = RPI * UN;
  const int tid = threadIdx.x;
  const int head = blockIdx.x;
  const int len = a.kv_len[head];
  if (len <= 0) return;
  const long long off = a.seg_off[head];
  const int len0 = len - a.appended;
  int keep = a.W;
  for (int m = 0; m < a.M; ++m) keep += a.budgets[(long long)head * a.M + m];
  const int sub = tid / LPR, piece = tid % LPR;
  ru32x4_t* kc = reinterpret_cast<ru32x4_t*>(a.k_c);
  ru32x4_t* vc = reinterpret_cast<ru32x4_t*>(a.v_c);
  for (int j0 = 0; j0 < keep; j0 += BATCH) {
    ru32x4_t kr[UN], vr[UN];
    int org[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int j = j0 + u * RPI + sub;
      const int src = j < keep ? a.sel[off + j] : 0;
      kr[u] = kc[(off + src) * LPR + piece];
      vr[u] = vc[(off + src) * LPR + piece];
      // original position: prompt rows and earlier generated rows carry theirs; rows appended since the
      // last (re-)eviction are generated tokens gen_base, gen_base + 1, ... after the prompt
      org[u] = src < len0 ? a.kept_idx[off + src] : a.L + a.gen_base + (src - len0);
    }
    __syncthreads();                              // every row of the batch is in registers before any is overwritten
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int j = j0 + u * RPI + sub;
      if (j < keep) {
        kc[(off + j) * LPR + piece] = kr[u];
        vc[(off + j) * LPR + piece] = vr[u];
        if (piece == 0) a.kept_idx[off + j] = org[u];
      }
    }
  }
  if (tid == 0) a.kv_len[head] = keep;
}

hipError_t launch_restats(const Dims& dm, const madakv_config& c, const float* psi_c, const int32_t* kept_idx, const uint8_t* mask,
                          const int64_t* seg_off, const int32_t* seg_len, int appended, float* pool_c, uint8_t* rowmod,
                          void* stats, int32_t* budgets, hipStream_t st) {
  RestatsArgs a;
  a.psi = psi_c; a.kept_idx = kept_idx; a.mask = mask; a.seg_off = seg_off; a.seg_len = seg_len; a.psi_pool = pool_c;
  a.rowmod = rowmod; a.stats = stats; a.budgets = budgets;
  a.B = dm.B; a.H = dm.H; a.L = dm.L; a.W = dm.W; a.M = c.n_modalities; a.appended = appended;
  a.pool_r = (c.pool_k - 1) / 2; a.pool_mode = c.pool_mode; a.share_mode = c.share_mode; a.mpa_mode = c.mpa_mode;
  hipLaunchKernelGGL(restats_kernel, dim3(dm.heads), dim3(RE_THREADS), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_compact(const Dims& dm, const madakv_config& c, void* k_c, void* v_c, int32_t* kept_idx, const int32_t* sel,
                          const int64_t* seg_off, int32_t* kv_len, const int32_t* budgets, int appended, int gen_base, hipStream_t st) {
  CompactArgs a;
  a.k_c = k_c; a.v_c = v_c; a.kept_idx = kept_idx; a.sel = sel; a.seg_off = seg_off; a.kv_len = kv_len; a.budgets = budgets;
  a.W = dm.W; a.M = c.n_modalities; a.L = dm.L; a.appended = appended; a.gen_base = gen_base;
  const int lpr = dm.d * (c.cache_fp8 ? 1 : (c.dtype == MADAKV_BF16 ? 2 : 4)) / 16;     // 16-byte pieces per cached row
  if (lpr == 4) hipLaunchKernelGGL((compact_kernel<4>), dim3(dm.heads), dim3(RE_THREADS), 0, st, a);
  else if (lpr == 8) hipLaunchKernelGGL((compact_kernel<8>), dim3(dm.heads), dim3(RE_THREADS), 0, st, a);
  else if (lpr == 16) hipLaunchKernelGGL((compact_kernel<16>), dim3(dm.heads), dim3(RE_THREADS), 0, st, a);
  else if (lpr == 32) hipLaunchKernelGGL((compact_kernel<32>), dim3(dm.heads), dim3(RE_THREADS), 0, st, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// ---- paged reduced cache ------------------------------------------------------------------------------
// A head's rows are its initial pages (which follow each other at kv_off) and pages taken later from the
// top of the batch item's region, listed in its table.  Re-eviction works on a linear copy: the rows of
// every head are laid end to end in the workspace (linear_offsets_kernel, linear_copy_kernel: as many rows
// as the cache itself holds), the kernels above run on that copy
// as they run on contiguous segments, and the surviving rows, never more than the initial pages hold, go
// back to the head's initial pages (write_back_kernel).  The pages taken since are free again afterwards:
// the call covers all layers, so the pools start over (pool_reset_kernel).
struct LinearArgs {
  ru32x4_t* k_c; ru32x4_t* v_c; int32_t* kept_idx;          // the paged cache
  ru32x4_t* k_lin; ru32x4_t* v_lin; int32_t* kept_lin;      // the linear copy: head i at rows [lin_off[i], + its length)
  int64_t* lin_off;                                         // [heads] running sum of the lengths (linear_offsets_kernel)
  const int64_t* seg_off; const int32_t* seg_len; const int32_t* page_tbl;
  int entries, shift, lpr;                                  // table entries per head, log2(page rows), 16-byte pieces per row
  int heads;
};
constexpr int LIN_ROWS = 64;                                // rows per workgroup

// lin_off[i] = sum of the lengths of the heads before i: one workgroup, every thread a stretch of consecutive heads
__global__ __launch_bounds__(1024) void linear_offsets_kernel(LinearArgs a) {
  __shared__ long long s_sum[1024];
  const int tid = threadIdx.x;
  const int per = (a.heads + 1023) / 1024;
  const int h0 = min(tid * per, a.heads), h1 = min(h0 + per, a.heads);
  long long mine = 0;
  for (int h = h0; h < h1; ++h) mine += max(a.seg_len[h], 0);
  s_sum[tid] = mine;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {                     // inclusive scan of the stretches' sums
    const long long add = tid >= o ? s_sum[tid - o] : 0;
    __syncthreads();
    s_sum[tid] += add;
    __syncthreads();
  }
  long long run = s_sum[tid] - mine;
  for (int h = h0; h < h1; ++h) { a.lin_off[h] = run; run += max(a.seg_len[h], 0); }
}

__global__ __launch_bounds__(RE_THREADS) void linear_copy_kernel(LinearArgs a) {
  const int head = blockIdx.y, tid = threadIdx.x;
  const int len = a.seg_len[head];
  const int r0 = blockIdx.x * LIN_ROWS;
  if (r0 >= len) return;
  const long long off = a.seg_off[head];
  const int32_t* tbl = a.page_tbl + (long long)head * a.entries;
  const int init_rows = tbl[0] << a.shift;
  const int rows = min(LIN_ROWS, len - r0);
  for (int e = tid; e < rows * a.lpr; e += RE_THREADS) {
    const int r = r0 + e / a.lpr, piece = e % a.lpr;
    long long src = off + r;
    if (r >= init_rows) { const int q = r - init_rows; src = ((long long)tbl[1 + (q >> a.shift)] << a.shift) + (q & ((1 << a.shift) - 1)); }
    const long long dst = a.lin_off[head] + r;
    a.k_lin[dst * a.lpr + piece] = __builtin_nontemporal_load(a.k_c + src * a.lpr + piece);
    a.v_lin[dst * a.lpr + piece] = __builtin_nontemporal_load(a.v_c + src * a.lpr + piece);
    if (piece == 0) a.kept_lin[dst] = r < init_rows ? a.kept_idx[src] : 0;   // (rows in later pages are generated tokens: their positions are computed)
  }
}

__global__ __launch_bounds__(RE_THREADS) void write_back_kernel(LinearArgs a) {
  const int head = blockIdx.y, tid = threadIdx.x;
  const int len = a.seg_len[head];                          // the length after compaction
  const int r0 = blockIdx.x * LIN_ROWS;
  if (r0 >= len) return;
  const long long off = a.seg_off[head];
  const int rows = min(LIN_ROWS, len - r0);
  for (int e = tid; e < rows * a.lpr; e += RE_THREADS) {
    const int r = r0 + e / a.lpr, piece = e % a.lpr;
    const long long src = a.lin_off[head] + r, dst = off + r;
    a.k_c[dst * a.lpr + piece] = a.k_lin[src * a.lpr + piece];
    a.v_c[dst * a.lpr + piece] = a.v_lin[src * a.lpr + piece];
    if (piece == 0) a.kept_idx[dst] = a.kept_lin[src];
  }
}

__global__ __launch_bounds__(256) void pool_reset_kernel(unsigned long long* pool_top, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) pool_top[i] = 0ULL;
}

// longest: at least the length of the longest head of the call (sizes the grids).  back = false: the copy (and the
// heads' offsets in it); true: the first seg_len rows of every head's copy go back to its initial pages
hipError_t launch_linear_copy(const Dims& dm, const madakv_config& c, void* k_c, void* v_c, int32_t* kept_idx, const int64_t* seg_off,
                              const int32_t* seg_len, const Paging& pg, long long head0, int longest, void* k_lin, void* v_lin,
                              int32_t* kept_lin, int64_t* lin_off, bool back, hipStream_t st) {
  LinearArgs a;
  a.k_c = static_cast<ru32x4_t*>(k_c); a.v_c = static_cast<ru32x4_t*>(v_c); a.kept_idx = kept_idx;
  a.k_lin = static_cast<ru32x4_t*>(k_lin); a.v_lin = static_cast<ru32x4_t*>(v_lin); a.kept_lin = kept_lin; a.lin_off = lin_off;
  a.seg_off = seg_off; a.seg_len = seg_len; a.page_tbl = pg.table + head0 * pg.entries;
  a.entries = pg.entries; a.shift = 0;
  while ((1 << a.shift) < pg.page_rows) ++a.shift;
  a.lpr = dm.d * (c.cache_fp8 ? 1 : (c.dtype == MADAKV_BF16 ? 2 : 4)) / 16;
  a.heads = dm.heads;
  const dim3 grid((unsigned)((std::max(longest, 1) + LIN_ROWS - 1) / LIN_ROWS), dm.heads);
  if (back) {
    hipLaunchKernelGGL(write_back_kernel, grid, dim3(RE_THREADS), 0, st, a);
  } else {
    hipLaunchKernelGGL(linear_offsets_kernel, dim3(1), dim3(1024), 0, st, a);
    hipLaunchKernelGGL(linear_copy_kernel, grid, dim3(RE_THREADS), 0, st, a);
  }
  return hipGetLastError();
}

hipError_t launch_pool_reset(const Paging& pg, int batch, hipStream_t st) {
  hipLaunchKernelGGL(pool_reset_kernel, dim3((batch + 255) / 256), dim3(256), 0, st, pg.pool_top, batch);
  return hipGetLastError();
}

}  // namespace madakv
