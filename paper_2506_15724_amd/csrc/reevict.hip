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

}  // namespace madakv
