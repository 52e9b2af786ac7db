// Budget allocation (paper Sec. 3.3): Eq. 10-11 layer compensation in integers, then the
// Eq. 8 modality split per head.
//
// One wavefront per batch item, one lane per KV head (H <= 64), layers in sequence.
// The recurrence phi^{l+1} = phi^l - K^l / (layers left) is carried as an integer pool R of
// candidate tokens for all remaining layers and heads: nominal per-head budget
// phi^l = R / (H * rem).  A head's demand is its Eq. 9 count k_t + k_v clamped to
// [phi/rho, rho*phi]; the layer draws the sum of demands, clamped so that every later layer
// can still get between beta_floor and n_cand tokens per head; the last layer draws what is
// left.  Heads share the layer total by largest remainder (ties to the lower head), scaled
// by demand when it has to shrink and by head-room when it has to grow.  All cross-head
// sums and ranks are wavefront shuffles; arithmetic is 64-bit integer except the double
// multiply (and, with more than two modalities, the subtraction) of the Eq. 8 share.  Those
// must round after every operation, as the reference arithmetic does: a fused multiply-add
// keeps the exact product and changes which of two nearly equal fractional parts is the
// larger, so contraction is switched off for this file.
#include "common.h"
#include "mpa_split.h"

#pragma clang fp contract(off)

namespace madakv {

struct AllocArgs {
  const void* stats; const int32_t* n_mod; int32_t* budgets; long long* pool;
  int n, B, H, NL, layer0, nc, beta, rho, mpa_mode, hcc_mode, keep_all, M;
};

// +1 for the `extra` lanes with the largest remainder (ties: lower lane first).
__device__ __forceinline__ long long largest_remainder(long long base, long long rem, long long extra,
                                                        int lane, int H) {
  int rank = 0;
  for (int o = 0; o < H; ++o) {
    long long ro = shfl_i64(rem, o);
    if (lane < H && (ro > rem || (ro == rem && o < lane))) ++rank;
  }
  return base + ((long long)rank < extra ? 1 : 0);
}

__global__ __launch_bounds__(64) void allocate_kernel(AllocArgs a) {
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const bool act = lane < a.H;
  constexpr int MAXM = 4;
  const int M = a.M;
  long long nm[MAXM];
#pragma unroll
  for (int m = 0; m < MAXM; ++m) nm[m] = m < M ? a.n_mod[b * M + m] : 0;
  const long long H = a.H, nc = a.nc, rho = a.rho, beta = a.beta;
  long long R = (a.layer0 == 0) ? (long long)a.NL * H * beta : a.pool[b];
  long long bf = beta / (rho * rho);
  if (bf < 1) bf = 1;

  for (int li = 0; li < a.n; ++li) {
    const int l = a.layer0 + li;
    const long long idx = ((long long)li * a.B + b) * a.H + lane;
    // the head's record: M float masses (Eq. 6) then M int32 counts (Eq. 9)
    float wm[MAXM]; long long km = 0;
    const float* rec = reinterpret_cast<const float*>(a.stats) + idx * 2 * M;
#pragma unroll
    for (int m = 0; m < MAXM; ++m) {
      wm[m] = (act && m < M) ? rec[m] : 0.f;
      if (act && m < M) km += reinterpret_cast<const int32_t*>(rec)[M + m];
    }
    long long ah;
    if (a.keep_all) {
#pragma unroll
      for (int m = 0; m < MAXM; ++m) if (act && m < M) a.budgets[idx * M + m] = (int32_t)nm[m];
      continue;
    }
    if (!a.hcc_mode) {
      ah = beta;
    } else {
      const long long rem = a.NL - l;
      long long lo = (R + rho * H * rem - 1) / (rho * H * rem);
      if (lo < 1) lo = 1;
      long long hi = (rho * R) / (H * rem);
      if (hi > nc) hi = nc;
      long long dem = km;
      dem = dem < lo ? lo : (dem > hi ? hi : dem);
      if (!act) dem = 0;
      const long long D = wave_sum_i64(dem);
      long long A;
      if (rem == 1) {
        A = R;
      } else {
        const long long amin = R - (rem - 1) * H * nc, amax = R - (rem - 1) * H * bf;
        A = D < amin ? amin : (D > amax ? amax : D);
      }
      if (a.hcc_mode == 2) {
        // Eq. 8 as printed: one budget per layer; the A mod H spare tokens go to the lowest heads
        ah = A / H + (lane < A % H ? 1 : 0);
      } else if (A == D) {
        ah = dem;
      } else if (A < D) {
        const long long num = A * dem;
        const long long base = num / D, r = num % D;
        const long long extra = A - wave_sum_i64(act ? base : 0);
        ah = largest_remainder(base, act ? r : -1, extra, lane, a.H);
      } else {
        const long long room = act ? nc - dem : 0;
        const long long S = A - D, Rm = wave_sum_i64(room);
        const long long num = S * room;
        const long long base = num / Rm, r = num % Rm;
        const long long extra = S - wave_sum_i64(act ? base : 0);
        ah = dem + largest_remainder(base, act ? r : -1, extra, lane, a.H);
      }
      R -= A;
    }
    if (act) {
      long long bm[MAXM];
      mpa_split_device(ah, wm, nm, M, a.mpa_mode, bm);
      for (int m = 0; m < M; ++m) a.budgets[idx * M + m] = (int32_t)bm[m];
    }
  }
  if (lane == 0 && !a.keep_all) a.pool[b] = R;
}

hipError_t launch_allocate(const Dims& dm, const madakv_config& c, int layer0, const void* stats,
                           const int32_t* n_mod, int32_t* budgets, long long* pool_state, hipStream_t st) {
  AllocArgs a;
  a.M = c.n_modalities;
  a.stats = stats; a.n_mod = n_mod; a.budgets = budgets; a.pool = pool_state;
  a.n = dm.n; a.B = dm.B; a.H = dm.H; a.NL = c.n_layers; a.layer0 = layer0; a.nc = dm.nc;
  a.beta = c.budget - c.window; a.rho = c.hcc_rho; a.mpa_mode = c.mpa_mode; a.hcc_mode = c.hcc_mode;
  a.keep_all = c.budget >= c.ctx_len ? 1 : 0;
  hipLaunchKernelGGL(allocate_kernel, dim3(dm.B), dim3(64), 0, st, a);
  return hipGetLastError();
}

}  // namespace madakv
