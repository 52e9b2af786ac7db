// Per-head modality statistics over the candidates [0, L-W) (paper Sec. 3.3):
//   Eq. 6  w_t, w_v   attention mass on text / image candidates
//   Eq. 9  k_t, k_v   fewest top-scored tokens of a modality that cover theta of its mass
// plus the max-pooled scores used for ranking, and the candidate counts per modality.
//
// One workgroup per (layer, batch, KV head).  Masses are summed in 64-bit fixed point
// (2^-44 units; a head's scores sum to G*W <= 256, so the total stays below 2^52): integer
// adds commute, so LDS atomics give the same bits on every run
// and the counts k_m, which are integers decided by a mass threshold, are reproducible.
// k_m is found without sorting by a radix descent on the float bit pattern (11 + 11 + 9
// bits): each level histograms count and mass per bin for the elements that match the
// prefix found so far and walks the bins from the top to the one where the running
// mass crosses theta * w_m; the last level pins the threshold value tau exactly, and
//   k_m = #{psi > tau} + ceil((theta w_m - mass{psi > tau}) / tau).
#include "common.h"


namespace madakv {

constexpr int STATS_THREADS = 512;
constexpr int STATS_EPT = 32;                    // consecutive candidates a thread owns per chunk
constexpr int BINS = 2048;
constexpr float FX_SCALE = 17592186044416.0f;    // 2^44
constexpr float PSI_MAX = 256.0f;                // G * W <= 256 bounds any column sum
constexpr int SPLIT_MAX_HEADS = 128;             // most heads of a launch whose chunks get workgroups of their own

// what the walk of one level hands to the next, per head and modality (phases 1 and 2)
struct StatsCarry {
  unsigned long long sum_gt, w, target, binsum, wwin;
  uint32_t prefix, cnt_gt, n, done, bincnt, pad;
};

struct StatsArgs {
  const float* psi; const uint8_t* mask; float* psi_pool; void* stats; int32_t* n_mod;
  int B, H, L, W, nc, pool_r, pool_mode, share_mode, M;
  double theta;
  // Long heads on few heads (see launch_stats): the chunks of a head go to workgroups of their own.
  // phase 0 = the whole head in one workgroup, all levels; 1 = histogram of one chunk at `level`, added
  // to the head's histogram in memory; 2 = the walk over that histogram (one workgroup per head).
  int phase, level, heads;
  unsigned long long* gsum; uint32_t* gcnt;      // [3 levels][heads][M][BINS]
  StatsCarry* carry;                             // [heads][4]
};

__device__ __forceinline__ unsigned long long to_fx(float v) {
  v = fminf(fmaxf(v, 0.f), PSI_MAX);
  return __float2ull_rn(v * FX_SCALE);            // exact product (power of two); exact integer for v >= 2^-21
}
__device__ __forceinline__ uint32_t nonneg_bits(float v) {
  v = fminf(fmaxf(v, 0.f), PSI_MAX);
  return __float_as_uint(v);                      // non-negative floats order like their bit patterns
}

typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

// Ownership inside a chunk of STATS_THREADS * STATS_EPT candidates: thread t owns the groups of four
// consecutive candidates number j * STATS_THREADS + t, j = 0 .. STATS_EPT / 4 - 1, so that a wave's
// loads and stores cover whole cache lines.  Element e = 4 j + q of the thread is candidate
// cbase + 4 (j * STATS_THREADS + t) + q.  Values and modality bits stay in registers through the three
// levels when the head fits one chunk (16384 candidates).
constexpr int STATS_GROUPS = STATS_EPT / 4;
constexpr int POOL_R_REG = 3;                    // widest pooling half-width served from registers
__device__ __forceinline__ int owned_start(int cbase, int tid, int j) { return cbase + 4 * (j * STATS_THREADS + tid); }

// Also fetches, for the first and the last lane of a wave, the POOL_R_REG values before / after each of
// its groups (the other lanes get theirs from the neighbouring lanes): edge[j][r] = psi[i - 3 + r] in
// lane 0, psi[i + 4 + r] in lane 63, where i is the group's first candidate.
__device__ __forceinline__ void load_owned(const float* psi, const uint8_t* mask, int cbase, int tid, int nc, int M, bool want_edges,
                                           float (&v)[STATS_EPT], unsigned long long& mbits, float (&edge)[STATS_GROUPS][POOL_R_REG]) {
  const bool al = (reinterpret_cast<uintptr_t>(psi + cbase) & 15u) == 0;
  const bool alm = (reinterpret_cast<uintptr_t>(mask + cbase) & 3u) == 0;
  const int lane = tid & 63;
  const uint32_t top = (uint32_t)(M - 1);
  uint32_t mw[STATS_GROUPS];
#pragma unroll
  for (int j = 0; j < STATS_GROUPS; ++j) {
    const int i = owned_start(cbase, tid, j);
    if (al && i + 4 <= nc) {
      const f32x4_t x = *reinterpret_cast<const f32x4_t*>(psi + i);
      v[j * 4 + 0] = x[0]; v[j * 4 + 1] = x[1]; v[j * 4 + 2] = x[2]; v[j * 4 + 3] = x[3];
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) v[j * 4 + q] = (i + q < nc) ? psi[i + q] : 0.f;
    }
    if (alm && i + 4 <= nc) mw[j] = *reinterpret_cast<const uint32_t*>(mask + i);
    else {
      mw[j] = 0u;
#pragma unroll
      for (int q = 0; q < 4; ++q) if (i + q < nc) mw[j] |= (uint32_t)mask[i + q] << (8 * q);
    }
    if (want_edges) {
#pragma unroll
      for (int r = 0; r < POOL_R_REG; ++r) {
        float x = 0.f;
        const int il = i - POOL_R_REG + r, ir = i + 4 + r;
        if (lane == 0 && il >= 0 && il < nc) x = psi[il];
        if (lane == 63 && ir < nc) x = psi[ir];
        edge[j][r] = x;
      }
    }
  }
  // modality ids, two bits per element (ids above the last modality count as the last one)
  mbits = 0ULL;
#pragma unroll
  for (int j = 0; j < STATS_GROUPS; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      mbits |= (unsigned long long)min((mw[j] >> (8 * q)) & 0xffu, top) << (2 * (j * 4 + q));
}

// pooling of half-width R <= POOL_R_REG over the candidates: a group's neighbours come from the lanes
// next to it (from memory at the ends of a wave); positions outside [0, nc) do not take part
template <int R, int AVG>
__device__ __forceinline__ void pool_owned(float* pool, int cbase, int tid, int nc, const float (&v)[STATS_EPT],
                                           const float (&edge)[STATS_GROUPS][POOL_R_REG]) {
  const float none = AVG ? 0.f : -__builtin_inff();          // what a position outside [0, nc) contributes
  const int lane = tid & 63;
  const bool alp = (reinterpret_cast<uintptr_t>(pool + cbase) & 15u) == 0;
#pragma unroll
  for (int j = 0; j < STATS_GROUPS; ++j) {
    const int i = owned_start(cbase, tid, j);
    float ext[4 + 2 * POOL_R_REG];
#pragma unroll
    for (int r = 0; r < POOL_R_REG; ++r) {
      // (all lanes take part in the shuffles; what is not needed for this R is dropped by the compiler)
      const float fl = __shfl_up(v[j * 4 + 1 + r], 1, 64);                 // previous lane's elements 1, 2, 3
      const float fr = __shfl_down(v[j * 4 + r], 1, 64);                   // next lane's elements 0, 1, 2
      const int il = i - POOL_R_REG + r, ir = i + 4 + r;
      const float xl = lane == 0 ? edge[j][r] : fl;
      const float xr = lane == 63 ? edge[j][r] : fr;
      ext[r] = (il >= 0 && il < nc) ? xl : none;
      ext[POOL_R_REG + 4 + r] = (ir < nc) ? xr : none;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) ext[POOL_R_REG + q] = (i + q < nc) ? v[j * 4 + q] : none;
    float o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (AVG) {
        float sm = 0.f;                                          // left to right over the clipped neighbourhood
#pragma unroll
        for (int r = -R; r <= R; ++r) sm += ext[POOL_R_REG + q + r];
        const int ii = i + q;
        const int cntw = min(ii + R, nc - 1) - max(ii - R, 0) + 1;
        o[q] = sm / (float)cntw;
      } else {
        float mx = ext[POOL_R_REG + q];
#pragma unroll
        for (int r = 1; r <= R; ++r) mx = fmaxf(mx, fmaxf(ext[POOL_R_REG + q - r], ext[POOL_R_REG + q + r]));
        o[q] = mx;
      }
    }
    if (alp && i + 4 <= nc) {
      f32x4_t x = {o[0], o[1], o[2], o[3]};
      *reinterpret_cast<f32x4_t*>(pool + i) = x;
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) if (i + q < nc) pool[i + q] = o[q];
    }
  }
}

template <int MM>   // modalities the kernel is built for (2 or 4)
__global__ __launch_bounds__(STATS_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) void stats_kernel(StatsArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char stats_smem[];
  unsigned long long* sum = reinterpret_cast<unsigned long long*>(stats_smem);      // [M][BINS] masses
  uint32_t* cnt = reinterpret_cast<uint32_t*>(sum + (size_t)a.M * BINS);             // [M][BINS] counts
  __shared__ uint32_t s_prefix[MM], s_cnt_gt[MM], s_n[MM], s_done[MM], s_bincnt[MM];
  __shared__ unsigned long long s_sum_gt[MM], s_w[MM], s_target[MM], s_binsum[MM], s_wwin[MM];
  const int M = a.M;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int phase = a.phase;
  const int head = phase == 1 ? blockIdx.y : blockIdx.x;      // phase 1: grid (chunks, heads)
  const int b = (head / a.H) % a.B;
  const float* psi = a.psi + (long long)head * a.L;
  const uint8_t* mask = a.mask + (long long)b * a.L;
  float* pool = a.psi_pool + (long long)head * a.nc;

  const int shifts[3] = {20, 9, 0};
  const int widths[3] = {11, 11, 9};
  constexpr int CH = STATS_THREADS * STATS_EPT;
  const int nchunks = (a.nc + CH - 1) / CH;
  const int c_first = phase == 1 ? blockIdx.x : 0, c_end = phase == 1 ? blockIdx.x + 1 : nchunks;
  const bool single = c_end - c_first == 1;      // the workgroup's candidates stay in registers through its levels
  const int lv_first = phase == 0 ? 0 : a.level, lv_end = phase == 0 ? 3 : a.level + 1;
  const size_t hist_words = (size_t)M * BINS;
  unsigned long long* gsum = phase ? a.gsum + ((size_t)a.level * a.heads + head) * hist_words : nullptr;
  uint32_t* gcnt = phase ? a.gcnt + ((size_t)a.level * a.heads + head) * hist_words : nullptr;
  StatsCarry* carry = phase ? a.carry + (size_t)head * 4 : nullptr;

  if (tid < MM) s_wwin[tid] = 0ULL;
  if (phase != 0 && a.level > 0 && tid < M) {    // what the walk of the level above left
    const StatsCarry cy = carry[tid];
    s_prefix[tid] = cy.prefix; s_cnt_gt[tid] = cy.cnt_gt; s_n[tid] = cy.n; s_done[tid] = cy.done; s_bincnt[tid] = cy.bincnt;
    s_sum_gt[tid] = cy.sum_gt; s_w[tid] = cy.w; s_target[tid] = cy.target; s_binsum[tid] = cy.binsum; s_wwin[tid] = cy.wwin;
  }
  __syncthreads();
  if (a.share_mode && tid < a.W && (phase == 0 || (phase == 2 && a.level == 0))) {
    // the other reading of Eq. 6: the proxy columns count towards the masses as well
    const int i = a.nc + tid;
    atomicAdd(&s_wwin[min((int)mask[i], M - 1)], to_fx(psi[i]));
  }
  float v[STATS_EPT];
  unsigned long long mbits = 0ULL;
  const bool reg_pool = a.pool_r <= POOL_R_REG;
  float edge[STATS_GROUPS][POOL_R_REG];
  if (single && phase != 2) load_owned(psi, mask, c_first * CH, tid, a.nc, M, reg_pool && lv_first == 0, v, mbits, edge);

  for (int level = lv_first; level < lv_end; ++level) {
    for (int e = tid; e < M * BINS; e += STATS_THREADS) { cnt[e] = 0; sum[e] = 0ULL; }
    __syncthreads();
    const int sh = shifts[level], wd = widths[level];
    const uint32_t binmask = (1u << wd) - 1u;
    uint32_t pfx[MM]; bool dn[MM];
#pragma unroll
    for (int m = 0; m < MM; ++m) { pfx[m] = (level > 0 && m < M) ? s_prefix[m] : 0u; dn[m] = (level > 0 && m < M) ? s_done[m] != 0 : false; }
    if (phase == 2) {                              // the head's histogram of this level, gathered by the chunks' workgroups
      for (int e = tid; e < M * BINS; e += STATS_THREADS) { cnt[e] = gcnt[e]; sum[e] = gsum[e]; }
    }
    for (int c = (phase == 2 ? c_end : c_first); c < c_end; ++c) {
      const int cbase = c * CH;
      if (!single) load_owned(psi, mask, cbase, tid, a.nc, M, level == 0 && reg_pool, v, mbits, edge);
      if (level == 0) {
        // pooled scores for ranking (raw values): windows up to 7 from registers, wider ones the slow way
        switch (a.pool_r + (a.pool_mode ? 100 : 0)) {
          case 0: case 100: pool_owned<0, 0>(pool, cbase, tid, a.nc, v, edge); break;
          case 1: pool_owned<1, 0>(pool, cbase, tid, a.nc, v, edge); break;
          case 2: pool_owned<2, 0>(pool, cbase, tid, a.nc, v, edge); break;
          case 3: pool_owned<3, 0>(pool, cbase, tid, a.nc, v, edge); break;
          case 101: pool_owned<1, 1>(pool, cbase, tid, a.nc, v, edge); break;
          case 102: pool_owned<2, 1>(pool, cbase, tid, a.nc, v, edge); break;
          case 103: pool_owned<3, 1>(pool, cbase, tid, a.nc, v, edge); break;
          default:
            for (int g = 0; g < STATS_GROUPS; ++g)
              for (int q = 0; q < 4; ++q) {
                const int i = owned_start(cbase, tid, g) + q;
                if (i >= a.nc) continue;
                const int lo = max(i - a.pool_r, 0), hi = min(i + a.pool_r, a.nc - 1);
                float acc = a.pool_mode ? 0.f : psi[i];
                for (int j = lo; j <= hi; ++j) acc = a.pool_mode ? acc + psi[j] : fmaxf(acc, psi[j]);
                pool[i] = a.pool_mode ? acc / (float)(hi - lo + 1) : acc;
              }
        }
      }
#pragma unroll
      for (int e = 0; e < STATS_EPT; ++e) {
        const int m = (int)((mbits >> (2 * e)) & 3ULL);
        const uint32_t key = nonneg_bits(v[e]);
        bool match = owned_start(cbase, tid, e >> 2) + (e & 3) < a.nc;
        // (the per-modality state is picked with selects: indexing a register array by m would spill it)
        uint32_t pm = pfx[0]; bool dm_ = dn[0];
#pragma unroll
        for (int j = 1; j < MM; ++j) { pm = (m == j) ? pfx[j] : pm; dm_ = (m == j) ? dn[j] : dm_; }
        if (level > 0) match = match && !dm_ && ((key >> (sh + wd)) == pm);
        if (match) {
          const uint32_t bin = (key >> sh) & binmask;
          atomicAdd(&cnt[m * BINS + bin], 1u);
          atomicAdd(&sum[m * BINS + bin], to_fx(v[e]));
        }
      }
    }
    __syncthreads();
    if (phase == 1) {                              // add the chunk's bins to the head's and leave
      for (int e = tid; e < M * BINS; e += STATS_THREADS)
        if (cnt[e]) { atomicAdd(&gcnt[e], cnt[e]); atomicAdd(&gsum[e], sum[e]); }
      return;
    }
    // wave m walks the histogram of modality m from the top bin down
    if (wave < M) {
      const int m = wave;
      const int nb = 1 << wd;
      const int per = (nb + 63) / 64;                 // bins per lane; lane 0 owns the top bins
      // lane l owns the `per` bins below nb - l * per; it sums them starting at a lane-dependent
      // offset so that the 64 lanes read different LDS banks
      unsigned long long ls = 0ULL; uint32_t lc = 0;
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        if (j < per) {
          const int bin = nb - 1 - (lane * per + ((j + lane) & (per - 1)));
          ls += sum[m * BINS + bin]; lc += cnt[m * BINS + bin];
        }
      }
      // inclusive scan over lanes (lane 0 first); a head's masses stay below 2^52
      const unsigned long long ss = wave_incl_scan_u63(ls);
      const uint32_t sc = wave_incl_scan_u32(lc);
      // totals, target and the state carried from the level above; at level 0 every lane
      // derives them from the scan, later levels read what was stored before the barrier
      unsigned long long target, base_s; uint32_t base_c, prefix_prev; bool done;
      if (level == 0) {
        const unsigned long long wtot = (unsigned long long)shfl_i64((long long)ss, 63);
        const uint32_t ntot = (uint32_t)__shfl((int)sc, 63, 64);
        // smallest integer >= theta * w: the running mass c reaches theta*w iff c >= it
        unsigned long long tg = (unsigned long long)ceil(a.theta * (double)wtot);
        target = tg < wtot ? tg : wtot;
        done = (wtot == 0ULL || ntot == 0u);
        base_s = 0ULL; base_c = 0u; prefix_prev = 0u;
        if (lane == 0) {
          s_w[m] = wtot; s_n[m] = ntot; s_target[m] = target; s_done[m] = done ? 1u : 0u;
          s_cnt_gt[m] = 0; s_sum_gt[m] = 0ULL; s_prefix[m] = 0; s_bincnt[m] = 0; s_binsum[m] = 0ULL;
        }
      } else {
        target = s_target[m]; base_s = s_sum_gt[m]; base_c = s_cnt_gt[m];
        prefix_prev = s_prefix[m]; done = s_done[m] != 0;
      }
      // the lane whose bins contain the crossing: mass before its bins < target <= mass after them
      const unsigned long long before = base_s + ss - ls;
      const unsigned long long owner = __ballot(!done && (before < target) && (before + ls >= target));
      if (owner) {
        // the owner's bins, one per lane, scanned the same way: the bin where the mass reaches the target
        const int src = __ffsll((long long)owner) - 1;
        const unsigned long long bs0 = (unsigned long long)shfl_i64((long long)before, src);
        const uint32_t bc0 = base_c + (uint32_t)__shfl((int)(sc - lc), src, 64);
        const int bin = nb - 1 - (src * per + min(lane, per - 1));
        const unsigned long long vs = lane < per ? sum[m * BINS + bin] : 0ULL;
        const uint32_t vc = lane < per ? cnt[m * BINS + bin] : 0u;
        const unsigned long long is = wave_incl_scan_u63(vs);
        const uint32_t ic = wave_incl_scan_u32(vc);
        const unsigned long long bef = bs0 + is - vs;
        const unsigned long long hit = __ballot(lane < per && bef < target && bef + vs >= target);
        const int hl = __ffsll((long long)hit) - 1;
        if (lane == hl) {
          s_prefix[m] = (prefix_prev << wd) | (uint32_t)bin;
          s_sum_gt[m] = bef; s_cnt_gt[m] = bc0 + ic - vc;
          s_binsum[m] = vs; s_bincnt[m] = vc;
        }
      }
    }
    __syncthreads();
  }

  if (phase == 2 && a.level < 2) {               // hand over to the next level
    if (tid < M) {
      StatsCarry cy;
      cy.prefix = s_prefix[tid]; cy.cnt_gt = s_cnt_gt[tid]; cy.n = s_n[tid]; cy.done = s_done[tid]; cy.bincnt = s_bincnt[tid]; cy.pad = 0;
      cy.sum_gt = s_sum_gt[tid]; cy.w = s_w[tid]; cy.target = s_target[tid]; cy.binsum = s_binsum[tid]; cy.wwin = s_wwin[tid];
      carry[tid] = cy;
    }
    return;
  }
  if (tid < M) {
    const int m = tid;
    int32_t k = 0;
    if (!s_done[m]) {
      // s_prefix is now the full bit pattern of tau; every element in the last bin equals tau
      const float tau = __uint_as_float(s_prefix[m]);
      const unsigned long long q = to_fx(tau);
      const unsigned long long need = s_target[m] - s_sum_gt[m];
      unsigned long long t = q ? (need + q - 1ULL) / q : 1ULL;
      if (t < 1ULL) t = 1ULL;
      if (t > (unsigned long long)s_bincnt[m]) t = s_bincnt[m];
      k = (int32_t)(s_cnt_gt[m] + (uint32_t)t);
    }
    const float w = (float)((double)(s_w[m] + s_wwin[m]) * (1.0 / (double)FX_SCALE));
    // a head's record: M float masses, then M int32 counts (two modalities: madakv_head_stats)
    float* rec = reinterpret_cast<float*>(a.stats) + (long long)head * 2 * M;
    rec[m] = w;
    reinterpret_cast<int32_t*>(rec)[M + m] = k;
    if (head < a.B * a.H && (head % a.H) == 0 && a.n_mod) a.n_mod[b * M + m] = (int32_t)s_n[m];
  }
}

__global__ __launch_bounds__(256) void split_zero_kernel(uint32_t* p, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

void launch_split_zero(uint32_t* p, long long words, hipStream_t st) {
  hipLaunchKernelGGL(split_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, p, words);
}

// Chunks per head that go to workgroups of their own, or 0: heads of at least four 16384-candidate chunks
// (with two, the 16 small launches cost what the parallelism gains: measured on 28 heads of 32K candidates),
// so few of them that one workgroup per head would leave most of the chip idle.
int split_chunks(const Dims& dm) {
  const int nchunks = (dm.nc + STATS_THREADS * STATS_EPT - 1) / (STATS_THREADS * STATS_EPT);
  return (nchunks >= 4 && dm.heads <= SPLIT_MAX_HEADS) ? nchunks : 0;
}
size_t split_buffer_bytes(int heads, int M, int nchunks) {
  const size_t hist = (size_t)3 * heads * M * BINS;
  return hist * (sizeof(unsigned long long) + sizeof(uint32_t)) + (size_t)heads * 4 * sizeof(StatsCarry) + (size_t)heads * nchunks * 16 + 256;
}

hipError_t launch_stats(const Dims& dm, const madakv_config& c, const float* psi, const uint8_t* mask,
                        float* psi_pool, void* stats, int32_t* n_mod, int layer0, hipStream_t st,
                        void* split_buf, size_t split_bytes) {
  StatsArgs a;
  a.psi = psi; a.mask = mask; a.psi_pool = psi_pool; a.stats = stats; a.n_mod = n_mod;
  a.B = dm.B; a.H = dm.H; a.L = dm.L; a.W = dm.W; a.nc = dm.nc; a.pool_r = (c.pool_k - 1) / 2;
  (void)layer0;
  a.pool_mode = c.pool_mode; a.share_mode = c.share_mode; a.theta = (double)c.theta;
  a.M = c.n_modalities;
  a.phase = 0; a.level = 0; a.heads = dm.heads; a.gsum = nullptr; a.gcnt = nullptr; a.carry = nullptr;
  const size_t lds = (size_t)a.M * BINS * (sizeof(unsigned long long) + sizeof(uint32_t));
  if (a.M == 2) {
    if (lds > 48 * 1024)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&stats_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  } else {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&stats_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  }
  const int nchunks = split_chunks(dm);
  if (nchunks && split_buf && split_bytes >= split_buffer_bytes(dm.heads, a.M, nchunks)) {
    // per level: the chunks' workgroups add their histograms into the head's (in memory), then one workgroup per
    // head walks it; the kernel boundary is the synchronisation
    const size_t hist = (size_t)3 * dm.heads * a.M * BINS;
    a.gsum = reinterpret_cast<unsigned long long*>(split_buf);
    a.gcnt = reinterpret_cast<uint32_t*>(a.gsum + hist);
    a.carry = reinterpret_cast<StatsCarry*>(a.gcnt + hist);
    const long long zw = (long long)(hist * 3);                // 32-bit words of the two histogram arrays
    launch_split_zero(reinterpret_cast<uint32_t*>(split_buf), zw, st);
    for (int level = 0; level < 3; ++level) {
      a.level = level;
      for (int phase = 1; phase <= 2; ++phase) {
        a.phase = phase;
        const dim3 grid = phase == 1 ? dim3(nchunks, dm.heads) : dim3(dm.heads);
        if (a.M == 2) hipLaunchKernelGGL((stats_kernel<2>), grid, dim3(STATS_THREADS), lds, st, a);
        else hipLaunchKernelGGL((stats_kernel<4>), grid, dim3(STATS_THREADS), lds, st, a);
      }
    }
    return hipGetLastError();
  }
  if (a.M == 2) hipLaunchKernelGGL((stats_kernel<2>), dim3(dm.heads), dim3(STATS_THREADS), lds, st, a);
  else hipLaunchKernelGGL((stats_kernel<4>), dim3(dm.heads), dim3(STATS_THREADS), lds, st, a);
  return hipGetLastError();
}

}  // namespace madakv
