// Eviction (paper Sec. 3.3, modality-specific eviction per attention head): for each head
// keep, per modality, the b_m candidates with the largest pooled score; equal scores go to
// the lower position.  Output: kept positions in ascending order, then the W window
// positions, written into the head's segment of the ragged index array.
//
// offsets_kernel   lays the segments out: batch item b owns a fixed region of the reduced
//                  cache, inside it layers and heads follow each other; a segment has
//                  kv_len = b_t + b_v + W rows plus max_new_tokens free rows.  It also fills
//                  a table "first head that overlaps each 64-row block" for the gather.
// select_kernel    one workgroup per head; a thread owns 32 consecutive candidates, whose keys
//                  and modality bits stay in registers (one trip to memory for contexts up to
//                  16K candidates, chunks of that size beyond).  A 3-level radix select
//                  (11 + 11 + 10 bits of the order-preserving key) on LDS count histograms
//                  finds, per modality, the threshold key tau_m and how many elements equal
//                  to tau_m are still needed; then key > tau_m is kept, and key == tau_m while
//                  its rank by position is below that number.  Workgroup prefix sums give
//                  the ranks and the output slots, so the result is ascending by construction.
#include "common.h"

namespace madakv {

constexpr int SEL_THREADS = 512;
constexpr int SEL_BINS = 2048;

constexpr int SEL_EPT = 32;                      // consecutive candidates a thread owns per chunk

// what the walk of one level hands on, per head and modality, and what a chunk reports (phases 1-4 of select_kernel)
struct SelCarry { uint32_t prefix, need, done, pad; };
struct SelChunk { uint32_t gt, pad; unsigned long long eq; };   // kept for sure; threshold-valued ones, 16 bits per modality

struct OffsetsArgs {
  const int32_t* budgets; int64_t* kv_off; int32_t* kv_len; long long* cursor; int32_t* blk2head; long long* call_range; int32_t* layer_maxlen;
  int n, B, H, L, W, layer0, max_new, keep_all, blocks_per_batch, M;
  long long region_tokens;       // rows of one batch item's region
  long long init_limit;          // rows of it the segments laid out here may fill
  int page_rows, tbl_entries;    // paged cache: segments are whole pages, no free rows reserved per head
  int32_t* page_tbl; unsigned long long* pool_top;
};

// One workgroup per batch item; thread f of a trip owns head f of the call's (layer, head)
// sequence.  Offsets are a prefix sum over that sequence (wave shuffles + one LDS hop).
// The workgroup is kept small (one wave per SIMD, few registers): it has to find room on a compute
// unit while the score sweeps or a gather of another layer group fill the chip, and a 1024-thread
// workgroup would wait there until that kernel's grid has drained.
constexpr int OFF_THREADS = 256;
constexpr int OFF_MAX_LAYERS = 1024;

__global__ __launch_bounds__(OFF_THREADS) void offsets_kernel(OffsetsArgs a) {
  __shared__ long long s_wtot[OFF_THREADS / 64];
  __shared__ long long s_used;
  __shared__ int s_first_bad;
  __shared__ int s_lmax[OFF_MAX_LAYERS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const int nh = a.n * a.H;
  const long long start = (a.layer0 == 0) ? 0 : a.cursor[b];
  const long long region = (long long)b * a.region_tokens;
  const long long blk_base = start / GATHER_ROWS;            // the block table is relative to the call's first block
  for (int li = tid; li < a.n; li += OFF_THREADS) s_lmax[li] = 0;
  if (tid == 0) { s_first_bad = 0x7fffffff; s_used = 0; }
  if (tid == 0 && a.page_rows && a.layer0 == 0) a.pool_top[b] = 0ULL;   // a new pass: every page taken for appended rows is free again
  __syncthreads();
  long long carry = 0;                                        // rows laid out by earlier trips
  bool overflowed = false;                                    // a head did not fit: every later head is empty
  for (int f0 = 0; f0 < nh; f0 += OFF_THREADS) {
    const int f = f0 + tid;
    const bool act = f < nh;
    const int li = act ? f / a.H : 0, h = act ? f % a.H : 0;
    const long long idx = ((long long)li * a.B + b) * a.H + h;
    long long len = 0;
    if (act) {
      len = a.keep_all ? a.L : a.W;
      if (!a.keep_all) for (int m = 0; m < a.M; ++m) len += a.budgets[idx * a.M + m];
    }
    long long seg = act ? len + a.max_new : 0;
    if (a.page_rows) seg = act ? (len + a.page_rows - 1) / a.page_rows * a.page_rows : 0;
    long long incl = seg;
    for (int o = 1; o < 64; o <<= 1) {
      long long t = shfl_i64(incl, max(lane - o, 0));
      if (lane >= o) incl += t;
    }
    if (lane == 63) s_wtot[wave] = incl;
    __syncthreads();
    long long before = 0, tot = 0;
    for (int w = 0; w < OFF_THREADS / 64; ++w) { const long long t = s_wtot[w]; if (w < wave) before += t; tot += t; }
    const long long abs_incl = carry + before + incl;         // rows up to and including this head's segment
    // Budgets that do not add up to the configured total could run past the batch item's
    // region: the first head that does not fit, and every head after it, gets an empty
    // segment (kv_len 0) at the end of what was laid out, so nothing is written outside.
    const bool bad = act && (overflowed || start + abs_incl > a.init_limit);
    if (bad && !overflowed) atomicMin(&s_first_bad, f);
    __syncthreads();
    const int first_bad = s_first_bad;
    if (!overflowed && first_bad == f) s_used = abs_incl - seg;
    __syncthreads();
    const bool now_over = first_bad != 0x7fffffff;
    const long long used = s_used;
    long long off;
    if (bad) { len = 0; seg = 0; off = start + used; }
    else off = start + abs_incl - seg;                        // relative to the region start
    if (act) {
      atomicMax(&s_lmax[li], (int)len);                       // longest segment of the layer, for the decode grid
      a.kv_off[idx] = region + off;
      a.kv_len[idx] = (int32_t)len;
      if (a.page_rows) a.page_tbl[(((long long)(a.layer0 + li) * a.B + b) * a.H + h) * a.tbl_entries] = (int32_t)(seg / a.page_rows);
      // blocks whose first row lies inside this segment
      const long long b0 = (off + GATHER_ROWS - 1) / GATHER_ROWS, b1 = seg > 0 ? (off + seg - 1) / GATHER_ROWS : b0 - 1;
      for (long long blk = b0; blk <= b1; ++blk) {
        const long long t = blk - blk_base;
        if (t >= 0 && t < a.blocks_per_batch) a.blk2head[(long long)b * a.blocks_per_batch + t] = f;
      }
      if (f == 0 && (start % GATHER_ROWS) != 0 && 0 < a.blocks_per_batch)
        a.blk2head[(long long)b * a.blocks_per_batch] = 0;    // the call starts inside a block: its first head is head 0
    }
    carry = now_over ? used : carry + tot;
    overflowed = now_over;
    __syncthreads();
  }
  for (int li = tid; li < a.n; li += OFF_THREADS) a.layer_maxlen[(long long)li * a.B + b] = s_lmax[li];
  if (tid == 0) {
    a.cursor[b] = start + carry;
    a.call_range[b * 2] = start;
    a.call_range[b * 2 + 1] = start + carry;
  }
}

struct SelectArgs {
  const float* psi_pool; const uint8_t* mask; const int32_t* budgets; const int64_t* kv_off; const int32_t* kv_len; int32_t* kept_idx;
  int B, H, L, W, nc, mpa_mode, keep_all, select_mode, sink_tokens, M;
  const int32_t* seg_len; const uint8_t* rowmod;   // ragged candidates (re-eviction), else null
  // Long heads on few heads (see launch_select): the chunks of a head go to workgroups of their own.
  // phase 0 = the whole head in one workgroup; 1 = count histogram of one chunk at `level`, added to the
  // head's histogram in memory; 2 = the walk over that histogram (one workgroup per head); 3 = a chunk's
  // numbers of kept and of threshold-valued candidates; 4 = a chunk's kept positions written behind those
  // of the chunks before it.
  int phase, level, heads, nchunks;
  uint32_t* gcnt;                 // [3 levels][heads][M][SEL_BINS]
  SelCarry* carry;                // [heads][4]
  SelChunk* chunkinfo;            // [heads][nchunks]
};

typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

// exclusive prefix over the workgroup of a packed pair of counts (lo16 | hi16; a chunk holds
// 16384 candidates, so each half stays below 2^16 unless every one of them counts: the
// caller keeps the totals in 32 bits and the halves are only used below that bound)
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* wave_tot, uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = v;
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t t = (uint32_t)__shfl((int)incl, max(lane - o, 0), 64);
    if (lane >= o) incl += t;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t before = 0, tot = 0;
  for (int w = 0; w < SEL_THREADS / 64; ++w) {
    uint32_t t = wave_tot[w];
    if (w < wave) before += t;
    tot += t;
  }
  __syncthreads();
  total = tot;
  return before + incl - v;
}

// the same for four 16-bit counts packed in 64 bits (one count per modality)
__device__ __forceinline__ unsigned long long block_excl_scan64(unsigned long long v, unsigned long long* wave_tot,
                                                                unsigned long long& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned long long incl = v;
  for (int o = 1; o < 64; o <<= 1) {
    unsigned long long t = (unsigned long long)shfl_i64((long long)incl, max(lane - o, 0));
    if (lane >= o) incl += t;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  unsigned long long before = 0, tot = 0;
  for (int w = 0; w < SEL_THREADS / 64; ++w) {
    unsigned long long t = wave_tot[w];
    if (w < wave) before += t;
    tot += t;
  }
  __syncthreads();
  total = tot;
  return before + incl - v;
}

template <typename T, int N>
__device__ __forceinline__ T pick(const T (&x)[N], int m) {              // x[m] without indexing registers by m
  T r = x[0];
#pragma unroll
  for (int j = 1; j < N; ++j) r = (m == j) ? x[j] : r;
  return r;
}

// Thread t of the workgroup owns SEL_EPT consecutive candidates of a chunk: their keys and
// modality bits live in registers through the three radix levels and the compaction.
__device__ __forceinline__ void load_owned(const float* sc, const uint8_t* mask, int i0, int nc, int use_mask, int M,
                                           uint32_t (&key)[SEL_EPT], unsigned long long& mbits) {
  const bool full = i0 + SEL_EPT <= nc;
  if (full && ((reinterpret_cast<uintptr_t>(sc + i0) & 15u) == 0)) {
#pragma unroll
    for (int j = 0; j < SEL_EPT / 4; ++j) {
      const f32x4_t v = *reinterpret_cast<const f32x4_t*>(sc + i0 + j * 4);
      key[j * 4 + 0] = float_key(v[0]); key[j * 4 + 1] = float_key(v[1]);
      key[j * 4 + 2] = float_key(v[2]); key[j * 4 + 3] = float_key(v[3]);
    }
  } else {
#pragma unroll
    for (int e = 0; e < SEL_EPT; ++e) key[e] = (i0 + e < nc) ? float_key(sc[i0 + e]) : 0u;
  }
  mbits = 0ULL;                                   // modality ids, two bits per element
  const uint32_t top = (uint32_t)(M - 1);
  if (use_mask) {
    if (full && ((reinterpret_cast<uintptr_t>(mask + i0) & 15u) == 0)) {
#pragma unroll
      for (int j = 0; j < SEL_EPT / 16; ++j) {
        const u32x4_t w = *reinterpret_cast<const u32x4_t*>(mask + i0 + j * 16);
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int bb = 0; bb < 4; ++bb)
            mbits |= (unsigned long long)min((w[q] >> (8 * bb)) & 0xffu, top) << (2 * (j * 16 + q * 4 + bb));
      }
    } else {
#pragma unroll
      for (int e = 0; e < SEL_EPT; ++e)
        if (i0 + e < nc) mbits |= (unsigned long long)min((uint32_t)mask[i0 + e], top) << (2 * e);
    }
  }
}

template <int MM>   // modalities the kernel is built for (2: the paper's text / image; 4: up to four)
__global__ __launch_bounds__(SEL_THREADS) __attribute__((amdgpu_waves_per_eu(MM == 2 ? 4 : 2, 4))) void select_kernel(SelectArgs a) {
  __shared__ uint32_t cnt[MM][SEL_BINS];
  __shared__ uint32_t s_prefix[MM], s_need[MM], s_done[MM];
  __shared__ uint32_t wave_tot[SEL_THREADS / 64];
  __shared__ unsigned long long wave_tot64[SEL_THREADS / 64];
  const int M = a.M;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int phase = a.phase;
  const bool per_chunk = phase == 1 || phase >= 3;             // grid (chunks, heads)
  const int head = per_chunk ? blockIdx.y : blockIdx.x;
  const int b = (head / a.H) % a.B;
  // candidates of this head: the L - W prompt positions before the window with the batch item's modality
  // mask, or (ragged: the rows of a reduced cache, re-eviction) the rows before the head's last W with a
  // modality byte per row; scores and output are indexed the same way
  const bool ragged = a.seg_len != nullptr;
  const int nc = ragged ? a.seg_len[head] - a.W : a.nc;
  const float* sc = ragged ? a.psi_pool + a.kv_off[head] : a.psi_pool + (long long)head * a.nc;
  const uint8_t* mask = ragged ? a.rowmod + a.kv_off[head] : a.mask + (long long)b * a.L;
  int32_t* out = a.kept_idx + a.kv_off[head];

  if (a.kv_len[head] == 0) return;               // the segment did not fit the region: nothing to write
  if (a.keep_all) {
    for (int i = tid; i < a.L; i += SEL_THREADS) out[i] = i;
    return;
  }
  uint32_t bud[MM];
#pragma unroll
  for (int m = 0; m < MM; ++m) bud[m] = m < M ? (uint32_t)a.budgets[(long long)head * M + m] : 0u;
  if (a.select_mode == 1) {
    // score-free baseline: the first `sink` candidates and the most recent ones, then the window
    uint32_t btot = 0;
#pragma unroll
    for (int m = 0; m < MM; ++m) btot += bud[m];
    const int total = min((int)btot, nc);
    const int sink = min(a.sink_tokens, total);
    for (int j = tid; j < total + a.W; j += SEL_THREADS)
      out[j] = j < sink ? j : (j < total ? nc - (total - j) : nc + (j - total));
    return;
  }
  const int shifts[3] = {21, 10, 0};
  const int widths[3] = {11, 11, 10};
  constexpr int CH = SEL_THREADS * SEL_EPT;      // candidates per chunk
  const int nchunks = (nc + CH - 1) / CH;
  const int c_first = per_chunk ? blockIdx.x : 0, c_end = per_chunk ? blockIdx.x + 1 : nchunks;
  const bool single = c_end - c_first == 1;      // the usual case: everything stays in registers
  const int lv_first = phase == 0 ? 0 : (phase <= 2 ? a.level : 3), lv_end = phase == 0 ? 3 : (phase <= 2 ? a.level + 1 : 3);
  uint32_t* gcnt = phase ? a.gcnt + ((size_t)(phase <= 2 ? a.level : 0) * a.heads + head) * (size_t)M * SEL_BINS : nullptr;
  SelCarry* carry = phase ? a.carry + (size_t)head * 4 : nullptr;
  if (phase != 0 && (phase >= 3 || a.level > 0) && tid < M) {   // what the walks before left
    const SelCarry cy = carry[tid];
    s_prefix[tid] = cy.prefix; s_need[tid] = cy.need; s_done[tid] = cy.done;
  }
  if (phase >= 3) __syncthreads();

  uint32_t key[SEL_EPT];
  unsigned long long mbits = 0ULL;
  if (single && phase != 2) load_owned(sc, mask, c_first * CH + tid * SEL_EPT, nc, a.mpa_mode, M, key, mbits);

  for (int level = lv_first; level < lv_end; ++level) {
    for (int e = tid; e < M * SEL_BINS; e += SEL_THREADS) (&cnt[0][0])[e] = 0;
    __syncthreads();
    const int sh = shifts[level], wd = widths[level];
    const uint32_t binmask = (1u << wd) - 1u;
    uint32_t pfx[MM]; bool dn[MM];
#pragma unroll
    for (int m = 0; m < MM; ++m) {
      pfx[m] = (level > 0 && m < M) ? s_prefix[m] : 0u;
      dn[m] = (level > 0 && m < M) ? s_done[m] != 0 : false;
    }
    if (phase == 2) {                              // the head's histogram of this level, gathered by the chunks' workgroups
      for (int e = tid; e < M * SEL_BINS; e += SEL_THREADS) (&cnt[0][0])[e] = gcnt[e];
    }
    for (int c = (phase == 2 ? c_end : c_first); c < c_end; ++c) {
      const int i0 = c * CH + tid * SEL_EPT;
      if (!single) load_owned(sc, mask, i0, nc, a.mpa_mode, M, key, mbits);
      const int nvalid = min(max(nc - i0, 0), SEL_EPT);
#pragma unroll
      for (int e = 0; e < SEL_EPT; ++e) {
        const int m = (int)((mbits >> (2 * e)) & 3ULL);
        bool match = e < nvalid;
        if (level > 0) match = match && !pick(dn, m) && ((key[e] >> (sh + wd)) == pick(pfx, m));
        if (match) atomicAdd(&cnt[m][(key[e] >> sh) & binmask], 1u);
      }
    }
    __syncthreads();
    if (phase == 1) {                              // add the chunk's bins to the head's and leave
      for (int e = tid; e < M * SEL_BINS; e += SEL_THREADS) {
        const uint32_t x = (&cnt[0][0])[e];
        if (x) atomicAdd(&gcnt[e], x);
      }
      return;
    }
    if (wave < M) {
      const int m = wave;
      const int nb = 1 << wd;
      const int per = (nb + 63) / 64;
      // lane l owns the `per` bins below nb - l * per; it sums them starting at a lane-dependent
      // offset so that the 64 lanes read different LDS banks
      uint32_t lc = 0;
#pragma unroll
      for (int j = 0; j < 32; ++j)
        if (j < per) lc += cnt[m][nb - 1 - (lane * per + ((j + lane) & (per - 1)))];
      const uint32_t incl = wave_incl_scan_u32(lc);
      uint32_t need, prefix_prev; bool done;
      if (level == 0) {
        const uint32_t ntot = (uint32_t)__shfl((int)incl, 63, 64);
        const uint32_t bm = pick(bud, m);
        need = bm < ntot ? bm : ntot;              // a budget above the candidate count keeps them all
        done = (need == 0);
        prefix_prev = 0;
        if (lane == 0) { s_need[m] = need; s_done[m] = done ? 1u : 0u; s_prefix[m] = 0; }
      } else {
        need = s_need[m]; prefix_prev = s_prefix[m]; done = s_done[m] != 0;
      }
      const uint32_t before = incl - lc;          // elements in higher bins than this lane's
      const unsigned long long owner = __ballot(!done && before < need && before + lc >= need);
      if (owner) {
        // the owner's bins, one per lane, scanned the same way: the bin where the count reaches `need`
        const int src = __ffsll((long long)owner) - 1;
        const uint32_t bsrc = (uint32_t)__shfl((int)before, src, 64);
        const uint32_t v = lane < per ? cnt[m][nb - 1 - (src * per + lane)] : 0u;
        const uint32_t inc2 = wave_incl_scan_u32(v);
        const uint32_t bef2 = bsrc + inc2 - v;
        const unsigned long long hit = __ballot(lane < per && bef2 < need && bef2 + v >= need);
        const int hl = __ffsll((long long)hit) - 1;
        const uint32_t acc = (uint32_t)__shfl((int)bef2, hl, 64);
        if (lane == 0) {
          s_prefix[m] = (prefix_prev << wd) | (uint32_t)(nb - 1 - (src * per + hl));
          s_need[m] = need - acc;                   // still needed from inside this bin
        }
      }
    }
    __syncthreads();
  }
  if (phase == 2) {                                // hand over to the next level, or to the chunks' compaction
    if (tid < M) { SelCarry cy; cy.prefix = s_prefix[tid]; cy.need = s_need[tid]; cy.done = s_done[tid]; cy.pad = 0; carry[tid] = cy; }
    return;
  }
  // tau_m = s_prefix (full key); take every key > tau_m and the first s_need[m] keys == tau_m.
  uint32_t tau[MM], ties[MM];
#pragma unroll
  for (int m = 0; m < MM; ++m) {
    if (m >= M || s_done[m]) { tau[m] = 0xffffffffu; ties[m] = 0; }   // nothing to keep: no key exceeds or (needed) equals it
    else { tau[m] = s_prefix[m]; ties[m] = s_need[m]; }
  }
  __syncthreads();

  uint32_t run_eq[MM];
#pragma unroll
  for (int m = 0; m < MM; ++m) run_eq[m] = 0;
  uint32_t run_out = 0;
  if (phase == 4) {
    // what the chunks in front of this one keep: their sure ones, and of the threshold-valued ones as many as are needed
    const SelChunk* ci = a.chunkinfo + (size_t)head * a.nchunks;
    for (int c = 0; c < c_first; ++c) {
      const SelChunk x = ci[c];
      run_out += x.gt;
#pragma unroll
      for (int m = 0; m < MM; ++m) run_eq[m] += (uint32_t)((x.eq >> (16 * m)) & 0xffffULL);
    }
#pragma unroll
    for (int m = 0; m < MM; ++m) run_out += min(run_eq[m], ties[m]);
  }
  for (int c = c_first; c < c_end; ++c) {
    const int i0 = c * CH + tid * SEL_EPT;
    if (!single) load_owned(sc, mask, i0, nc, a.mpa_mode, M, key, mbits);
    const int nvalid = min(max(nc - i0, 0), SEL_EPT);
    // ties of this thread's stretch, per modality (four 16-bit counts), then their rank by
    // position over the workgroup
    unsigned long long eqbits = 0ULL, gtbits = 0ULL, eqcnt = 0ULL;
#pragma unroll
    for (int e = 0; e < SEL_EPT; ++e) {
      const int m = (int)((mbits >> (2 * e)) & 3ULL);
      const bool ok = e < nvalid;
      const uint32_t tm = pick(tau, m);
      const bool gt = ok && key[e] > tm;
      const bool eq = ok && key[e] == tm && pick(ties, m) > 0;
      gtbits |= (unsigned long long)gt << e;
      eqbits |= (unsigned long long)eq << e;
      eqcnt += (unsigned long long)eq << (16 * m);
    }
    unsigned long long eqtot;
    const unsigned long long eqbefore = block_excl_scan64(eqcnt, wave_tot64, eqtot);
    if (phase == 3) {                              // report and leave
      uint32_t gttot;
      (void)block_excl_scan((uint32_t)__popcll(gtbits), wave_tot, gttot);
      if (tid == 0) { SelChunk x; x.gt = gttot; x.pad = 0; x.eq = eqtot; a.chunkinfo[(size_t)head * a.nchunks + c] = x; }
      return;
    }
    uint32_t rank[MM];
#pragma unroll
    for (int m = 0; m < MM; ++m) rank[m] = run_eq[m] + (uint32_t)((eqbefore >> (16 * m)) & 0xffffULL);
    unsigned long long keepbits = gtbits;
    if (eqbits) {
#pragma unroll
      for (int e = 0; e < SEL_EPT; ++e) {
        if ((eqbits >> e) & 1ULL) {
          const int m = (int)((mbits >> (2 * e)) & 3ULL);
          if (pick(rank, m) < pick(ties, m)) keepbits |= 1ULL << e;
#pragma unroll
          for (int mm = 0; mm < MM; ++mm) rank[mm] += (mm == m) ? 1u : 0u;
        }
      }
    }
    uint32_t ktot;
    uint32_t pos = run_out + block_excl_scan((uint32_t)__popcll(keepbits), wave_tot, ktot);
    while (keepbits) {                            // ascending by construction: lowest set bit first
      const int e = __ffsll((long long)keepbits) - 1;
      out[pos++] = i0 + e;
      keepbits &= keepbits - 1ULL;
    }
#pragma unroll
    for (int m = 0; m < MM; ++m) run_eq[m] += (uint32_t)((eqtot >> (16 * m)) & 0xffffULL);
    run_out += ktot;
  }
  if (phase == 4 && c_end != nchunks) return;      // the window positions follow the last chunk's
  for (int r = tid; r < a.W; r += SEL_THREADS) out[run_out + r] = nc + r;
}

size_t select_ws_bytes(const Dims& dm, const madakv_config& c) {
  long long per_batch_model = region_tokens_of(c);
  long long per_batch_call = (long long)dm.n * dm.H * ((long long)dm.L + c.max_new_tokens + 2 * c.page_rows);
  long long tokens = std::min(per_batch_model, per_batch_call);
  long long blocks = tokens / GATHER_ROWS + 2;
  return (size_t)dm.B * blocks * sizeof(int32_t) + (size_t)dm.B * 2 * sizeof(long long) + 64;
}

hipError_t launch_offsets(const Dims& dm, const madakv_config& c, int layer0, const int32_t* budgets,
                          int64_t* kv_off, int32_t* kv_len, long long* cursor_state, int32_t* layer_maxlen, void* ws,
                          const Paging& pg, int blocks_per_batch, hipStream_t st) {
  OffsetsArgs a;
  a.layer_maxlen = layer_maxlen;
  a.budgets = budgets; a.kv_off = kv_off; a.kv_len = kv_len; a.cursor = cursor_state;
  a.call_range = reinterpret_cast<long long*>(ws);
  a.blk2head = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(ws) + ((size_t)dm.B * 2 * sizeof(long long) + 63) / 64 * 64);
  a.n = dm.n; a.B = dm.B; a.H = dm.H; a.L = dm.L; a.W = dm.W; a.layer0 = layer0; a.M = c.n_modalities;
  a.max_new = c.max_new_tokens; a.keep_all = c.budget >= c.ctx_len ? 1 : 0;
  a.blocks_per_batch = blocks_per_batch; a.region_tokens = pg.region_tokens; a.init_limit = pg.init_limit;
  a.page_rows = pg.page_rows; a.tbl_entries = pg.entries; a.page_tbl = pg.table; a.pool_top = pg.pool_top;
  hipLaunchKernelGGL(offsets_kernel, dim3(dm.B), dim3(OFF_THREADS), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_select(const Dims& dm, const madakv_config& c, const float* psi_pool, const uint8_t* mask,
                         const int32_t* budgets, const int64_t* kv_off, const int32_t* kv_len, int32_t* kept_idx,
                         hipStream_t st, const int32_t* seg_len, const uint8_t* rowmod, void* split_buf, size_t split_bytes) {
  SelectArgs a;
  a.seg_len = seg_len; a.rowmod = rowmod;
  a.psi_pool = psi_pool; a.mask = mask; a.budgets = budgets; a.kv_off = kv_off; a.kv_len = kv_len; a.kept_idx = kept_idx;
  a.B = dm.B; a.H = dm.H; a.L = dm.L; a.W = dm.W; a.nc = dm.nc; a.mpa_mode = c.mpa_mode;
  a.keep_all = (c.budget >= c.ctx_len && !seg_len) ? 1 : 0;
  a.select_mode = c.select_mode; a.sink_tokens = c.sink_tokens; a.M = c.n_modalities;
  a.phase = 0; a.level = 0; a.heads = dm.heads; a.nchunks = 0; a.gcnt = nullptr; a.carry = nullptr; a.chunkinfo = nullptr;
  const int nchunks = split_chunks(dm);
  if (nchunks && !seg_len && !a.keep_all && a.select_mode != 1 && split_buf &&
      split_bytes >= split_buffer_bytes(dm.heads, a.M, nchunks)) {
    // per level: the chunks' workgroups add their count histograms into the head's (in memory), one workgroup per head
    // walks it; then every chunk reports what it keeps and writes it behind the chunks in front of it
    const size_t hist = (size_t)3 * dm.heads * a.M * SEL_BINS;
    a.gcnt = reinterpret_cast<uint32_t*>(split_buf);
    a.carry = reinterpret_cast<SelCarry*>(a.gcnt + hist);
    a.chunkinfo = reinterpret_cast<SelChunk*>(a.carry + (size_t)dm.heads * 4);
    a.nchunks = nchunks;
    launch_split_zero(a.gcnt, (long long)hist, st);
    for (int step = 0; step < 8; ++step) {
      a.phase = step < 6 ? 1 + (step & 1) : step - 3;          // 1, 2, 1, 2, 1, 2, 3, 4
      a.level = step < 6 ? step / 2 : 0;
      const dim3 grid = a.phase == 2 ? dim3(dm.heads) : dim3(nchunks, dm.heads);
      if (a.M == 2) hipLaunchKernelGGL((select_kernel<2>), grid, dim3(SEL_THREADS), 0, st, a);
      else hipLaunchKernelGGL((select_kernel<4>), grid, dim3(SEL_THREADS), 0, st, a);
    }
    return hipGetLastError();
  }
  if (a.M == 2) hipLaunchKernelGGL((select_kernel<2>), dim3(dm.heads), dim3(SEL_THREADS), 0, st, a);
  else hipLaunchKernelGGL((select_kernel<4>), dim3(dm.heads), dim3(SEL_THREADS), 0, st, a);
  return hipGetLastError();
}

}  // namespace madakv
