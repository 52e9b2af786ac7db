// Proxy-token scores (paper Sec. 3.3 Eq. 7): psi[i] = sum over the G*W proxy rows of the
// causal softmax(scale * q k^T) they pay to key i.
//
// The softmax normaliser of a row needs the whole row, the column sum needs the
// normalisers, so the scores are produced in two sweeps over K:
//   sweep 1  per row: running max and sum of exp2 (log2 domain), per L-chunk
//   sweep 2  recompute the logits, p = exp2(s - (m + log2 l)), sum p over the rows
// Both sweeps are the same small-M contraction S^T = Q K^T (M = G*W rows, N = keys).
// bf16 inputs run on the 32x32x16 bf16 MFMA with fp32 accumulation; fp32 inputs (and
// head dims other than 64/128) take a plain FMA kernel.  All reductions have a fixed
// order: psi feeds integer decisions downstream and must not change from run to run.
#include "common.h"

#include <algorithm>
#include <cstdlib>

namespace madakv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr float NEG_BIG = -1.0e30f;
constexpr int SCORE_THREADS = 256;

struct ScoreArgs {
  const void* q_win;   // [heads/H * Hq, W, d]
  const void* k;       // [heads, L, d]
  float* psi;          // [heads, L]
  float* rowstat;      // [heads, nsplit, mpad, 2]
  const float* lse;    // optional [heads/H * Hq, W]: natural log-sum-exp of each proxy row's scaled logits (sweep 1 not needed)
  float* sink;         // 32 floats nobody reads: keeps the psi store of sweep 2 unconditional (both half-waves
                       // store the same value; a store under a branch makes the load waits pessimistic)
  int H, G, d, L, W, M, mpad, nsplit, chunk;
  int nmerge;          // chunks whose row statistics sweep 2 still has to merge (1 after score_combine_kernel)
  // one-sweep kernel: row statistics of the head's chunks as (max, sum) pairs in one 64-bit word each,
  // [heads, fsplit, mpad], all ones = not yet there; status[0] != 0 = a workgroup gave up waiting
  unsigned long long* xchg;
  int k_fp8;              // keys are E4M3 bytes (rows of d bytes: the 8-bit reduced cache), else bf16
  int xgroups;            // 0: every workgroup reads every chunk's words; else the number of groups of XCHG_GROUP chunks (two levels)
  long long xstride;      // exchange words per head: (fsplit + xgroups) * mpad
  int* status;         // status[0]: workgroups of one-sweep launches that gave up waiting so far (diagnostic counter,
                       // the first word of the workspace; never cleared here)
  int fsplit;          // chunks per head of the one-sweep kernel
  const int64_t* seg_off;   // one-sweep kernel on ragged heads (null: every head has L keys at head * L): first row and
  const int32_t* seg_len;   // number of rows of each head in k; psi is indexed the same way
  // one-sweep kernel with more than 64 proxy rows: the rows are cut into rb_count blocks of 64, each handled
  // like a head of its own (grid.y = heads * rb_count); their column sums go to psi_part [rb][heads][L stride]
  // and are added in block order afterwards
  int rb_count;
  float* psi_part;
  long long psi_part_stride;   // floats between two row blocks' copies
  int spin_limit;      // polls a workgroup of the one-sweep kernel spends on one missing word before it goes its own way
  // one-sweep kernel on long heads whose chunks do not pack the chip's workgroup slots (see launch_fused): the last
  // nstrag chunks of every head come first in the grid (x < nstrag), leave their row statistics as exchange words
  // of the group level and their logits in `park`, and do not wait; the other chunks' workgroups leave the heads'
  // row offsets in offs_out, a small kernel finishes the parked chunks
  int nstrag = 0;
  float* park = nullptr;
  float* offs_out = nullptr;
  int head0;           // first head of this launch (grid.y indexes head0 + y)
  float scale_log2;    // softmax scale * log2(e)
};

__device__ __forceinline__ void merge_ml(float& m, float& l, float m2, float l2) {
  float mn = fmaxf(m, m2);
  l = l * exp2f(m - mn) + l2 * exp2f(m2 - mn);
  m = mn;
}

// ------------------------------------------------------------------------------------
// bf16 MFMA path.  One workgroup = 4 waves works on one (head, L-chunk); a wave streams
// 32-key subtiles of K:
//   D[i = proxy row][j = key] = sum_k A[i][k] * B[k][j],  A = 32-row block of Q, B = K subtile^T.
// HBM side: a subtile (32 rows of 256 B) is fetched with fully coalesced 16-byte loads (16
// lanes cover one row), PF subtiles ahead of the arithmetic, into registers.  That is
// what hides the HBM latency: a subtile's arithmetic takes a fraction of a microsecond.
// MFMA side: an operand lane needs the whole row of "its" key, a layout that would touch 64
// different cache lines per load instruction if read from global memory directly; so the
// subtile is parked in a wave-private LDS tile (rows padded by 16 bytes: the 128-bit reads of
// 32 different rows fall into different banks) and the B fragments are read from there.  The
// tile is private to the wave: no workgroup barrier in the loop, LDS operations of one wave
// execute in order.
// In D a lane holds one key column and 16 rows: the column sum is in-lane, the row
// statistics need one cross-lane merge at the end of the chunk.
// Every wave has its own keys and all (at most two) row blocks; more than 64 proxy rows take the
// kernels further down, whose waves share the keys and own row blocks.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }   // x <= ~0 here; tiny results may flush to 0

template <int OP>   // 0 = max, 1 = sum over the 32 lanes of a half-wave; every lane gets the result
__device__ __forceinline__ float half_reduce(float x) {
#define MADAKV_DPP(ctrl) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), ctrl, 0xF, 0xF, true))
  float y;
  y = MADAKV_DPP(0xB1);  x = OP ? x + y : fmaxf(x, y);     // quad_perm [1,0,3,2]
  y = MADAKV_DPP(0x4E);  x = OP ? x + y : fmaxf(x, y);     // quad_perm [2,3,0,1]
  y = MADAKV_DPP(0x141); x = OP ? x + y : fmaxf(x, y);     // row_half_mirror
  y = MADAKV_DPP(0x140); x = OP ? x + y : fmaxf(x, y);     // row_mirror
#undef MADAKV_DPP
  y = __shfl_xor(x, 16, 64); x = OP ? x + y : fmaxf(x, y); // the two 16-lane rows of the half
  return x;
}

template <int D, int NRB, int PASS>
__global__ __launch_bounds__(SCORE_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void score_mfma_kernel(ScoreArgs a) {
  constexpr int KS = D / 16;                  // MFMA k-steps
  constexpr int RS = D + 8;                   // bf16 elements per LDS row (16 B pad)
  constexpr int KG = 4;                       // key groups: the waves
  constexpr int PPR = D / 8;                  // 16-byte pieces per row
  constexpr int LPS = 32 * PPR / 64;          // 16-byte loads per lane per subtile
  constexpr int PF = 2;                       // subtiles in flight per wave
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* qs = reinterpret_cast<uint16_t*>(smem);                       // [mpad][RS]
  uint16_t* kt_all = qs + (size_t)a.mpad * RS;                            // [4 waves][32][RS]
  float* fbuf = reinterpret_cast<float*>(kt_all + 4 * 32 * RS);           // pass 1: [KG][mpad][2]; pass 2: off[mpad]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x;
  const int head = a.head0 + blockIdx.y;
  const int kvh = head % a.H;
  const long long lb = head / a.H;            // (layer, batch) index
  const uint16_t* qg = reinterpret_cast<const uint16_t*>(a.q_win) + (lb * a.H + kvh) * (long long)a.G * a.W * D;
  const uint16_t* kg = reinterpret_cast<const uint16_t*>(a.k) + (long long)head * a.L * D;
  const int chunk0 = split * a.chunk;
  const int chunk1 = min(a.L, chunk0 + a.chunk);
  const int nsub = (chunk1 - chunk0 + 31) / 32;
  const int niter = (nsub + KG - 1) / KG;
  const int kgid = wave;                      // subtiles of this wave: kgid, kgid + KG, ...
  uint16_t* kt = kt_all + (size_t)wave * 32 * RS;

  // PF subtiles of K on their way before anything else
  u32x4_t pre0[LPS], pre1[LPS];                // two register sets = PF subtiles in flight
  static_assert(PF == 2, "the loop body below is written out for two register sets");
#define MADAKV_LOAD_SUB(DST, IT)                                                                 \
  {                                                                                              \
    const int lt0 = chunk0 + ((IT) * KG + kgid) * 32;                                            \
    _Pragma("unroll") for (int i = 0; i < LPS; ++i) {                                            \
      const int idx = i * 64 + lane;                                                             \
      const int lkey = min(lt0 + idx / PPR, a.L - 1); /* past the end: a valid row, masked later */ \
      DST[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(kg + (long long)lkey * D + (idx % PPR) * 8)); \
    }                                                                                            \
  }
  MADAKV_LOAD_SUB(pre0, 0)
  MADAKV_LOAD_SUB(pre1, 1)

  // stage Q (the G*W rows of this KV head are contiguous), zero the padding rows
  for (int e = tid; e < a.mpad * PPR; e += SCORE_THREADS) {
    const int r = e / PPR, c = e % PPR;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (r < a.M) val = *reinterpret_cast<const uint4*>(qg + (long long)r * D + c * 8);
    *reinterpret_cast<uint4*>(qs + r * RS + c * 8) = val;
  }
  float* offs = fbuf;                          // pass 2 only
  if (PASS == 2) {
    const float* rs = a.rowstat + (long long)head * a.nsplit * a.mpad * 2;
    for (int r = tid; r < a.mpad; r += SCORE_THREADS) {
      float m = NEG_BIG, l = 0.f;
      if (a.lse) {                                               // the caller's prefill attention already has the row normalisers
        if (r < a.M) { m = a.lse[(lb * a.H + kvh) * (long long)a.G * a.W + r] * 1.4426950408889634f; l = 1.f; }
      } else {
        for (int s = 0; s < a.nmerge; ++s) merge_ml(m, l, rs[(s * a.mpad + r) * 2], rs[(s * a.mpad + r) * 2 + 1]);
      }
      offs[r] = (r < a.M) ? m + log2f(l) : __builtin_inff();     // padding rows contribute exp2(-inf) = 0
    }
  }
  __syncthreads();

  const int half = lane >> 5, col = lane & 31;
  const int first_masked = a.L - a.W + 1;      // keys below this are visible to every proxy row

  float st_m[NRB][16], st_l[NRB][16], off_r[NRB][16];
#pragma unroll
  for (int b = 0; b < NRB; ++b)
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      st_m[b][j] = NEG_BIG; st_l[b][j] = 0.f;
      const int row = min(b * 32 + (j >> 2) * 8 + half * 4 + (j & 3), a.mpad - 1);
      off_r[b][j] = (PASS == 2) ? offs[row] : 0.f;
    }
  // with a single row block per wave the Q fragments stay in registers (no LDS reads in the loop)
  bf16x8_t areg[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    areg[ks] = *reinterpret_cast<const bf16x8_t*>(qs + col * RS + half * (D / 2) + ks * 8);
  const int MB = a.mpad / 32;

  // one subtile per step: registers -> LDS tile -> MFMA -> statistics / column sums.
  // (Written as a macro applied to each register set: the sets must stay in registers, and
  // any indirection over them makes the compiler park them in scratch memory.)
#define MADAKV_STEP(SRC, IT)  {  const int it = (IT);  { \
_Pragma("unroll") \
    for (int i = 0; i < LPS; ++i) { \
      const int idx = i * 64 + lane; \
      *reinterpret_cast<u32x4_t*>(kt + (idx / PPR) * RS + (idx % PPR) * 8) = SRC[i]; \
    } \
    MADAKV_LOAD_SUB(SRC, it + PF) \
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); \
    __builtin_amdgcn_wave_barrier(); \
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront"); \
    const int t0 = chunk0 + (it * KG + kgid) * 32; \
    const int key = t0 + col; \
    const bool tail = (t0 + 32 > first_masked) || (t0 + 32 > chunk1); \
    const uint16_t* krow = kt + col * RS + half * (D / 2); \
    bf16x8_t bfrag[KS]; \
_Pragma("unroll") \
    for (int ks = 0; ks < KS; ++ks) bfrag[ks] = *reinterpret_cast<const bf16x8_t*>(krow + ks * 8); \
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); \
    __builtin_amdgcn_wave_barrier(); \
    float colsum = 0.f; \
_Pragma("unroll") \
    for (int b = 0; b < NRB; ++b) { \
      const int rb = b; \
      if (rb < MB) { \
        f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}; \
        const uint16_t* qrow = qs + (rb * 32 + col) * RS + half * (D / 2); \
_Pragma("unroll") \
        for (int ks = 0; ks < KS; ++ks) { \
          const bf16x8_t afrag = (NRB == 1) ? areg[ks] : *reinterpret_cast<const bf16x8_t*>(qrow + ks * 8); \
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[ks], acc, 0, 0, 0); \
        } \
        if (!tail) { \
_Pragma("unroll") \
          for (int j = 0; j < 16; ++j) { \
            const float s2 = acc[j] * a.scale_log2; \
            if (PASS == 1) { \
              const float dlt = s2 - st_m[b][j]; \
              const float e = fast_exp2(-fabsf(dlt)); \
              st_l[b][j] = dlt > 0.f ? fmaf(st_l[b][j], e, 1.0f) : st_l[b][j] + e; \
              st_m[b][j] = fmaxf(st_m[b][j], s2); \
            } else { \
              colsum += fast_exp2(s2 - off_r[b][j]); \
            } \
          } \
        } else { \
_Pragma("unroll") \
          for (int j = 0; j < 16; ++j) { \
            const float s2 = acc[j] * a.scale_log2; \
            const int row = rb * 32 + (j >> 2) * 8 + half * 4 + (j & 3); \
            const int pos = a.L - a.W + (row % a.W); \
            const bool valid = (key < chunk1) && (key <= pos) && (row < a.M); \
            if (PASS == 1) { \
              const float dlt = s2 - st_m[b][j]; \
              const float e = fast_exp2(-fabsf(dlt)); \
              const float nl = dlt > 0.f ? fmaf(st_l[b][j], e, 1.0f) : st_l[b][j] + e; \
              st_l[b][j] = valid ? nl : st_l[b][j]; \
              st_m[b][j] = valid ? fmaxf(st_m[b][j], s2) : st_m[b][j]; \
            } else { \
              const float pr = fast_exp2(s2 - off_r[b][j]); \
              colsum += valid ? pr : 0.f; \
            } \
          } \
        } \
      } \
    } \
    if (PASS == 2) { \
      colsum += __shfl_xor(colsum, 32, 64); \
      { float* dst = (key < chunk1) ? a.psi + ((long long)head * a.L + key) : a.sink + col; __builtin_nontemporal_store(colsum, dst); } \
    } \
  } }
  // Four unconditional steps per trip; the step count is rounded up (a step past the end works on
  // clamped rows and is fully masked).  A step under a condition would leave the compiler unsure how
  // many loads are in flight after it, and it would then wait for all of them at every step.
  const int niter4 = (niter + 2 * PF - 1) / (2 * PF) * (2 * PF);
  for (int it0 = 0; it0 < niter4; it0 += 2 * PF) {
    MADAKV_STEP(pre0, it0)
    MADAKV_STEP(pre1, it0 + 1)
    MADAKV_STEP(pre0, it0 + 2)
    MADAKV_STEP(pre1, it0 + 3)
  }
#undef MADAKV_STEP
#undef MADAKV_LOAD_SUB

  if (PASS == 1) {
    // per row: maximum over the 32 key columns of the half, sums rescaled to it and added;
    // then the key groups meet in LDS
    float* part = fbuf;                        // [KG][mpad][2]
#pragma unroll
    for (int b = 0; b < NRB; ++b) {
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const float m = half_reduce<0>(st_m[b][j]);
        const float l = half_reduce<1>(st_l[b][j] * fast_exp2(st_m[b][j] - m));
        const int rb = b;
        if (rb < MB && col == 0) {
          const int row = rb * 32 + (j >> 2) * 8 + half * 4 + (j & 3);
          part[(kgid * a.mpad + row) * 2] = m;
          part[(kgid * a.mpad + row) * 2 + 1] = l;
        }
      }
    }
    __syncthreads();
    float* rs = a.rowstat + ((long long)head * a.nsplit + split) * a.mpad * 2;
    for (int r = tid; r < a.mpad; r += SCORE_THREADS) {
      float m = NEG_BIG, l = 0.f;
      for (int g = 0; g < KG; ++g) merge_ml(m, l, part[(g * a.mpad + r) * 2], part[(g * a.mpad + r) * 2 + 1]);
      rs[r * 2] = m; rs[r * 2 + 1] = l;
    }
  }
}

// ------------------------------------------------------------------------------------
// More than 64 proxy rows (grouped queries: G*W up to 256), the same two sweeps.  The arithmetic per
// key grows with the rows and is what bounds these kernels (one exp2 per logit and sweep on the vector
// unit; the contraction is a fraction of that), so the layout serves the vector unit: wave w owns
// proxy rows [32 NRB w, 32 NRB (w + 1)) for all keys of the workgroup's chunk and keeps their Q
// fragments in registers; the waves share the keys.  Sweep 1 needs no merge among the waves (a row's
// statistics over the chunk are complete in its wave) and multiplies the other way round, S^T = K Q^T:
// a lane then holds one row against 16 keys, the running (max, sum) of a row is one register pair and
// in-lane work.  Sweep 2 (S = Q K^T: a lane holds one key against 16 rows, the column sum is in-lane)
// adds the waves' partial column sums through LDS, in wave order, one tile behind the arithmetic.
// The keys are fetched straight into LDS (global_load_lds, 16 bytes per lane): no register holds a
// key on its way, so three tiles form a ring with two tiles in flight while the third is multiplied.
// A wave's load instruction fills 1 KB of consecutive LDS (lane i at base + 16 i), so rows cannot be
// padded; instead the 16-byte pieces of a row are stored permuted, piece c of row r at slot
// c ^ (r mod pieces per row): the lane that writes slot s of row r fetches piece s ^ (r mod ...) from
// memory (a row's pieces are still one contiguous stretch per 16 lanes), and the operand reads of 16
// lanes with consecutive rows fall into 16 different slots.
// The compiler cannot tell which LDS bytes such a load writes and would wait for ALL outstanding loads
// before every LDS access it sees; so inside the loop every LDS access and every wait is written out:
// loads are counted (they complete in order), "tile t is there" is s_waitcnt vmcnt(loads of one tile),
// and the barrier that follows also tells that everybody is done with the tile the next load overwrites.
// ------------------------------------------------------------------------------------
constexpr int DMA_NBUF = 3;
#ifndef MADAKV_P1_WPE
#define MADAKV_P1_WPE 3      // waves per SIMD of sweep 1 (its registers allow three)
#endif

typedef __attribute__((address_space(3))) void* lds_void_ptr_t;
typedef const __attribute__((address_space(1))) void* global_void_ptr_t;

template <int D, int NW, int NRB, int DMA_TK, int BS, int PASS>   // NW waves of NRB row blocks each; tiles of DMA_TK keys; the vector arithmetic runs on BS subtiles at a time
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(PASS == 1 ? MADAKV_P1_WPE : 2, PASS == 1 ? MADAKV_P1_WPE : 2))) void score_wide_dma_kernel(ScoreArgs a) {
  constexpr int NT = NW * 64;
  constexpr int KS = D / 16;                  // MFMA k-steps
  constexpr int PPR = D / 8;                  // 16-byte pieces per row
  constexpr int ROWB = D * 2;                 // bytes per row
  constexpr int LPT = DMA_TK * PPR / NT;              // load instructions per thread and tile (each fills 1 KB per wave)
  constexpr int NSUB = DMA_TK / 32;
  constexpr int TILEB = DMA_TK * ROWB;
  static_assert((LPT == 4 || LPT == 2 || LPT == 1) && NSUB % BS == 0 && (PASS == 1 || DMA_TK == 64), "the waits below are written for these");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* ring = smem;                                              // [DMA_NBUF][DMA_TK][ROWB], pieces permuted
  float* offs = reinterpret_cast<float*>(smem + DMA_NBUF * TILEB);         // sweep 2: [mpad]
  float* red = offs + a.mpad;                                              // sweep 2: [2][NW][DMA_TK]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x;
  const int head = a.head0 + blockIdx.y;
  const int kvh = head % a.H;
  const long long lb = head / a.H;            // (layer, batch) index
  const uint16_t* qg = reinterpret_cast<const uint16_t*>(a.q_win) + (lb * a.H + kvh) * (long long)a.G * a.W * D;
  const unsigned char* kg = reinterpret_cast<const unsigned char*>(a.k) + (long long)head * a.L * ROWB;
  const int chunk0 = split * a.chunk;
  const int chunk1 = min(a.L, chunk0 + a.chunk);
  const int ntiles = (chunk1 - chunk0 + DMA_TK - 1) / DMA_TK;
  const int half = lane >> 5, col = lane & 31;
  const int MB = a.mpad / 32;
  const int rb0 = wave * NRB;                  // first row block of this wave
  const int first_masked = a.L - a.W + 1;      // keys below this are visible to every proxy row

  // sweep 2: the rows' offsets (ordinary LDS traffic, so before the first key is on its way)
  // sweep 2: st_m holds the offsets of the 16 rows a lane has of each block.  Sweep 1 runs the contraction the
  // other way round (S^T = K Q^T: a lane holds ONE row and 16 keys of a subtile), so its running (max in
  // accumulator units, sum) is one pair per lane and block: row_m, row_l.
  float st_m[PASS == 2 ? NRB : 1][16];
  float row_m[NRB], row_l[NRB];
  if (PASS == 2) {
    const float* rs = a.rowstat + (long long)head * a.nsplit * a.mpad * 2;
    for (int r = tid; r < a.mpad; r += NT) {
      float m = NEG_BIG, l = 0.f;
      if (a.lse) {                                               // the caller's prefill attention already has the row normalisers
        if (r < a.M) { m = a.lse[(lb * a.H + kvh) * (long long)a.G * a.W + r] * 1.4426950408889634f; l = 1.f; }
      } else {
        for (int s = 0; s < a.nmerge; ++s) merge_ml(m, l, rs[(s * a.mpad + r) * 2], rs[(s * a.mpad + r) * 2 + 1]);
      }
      offs[r] = (r < a.M) ? m + log2f(l) : __builtin_inff();     // padding rows contribute exp2(-inf) = 0
    }
    __syncthreads();
  }
#pragma unroll
  for (int b = 0; b < NRB; ++b)
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int row = (rb0 + b) * 32 + (j >> 2) * 8 + half * 4 + (j & 3);     // (a block past the last: rows that count for nothing)
      if (PASS == 2) st_m[b][j] = row < a.mpad ? offs[row] : __builtin_inff();
    }
#pragma unroll
  for (int b = 0; b < NRB; ++b) { row_m[b] = NEG_BIG; row_l[b] = 0.f; }
  __syncthreads();                             // (the last ordinary LDS access of the kernel)

  // tile T of the chunk -> ring slot T mod 3.  Load j of wave w fills bytes [(w LPT + j) 1024, + 1024) of the slot:
  // lane i writes piece P = (w LPT + j) 64 + i, i.e. slot P mod PPR of row P / PPR, and fetches that row's piece
  // (P mod PPR) ^ (row mod PPR).  Rows past the head's end: its last row (masked where it is used).
  const uint32_t ring_lds = (uint32_t)(uintptr_t)ring;
#define MADAKV_DMA_ISSUE(T)                                                                          \
  {                                                                                                  \
    const int tt = (T);                                                                              \
    const int lt0 = chunk0 + tt * DMA_TK;                                                            \
    const uint32_t slot_lds = ring_lds + (uint32_t)(tt % DMA_NBUF) * TILEB;                          \
    _Pragma("unroll") for (int j = 0; j < LPT; ++j) {                                                \
      const int piece = (wave * LPT + j) * 64 + lane;                                                \
      const int row = piece / PPR;                                                                   \
      const int lkey = min(lt0 + row, a.L - 1);                                                      \
      const unsigned char* src = kg + (long long)lkey * ROWB + (((piece % PPR) ^ (row % PPR)) * 16); \
      const uint32_t dst = __builtin_amdgcn_readfirstlane(slot_lds + (uint32_t)(wave * LPT + j) * 1024u); \
      __builtin_amdgcn_global_load_lds((global_void_ptr_t)(uintptr_t)src, (lds_void_ptr_t)(uintptr_t)dst, 16, 0, 0); \
    }                                                                                                \
  }
  MADAKV_DMA_ISSUE(0)
  MADAKV_DMA_ISSUE(min(1, ntiles - 1))

  // Q fragments of the wave's rows straight from memory (rows past M: zeros); a lane holds, for k-step ks,
  // elements [half * D/2 + ks * 8, + 8) of row `col` of the block
  bf16x8_t areg[NRB][KS];
#pragma unroll
  for (int b = 0; b < NRB; ++b) {
    const int row = (rb0 + b) * 32 + col;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 val = make_uint4(0, 0, 0, 0);
      if (row < a.M) val = *reinterpret_cast<const uint4*>(qg + (long long)row * D + half * (D / 2) + ks * 8);
      areg[b][ks] = __builtin_bit_cast(bf16x8_t, val);
    }
  }
  // where this lane's operand pieces of row `col` of a subtile sit, relative to the subtile's first byte
  uint32_t frag_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) frag_off[ks] = (uint32_t)(col * ROWB + (((half * KS + ks) ^ (col % PPR)) * 16));
  const uint32_t red_lds = (uint32_t)(uintptr_t)red;

  for (int t = 0; t < ntiles; ++t) {
    // tile t has landed (the loads of tile t + 1 may still be out), this wave's LDS stores of the last trip are
    // done; after the barrier that holds for every wave, and nobody reads tile t - 1 any more
    if (LPT == 4) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else if (LPT == 2) asm volatile("s_waitcnt vmcnt(2) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(1) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    MADAKV_DMA_ISSUE(min(t + 2, ntiles - 1))   // into the slot of tile t - 1 (past the end: the last tile once more, which keeps the count of loads in flight)
    if (PASS == 2 && t > 0 && tid < DMA_TK) {  // the column sums of tile t - 1, the waves' shares added in wave order
      const int key = chunk0 + (t - 1) * DMA_TK + tid;
      const uint32_t r4 = red_lds + (uint32_t)((((t - 1) & 1) * NW * DMA_TK + tid) * 4);
      static_assert(NW == 4 || PASS == 1, "sweep 2 adds four waves' shares");
      float c0, c1, c2, c3;
      asm volatile("ds_read_b32 %0, %4\n\tds_read_b32 %1, %4 offset:256\n\tds_read_b32 %2, %4 offset:512\n\tds_read_b32 %3, %4 offset:768\n\ts_waitcnt lgkmcnt(0)"
                   : "=&v"(c0), "=&v"(c1), "=&v"(c2), "=&v"(c3) : "v"(r4) : "memory");
      if (key < chunk1) __builtin_nontemporal_store(((c0 + c1) + c2) + c3, a.psi + ((long long)head * a.L + key));
    }
    const uint32_t tile_lds = ring_lds + (uint32_t)(t % DMA_NBUF) * TILEB;
    const int tile_end = chunk0 + (t + 1) * DMA_TK;
    const bool tail = tile_end > first_masked || tile_end > chunk1;

    // Sweep 2's vector arithmetic runs on the BS logits a lane holds of every row after the contractions of BS
    // subtiles.  In a tail tile (it holds keys that some proxy row must not see: the last W - 1 keys of the head,
    // keys past the chunk's end) such logits become NEG_BIG, in both sweeps.
#define MADAKV_DMA_VECTOR(TAIL)                                                                      \
    _Pragma("unroll") for (int b = 0; b < NRB; ++b) {                                                \
      _Pragma("unroll") for (int j = 0; j < 16; ++j) {                                               \
        float x[BS];                                                                                 \
        _Pragma("unroll") for (int u = 0; u < BS; ++u) {                                             \
          x[u] = acc[u][b][j];                                                                       \
          if (TAIL) {                                                                                \
            const int key = chunk0 + t * DMA_TK + (s0 + u) * 32 + col;                               \
            const int row = (rb0 + b) * 32 + (j >> 2) * 8 + half * 4 + (j & 3);                      \
            const int pos = a.L - a.W + (row % a.W);                                                 \
            const bool valid = (key < chunk1) && (key <= pos) && (row < a.M);                        \
            x[u] = valid ? x[u] : NEG_BIG;                                                           \
          }                                                                                          \
        }                                                                                            \
        _Pragma("unroll") for (int u = 0; u < BS; ++u) colsum[u] += fast_exp2(fmaf(x[u], a.scale_log2, -st_m[b][j])); \
      }                                                                                              \
    }
    // Sweep 1 on one subtile: S^T = K Q^T, so that D[key][row] leaves a lane with the logits of its own row
    // (row `col` of the block) against 16 keys: keys t0 + 8 (j >> 2) + 4 half + (j & 3).  The row's maximum and sum
    // are then in-lane work, one rescaling of the sum per subtile; the two halves of a row meet after the last tile.
    // The running maximum stays in accumulator units (scale > 0).  A row that has seen no key yet holds NEG_BIG and
    // a meaningless, finite sum, which the first real key (and any merge with real statistics) multiplies by
    // exp2(-huge) = 0.
#define MADAKV_DMA_ROWS(TAIL)                                                                        \
    _Pragma("unroll") for (int b = 0; b < NRB; ++b) {                                                \
      f32x16_t xt = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}; \
      _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                              \
        xt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag[0][ks], areg[b][ks], xt, 0, 0, 0);        \
      if (TAIL) {                                                                                    \
        const int row = (rb0 + b) * 32 + col;                                                        \
        const int pos = a.L - a.W + (row % a.W);                                                     \
        _Pragma("unroll") for (int j = 0; j < 16; ++j) {                                             \
          const int key = chunk0 + t * DMA_TK + s0 * 32 + 8 * (j >> 2) + 4 * half + (j & 3);         \
          xt[j] = ((key < chunk1) && (key <= pos) && (row < a.M)) ? xt[j] : NEG_BIG;                 \
        }                                                                                            \
      }                                                                                              \
      float mn = row_m[b];                                                                           \
      _Pragma("unroll") for (int j = 0; j < 16; ++j) mn = fmaxf(mn, xt[j]);                          \
      float l = row_l[b] * fast_exp2((row_m[b] - mn) * a.scale_log2);                                \
      /* (no key of the row seen yet: every x is NEG_BIG too, and x * scale - round(NEG_BIG * scale) would be the   \
         product's rounding error, some 1e21 of either sign; against 0 the terms are exp2(-huge) = 0) */            \
      const float ms = mn > 0.5f * NEG_BIG ? mn * a.scale_log2 : 0.f;                                \
      _Pragma("unroll") for (int j = 0; j < 16; ++j) l += fast_exp2(fmaf(xt[j], a.scale_log2, -ms)); \
      row_m[b] = mn; row_l[b] = l;                                                                   \
    }
#pragma unroll 1
    for (int s0 = 0; s0 < NSUB; s0 += BS) {
      f32x16_t acc[BS][NRB];
      float colsum[BS];
#pragma unroll
      for (int u = 0; u < BS; ++u) colsum[u] = 0.f;
      bf16x8_t bfrag[BS][KS];
#pragma unroll
      for (int u = 0; u < BS; ++u) {
        const uint32_t sub_lds = tile_lds + (uint32_t)(s0 + u) * 32 * ROWB;
        if (KS == 8) {
          asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %10\n\tds_read_b128 %3, %11\n\t"
                       "ds_read_b128 %4, %12\n\tds_read_b128 %5, %13\n\tds_read_b128 %6, %14\n\tds_read_b128 %7, %15\n\t"
                       "s_waitcnt lgkmcnt(0)"
                       : "=&v"(bfrag[u][0]), "=&v"(bfrag[u][1]), "=&v"(bfrag[u][2]), "=&v"(bfrag[u][3]), "=&v"(bfrag[u][4 % KS]), "=&v"(bfrag[u][5 % KS]), "=&v"(bfrag[u][6 % KS]), "=&v"(bfrag[u][7 % KS])
                       : "v"(sub_lds + frag_off[0]), "v"(sub_lds + frag_off[1]), "v"(sub_lds + frag_off[2]), "v"(sub_lds + frag_off[3]),
                         "v"(sub_lds + frag_off[4 % KS]), "v"(sub_lds + frag_off[5 % KS]), "v"(sub_lds + frag_off[6 % KS]), "v"(sub_lds + frag_off[7 % KS])
                       : "memory");
        } else {
          asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b128 %3, %7\n\t"
                       "s_waitcnt lgkmcnt(0)"
                       : "=&v"(bfrag[u][0]), "=&v"(bfrag[u][1]), "=&v"(bfrag[u][2]), "=&v"(bfrag[u][3])
                       : "v"(sub_lds + frag_off[0]), "v"(sub_lds + frag_off[1]), "v"(sub_lds + frag_off[2]), "v"(sub_lds + frag_off[3])
                       : "memory");
        }
        if (BS > 1) {                            // (a batch of several subtiles: its contractions as the fragments come)
#pragma unroll
          for (int b = 0; b < NRB; ++b) {
            acc[u][b] = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
              acc[u][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(areg[b][ks], bfrag[u][ks], acc[u][b], 0, 0, 0);
          }
        }
      }
      // One subtile per batch: contractions and vector arithmetic of the subtile in one stretch of straight-line
      // code, so that the second row block's contraction can be issued between the first block's vector
      // instructions (a wave issues in order: what follows a matrix instruction that waits for its predecessor
      // waits with it).
#define MADAKV_DMA_CONTRACT                                                                          \
      if (BS == 1) {                                                                                 \
        _Pragma("unroll") for (int b = 0; b < NRB; ++b) {                                            \
          acc[0][b] = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}; \
          _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                          \
            acc[0][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(areg[b][ks], bfrag[0][ks], acc[0][b], 0, 0, 0); \
        }                                                                                            \
      }
      if (PASS == 1) {
        static_assert(PASS == 2 || BS == 1, "sweep 1 takes one subtile at a time");
        (void)acc;
        if (tail) { MADAKV_DMA_ROWS(true) } else { MADAKV_DMA_ROWS(false) }
      } else if (tail) {
        MADAKV_DMA_CONTRACT
        MADAKV_DMA_VECTOR(true)
      } else {
        MADAKV_DMA_CONTRACT
        MADAKV_DMA_VECTOR(false)
        if (BS == 1 && NRB == 2 && PASS == 2 && KS == 8) {
          // the order asked of the compiler: the first block's eight matrix instructions, then each of the second
          // block's followed by four plain and two exp2 instructions of the first block's arithmetic
          __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
          }
        }
      }
#undef MADAKV_DMA_CONTRACT
      if (PASS == 2) {
#pragma unroll
        for (int u = 0; u < BS; ++u) {
          const float cs = colsum[u] + __shfl_xor(colsum[u], 32, 64);
          const uint32_t dst = red_lds + (uint32_t)((((t & 1) * NW + wave) * DMA_TK + (s0 + u) * 32 + col) * 4);
          if (half == 0) asm volatile("ds_write_b32 %0, %1" :: "v"(dst), "v"(cs) : "memory");
        }
      }
    }
#undef MADAKV_DMA_VECTOR
#undef MADAKV_DMA_ROWS
  }
#undef MADAKV_DMA_ISSUE
  // nothing may still be on its way into this workgroup's LDS when it ends
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

  if (PASS == 2) {
    if (tid < DMA_TK) {
      const int key = chunk0 + (ntiles - 1) * DMA_TK + tid;
      const uint32_t r4 = red_lds + (uint32_t)((((ntiles - 1) & 1) * NW * DMA_TK + tid) * 4);
      float c0, c1, c2, c3;
      asm volatile("ds_read_b32 %0, %4\n\tds_read_b32 %1, %4 offset:256\n\tds_read_b32 %2, %4 offset:512\n\tds_read_b32 %3, %4 offset:768\n\ts_waitcnt lgkmcnt(0)"
                   : "=&v"(c0), "=&v"(c1), "=&v"(c2), "=&v"(c3) : "v"(r4) : "memory");
      if (key < chunk1) __builtin_nontemporal_store(((c0 + c1) + c2) + c3, a.psi + ((long long)head * a.L + key));
    }
  } else {
    // the two halves of a row (their keys interleave in groups of four) meet; lanes 0..31 hold rows 0..31 of a block
    float* rs = a.rowstat + ((long long)head * a.nsplit + split) * a.mpad * 2;
#pragma unroll
    for (int b = 0; b < NRB; ++b) {
      const float m2 = __shfl_xor(row_m[b], 32, 64), l2 = __shfl_xor(row_l[b], 32, 64);
      const float m = fmaxf(row_m[b], m2);
      const float l = row_l[b] * fast_exp2((row_m[b] - m) * a.scale_log2) + l2 * fast_exp2((m2 - m) * a.scale_log2);
      if (rb0 + b < MB && half == 0) {
        const int row = (rb0 + b) * 32 + col;
        rs[row * 2] = m * a.scale_log2; rs[row * 2 + 1] = l;
      }
    }
  }
}

// ------------------------------------------------------------------------------------
// One sweep over K (bf16, at most two row blocks: G*W <= 64).  The logits of a workgroup's
// keys fit in its registers: a wave keeps the D tiles of its NS subtiles (NS * NRB * 16 floats
// per lane) instead of reducing them on the fly.  After its last subtile a workgroup knows the
// (max, sum) of every proxy row over its own keys; the workgroups of a head exchange these
// through memory, every one merges all of them in the same fixed order, and the column sums
// come out of the registers: K is read once and multiplied once.
//
// The exchange: a (max, sum) pair is one 64-bit word, stored with a relaxed agent-scope atomic
// store and read with relaxed agent-scope atomic loads until it differs from the all-ones
// pattern the array is filled with before the launch; the word carries its own arrival, so no
// fence and no counter is needed.  A workgroup waits only for workgroups of its own head.  Those
// have consecutive workgroup ids (the chunk index is the fast grid dimension), workgroups are
// dispatched in id order, and a head has far fewer chunks than the chip has workgroup slots, so
// the workgroups waited for are already running or next in line for the slots that free up.
// The wait is bounded all the same: a workgroup that runs out of patience counts itself in
// status[0] and computes the row statistics of the whole head on its own with plain FMA code
// (slow, and its last bits differ from the exchanged ones, but it depends on nobody).
// ------------------------------------------------------------------------------------
// 4 E4M3 bytes -> 4 bf16 (exact: 3 mantissa bits fit bf16's 7), as two packed dwords
__device__ __forceinline__ u32x2_t e4m3x4_as_bf16x4(uint32_t w) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
  u32x2_t o;
  o[0] = (__float_as_uint(a[0]) >> 16) | (__float_as_uint(a[1]) & 0xffff0000u);
  o[1] = (__float_as_uint(b[0]) >> 16) | (__float_as_uint(b[1]) & 0xffff0000u);
  return o;
}

constexpr unsigned long long XCHG_EMPTY = ~0ULL;
constexpr int FUSED_SPIN_LIMIT = 1 << 16;     // default spin_limit: polls of ~1 us each

__global__ __launch_bounds__(256) void score_xchg_init_kernel(unsigned long long* xchg, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) xchg[i] = XCHG_EMPTY;
}

// Row statistics of a whole head by one workgroup, without matrix cores and without anybody
// else: wave w takes rows w, w + 4, ...; lanes stride over the keys the row sees.  Q comes from
// the staged tile.  Leaves offs[r] = max + log2(sum) (log2 domain), +inf for padding rows.
template <int D, bool F8 = false>
__device__ __forceinline__ void score_head_stats_alone(const ScoreArgs& a, int Lh, int Mh, int rowbase, const uint16_t* kg, const uint16_t* qs, float* offs) {
  constexpr int RS = D + 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int r = wave; r < a.mpad; r += 4) {
    float m = NEG_BIG, l = 0.f;
    if (r < Mh) {
      const int pos = Lh - a.W + ((rowbase + r) % a.W);
      for (int key = lane; key <= pos; key += 64) {
        float sdot = 0.f;
        for (int c = 0; c < D / 8; ++c) {
          uint4 kk;
          if (F8) {      // 8 of the row's D bytes -> 8 bf16
            const u32x2_t raw = *reinterpret_cast<const u32x2_t*>(reinterpret_cast<const unsigned char*>(kg) + (long long)key * D + c * 8);
            const u32x2_t lo = e4m3x4_as_bf16x4(raw[0]), hi = e4m3x4_as_bf16x4(raw[1]);
            kk = make_uint4(lo[0], lo[1], hi[0], hi[1]);
          } else {
            kk = *reinterpret_cast<const uint4*>(kg + (long long)key * D + c * 8);
          }
          const uint4 qq = *reinterpret_cast<const uint4*>(qs + r * RS + c * 8);
          sdot = fmaf(bf16_lo(kk.x), bf16_lo(qq.x), sdot); sdot = fmaf(bf16_hi(kk.x), bf16_hi(qq.x), sdot);
          sdot = fmaf(bf16_lo(kk.y), bf16_lo(qq.y), sdot); sdot = fmaf(bf16_hi(kk.y), bf16_hi(qq.y), sdot);
          sdot = fmaf(bf16_lo(kk.z), bf16_lo(qq.z), sdot); sdot = fmaf(bf16_hi(kk.z), bf16_hi(qq.z), sdot);
          sdot = fmaf(bf16_lo(kk.w), bf16_lo(qq.w), sdot); sdot = fmaf(bf16_hi(kk.w), bf16_hi(qq.w), sdot);
        }
        const float s2 = sdot * a.scale_log2;
        const float mn = fmaxf(m, s2);
        l = l * exp2f(m - mn) + exp2f(s2 - mn);
        m = mn;
      }
      for (int o = 1; o < 64; o <<= 1) {
        const float m2 = __shfl_xor(m, o, 64), l2 = __shfl_xor(l, o, 64);
        merge_ml(m, l, m2, l2);
      }
    }
    if (lane == 0) offs[r] = (r < Mh) ? m + log2f(l) : __builtin_inff();
  }
}

// After a workgroup has left the (max, sum) of every proxy row over its own keys in part[4 waves][mpad][2]
// (LDS, behind a barrier): the head-wide exchange described above, in two halves.  post_row_stats
// publishes this workgroup's words and waits for nobody; collect_row_stats gathers the head's words and
// leaves offs[r] = max + log2(sum) over all keys of the head (log2 domain; +inf for padding rows).
// All threads call both; work that needs nobody else's statistics can sit between them.  The caller
// adds the barrier after collect_row_stats.
__device__ __forceinline__ void post_row_stats(const ScoreArgs& a, int head, int slot, int fs, const float* part) {   // slot: the chunk, or a word of the group level
  const int tid = threadIdx.x;
  if (fs == 1 || tid >= a.mpad) return;
  // a row none of whose keys here is visible has max NEG_BIG and a meaningless sum: merging it with
  // anything real scales it by exp2(NEG_BIG - m) = 0
  unsigned long long* xh = a.xchg + (long long)head * a.xstride;
  float m = NEG_BIG, l = 0.f;
  for (int w = 0; w < 4; ++w) merge_ml(m, l, part[(w * a.mpad + tid) * 2], part[(w * a.mpad + tid) * 2 + 1]);
  unsigned long long word = ((unsigned long long)__float_as_uint(l) << 32) | __float_as_uint(m);
  if (word == XCHG_EMPTY) word = 0x7fc000007fc00000ULL;            // cannot happen with finite inputs
  __hip_atomic_store(xh + (long long)slot * a.mpad + tid, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Thread (r, pt) of the workgroup merges, in order, its share of the `n` words base[item * mpad + r]
// (items [pt * cpp, (pt + 1) * cpp), cpp = ceil(n / parts)), waiting for each at most spin_limit polls,
// eight loads at a time; leaves (max, sum) in pm[(pt * mpad + r) * 2 ..] and raises *s_fail if a word stayed away.
__device__ __forceinline__ void poll_row_words(const ScoreArgs& a, const unsigned long long* base, int n, float* pm, int* s_fail) {
  const int tid = threadIdx.x;
  const int nparts = SCORE_THREADS / a.mpad;    // mpad is 32 or 64
  const int r = tid % a.mpad, pt = tid / a.mpad;
  const int cpp = (n + nparts - 1) / nparts;
  int s = min(pt * cpp, n);
  const int s1 = min(s + cpp, n);
  float m = NEG_BIG, l = 0.f;
  int patience = a.spin_limit;
  bool fail = false;
  while (s < s1) {
    unsigned long long v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
      v[j] = __hip_atomic_load(base + (long long)min(s + j, s1 - 1) * a.mpad + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int got = 0;
    bool open = true;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      open = open && (s + j < s1) && (v[j] != XCHG_EMPTY);
      if (open) { merge_ml(m, l, __uint_as_float((uint32_t)v[j]), __uint_as_float((uint32_t)(v[j] >> 32))); ++got; }
    }
    s += got;
    if (got == 0) {
      if (--patience == 0) { fail = true; break; }
      __builtin_amdgcn_s_sleep(8);
    }
  }
  if (fail) *s_fail = 1;
  pm[(pt * a.mpad + r) * 2] = m;
  pm[(pt * a.mpad + r) * 2 + 1] = l;
}

constexpr int XCHG_GROUP = 16;       // chunks per group when the exchange has two levels

template <int D, bool F8 = false>
__device__ __forceinline__ void collect_row_stats(const ScoreArgs& a, int head, int split, int fs, int Lh, int Mh, int rowbase,
                                                  const uint16_t* kg, const uint16_t* qs, const float* part, float* offs, float* pm, int* s_fail) {
  const int tid = threadIdx.x;
  const int nparts = SCORE_THREADS / a.mpad;
  if (fs == 1) {
    if (tid < a.mpad) {
      float m = NEG_BIG, l = 0.f;
      for (int w = 0; w < 4; ++w) merge_ml(m, l, part[(w * a.mpad + tid) * 2], part[(w * a.mpad + tid) * 2 + 1]);
      offs[tid] = (tid < Mh) ? m + log2f(l) : __builtin_inff();
    }
    return;
  }
  unsigned long long* xh = a.xchg + (long long)head * a.xstride;
  if (a.xgroups == 0) {
    poll_row_words(a, xh, fs, pm, s_fail);
  } else {
    // Two levels, so that a workgroup reads tens of words per row instead of one per chunk of a long head.
    // The workgroup of a group's last chunk (it starts after the group's others) merges the group's
    // words and leaves one word per row for the group; everybody merges the groups' words.
    unsigned long long* gw = xh + (long long)fs * a.mpad;
    const int g = split / XCHG_GROUP, c0 = g * XCHG_GROUP, c1 = min(c0 + XCHG_GROUP, fs);
    if (split == c1 - 1) {
      poll_row_words(a, xh + (long long)c0 * a.mpad, c1 - c0, pm, s_fail);
      __syncthreads();
      if (!*s_fail && tid < a.mpad) {
        float mm = NEG_BIG, ll = 0.f;
        for (int q = 0; q < nparts; ++q) merge_ml(mm, ll, pm[(q * a.mpad + tid) * 2], pm[(q * a.mpad + tid) * 2 + 1]);
        unsigned long long word = ((unsigned long long)__float_as_uint(ll) << 32) | __float_as_uint(mm);
        if (word == XCHG_EMPTY) word = 0x7fc000007fc00000ULL;
        __hip_atomic_store(gw + (long long)g * a.mpad + tid, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __syncthreads();                              // pm is written again below
    }
    if (!*s_fail) poll_row_words(a, gw, a.xgroups, pm, s_fail);   // (uniform: s_fail was read behind a barrier)
  }
  __syncthreads();
  if (__builtin_expect(*s_fail, 0)) {         // uniform over the workgroup
    if (tid == 0) atomicAdd(a.status, 1);
    score_head_stats_alone<D, F8>(a, Lh, Mh, rowbase, kg, qs, offs);
  } else if (tid < a.mpad) {
    float mm = NEG_BIG, ll = 0.f;
    for (int q = 0; q < nparts; ++q) merge_ml(mm, ll, pm[(q * a.mpad + tid) * 2], pm[(q * a.mpad + tid) * 2 + 1]);
    offs[tid] = (tid < Mh) ? mm + log2f(ll) : __builtin_inff();
  }
}

template <int D, bool F8 = false>
__device__ __forceinline__ void exchange_row_stats(const ScoreArgs& a, int head, int split, int fs, int Lh, int Mh, int rowbase,
                                                   const uint16_t* kg, const uint16_t* qs, const float* part, float* offs, float* pm, int* s_fail) {
  post_row_stats(a, head, split, fs, part);
  collect_row_stats<D, F8>(a, head, split, fs, Lh, Mh, rowbase, kg, qs, part, offs, pm, s_fail);
}

#ifndef MADAKV_FUSED_NS1      // tuning constants of the one-sweep kernel (measured on MI355X)
#define MADAKV_FUSED_NS1 8    // subtiles per wave with one row block
#define MADAKV_FUSED_NS2 6    // ... with two row blocks
#define MADAKV_FUSED_PF 2     // subtiles in flight per wave
#define MADAKV_FUSED_WPE 2    // waves per SIMD
#endif
#ifndef MADAKV_FUSED_MAX_SPLIT
#define MADAKV_FUSED_MAX_SPLIT 64   // most chunks per head the one-sweep kernel is used for
#endif
template <int D, int NRB, int NS, bool F8 = false>   // F8: the keys are E4M3 bytes (the 8-bit reduced cache), turned into bf16 when parked in LDS
__global__ __launch_bounds__(SCORE_THREADS) __attribute__((amdgpu_waves_per_eu(MADAKV_FUSED_WPE, MADAKV_FUSED_WPE))) void score_fused_kernel(ScoreArgs a) {
  constexpr int PF = MADAKV_FUSED_PF < NS ? MADAKV_FUSED_PF : NS;
  constexpr int KS = D / 16;                  // MFMA k-steps
  constexpr int RS = D + 8;                   // bf16 elements per LDS row (16 B pad)
  constexpr int PPR = D / 8;                  // 16-byte pieces per row
  constexpr int LPS = 32 * PPR / 64;          // 16-byte loads per lane per subtile
  constexpr int CK = 4 * NS * 32;             // keys per workgroup
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* qs = reinterpret_cast<uint16_t*>(smem);                       // [mpad][RS]
  uint16_t* kt_all = qs + (size_t)a.mpad * RS;                            // [4 waves][32][RS]
  float* part = reinterpret_cast<float*>(kt_all + 4 * 32 * RS);           // [4 waves][mpad][2]
  float* offs = part + 4 * a.mpad * 2;                                    // [mpad]
  float* pm = offs + a.mpad;                                              // [256 / mpad parts][mpad][2]
  __shared__ int s_fail;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int bx = blockIdx.x;                  // (the parked chunks first: split is set below, once fs is known)
  const int hv = a.head0 + blockIdx.y;        // head, or (head, block of 64 proxy rows) when there are more than 64
  const int head = hv / a.rb_count;
  const int rowbase = (hv % a.rb_count) * 64; // first proxy row of this workgroup's block
  const int Mh = min(a.M - rowbase, a.mpad);  // its rows
  const int kvh = head % a.H;
  const long long lb = head / a.H;            // (layer, batch) index
  const uint16_t* qg = reinterpret_cast<const uint16_t*>(a.q_win) + ((lb * a.H + kvh) * (long long)a.G * a.W + rowbase) * D;
  // keys of this head: L rows at head * L, or (ragged: the rows of a reduced cache) seg_len rows at seg_off
  const int Lh = a.seg_len ? a.seg_len[head] : a.L;
  const long long base = a.seg_off ? a.seg_off[head] : (long long)head * a.L;
  const int fs = a.seg_len ? (Lh + CK - 1) / CK : a.fsplit;      // chunks of this head (the grid is sized for the longest)
  const int split = bx < a.nstrag ? fs + bx : bx - a.nstrag;
  if (split >= fs + a.nstrag) return;
  const bool parked = split >= fs;            // one of the head's last chunks, run ahead of the others
  // (F8: rows of D bytes; kg then counts in 2-byte units from a byte address that is base * D)
  const uint16_t* kg = F8 ? reinterpret_cast<const uint16_t*>(reinterpret_cast<const unsigned char*>(a.k) + base * D)
                          : reinterpret_cast<const uint16_t*>(a.k) + base * D;
  const int chunk0 = split * CK;
  const int chunk1 = min(Lh, chunk0 + CK);
  uint16_t* kt = kt_all + (size_t)wave * 32 * RS;
  if (tid == 0) s_fail = 0;

  // subtile `it` of this wave: keys chunk0 + (it * 4 + wave) * 32 ...; PF subtiles in flight
  constexpr int CPR = F8 ? PPR / 2 : PPR;      // 16-byte pieces per cached row
  constexpr int LPSK = F8 ? LPS / 2 : LPS;     // loads per lane and subtile
  u32x4_t pre[PF][LPSK];
#define MADAKV_FUSED_LOAD(SET, IT)                                                               \
  {                                                                                              \
    const int lt0 = chunk0 + ((IT) * 4 + wave) * 32;                                             \
    _Pragma("unroll") for (int i = 0; i < LPSK; ++i) {                                           \
      const int idx = i * 64 + lane;                                                             \
      const int lkey = min(lt0 + idx / CPR, Lh - 1); /* past the end: a valid row, masked later */ \
      pre[SET][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(                 \
          reinterpret_cast<const unsigned char*>(kg) + ((long long)lkey * CPR + (idx % CPR)) * 16)); \
    }                                                                                            \
  }
#pragma unroll
  for (int it = 0; it < PF; ++it) MADAKV_FUSED_LOAD(it, it)

  for (int e = tid; e < a.mpad * PPR; e += SCORE_THREADS) {               // Q tile, padding rows zero
    const int r = e / PPR, c = e % PPR;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (r < Mh) val = *reinterpret_cast<const uint4*>(qg + (long long)r * D + c * 8);
    *reinterpret_cast<uint4*>(qs + r * RS + c * 8) = val;
  }
  __syncthreads();

  const int half = lane >> 5, col = lane & 31;
  const int first_masked = Lh - a.W + 1;      // keys below this are visible to every proxy row
  bf16x8_t areg[KS];                           // one row block: its Q fragments stay in registers
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    areg[ks] = *reinterpret_cast<const bf16x8_t*>(qs + col * RS + half * (D / 2) + ks * 8);

  float lg[NS][NRB][16];                       // scaled logits (log2 domain); masked entries hold NEG_BIG
#pragma unroll
  for (int it = 0; it < NS; ++it) {
#pragma unroll
    for (int i = 0; i < LPSK; ++i) {
      const int idx = i * 64 + lane;
      if (F8) {                                   // 16 bytes of a row -> 16 bf16
        const u32x4_t raw = pre[it % PF][i];
        const u32x2_t c0 = e4m3x4_as_bf16x4(raw[0]), c1 = e4m3x4_as_bf16x4(raw[1]), c2 = e4m3x4_as_bf16x4(raw[2]), c3 = e4m3x4_as_bf16x4(raw[3]);
        *reinterpret_cast<u32x4_t*>(kt + (idx / CPR) * RS + (idx % CPR) * 16) = u32x4_t{c0[0], c0[1], c1[0], c1[1]};
        *reinterpret_cast<u32x4_t*>(kt + (idx / CPR) * RS + (idx % CPR) * 16 + 8) = u32x4_t{c2[0], c2[1], c3[0], c3[1]};
      } else {
        *reinterpret_cast<u32x4_t*>(kt + (idx / PPR) * RS + (idx % PPR) * 8) = pre[it % PF][i];
      }
    }
    if (it + PF < NS) MADAKV_FUSED_LOAD(it % PF, it + PF)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int t0 = chunk0 + (it * 4 + wave) * 32;
    const int key = t0 + col;
    const bool tail = (t0 + 32 > first_masked) || (t0 + 32 > chunk1);     // (padding rows need no mask: their offset is +inf)
    const uint16_t* krow = kt + col * RS + half * (D / 2);
    bf16x8_t bfrag[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) bfrag[ks] = *reinterpret_cast<const bf16x8_t*>(krow + ks * 8);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int b = 0; b < NRB; ++b) {
      f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      const uint16_t* qrow = qs + (b * 32 + col) * RS + half * (D / 2);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8_t afrag = (NRB == 1) ? areg[ks] : *reinterpret_cast<const bf16x8_t*>(qrow + ks * 8);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[ks], acc, 0, 0, 0);
      }
      if (!tail) {
#pragma unroll
        for (int j = 0; j < 16; ++j) lg[it][b][j] = acc[j] * a.scale_log2;
      } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int row = b * 32 + (j >> 2) * 8 + half * 4 + (j & 3);
          const int pos = Lh - a.W + ((rowbase + row) % a.W);
          const bool valid = (key < chunk1) && (key <= pos) && (row < Mh);
          lg[it][b][j] = valid ? acc[j] * a.scale_log2 : NEG_BIG;
        }
      }
    }
  }
#undef MADAKV_FUSED_LOAD

  // ---- (max, sum) of every row over this workgroup's keys: lanes, then waves (fixed order)
#pragma unroll
  for (int b = 0; b < NRB; ++b) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      float mx = lg[0][b][j];
#pragma unroll
      for (int it = 1; it < NS; ++it) mx = fmaxf(mx, lg[it][b][j]);
      const float m = half_reduce<0>(mx);
      float sm = 0.f;
#pragma unroll
      for (int it = 0; it < NS; ++it) sm += fast_exp2(lg[it][b][j] - m);   // masked entries against a real maximum: 0
      const float l = half_reduce<1>(sm);
      if (col == 0) {
        const int row = b * 32 + (j >> 2) * 8 + half * 4 + (j & 3);
        part[(wave * a.mpad + row) * 2] = m;
        part[(wave * a.mpad + row) * 2 + 1] = l;
      }
    }
  }
  __syncthreads();
  if (parked) {
    // its statistics as a word of the group level (behind the groups' own), its logits to memory; nobody is waited for
    post_row_stats(a, hv, fs + (a.xgroups - a.nstrag) + (split - fs), fs, part);
    float* pk = a.park + ((long long)hv * a.nstrag + (split - fs)) * (NS * NRB * 16 * SCORE_THREADS);
#pragma unroll
    for (int it = 0; it < NS; ++it)
#pragma unroll
      for (int b = 0; b < NRB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) __builtin_nontemporal_store(lg[it][b][j], pk + ((it * NRB + b) * 16 + j) * SCORE_THREADS + tid);
    return;
  }
  exchange_row_stats<D, F8>(a, hv, split, fs, Lh, Mh, rowbase, kg, qs, part, offs, pm, &s_fail);
  __syncthreads();
  if (a.offs_out && split == 0 && tid < a.mpad) a.offs_out[(long long)hv * a.mpad + tid] = offs[tid];

  // ---- column sums from the registers
  float off_r[NRB][16];
#pragma unroll
  for (int b = 0; b < NRB; ++b)
#pragma unroll
    for (int j = 0; j < 16; ++j) off_r[b][j] = offs[b * 32 + (j >> 2) * 8 + half * 4 + (j & 3)];
#pragma unroll
  for (int it = 0; it < NS; ++it) {
    float colsum = 0.f;
#pragma unroll
    for (int b = 0; b < NRB; ++b)
#pragma unroll
      for (int j = 0; j < 16; ++j) colsum += fast_exp2(lg[it][b][j] - off_r[b][j]);
    colsum += __shfl_xor(colsum, 32, 64);
    const int key = chunk0 + (it * 4 + wave) * 32 + col;
    if (half == 0 && key < chunk1) __builtin_nontemporal_store(colsum, (a.rb_count > 1 ? a.psi_part + (hv % a.rb_count) * a.psi_part_stride : a.psi) + (base + key));
  }
}

// The parked chunks' column sums, from their logits and the heads' row offsets: the arithmetic (and its order) of the
// kernel's own last step.  Grid (parked chunk, head).
template <int NRB, int NS>
__global__ __launch_bounds__(SCORE_THREADS) void score_fused_finish_kernel(ScoreArgs a) {
  constexpr int CK = 4 * NS * 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int hv = a.head0 + blockIdx.y, sidx = blockIdx.x;
  const int chunk0 = (a.fsplit + sidx) * CK;
  const int chunk1 = min(a.L, chunk0 + CK);
  const float* pk = a.park + ((long long)hv * a.nstrag + sidx) * (NS * NRB * 16 * SCORE_THREADS);
  const float* offs = a.offs_out + (long long)hv * a.mpad;
  float off_r[NRB][16];
#pragma unroll
  for (int b = 0; b < NRB; ++b)
#pragma unroll
    for (int j = 0; j < 16; ++j) off_r[b][j] = offs[b * 32 + (j >> 2) * 8 + half * 4 + (j & 3)];
#pragma unroll
  for (int it = 0; it < NS; ++it) {
    float colsum = 0.f;
#pragma unroll
    for (int b = 0; b < NRB; ++b)
#pragma unroll
      for (int j = 0; j < 16; ++j) colsum += fast_exp2(__builtin_nontemporal_load(pk + ((it * NRB + b) * 16 + j) * SCORE_THREADS + tid) - off_r[b][j]);
    colsum += __shfl_xor(colsum, 32, 64);
    const int key = chunk0 + (it * 4 + wave) * 32 + col;
    if (half == 0 && key < chunk1) __builtin_nontemporal_store(colsum, a.psi + ((long long)hv * a.L + key));
  }
}

// ------------------------------------------------------------------------------------
// The prefill attention of the last W prompt positions (paper Sec. 3.1 Eq. 5 for the proxy rows of
// Sec. 3.3) with the proxy-token scores of Eq. 7 as a by-product: out = softmax(scale Q K^T) V for
// a block of up to 32 of the G*W proxy rows of a KV head (more rows: more blocks, each with a pass of its own over
// K and V, their column sums added in block order afterwards), their log-sum-exp, and psi = the column sums of the same
// softmax rows.  A model's prefill runs this attention anyway; taking psi from it removes the
// eviction's own sweep over K.
// Same structure as score_fused_kernel (a workgroup's logits stay in registers while the row
// statistics travel among the head's workgroups), with the contraction transposed: S^T = K Q^T, so a
// lane holds one proxy row and 16 keys of a subtile.  Row statistics are then in-lane, the
// column sums of Eq. 7 one half-wave reduction per key, and P is already laid out as the A
// operand of O += P V: the contraction index of that product is numbered so that a lane's
// eight keys of a 16-key step are the eight it holds.  V subtiles are streamed through the same
// wave-private LDS tile as K was; a B fragment (eight keys of one output column) is gathered
// from it two bytes at a time.  P goes in as bf16 hi + lo parts (two MFMAs), which keeps
// fp32-level accuracy.  The V sweep does not wait for the exchange: it exponentiates against the
// wave's own row maxima, and the head-wide statistics, collected after it, enter as one factor per
// row (for O and for the column sums alike).  Every workgroup leaves its share of O, normalised
// that way, in memory; window_attn_reduce_kernel adds the shares in chunk order.
// ------------------------------------------------------------------------------------
struct WinArgs {
  ScoreArgs s;
  const void* v;       // [heads, L, d]
  float* opart;        // [heads, fsplit, 32, d] shares of O
  float* lse;          // optional [heads/H * Hq, W] natural log-sum-exp of every proxy row
  void* out;           // [heads/H * Hq, W, d]
  int out_fp32;
};

template <int D, int NS>
__global__ __launch_bounds__(SCORE_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void window_attn_kernel(WinArgs wa) {
  const ScoreArgs& a = wa.s;
  constexpr int KS = D / 16, RS = D + 8, PPR = D / 8, LPS = 32 * PPR / 64, CK = 4 * NS * 32, PF = 2, DB = D / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* qs = reinterpret_cast<uint16_t*>(smem);                       // [32][RS]
  uint16_t* kt_all = qs + 32 * RS;                                        // [4 waves][32][RS]
  float* part = reinterpret_cast<float*>(kt_all + 4 * 32 * RS);           // [4 waves][32][2]
  float* offs = part + 4 * 32 * 2;                                        // [32]
  float* pm = offs + 32;                                                  // [8 parts][32][2]
  __shared__ int s_fail;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x;
  const int hv = a.head0 + blockIdx.y;        // head, or (head, block of 32 proxy rows) when there are more than 32
  const int head = hv / a.rb_count;
  const int rowbase = (hv % a.rb_count) * 32; // first proxy row of this workgroup's block
  const int Mh = min(a.M - rowbase, 32);      // its rows
  const int kvh = head % a.H;
  const long long lb = head / a.H;
  const uint16_t* qg = reinterpret_cast<const uint16_t*>(a.q_win) + ((lb * a.H + kvh) * (long long)a.G * a.W + rowbase) * D;
  const uint16_t* kg = reinterpret_cast<const uint16_t*>(a.k) + (long long)head * a.L * D;
  const uint16_t* vg = reinterpret_cast<const uint16_t*>(wa.v) + (long long)head * a.L * D;
  const int Lh = a.L, fs = a.fsplit;
  const int chunk0 = split * CK;
  const int chunk1 = min(Lh, chunk0 + CK);
  uint16_t* kt = kt_all + (size_t)wave * 32 * RS;
  if (tid == 0) s_fail = 0;

  u32x4_t pre[PF][LPS];
#define MADAKV_WIN_LOAD(BASE, SET, IT)                                                           \
  {                                                                                              \
    const int lt0 = chunk0 + ((IT) * 4 + wave) * 32;                                             \
    _Pragma("unroll") for (int i = 0; i < LPS; ++i) {                                            \
      const int idx = i * 64 + lane;                                                             \
      const int lkey = min(lt0 + idx / PPR, Lh - 1); /* past the end: a valid row, masked */     \
      pre[SET][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(BASE + (long long)lkey * D + (idx % PPR) * 8)); \
    }                                                                                            \
  }
#define MADAKV_WIN_PARK(SET)                                                                     \
  _Pragma("unroll") for (int i = 0; i < LPS; ++i) {                                              \
    const int idx = i * 64 + lane;                                                               \
    *reinterpret_cast<u32x4_t*>(kt + (idx / PPR) * RS + (idx % PPR) * 8) = pre[SET][i];          \
  }
#pragma unroll
  for (int it = 0; it < PF; ++it) MADAKV_WIN_LOAD(kg, it, it)

  for (int e = tid; e < 32 * PPR; e += SCORE_THREADS) {                   // Q tile, padding rows zero
    const int r = e / PPR, c = e % PPR;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (r < Mh) val = *reinterpret_cast<const uint4*>(qg + (long long)r * D + c * 8);
    *reinterpret_cast<uint4*>(qs + r * RS + c * 8) = val;
  }
  __syncthreads();

  const int half = lane >> 5, col = lane & 31;            // col = this lane's proxy row (of the block)
  const int first_masked = Lh - a.W + 1;
  const int pos = Lh - a.W + ((rowbase + col) % a.W);     // last key the row sees
  bf16x8_t qfrag[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qfrag[ks] = *reinterpret_cast<const bf16x8_t*>(qs + col * RS + half * (D / 2) + ks * 8);

  // ---- S^T = K Q^T: lg[it][j] = scaled logit of row `col` and key t0 + 8 (j >> 2) + 4 half + (j & 3)
  float lg[NS][16];
#pragma unroll
  for (int it = 0; it < NS; ++it) {
    MADAKV_WIN_PARK(it % PF)
    if (it + PF < NS) MADAKV_WIN_LOAD(kg, it % PF, it + PF)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int t0 = chunk0 + (it * 4 + wave) * 32;
    const bool tail = (t0 + 32 > first_masked) || (t0 + 32 > chunk1) || (Mh < 32);
    const uint16_t* krow = kt + col * RS + half * (D / 2);
    f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8_t kfrag = *reinterpret_cast<const bf16x8_t*>(krow + ks * 8);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag, qfrag[ks], acc, 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int key = t0 + 8 * (j >> 2) + 4 * half + (j & 3);
      const bool valid = !tail || ((key < chunk1) && (key <= pos) && (col < Mh));
      lg[it][j] = valid ? acc[j] * a.scale_log2 : NEG_BIG;
    }
  }

  // ---- (max, sum) of the lane's row over this wave's keys: in-lane, then the two halves
  float mx = NEG_BIG;
#pragma unroll
  for (int it = 0; it < NS; ++it)
#pragma unroll
    for (int j = 0; j < 16; ++j) mx = fmaxf(mx, lg[it][j]);
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float mloc = mx > NEG_BIG ? mx : 0.f;              // NEG_BIG: the row sees none of this wave's keys
  {
    float sm = 0.f;
#pragma unroll
    for (int it = 0; it < NS; ++it)
#pragma unroll
      for (int j = 0; j < 16; ++j) sm += fast_exp2(lg[it][j] - mx);
    sm += __shfl_xor(sm, 32, 64);
    if (half == 0) { part[(wave * 32 + col) * 2] = mx; part[(wave * 32 + col) * 2 + 1] = sm; }
  }
#pragma unroll
  for (int it = 0; it < PF; ++it) MADAKV_WIN_LOAD(vg, it, it)
  __syncthreads();
  post_row_stats(a, hv, split, fs, part);

  // ---- O += P V with p taken against the wave's own row maxima, so that nothing here waits for the
  // other workgroups of the head; the head-wide statistics come in as one factor per row afterwards
  f32x16_t oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) oacc[db] = f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int it = 0; it < NS; ++it) {
    MADAKV_WIN_PARK(it % PF)
    if (it + PF < NS) MADAKV_WIN_LOAD(vg, it % PF, it + PF)
#pragma unroll
    for (int j = 0; j < 16; ++j) lg[it][j] = fast_exp2(lg[it][j] - mloc);   // masked: exp2(NEG_BIG) = 0
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int st = 0; st < 2; ++st) {                       // two 16-key steps of the subtile
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float pv = lg[it][8 * st + i];
        const uint32_t hb = f32_to_bf16_rne(pv);
        const uint32_t lb2 = f32_to_bf16_rne(pv - bf16_bits_to_f32(hb));
        if (i & 1) { hi[i >> 1] |= hb << 16; lo[i >> 1] |= lb2 << 16; }
        else { hi[i >> 1] = hb; lo[i >> 1] = lb2; }
      }
      const bf16x8_t pa_hi = __builtin_bit_cast(bf16x8_t, u32x4_t{hi[0], hi[1], hi[2], hi[3]});
      const bf16x8_t pa_lo = __builtin_bit_cast(bf16x8_t, u32x4_t{lo[0], lo[1], lo[2], lo[3]});
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 8; ++i) {                      // V[key of contraction index 8 half + i][32 db + col]
          const int row = 16 * st + 8 * (i >> 2) + 4 * half + (i & 3);
          const uint32_t x = kt[row * RS + db * 32 + col];
          if (i & 1) w[i >> 1] |= x << 16; else w[i >> 1] = x;
        }
        const bf16x8_t vb = __builtin_bit_cast(bf16x8_t, u32x4_t{w[0], w[1], w[2], w[3]});
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa_hi, vb, oacc[db], 0, 0, 0);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa_lo, vb, oacc[db], 0, 0, 0);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
#undef MADAKV_WIN_LOAD
#undef MADAKV_WIN_PARK

  // ---- the head-wide statistics (by now the other workgroups have normally posted theirs)
  collect_row_stats<D>(a, hv, split, fs, Lh, Mh, rowbase, kg, qs, part, offs, pm, &s_fail);
  __syncthreads();
  if (split == 0 && wa.lse && tid < Mh) wa.lse[(lb * a.H + kvh) * (long long)a.G * a.W + rowbase + tid] = offs[tid] * 0.6931471805599453f;
  const float mxw = part[(wave * 32 + col) * 2];           // the wave's own row maximum again
  const float rs = mxw > NEG_BIG ? fast_exp2(mxw - offs[col]) : 0.f;   // this wave's p times rs = the softmax entry

  // ---- Eq. 7 column sums
#pragma unroll
  for (int it = 0; it < NS; ++it) {
    const int t0 = chunk0 + (it * 4 + wave) * 32;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float cs = half_reduce<1>(lg[it][j] * rs);     // over the 32 rows: psi of this key
      const int key = t0 + 8 * (j >> 2) + 4 * half + (j & 3);
      // (more than 32 proxy rows: the block's share of psi, added to the other blocks' in block order afterwards)
      float* psi_dst = a.rb_count > 1 ? a.psi_part + (hv % a.rb_count) * a.psi_part_stride : a.psi;
      if (col == 0 && key < chunk1) psi_dst[(long long)head * a.L + key] = cs;
    }
  }
  // ---- O rows take their factor: row m of the tile sits in lane m's rs
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const float f = __shfl(rs, 8 * (j >> 2) + 4 * half + (j & 3), 64);
#pragma unroll
    for (int db = 0; db < DB; ++db) oacc[db][j] *= f;
  }

  // ---- the four waves' shares of O, added in wave order, CR output columns at a time through the K/V tiles' space
  constexpr int DPR = D == 128 ? 2 : 1, CR = 32 * DPR;     // 4 waves x 32 rows x CR floats fit the four tiles
  static_assert(4 * 32 * CR * sizeof(float) <= 4 * 32 * RS * sizeof(uint16_t), "the shares must fit the tiles");
  float* fl = reinterpret_cast<float*>(kt_all);           // [4 waves][32 rows][CR]
  float* op = wa.opart + ((long long)hv * fs + split) * 32 * D;
  for (int rd = 0; rd < DB / DPR; ++rd) {
    __syncthreads();
#pragma unroll
    for (int dd = 0; dd < DPR; ++dd)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int m = 8 * (j >> 2) + 4 * half + (j & 3);   // O[row m][column 32 db + col] sits in oacc[db][j]
        fl[(wave * 32 + m) * CR + dd * 32 + col] = oacc[rd * DPR + dd][j];
      }
    __syncthreads();
    for (int e = tid; e < 32 * CR; e += SCORE_THREADS) {
      const int m = e / CR, c = e % CR;
      op[m * D + rd * CR + c] = ((fl[(0 * 32 + m) * CR + c] + fl[(1 * 32 + m) * CR + c]) + fl[(2 * 32 + m) * CR + c]) + fl[(3 * 32 + m) * CR + c];
    }
  }
}

// out[row][c] = sum over the head's chunks, in chunk order, of their shares.  Grid (head, slice of
// 256 float4 of the 32 x d tile); eight shares in flight per thread.
__global__ __launch_bounds__(256) void window_attn_reduce_kernel(WinArgs wa) {
  const ScoreArgs& a = wa.s;
  const int hv = a.head0 + blockIdx.x;
  const int head = hv / a.rb_count, rowbase = (hv % a.rb_count) * 32;
  const int kvh = head % a.H;
  const long long lb = head / a.H;
  const int e4 = blockIdx.y * 256 + threadIdx.x;           // float4 index in the [32][d] tile
  const int tile4 = 32 * a.d / 4;
  if (e4 >= min(a.M - rowbase, 32) * a.d / 4) return;
  const f32x4_t* op = reinterpret_cast<const f32x4_t*>(wa.opart) + (long long)hv * a.fsplit * tile4 + e4;
  f32x4_t sum = {0.f, 0.f, 0.f, 0.f};
  int sp = 0;
  for (; sp + 8 <= a.fsplit; sp += 8) {
    f32x4_t x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = __builtin_nontemporal_load(op + (long long)(sp + j) * tile4);
#pragma unroll
    for (int j = 0; j < 8; ++j) sum += x[j];
  }
  for (; sp < a.fsplit; ++sp) sum += __builtin_nontemporal_load(op + (long long)sp * tile4);
  const long long o = ((lb * a.H + kvh) * (long long)a.G * a.W + rowbase) * a.d + (long long)e4 * 4;
  if (wa.out_fp32) *reinterpret_cast<f32x4_t*>(reinterpret_cast<float*>(wa.out) + o) = sum;
  else {
    u32x2_t pk;
    pk[0] = (uint32_t)f32_to_bf16_rne(sum[0]) | ((uint32_t)f32_to_bf16_rne(sum[1]) << 16);
    pk[1] = (uint32_t)f32_to_bf16_rne(sum[2]) | ((uint32_t)f32_to_bf16_rne(sum[3]) << 16);
    *reinterpret_cast<u32x2_t*>(reinterpret_cast<uint16_t*>(wa.out) + o) = pk;
  }
}

// ------------------------------------------------------------------------------------
// Plain FMA path (fp32 inputs, or bf16 with an odd head_dim).  Same two sweeps.
// Sweep 1: wave w takes rows w, w+4, ...; lanes stride over the keys of the chunk.
// Sweep 2: one thread per key, loop over the rows.
// ------------------------------------------------------------------------------------
template <typename T, int PASS>
__global__ __launch_bounds__(SCORE_THREADS) void score_simple_kernel(ScoreArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* qs = reinterpret_cast<float*>(smem);          // [M][d]
  float* offs = qs + a.M * a.d;                        // [M]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x;
  const int head = a.head0 + blockIdx.y;
  const int kvh = head % a.H;
  const long long lb = head / a.H;
  const T* qg = reinterpret_cast<const T*>(a.q_win) + (lb * a.H + kvh) * (long long)a.G * a.W * a.d;
  const T* kg = reinterpret_cast<const T*>(a.k) + (long long)head * a.L * a.d;
  for (int e = tid; e < a.M * a.d; e += SCORE_THREADS) qs[e] = load_elem(qg, e);
  if (PASS == 2) {
    const float* rs = a.rowstat + (long long)head * a.nsplit * a.mpad * 2;
    for (int r = tid; r < a.M; r += SCORE_THREADS) {
      float m = NEG_BIG, l = 0.f;
      if (a.lse) { m = a.lse[(lb * a.H + kvh) * (long long)a.G * a.W + r] * 1.4426950408889634f; l = 1.f; }
      else for (int s = 0; s < a.nmerge; ++s) merge_ml(m, l, rs[(s * a.mpad + r) * 2], rs[(s * a.mpad + r) * 2 + 1]);
      offs[r] = m + log2f(l);
    }
  }
  __syncthreads();
  const int chunk0 = split * a.chunk, chunk1 = min(a.L, chunk0 + a.chunk);
  if (PASS == 1) {
    float* rs = a.rowstat + ((long long)head * a.nsplit + split) * a.mpad * 2;
    for (int r = wave; r < a.mpad; r += 4) {
      float m = NEG_BIG, l = 0.f;
      if (r < a.M) {
        const int pos = a.L - a.W + (r % a.W);
        for (int key = chunk0 + lane; key < chunk1 && key <= pos; key += 64) {
          float s = 0.f;
          for (int e = 0; e < a.d; ++e) s = fmaf(qs[r * a.d + e], load_elem(kg, (long long)key * a.d + e), s);
          float s2 = s * a.scale_log2;
          float mn = fmaxf(m, s2);
          l = l * exp2f(m - mn) + exp2f(s2 - mn);
          m = mn;
        }
        for (int o = 1; o < 64; o <<= 1) {
          float m2 = __shfl_xor(m, o, 64), l2 = __shfl_xor(l, o, 64);
          merge_ml(m, l, m2, l2);
        }
      }
      if (lane == 0) { rs[r * 2] = m; rs[r * 2 + 1] = l; }
    }
  } else {
    for (int key = chunk0 + tid; key < chunk1; key += SCORE_THREADS) {
      float sum = 0.f;
      for (int r = 0; r < a.M; ++r) {
        const int pos = a.L - a.W + (r % a.W);
        if (key > pos) continue;
        float s = 0.f;
        for (int e = 0; e < a.d; ++e) s = fmaf(qs[r * a.d + e], load_elem(kg, (long long)key * a.d + e), s);
        sum += exp2f(s * a.scale_log2 - offs[r]);
      }
      a.psi[(long long)head * a.L + key] = sum;
    }
  }
}

// ------------------------------------------------------------------------------------
// With many chunks per head every sweep-2 workgroup would redo the same merge of the chunks' row
// statistics: this small kernel does it once per head and leaves the result in the first chunk's slot.
__global__ __launch_bounds__(256) void score_combine_kernel(ScoreArgs a) {
  const int head = a.head0 + blockIdx.x;
  float* rs = a.rowstat + (long long)head * a.nsplit * a.mpad * 2;
  for (int r = threadIdx.x; r < a.mpad; r += blockDim.x) {
    float m = NEG_BIG, l = 0.f;
    for (int s = 0; s < a.nsplit; ++s) merge_ml(m, l, rs[(s * a.mpad + r) * 2], rs[(s * a.mpad + r) * 2 + 1]);
    rs[r * 2] = m; rs[r * 2 + 1] = l;
  }
}

// chunks per head from which the merge is hoisted out of sweep 2
constexpr int COMBINE_FROM = 8;
#ifndef MADAKV_WIDE_WGS
#define MADAKV_WIDE_WGS 768
#endif
#ifndef MADAKV_WIDE_WGS2
#define MADAKV_WIDE_WGS2 512
#endif
constexpr int WIDE_WGS = MADAKV_WIDE_WGS, WIDE_WGS2 = MADAKV_WIDE_WGS2;   // workgroups per launch the chunking aims at with more than 64 proxy rows: sweep 1, sweep 2

static bool use_mfma(const Dims& dm, int dtype) { return dtype == MADAKV_BF16 && (dm.d == 64 || dm.d == 128); }

ScorePlan score_plan(const Dims& dm, int dtype) {
  (void)dtype;
  ScorePlan p;
  p.mpad = (dm.M + 31) / 32 * 32;
  // Both sweeps run over all heads of the call in one launch each, at most 65535 heads at a
  // time (the grid's y limit).  (Splitting a call into groups of heads whose K fits the 256 MB
  // memory-side cache, so that the second sweep finds its data there, was measured slower at
  // every group size.)
  p.group_heads = std::min(dm.heads, 65535);
  // enough workgroups per launch to fill 256 CUs several times over; chunks are a multiple
  // of 128 keys (4 waves x 32-key tiles) and at least 256 keys long
  int want = std::max(1, (2048 + p.group_heads - 1) / p.group_heads);
  int max_split = std::max(1, dm.L / 256);
  // (more than 64 proxy rows: the arithmetic per key is several times larger and a workgroup's start, its Q
  // fragments and first tile, costs more, so about two workgroups per CU with long chunks)
  if (p.mpad > 64) { want = std::max(1, (WIDE_WGS + p.group_heads / 2) / p.group_heads); max_split = std::max(1, dm.L / 1024); }
  int ns = std::min(std::min(want, max_split), 128);
  int chunk = ((dm.L + ns - 1) / ns + 127) / 128 * 128;
  p.nsplit = (dm.L + chunk - 1) / chunk;
  p.chunk = chunk;
  return p;
}

// One sweep when the logits of a workgroup's keys fit in registers (at most two row blocks) and a
// head has few enough chunks that all its workgroups are certain to be on the chip together.
constexpr int FUSED_NS1 = MADAKV_FUSED_NS1, FUSED_NS2 = MADAKV_FUSED_NS2;
constexpr int FUSED_MAX_SPLIT = MADAKV_FUSED_MAX_SPLIT;
static int fused_chunk(const Dims& dm) { return 4 * 32 * ((dm.M + 31) / 32 == 1 ? FUSED_NS1 : FUSED_NS2); }
static int fused_split(const Dims& dm) { return (dm.L + fused_chunk(dm) - 1) / fused_chunk(dm); }
static int fused_mpad(const Dims& dm) { return dm.M <= 32 ? 32 : 64; }
static int fused_blocks(const Dims& dm) { return dm.M <= 64 ? 1 : (dm.M + 63) / 64; }   // blocks of 64 proxy rows handled like heads
// exchange levels: one up to FUSED_MAX_SPLIT chunks per head, two (groups of XCHG_GROUP chunks) up to
// FUSED_MAX_SPLIT_2L.  All workgroups of a head wait for each other, so a head must never need more
// workgroups than the chip holds at once (512 of this kernel): half of that is the limit.
constexpr int FUSED_MAX_SPLIT_2L = 256;
static int xchg_groups(int split) { return split <= FUSED_MAX_SPLIT ? 0 : (split + XCHG_GROUP - 1) / XCHG_GROUP; }
// (More than 64 proxy rows: the prompt's keys take the two-sweep kernels above, which are bound by their vector
// arithmetic either way and twice as fast as one sweep per block of 64 rows; the ragged rows of a reduced cache
// still go through the one-sweep kernel in blocks.)
// Long heads whose chunks pack the workgroup slots badly.  A workgroup keeps its slot until its whole head is
// through; the chip holds FUSED_SLOTS workgroups of the kernel; k = slots / chunks heads fit at once, and when a
// few chunks fewer per head would let k + 1 fit (171 chunks at a 128K context: 3 x 171 = 513), every (k + 1)-th
// head's last chunk waits for a slot while its head-mates hold theirs idle.  Those few last chunks per head then
// run ahead of the launch of the others (ScoreArgs::nstrag).  Returns their number (0: nothing to gain).
constexpr int FUSED_SLOTS = 512, FUSED_MAX_PARKED = 8;
static int fused_parked_chunks(int split) {
  if (split <= FUSED_MAX_SPLIT) return 0;                 // (the parked chunks' words live at the group level)
  const int k = FUSED_SLOTS / split, fewer = FUSED_SLOTS / (k + 1);
  const int n = split - fewer;
  return (fewer > FUSED_MAX_SPLIT && n >= 1 && n <= FUSED_MAX_PARKED && k * split * 10 < FUSED_SLOTS * 9) ? n : 0;
}
static size_t fused_park_bytes(const Dims& dm, int dtype);
static bool fused_fits(const Dims& dm, int dtype) {
  return use_mfma(dm, dtype) && dm.M <= 64 && fused_split(dm) <= FUSED_MAX_SPLIT_2L && dm.heads <= 65535;
}
static bool use_fused(const Dims& dm, int dtype) {
  const char* e = getenv("MADAKV_SCORE_TWO_SWEEPS");      // diagnostic switch: the two-sweep kernels everywhere
  const bool off = e && atoi(e) != 0;
  return !off && fused_fits(dm, dtype);
}

static size_t rowstat_bytes(const Dims& dm, int dtype) {
  ScorePlan p = score_plan(dm, dtype);
  return ((size_t)dm.heads * p.nsplit * p.mpad * 2 * sizeof(float) + 255) / 256 * 256;
}
static size_t xchg_bytes(const Dims& dm, int dtype) {
  const size_t per_head = (size_t)(fused_split(dm) + xchg_groups(fused_split(dm))) * fused_mpad(dm);
  return fused_fits(dm, dtype) ? ((size_t)dm.heads * fused_blocks(dm) * per_head * 8 + 255) / 256 * 256 : 0;
}
static size_t fused_park_bytes(const Dims& dm, int dtype) {
  if (!fused_fits(dm, dtype)) return 0;
  const int n = fused_parked_chunks(fused_split(dm));
  const int ns = fused_mpad(dm) == 32 ? FUSED_NS1 : FUSED_NS2, nrb = fused_mpad(dm) / 32;
  // the parked logits (one float per thread and logit register) and the heads' row offsets
  return n ? ((size_t)dm.heads * n * ns * nrb * 16 * SCORE_THREADS * sizeof(float) + (size_t)dm.heads * fused_mpad(dm) * sizeof(float) + 255) / 256 * 256 : 0;
}
size_t score_ws_bytes(const Dims& dm, int dtype) {
  // the counter of lone workgroups, the row statistics of the two sweeps, the store sink, the exchange array of the
  // one-sweep kernel, its per-row-block copies of psi when there are more than 64 proxy rows
  const size_t part = fused_fits(dm, dtype) && fused_blocks(dm) > 1 ? (size_t)fused_blocks(dm) * dm.heads * dm.L * sizeof(float) : 0;
  return 256 + rowstat_bytes(dm, dtype) + 256 + xchg_bytes(dm, dtype) + part + fused_park_bytes(dm, dtype);
}

// psi = the row blocks' column sums added in block order (more than 64 proxy rows)
__global__ __launch_bounds__(256) void score_blocks_sum_kernel(const float* part, long long stride, int blocks, float* psi, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float acc = part[i];
  for (int b = 1; b < blocks; ++b) acc += part[b * stride + i];
  psi[i] = acc;
}

// the one-sweep kernel over `heads` heads (each cut into a.rb_count blocks of proxy rows)
template <int D>
static void launch_fused(const ScoreArgs& a, int heads, hipStream_t st) {
  const int vheads = heads * a.rb_count;
  const long long nx = (long long)vheads * a.xstride;
  if (a.fsplit > 1)
    hipLaunchKernelGGL(score_xchg_init_kernel, dim3((unsigned)((nx + 255) / 256)), dim3(256), 0, st,
                       a.xchg + (long long)a.head0 * a.rb_count * a.xstride, nx);
  const size_t ldsf = ((size_t)a.mpad + 4 * 32) * (D + 8) * 2 + ((size_t)4 * a.mpad * 2 + a.mpad + 512) * sizeof(float);
  ScoreArgs b = a;
  b.head0 = a.head0 * a.rb_count;
  // (a.nstrag > 0: a.fsplit counts the chunks that wait for each other; the parked ones are the first in the grid)
  const dim3 grid(a.nstrag + a.fsplit, vheads);
  if (a.mpad == 32) {
    if (a.k_fp8) hipLaunchKernelGGL((score_fused_kernel<D, 1, FUSED_NS1, true>), grid, dim3(SCORE_THREADS), ldsf, st, b);
    else hipLaunchKernelGGL((score_fused_kernel<D, 1, FUSED_NS1>), grid, dim3(SCORE_THREADS), ldsf, st, b);
  } else if (a.k_fp8) {
    if (ldsf > 48 * 1024)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_fused_kernel<D, 2, FUSED_NS2, true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldsf);
    hipLaunchKernelGGL((score_fused_kernel<D, 2, FUSED_NS2, true>), grid, dim3(SCORE_THREADS), ldsf, st, b);
  } else {
    if (ldsf > 48 * 1024)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_fused_kernel<D, 2, FUSED_NS2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldsf);
    hipLaunchKernelGGL((score_fused_kernel<D, 2, FUSED_NS2>), grid, dim3(SCORE_THREADS), ldsf, st, b);
  }
  if (a.nstrag) {
    if (a.mpad == 32) hipLaunchKernelGGL((score_fused_finish_kernel<1, FUSED_NS1>), dim3(a.nstrag, vheads), dim3(SCORE_THREADS), 0, st, b);
    else hipLaunchKernelGGL((score_fused_finish_kernel<2, FUSED_NS2>), dim3(a.nstrag, vheads), dim3(SCORE_THREADS), 0, st, b);
  }
  if (a.rb_count > 1) {
    const long long n = (long long)heads * a.L;
    hipLaunchKernelGGL(score_blocks_sum_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       a.psi_part + (long long)a.head0 * a.L, a.psi_part_stride, a.rb_count, a.psi + (long long)a.head0 * a.L, n);
  }
}

template <int D, int NRB>
static void launch_mfma_pair(const ScoreArgs& a0, int heads, size_t lds1, size_t lds2, hipStream_t st) {
  ScoreArgs a = a0;
  dim3 grid(a.nsplit, heads);
  if (lds1 > 48 * 1024 || lds2 > 48 * 1024) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_mfma_kernel<D, NRB, 1>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_mfma_kernel<D, NRB, 2>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
  }
  if (!a.lse) {
    hipLaunchKernelGGL((score_mfma_kernel<D, NRB, 1>), grid, dim3(SCORE_THREADS), lds1, st, a);
    if (a.nsplit >= COMBINE_FROM) { hipLaunchKernelGGL(score_combine_kernel, dim3(heads), dim3(256), 0, st, a); a.nmerge = 1; }
  }
  hipLaunchKernelGGL((score_mfma_kernel<D, NRB, 2>), grid, dim3(SCORE_THREADS), lds2, st, a);
}

// more than 64 proxy rows (up to 128 with WIDE8 = false, else up to 256)
template <int D, bool WIDE8>
static void launch_wide_pair(const ScoreArgs& a0, int heads, hipStream_t st) {
  ScoreArgs a = a0;
  dim3 grid(a.nsplit, heads);
  // both sweeps: four waves of one (up to 128 rows) or two row blocks, tiles of 64 keys, two workgroups per CU
  constexpr int NW1 = 4, NRB1 = WIDE8 ? 2 : 1, NRB2 = NRB1;
  constexpr int TK1 = 64, BS1 = 1, BS2 = WIDE8 ? 1 : 2;     // (sweep 2: what the registers hold)
  const size_t lds1 = (size_t)DMA_NBUF * TK1 * D * 2;
  const size_t lds2 = (size_t)DMA_NBUF * 64 * D * 2 + ((size_t)a.mpad + 2 * 4 * 64) * sizeof(float);
  static size_t allowed[2][64] = {};            // (per instantiation and device; set again only when a call needs more)
  int dev = 0;
  (void)hipGetDevice(&dev);
  size_t& allowed1 = allowed[0][dev & 63];
  size_t& allowed2 = allowed[1][dev & 63];
  if (lds1 > allowed1) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_wide_dma_kernel<D, NW1, NRB1, TK1, BS1, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
    allowed1 = lds1;
  }
  if (lds2 > allowed2) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_wide_dma_kernel<D, 4, NRB2, 64, BS2, 2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
    allowed2 = lds2;
  }
  if (!a.lse) {
    hipLaunchKernelGGL((score_wide_dma_kernel<D, NW1, NRB1, TK1, BS1, 1>), grid, dim3(NW1 * 64), lds1, st, a);
    hipLaunchKernelGGL(score_combine_kernel, dim3(heads), dim3(256), 0, st, a);
    a.nmerge = 1;
  }
  // sweep 2 in chunks of its own (about two workgroups per CU); a.nsplit stays what the row statistics are laid out by
  const int want2 = std::max(1, (WIDE_WGS2 + heads / 2) / heads);
  const int ns2 = std::min(want2, std::max(1, a.L / 512));
  a.chunk = ((a.L + ns2 - 1) / ns2 + 63) / 64 * 64;
  dim3 grid2((a.L + a.chunk - 1) / a.chunk, heads);
  hipLaunchKernelGGL((score_wide_dma_kernel<D, 4, NRB2, 64, BS2, 2>), grid2, dim3(SCORE_THREADS), lds2, st, a);
}

// ---- the one-sweep kernel on ragged heads: the rows of a reduced cache, scored against the most recent queries
static int ragged_split(const Dims& dm, int longest_rows) { return (std::max(longest_rows, 1) + fused_chunk(dm) - 1) / fused_chunk(dm); }
bool score_ragged_supported(const Dims& dm, const madakv_config& c, int longest_rows) {
  return use_mfma(dm, c.dtype) && dm.M <= 256 && ragged_split(dm, longest_rows) <= FUSED_MAX_SPLIT &&
         (long long)dm.heads * fused_blocks(dm) <= 65535;
}
static size_t ragged_xchg_bytes(const Dims& dm, int longest_rows) {
  return ((size_t)dm.heads * fused_blocks(dm) * ragged_split(dm, longest_rows) * fused_mpad(dm) * 8 + 255) / 256 * 256;
}
// cache_rows: rows of the whole reduced cache (psi_c is indexed like it; so are the row blocks' copies)
size_t score_ragged_ws_bytes(const Dims& dm, const madakv_config& c, int longest_rows, long long cache_rows) {
  (void)c;
  return 256 + ragged_xchg_bytes(dm, longest_rows) + (fused_blocks(dm) > 1 ? (size_t)fused_blocks(dm) * cache_rows * sizeof(float) : 0);
}
hipError_t launch_score_ragged(const Dims& dm, const madakv_config& c, const void* q_recent, const void* k_c,
                               const int64_t* seg_off, const int32_t* seg_len, int longest_rows, long long cache_rows,
                               float* psi_c, void* ws, hipStream_t st) {
  ScoreArgs a;
  a.lse = nullptr; a.q_win = q_recent; a.k = k_c; a.psi = psi_c;
  a.status = reinterpret_cast<int*>(ws);
  a.rowstat = nullptr; a.sink = nullptr;
  a.xchg = reinterpret_cast<unsigned long long*>(static_cast<char*>(ws) + 256);
  a.seg_off = seg_off; a.seg_len = seg_len;
  a.H = dm.H; a.G = dm.G; a.d = dm.d; a.L = dm.L; a.W = dm.W; a.M = dm.M;
  a.mpad = fused_mpad(dm); a.nsplit = 0; a.nmerge = 0; a.chunk = 0; a.head0 = 0;
  a.fsplit = ragged_split(dm, longest_rows);
  a.xgroups = 0; a.xstride = (long long)a.fsplit * fused_mpad(dm);
  a.k_fp8 = c.cache_fp8 ? 1 : 0;                  // the reduced cache is what is scored here
  const char* spin = getenv("MADAKV_SCORE_SPIN_LIMIT");
  a.spin_limit = spin && atoi(spin) > 0 ? atoi(spin) : FUSED_SPIN_LIMIT;
  const float scale = c.softmax_scale > 0.f ? c.softmax_scale : 1.0f / sqrtf((float)dm.d);
  a.scale_log2 = scale * 1.4426950408889634f;
  a.rb_count = fused_blocks(dm);
  a.psi_part = reinterpret_cast<float*>(static_cast<char*>(ws) + 256 + ragged_xchg_bytes(dm, longest_rows));
  a.psi_part_stride = cache_rows;
  if (a.rb_count == 1) {
    if (dm.d == 128) launch_fused<128>(a, dm.heads, st); else launch_fused<64>(a, dm.heads, st);
  } else {
    // the kernel writes the row blocks' copies at the rows' own places; they are added over the whole cache
    // (rows outside the call's segments hold old values of the workspace and are not read by anybody)
    const ScoreArgs& b = a;
    const int vheads = dm.heads * a.rb_count;
    const long long nx = (long long)vheads * a.fsplit * a.mpad;
    if (a.fsplit > 1) hipLaunchKernelGGL(score_xchg_init_kernel, dim3((unsigned)((nx + 255) / 256)), dim3(256), 0, st, a.xchg, nx);
    const size_t ldsf = ((size_t)a.mpad + 4 * 32) * (dm.d + 8) * 2 + ((size_t)4 * a.mpad * 2 + a.mpad + 512) * sizeof(float);
    const dim3 grid(a.fsplit, vheads);
    if (dm.d == 128 && a.k_fp8) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_fused_kernel<128, 2, FUSED_NS2, true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldsf);
      hipLaunchKernelGGL((score_fused_kernel<128, 2, FUSED_NS2, true>), grid, dim3(SCORE_THREADS), ldsf, st, b);
    } else if (dm.d == 128) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_fused_kernel<128, 2, FUSED_NS2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldsf);
      hipLaunchKernelGGL((score_fused_kernel<128, 2, FUSED_NS2>), grid, dim3(SCORE_THREADS), ldsf, st, b);
    } else if (a.k_fp8) {
      hipLaunchKernelGGL((score_fused_kernel<64, 2, FUSED_NS2, true>), grid, dim3(SCORE_THREADS), ldsf, st, b);
    } else {
      hipLaunchKernelGGL((score_fused_kernel<64, 2, FUSED_NS2>), grid, dim3(SCORE_THREADS), ldsf, st, b);
    }
    hipLaunchKernelGGL(score_blocks_sum_kernel, dim3((unsigned)((cache_rows + 255) / 256)), dim3(256), 0, st,
                       a.psi_part, a.psi_part_stride, a.rb_count, psi_c, cache_rows);
  }
  return hipGetLastError();
}

// ---- the last-window attention with the scores as a by-product
constexpr int WIN_NS_128 = 4, WIN_NS_64 = 6;             // subtiles per wave (registers: logits + the O tile)
static int win_split(const Dims& dm) { const int ck = 4 * 32 * (dm.d == 128 ? WIN_NS_128 : WIN_NS_64); return (dm.L + ck - 1) / ck; }
static int win_blocks(const Dims& dm) { return (dm.M + 31) / 32; }   // blocks of 32 proxy rows, each handled like a head of its own
bool window_attn_supported(const Dims& dm, const madakv_config& c) {
  return use_mfma(dm, c.dtype) && dm.M <= 256 && win_split(dm) <= FUSED_MAX_SPLIT_2L;
}
static size_t win_xchg_bytes(const Dims& dm) {
  return ((size_t)dm.heads * win_blocks(dm) * (win_split(dm) + xchg_groups(win_split(dm))) * 32 * 8 + 255) / 256 * 256;
}
static size_t win_opart_bytes(const Dims& dm) { return ((size_t)dm.heads * win_blocks(dm) * win_split(dm) * 32 * dm.d * sizeof(float) + 255) / 256 * 256; }
size_t window_attn_ws_bytes(const Dims& dm, const madakv_config& c) {
  if (!window_attn_supported(dm, c)) return 256;
  // the counter of lone workgroups, the exchange words, the workgroups' shares of O, the row blocks' shares of psi
  return 256 + win_xchg_bytes(dm) + win_opart_bytes(dm) + (win_blocks(dm) > 1 ? (size_t)win_blocks(dm) * dm.heads * dm.L * sizeof(float) : 0);
}
hipError_t launch_window_attn(const Dims& dm, const madakv_config& c, const void* q_win, const void* k, const void* v,
                              void* out, float* row_lse, float* psi, void* ws, hipStream_t st) {
  WinArgs wa;
  ScoreArgs& a = wa.s;
  a.lse = nullptr; a.q_win = q_win; a.k = k; a.psi = psi;
  a.status = reinterpret_cast<int*>(ws);
  a.rowstat = nullptr; a.sink = nullptr; a.seg_off = nullptr; a.seg_len = nullptr;
  a.xchg = reinterpret_cast<unsigned long long*>(static_cast<char*>(ws) + 256);
  a.H = dm.H; a.G = dm.G; a.d = dm.d; a.L = dm.L; a.W = dm.W; a.M = dm.M;
  a.mpad = 32; a.nsplit = 0; a.nmerge = 0; a.chunk = 0; a.head0 = 0;
  const int rb = win_blocks(dm);
  a.rb_count = rb;
  a.psi_part = reinterpret_cast<float*>(static_cast<char*>(ws) + 256 + win_xchg_bytes(dm) + win_opart_bytes(dm));
  a.psi_part_stride = (long long)dm.heads * dm.L;
  a.fsplit = win_split(dm);
  a.xgroups = xchg_groups(a.fsplit); a.xstride = (long long)(a.fsplit + a.xgroups) * 32; a.k_fp8 = 0;   // (two exchange levels above 64 chunks)
  const char* spin = getenv("MADAKV_SCORE_SPIN_LIMIT");
  a.spin_limit = spin && atoi(spin) > 0 ? atoi(spin) : FUSED_SPIN_LIMIT;
  const float scale = c.softmax_scale > 0.f ? c.softmax_scale : 1.0f / sqrtf((float)dm.d);
  a.scale_log2 = scale * 1.4426950408889634f;
  wa.v = v; wa.lse = row_lse; wa.out = out; wa.out_fp32 = c.out_fp32;
  wa.opart = reinterpret_cast<float*>(static_cast<char*>(ws) + 256 + win_xchg_bytes(dm));
  const long long nx = (long long)dm.heads * rb * a.xstride;
  if (a.fsplit > 1) hipLaunchKernelGGL(score_xchg_init_kernel, dim3((unsigned)((nx + 255) / 256)), dim3(256), 0, st, a.xchg, nx);
  const size_t lds = ((size_t)32 + 4 * 32) * (dm.d + 8) * 2 + ((size_t)4 * 32 * 2 + 32 + 512) * sizeof(float);
  const int vheads = dm.heads * rb, step = 65535 / rb * rb;       // whole heads per launch (the grid's y limit)
  for (int h0 = 0; h0 < vheads; h0 += step) {
    const int nh = std::min(step, vheads - h0);
    a.head0 = h0;
    if (dm.d == 128) hipLaunchKernelGGL((window_attn_kernel<128, WIN_NS_128>), dim3(a.fsplit, nh), dim3(SCORE_THREADS), lds, st, wa);
    else hipLaunchKernelGGL((window_attn_kernel<64, WIN_NS_64>), dim3(a.fsplit, nh), dim3(SCORE_THREADS), lds, st, wa);
    hipLaunchKernelGGL(window_attn_reduce_kernel, dim3(nh, (32 * dm.d / 4 + 255) / 256), dim3(256), 0, st, wa);
  }
  if (rb > 1) {
    const long long n = (long long)dm.heads * dm.L;
    hipLaunchKernelGGL(score_blocks_sum_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a.psi_part, a.psi_part_stride, rb, psi, n);
  }
  return hipGetLastError();
}

hipError_t launch_score(const Dims& dm, const madakv_config& c, const void* q_win, const void* k, const float* row_lse,
                        float* psi, void* ws, hipStream_t st) {
  ScorePlan p = score_plan(dm, c.dtype);
  ScoreArgs a;
  a.lse = row_lse;
  a.q_win = q_win; a.k = k; a.psi = psi;
  a.status = reinterpret_cast<int*>(ws);
  a.rowstat = reinterpret_cast<float*>(static_cast<char*>(ws) + 256);
  a.sink = reinterpret_cast<float*>(static_cast<char*>(ws) + 256 + rowstat_bytes(dm, c.dtype));
  a.xchg = reinterpret_cast<unsigned long long*>(static_cast<char*>(ws) + 256 + rowstat_bytes(dm, c.dtype) + 256);
  a.rb_count = fused_blocks(dm);
  a.psi_part = reinterpret_cast<float*>(static_cast<char*>(ws) + 256 + rowstat_bytes(dm, c.dtype) + 256 + xchg_bytes(dm, c.dtype));
  a.psi_part_stride = (long long)dm.heads * dm.L;
  a.fsplit = (!row_lse && use_fused(dm, c.dtype)) ? fused_split(dm) : 0;
  a.nstrag = a.fsplit ? fused_parked_chunks(a.fsplit) : 0;
  if (getenv("MADAKV_SCORE_NO_PARKED_CHUNKS")) a.nstrag = 0;                      // (measurement switch)
  a.fsplit -= a.nstrag;                                                            // the chunks of the main launch
  a.xgroups = xchg_groups(a.fsplit) + a.nstrag; a.xstride = (long long)(a.fsplit + a.xgroups) * fused_mpad(dm); a.k_fp8 = 0;
  {
    char* pk = static_cast<char*>(ws) + 256 + rowstat_bytes(dm, c.dtype) + 256 + xchg_bytes(dm, c.dtype) +
               (fused_fits(dm, c.dtype) && fused_blocks(dm) > 1 ? (size_t)fused_blocks(dm) * dm.heads * dm.L * sizeof(float) : 0);
    a.offs_out = a.nstrag ? reinterpret_cast<float*>(pk) : nullptr;
    a.park = a.nstrag ? reinterpret_cast<float*>(pk) + (size_t)dm.heads * fused_mpad(dm) : nullptr;
  }
  a.seg_off = nullptr; a.seg_len = nullptr;
  // (a test can force the lone-workgroup path of the one-sweep kernel from the host with a spin limit of 1)
  const char* spin = getenv("MADAKV_SCORE_SPIN_LIMIT");
  a.spin_limit = spin && atoi(spin) > 0 ? atoi(spin) : FUSED_SPIN_LIMIT;
  a.H = dm.H; a.G = dm.G; a.d = dm.d; a.L = dm.L; a.W = dm.W; a.M = dm.M;
  a.mpad = p.mpad; a.nsplit = p.nsplit; a.nmerge = p.nsplit; a.chunk = p.chunk; a.head0 = 0;
  float scale = c.softmax_scale > 0.f ? c.softmax_scale : 1.0f / sqrtf((float)dm.d);
  a.scale_log2 = scale * 1.4426950408889634f;
  if (a.fsplit > 0) {                                      // one sweep (heads * row blocks fit one launch)
    a.mpad = fused_mpad(dm);
    if (dm.d == 128) launch_fused<128>(a, dm.heads, st); else launch_fused<64>(a, dm.heads, st);
    return hipGetLastError();
  }
  for (int h0 = 0; h0 < dm.heads; h0 += p.group_heads) {
    int nh = std::min(p.group_heads, dm.heads - h0);
    a.head0 = h0;
    if (use_mfma(dm, c.dtype)) {
      // row blocks of 32 proxy rows: 1-2 -> every wave its own keys and all rows; 3-8 -> the waves share the
      // keys and own row blocks (the kernels with the LDS ring)
      const int MB = p.mpad / 32;
      const size_t qbytes = ((size_t)p.mpad + 4 * 32) * (dm.d + 8) * 2;      // Q tile + one K subtile per wave
      const size_t lds1 = qbytes + (size_t)4 * p.mpad * 2 * sizeof(float);
      const size_t lds2 = qbytes + (size_t)p.mpad * sizeof(float);
#define MADAKV_SCORE_CASE(DD, NN) launch_mfma_pair<DD, NN>(a, nh, lds1, lds2, st)
#define MADAKV_SCORE_BY_MB(DD) \
      if (MB == 1) MADAKV_SCORE_CASE(DD, 1); else if (MB == 2) MADAKV_SCORE_CASE(DD, 2); \
      else if (MB <= 4) launch_wide_pair<DD, false>(a, nh, st); else launch_wide_pair<DD, true>(a, nh, st)
      if (dm.d == 128) { MADAKV_SCORE_BY_MB(128); } else { MADAKV_SCORE_BY_MB(64); }
#undef MADAKV_SCORE_BY_MB
#undef MADAKV_SCORE_CASE
    } else {
      size_t lds = ((size_t)dm.M * dm.d + dm.M) * sizeof(float);
      dim3 grid(a.nsplit, nh);
      if (c.dtype == MADAKV_BF16) {
        if (!a.lse) hipLaunchKernelGGL((score_simple_kernel<uint16_t, 1>), grid, dim3(SCORE_THREADS), lds, st, a);
        hipLaunchKernelGGL((score_simple_kernel<uint16_t, 2>), grid, dim3(SCORE_THREADS), lds, st, a);
      } else {
        if (!a.lse) hipLaunchKernelGGL((score_simple_kernel<float, 1>), grid, dim3(SCORE_THREADS), lds, st, a);
        hipLaunchKernelGGL((score_simple_kernel<float, 2>), grid, dim3(SCORE_THREADS), lds, st, a);
      }
    }
  }
  return hipGetLastError();
}

}  // namespace madakv
