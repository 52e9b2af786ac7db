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

constexpr float NEG_BIG = -1.0e30f;
constexpr int SCORE_THREADS = 256;

struct ScoreArgs {
  const void* q_win;   // [heads/H * Hq, W, d]
  const void* k;       // [heads, L, d]
  float* psi;          // [heads, L]
  float* rowstat;      // [heads, nsplit, mpad, 2]
  int H, G, d, L, W, M, mpad, nsplit, chunk;
  int head0;           // first head of this launch (grid.y indexes head0 + y)
  float scale_log2;    // softmax scale * log2(e)
};

__device__ __forceinline__ void merge_ml(float& m, float& l, float m2, float l2) {
  float mn = fmaxf(m, m2);
  l = l * exp2f(m - mn) + l2 * exp2f(m2 - mn);
  m = mn;
}

// ------------------------------------------------------------------------------------
// bf16 MFMA path.  One workgroup = 4 waves works on one (head, L-chunk).  A wave owns up
// to two 32-row blocks of Q and a 32-key tile of K at a time:
//   D[i = proxy row][j = key] = sum_k A[i][k] * B[k][j],  A = Q block, B = K tile^T.
// Lane l feeds key (l & 31): its B fragments are 16-byte pieces of that key's row, read
// straight from global memory (half (l >> 5) of the row, contiguous); the A fragments
// come from the Q tile staged in LDS.  In D a lane holds one key column and 16 rows, so
// the column sum is in-lane and the row statistics need one cross-lane merge at the end.
// WPT waves share a key tile when there are more than two row blocks.
// ------------------------------------------------------------------------------------
template <int D, int WPT, int PASS>
__global__ __launch_bounds__(SCORE_THREADS) void score_mfma_kernel(ScoreArgs a) {
  constexpr int KS = D / 16;                  // MFMA k-steps
  constexpr int QSTRIDE = D + 8;              // bf16 elements per LDS row (16 B pad: conflict-free b128 reads)
  constexpr int KG = 4 / WPT;                 // key groups (waves that own different tiles)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint16_t* qs = reinterpret_cast<uint16_t*>(smem);                                 // [mpad][QSTRIDE]
  float* fbuf = reinterpret_cast<float*>(smem + (size_t)a.mpad * QSTRIDE * 2);      // pass 1: [4][mpad][2]; pass 2: off[mpad] + red[4][32]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x;
  const int head = a.head0 + blockIdx.y;
  const int kvh = head % a.H;
  const long long lb = head / a.H;            // (layer, batch) index
  const uint16_t* qg = reinterpret_cast<const uint16_t*>(a.q_win) + (lb * a.H + kvh) * (long long)a.G * a.W * D;
  const uint16_t* kg = reinterpret_cast<const uint16_t*>(a.k) + (long long)head * a.L * D;
  const int MB = a.mpad / 32;

  // stage Q (the G*W rows of this KV head are contiguous), zero the padding rows
  for (int e = tid; e < a.mpad * (D / 8); e += SCORE_THREADS) {
    int r = e / (D / 8), c = e % (D / 8);
    uint4 val = make_uint4(0, 0, 0, 0);
    if (r < a.M) val = *reinterpret_cast<const uint4*>(qg + (long long)r * D + c * 8);
    *reinterpret_cast<uint4*>(qs + r * QSTRIDE + c * 8) = val;
  }
  float* offs = fbuf;                          // pass 2 only
  if (PASS == 2) {
    const float* rs = a.rowstat + (long long)head * a.nsplit * a.mpad * 2;
    for (int r = tid; r < a.mpad; r += SCORE_THREADS) {
      float m = NEG_BIG, l = 0.f;
      for (int s = 0; s < a.nsplit; ++s) merge_ml(m, l, rs[(s * a.mpad + r) * 2], rs[(s * a.mpad + r) * 2 + 1]);
      offs[r] = (r < a.M) ? m + log2f(l) : __builtin_inff();     // padding rows contribute exp2(-inf) = 0
    }
  }
  __syncthreads();

  const int wsub = wave % WPT;                 // which row blocks of the tile this wave owns
  const int kgid = wave / WPT;                 // which tiles of the chunk
  const int nrb = (MB - wsub + WPT - 1) / WPT; // 0, 1 or 2 row blocks: wsub, wsub + WPT
  const int half = lane >> 5, col = lane & 31;
  const int chunk0 = split * a.chunk;
  const int chunk1 = min(a.L, chunk0 + a.chunk);
  const int first_masked = a.L - a.W + 1;      // keys below this are visible to every proxy row

  float st_m[2][16], st_l[2][16], off_r[2][16];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      st_m[b][j] = NEG_BIG; st_l[b][j] = 0.f;
      int row = (wsub + b * WPT) * 32 + (j >> 2) * 8 + half * 4 + (j & 3);
      off_r[b][j] = (PASS == 2 && b < nrb) ? offs[row] : 0.f;
    }
  float* red = fbuf + a.mpad;                  // pass 2, WPT > 1: [4][32] partial column sums

  // every wave runs the same number of iterations (the loop holds workgroup barriers);
  // a tile that starts past the chunk is computed on clamped rows and fully masked
  const int niter = (chunk1 - chunk0 + KG * 32 - 1) / (KG * 32);
  for (int it = 0; it < niter; ++it) {
    const int t0 = chunk0 + (it * KG + kgid) * 32;
    const int key = t0 + col;
    const int keyc = min(key, a.L - 1);        // ragged tail: load a valid row, mask it below
    bf16x8_t bfrag[KS];
    const uint16_t* kp = kg + (long long)keyc * D + half * (D / 2);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) bfrag[ks] = *reinterpret_cast<const bf16x8_t*>(kp + ks * 8);
    const bool tail = (t0 + 32 > first_masked) || (t0 + 32 > chunk1);
    float colsum = 0.f;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if (b < nrb) {
        const int rb = wsub + b * WPT;
        f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const uint16_t* qrow = qs + (rb * 32 + col) * QSTRIDE + half * (D / 2);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          bf16x8_t afrag = *reinterpret_cast<const bf16x8_t*>(qrow + ks * 8);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[ks], acc, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const float s2 = acc[j] * a.scale_log2;
          bool valid = true;
          if (tail) {
            const int row = rb * 32 + (j >> 2) * 8 + half * 4 + (j & 3);
            const int pos = a.L - a.W + (row % a.W);            // absolute position of the proxy row
            valid = (key < chunk1) && (key <= pos) && (row < a.M);
          }
          if (PASS == 1) {
            const float mn = valid ? fmaxf(st_m[b][j], s2) : st_m[b][j];
            st_l[b][j] = st_l[b][j] * exp2f(st_m[b][j] - mn) + (valid ? exp2f(s2 - mn) : 0.f);
            st_m[b][j] = mn;
          } else {
            const float p = exp2f(s2 - off_r[b][j]);
            colsum += valid ? p : 0.f;
          }
        }
      }
    }
    if (PASS == 2) {
      colsum += __shfl_xor(colsum, 32, 64);    // the two halves hold different rows of the same key
      if (WPT == 1) {
        if (half == 0 && key < chunk1) a.psi[(long long)head * a.L + key] = colsum;
      } else {
        if (half == 0) red[wave * 32 + col] = colsum;
        __syncthreads();
        if (wsub == 0 && half == 0 && key < chunk1) {
          float s = 0.f;
#pragma unroll
          for (int w = 0; w < WPT; ++w) s += red[(kgid * WPT + w) * 32 + col];
          a.psi[(long long)head * a.L + key] = s;
        }
        __syncthreads();
      }
    }
  }

  if (PASS == 1) {
    // merge over the 32 key columns of each half, then over the key groups through LDS
    float* part = fbuf;                        // [4 waves][mpad][2]
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        float m = st_m[b][j], l = st_l[b][j];
        for (int o = 1; o < 32; o <<= 1) {
          float m2 = __shfl_xor(m, o, 64), l2 = __shfl_xor(l, o, 64);
          merge_ml(m, l, m2, l2);
        }
        if (b < nrb && col == 0) {
          int row = (wsub + b * WPT) * 32 + (j >> 2) * 8 + half * 4 + (j & 3);
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
      for (int s = 0; s < a.nsplit; ++s) merge_ml(m, l, rs[(s * a.mpad + r) * 2], rs[(s * a.mpad + r) * 2 + 1]);
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
static bool use_mfma(const Dims& dm, int dtype) { return dtype == MADAKV_BF16 && (dm.d == 64 || dm.d == 128); }

ScorePlan score_plan(const Dims& dm, int dtype) {
  ScorePlan p;
  p.mpad = (dm.M + 31) / 32 * 32;
  // enough workgroups to fill 256 CUs a few times over, chunks a multiple of 128 keys
  int want = std::max(1, (2048 + dm.heads - 1) / dm.heads);
  int max_split = std::max(1, dm.L / 512);
  int ns = std::min(std::min(want, max_split), 64);
  int chunk = ((dm.L + ns - 1) / ns + 127) / 128 * 128;
  p.nsplit = (dm.L + chunk - 1) / chunk;
  p.chunk = chunk;
  // heads per launch pair: keep the K bytes of a group small enough that the second
  // sweep can find them in the memory-side cache
  long long head_bytes = (long long)dm.L * dm.d * (dtype == MADAKV_BF16 ? 2 : 4);
  long long group_mb = 96;
  if (const char* e = getenv("MADAKV_SCORE_GROUP_MB")) group_mb = std::max(1, atoi(e));
  long long gh = std::max(1LL, group_mb * 1024 * 1024 / head_bytes);
  p.group_heads = (int)std::min<long long>(gh, dm.heads);
  return p;
}

size_t score_ws_bytes(const Dims& dm, int dtype) {
  ScorePlan p = score_plan(dm, dtype);
  return (size_t)dm.heads * p.nsplit * p.mpad * 2 * sizeof(float);
}

template <int D, int WPT>
static void launch_mfma_pair(const ScoreArgs& a0, int heads, size_t lds1, size_t lds2, hipStream_t st) {
  ScoreArgs a = a0;
  dim3 grid(a.nsplit, heads);
  if (lds1 > 48 * 1024 || lds2 > 48 * 1024) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_mfma_kernel<D, WPT, 1>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&score_mfma_kernel<D, WPT, 2>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
  }
  hipLaunchKernelGGL((score_mfma_kernel<D, WPT, 1>), grid, dim3(SCORE_THREADS), lds1, st, a);
  hipLaunchKernelGGL((score_mfma_kernel<D, WPT, 2>), grid, dim3(SCORE_THREADS), lds2, st, a);
}

hipError_t launch_score(const Dims& dm, const madakv_config& c, const void* q_win, const void* k,
                        float* psi, void* ws, hipStream_t st) {
  ScorePlan p = score_plan(dm, c.dtype);
  ScoreArgs a;
  a.q_win = q_win; a.k = k; a.psi = psi; a.rowstat = reinterpret_cast<float*>(ws);
  a.H = dm.H; a.G = dm.G; a.d = dm.d; a.L = dm.L; a.W = dm.W; a.M = dm.M;
  a.mpad = p.mpad; a.nsplit = p.nsplit; a.chunk = p.chunk; a.head0 = 0;
  float scale = c.softmax_scale > 0.f ? c.softmax_scale : 1.0f / sqrtf((float)dm.d);
  a.scale_log2 = scale * 1.4426950408889634f;
  for (int h0 = 0; h0 < dm.heads; h0 += p.group_heads) {
    int nh = std::min(p.group_heads, dm.heads - h0);
    a.head0 = h0;
    if (use_mfma(dm, c.dtype)) {
      int MB = p.mpad / 32;
      int wpt = MB <= 2 ? 1 : (MB <= 4 ? 2 : 4);
      size_t qbytes = (size_t)p.mpad * (dm.d + 8) * 2;
      size_t lds1 = qbytes + (size_t)4 * p.mpad * 2 * sizeof(float);
      size_t lds2 = qbytes + ((size_t)p.mpad + 128) * sizeof(float);
#define MADAKV_SCORE_CASE(DD, WW) launch_mfma_pair<DD, WW>(a, nh, lds1, lds2, st)
      if (dm.d == 128) { if (wpt == 1) MADAKV_SCORE_CASE(128, 1); else if (wpt == 2) MADAKV_SCORE_CASE(128, 2); else MADAKV_SCORE_CASE(128, 4); }
      else             { if (wpt == 1) MADAKV_SCORE_CASE(64, 1);  else if (wpt == 2) MADAKV_SCORE_CASE(64, 2);  else MADAKV_SCORE_CASE(64, 4); }
#undef MADAKV_SCORE_CASE
    } else {
      size_t lds = ((size_t)dm.M * dm.d + dm.M) * sizeof(float);
      dim3 grid(a.nsplit, nh);
      if (c.dtype == MADAKV_BF16) {
        hipLaunchKernelGGL((score_simple_kernel<uint16_t, 1>), grid, dim3(SCORE_THREADS), lds, st, a);
        hipLaunchKernelGGL((score_simple_kernel<uint16_t, 2>), grid, dim3(SCORE_THREADS), lds, st, a);
      } else {
        hipLaunchKernelGGL((score_simple_kernel<float, 1>), grid, dim3(SCORE_THREADS), lds, st, a);
        hipLaunchKernelGGL((score_simple_kernel<float, 2>), grid, dim3(SCORE_THREADS), lds, st, a);
      }
    }
  }
  return hipGetLastError();
}

}  // namespace madakv
