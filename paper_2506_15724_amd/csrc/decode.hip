// Decode over the reduced, ragged cache (paper Sec. 3.1 Eq. 3-5): append the new K/V row to
// every head's segment (Eq. 4), then out = softmax(scale * q K_c^T) V_c over the rows the
// head kept (Eq. 5).  The G query heads of a KV head share one pass over its K_c and V_c.
//
// This is bandwidth work: 2 * len * d * sizeof(T) bytes per KV head and step, a few flops
// per byte.  A row is LPR lanes x 16 bytes; a wave reads 64 / LPR rows per load
// instruction and keeps UNROLL K rows and UNROLL V rows in flight.  The dot product is
// reduced over the LPR lanes of a row with DPP row operations, the softmax is the usual
// running max / running sum in the log2 domain with fp32 accumulation.  Each head's rows
// are cut into chunks of `chunk_rows` (one workgroup each): a single layer's 128 ragged heads
// become ~2000 equal pieces of work that the hardware scheduler spreads over 256 CUs.  The
// grid is (heads, longest possible head / chunk_rows): workgroups past a head's real length
// exit at once, and since the chunk index is the slow grid dimension they are dispatched
// after all the real work.  A second, small kernel merges the partial (max, sum, acc) triples
// of each head in chunk order.  (Merging inside the first kernel by the last workgroup to
// arrive was measured three times and lost every time: with device-scope fences, which write back and
// invalidate the whole L2 of an XCD per workgroup, 15x slower; with fence-free agent-scope
// atomic stores / loads of the partials and one arrival counter per head, 10% slower per call
// on 128 heads of ~2K rows and 4x slower on 32 heads of ~4K rows: every workgroup then ends in
// a store acknowledgement plus an atomic round trip, and the last one adds a dependent read.
// Without any counter: the workgroup of a head's last chunk, which is
// dispatched after the others, polls their partials, written as self-validating 64-bit words
// {value, call number}; 30.2 against 29.5 us per call for the same kernel followed by the merge
// kernel, and the extra state costs the attention loop registers: 142 instead of 122, or spills.
// Cutting the rows of all heads, laid end to end, into equal stretches per workgroup, so that
// the launch has a single, perfectly balanced round of workgroups, was measured too: 27.3 us
// against 26.9 us for the attention part on 128 heads of ~2K rows, the table of head starts
// every workgroup has to build first costs what the balance gains.)
// The appended row is taken from k_new / v_new by the
// workgroup whose chunk holds it, which also stores it in the cache; kv_len is bumped by
// whoever finalises the head.
#include "common.h"

#include <algorithm>

namespace madakv {

constexpr float DNEG_BIG = -1.0e30f;
constexpr int DEC_THREADS = 256;

struct DecodeArgs {
  const void* q; const void* k_new; const void* v_new; void* k_c; void* v_c;
  const int64_t* kv_off; int32_t* kv_len; void* out; float* part;
  int B, H, G, d, chunk_rows, max_chunks, out_fp32, has_new;
  long long capacity;   // rows in k_c / v_c
  // paged cache (page_rows > 0): see struct Paging
  int page_rows, page_shift, tbl_entries;
  int32_t* page_tbl; unsigned long long* pool_top;
  long long region_pages;      // pages in one batch item's region
  long long head0;             // index of the call's first head in the whole model (layer0 * B * H)
  float scale_log2;
};

// 16 bytes that are read once per launch (cache rows): a non-temporal load, so that the stream
// does not push anything useful out of the caches.  Measured: 10-15% off the decode step.
typedef __attribute__((ext_vector_type(4))) unsigned int stream_u32x4_t;
__device__ __forceinline__ uint4 stream_load16(const void* p) {
  const stream_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const stream_u32x4_t*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}

template <int LPR> __device__ __forceinline__ float row_sum(float x);
template <> __device__ __forceinline__ float row_sum<16>(float x) { return row16_sum(x); }
template <> __device__ __forceinline__ float row_sum<8>(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));
  return x;
}
template <> __device__ __forceinline__ float row_sum<4>(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));
  return x;
}
template <> __device__ __forceinline__ float row_sum<32>(float x) {
  x = row16_sum(x);
  return x + __shfl_xor(x, 16, 64);
}

template <typename T> struct Elems;
template <> struct Elems<uint16_t> {
  static constexpr int EPL = 8;
  static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
  }
};
template <> struct Elems<uint8_t> {                  // E4M3 bytes of the 8-bit reduced cache
  static constexpr int EPL = 16;
  static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {                     // the hardware conversion is exact (every code is a float)
      const f32x2_t lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
      const f32x2_t hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
      f[i * 4] = lo[0]; f[i * 4 + 1] = lo[1]; f[i * 4 + 2] = hi[0]; f[i * 4 + 3] = hi[1];
    }
  }
};
template <> struct Elems<float> {
  static constexpr int EPL = 4;
  static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};

// EPL consecutive elements of the caller's type T (Q, k_new, v_new) as floats
template <typename T, int EPL>
__device__ __forceinline__ void load_floats(const T* p, float* f) {
  constexpr int PER = 16 / sizeof(T);                 // elements per 16-byte load
#pragma unroll
  for (int j = 0; j < EPL / PER; ++j) Elems<T>::unpack(*reinterpret_cast<const uint4*>(p + j * PER), f + j * PER);
}
// 16 bytes of a reduced-cache row made from the caller's new row: a plain copy when the cache
// has the caller's type, an E4M3 encoding of 16 bf16 values otherwise
template <typename T, typename CT>
__device__ __forceinline__ uint4 cache_piece(const T* p) {
  if (sizeof(T) == sizeof(CT)) return *reinterpret_cast<const uint4*>(p);
  float f[16];
  load_floats<T, 16>(p, f);
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = f32_to_e4m3(f[i * 4]) | (f32_to_e4m3(f[i * 4 + 1]) << 8) | (f32_to_e4m3(f[i * 4 + 2]) << 16) | (f32_to_e4m3(f[i * 4 + 3]) << 24);
  return make_uint4(w[0], w[1], w[2], w[3]);
}

template <typename T>
__device__ __forceinline__ void store_out(void* out, int out_fp32, long long o, float val) {
  if (out_fp32 || sizeof(T) == 4) reinterpret_cast<float*>(out)[o] = val;
  else reinterpret_cast<uint16_t*>(out)[o] = f32_to_bf16_rne(val);
}

// ---- where row r of a head lives ---------------------------------------------------------
// Contiguous segments: at off + r.  Paged cache: the first init_rows rows (the head's initial pages,
// which follow each other) likewise; later rows in pages listed in the head's table.  `fresh`
// is the page this workgroup has just taken for the row being appended, if it had to take one
// (the table entry it wrote is not yet visible to its other threads).
struct RowMap {
  long long off;
  int init_rows;               // INT_MAX without paging
  const int32_t* tbl;          // the head's table (entries 1.. = pages taken later)
  int shift, fresh_slot;
  long long fresh_page;
  __device__ __forceinline__ long long operator()(int r) const {
    if (r < init_rows) return off + r;
    const int q = r - init_rows, j = q >> shift;
    const long long pg = (j == fresh_slot) ? fresh_page : (long long)tbl[1 + j];
    return (pg << shift) + (q & ((1 << shift) - 1));
  }
};

__device__ __forceinline__ bool can_append_to(const DecodeArgs& a, long long off, int len_old) {
  // an empty segment (its budgets did not fit the cache) stays empty; contiguous segments also end at the cache's end
  return a.has_new && len_old > 0 && (a.page_rows ? true : off + len_old < a.capacity);
}

// All threads of the workgroup.  rows [r_begin, r_end) are the workgroup's; when the appended row is
// among them and starts a new page, thread 0 takes the next page from the top of the batch item's region.
__device__ __forceinline__ RowMap make_row_map(const DecodeArgs& a, long long hidx, long long off, int len_old, bool can_append,
                                               int r_begin, int r_end) {
  RowMap m;
  m.off = off; m.init_rows = 0x7fffffff; m.tbl = nullptr; m.shift = 0; m.fresh_slot = -1; m.fresh_page = 0;
  if (!a.page_rows) return m;
  __shared__ long long s_fresh;
  int32_t* tbl = a.page_tbl + (a.head0 + hidx) * a.tbl_entries;
  m.tbl = tbl; m.shift = a.page_shift;
  m.init_rows = tbl[0] << a.page_shift;
  const int q = len_old - m.init_rows;
  const bool takes = can_append && len_old >= r_begin && len_old < r_end && q >= 0 && (q & (a.page_rows - 1)) == 0;   // uniform
  if (takes) {
    if (threadIdx.x == 0) {
      const long long b = ((a.head0 + hidx) / a.H) % a.B;
      const unsigned long long nth = atomicAdd(a.pool_top + b, 1ULL);
      const long long page = (b + 1) * a.region_pages - 1 - (long long)nth;
      tbl[1 + (q >> a.page_shift)] = (int32_t)page;
      s_fresh = page;
    }
    __syncthreads();
    m.fresh_slot = q >> a.page_shift;
    m.fresh_page = s_fresh;
  }
  return m;
}

template <typename T, typename CT, int LPR, int GT, int UNROLL, int NW>   // T: Q / new rows / out; CT: cache elements
__global__ __launch_bounds__(NW * 64) void decode_attn_kernel(DecodeArgs a) {
  constexpr int EPL = Elems<CT>::EPL;
  constexpr int RPI = 64 / LPR;
  constexpr int D = LPR * EPL;
  __shared__ float s_ml[NW][GT][2];
  __shared__ float s_acc[NW][GT][D];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / LPR, piece = lane % LPR;
  const long long hidx = blockIdx.x;                 // (layer, batch, kv head) of the call
  const int chunk = blockIdx.y;                      // which `chunk_rows` rows of the head
  const int len_old = a.kv_len[hidx];
  const long long off = a.kv_off[hidx];
  // an empty segment (its budgets did not fit the cache) stays empty: no append, output 0/0 = NaN
  const bool can_append = can_append_to(a, off, len_old);
  const int len = len_old + (can_append ? 1 : 0);
  const int nch = max(1, (len + a.chunk_rows - 1) / a.chunk_rows);
  if (chunk >= nch) return;                          // the grid is sized for the longest possible head
  const long long lb = hidx / a.H;
  const int h = (int)(hidx % a.H);
  const int r_begin = chunk * a.chunk_rows;
  const int r_end = min(len, r_begin + a.chunk_rows);
  const RowMap at = make_row_map(a, hidx, off, len_old, can_append, r_begin, r_end);
  // the NW waves take turns on consecutive RPI * UNROLL-row slices, so that at any moment the
  // workgroup reads one contiguous stretch of K and one of V
  constexpr int WSTEP = RPI * UNROLL;

  // queries of the group, pre-multiplied by scale * log2(e)
  float qf[GT][EPL];
  const T* qg = reinterpret_cast<const T*>(a.q) + (lb * a.H + h) * (long long)a.G * D;
#pragma unroll
  for (int g = 0; g < GT; ++g) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[g][e] = 0.f;
    if (g < a.G) load_floats<T, EPL>(qg + (long long)g * D + piece * EPL, qf[g]);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[g][e] *= a.scale_log2;
  }

  float m[GT], l[GT], acc[GT][EPL];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    m[g] = DNEG_BIG; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  const uint4* kc = reinterpret_cast<const uint4*>(a.k_c);
  const uint4* vc = reinterpret_cast<const uint4*>(a.v_c);
  const T* kn = reinterpret_cast<const T*>(a.k_new);
  const T* vn = reinterpret_cast<const T*>(a.v_new);

  for (int row0 = r_begin + wave * WSTEP; row0 < r_end; row0 += NW * WSTEP) {
    uint4 kraw[UNROLL], vraw[UNROLL];
    bool valid[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int r = row0 + u * RPI + sub;
      valid[u] = r < r_end;
      kraw[u] = make_uint4(0, 0, 0, 0); vraw[u] = make_uint4(0, 0, 0, 0);
      if (valid[u]) {
        if (can_append && r == len_old) {
          kraw[u] = cache_piece<T, CT>(kn + hidx * D + piece * EPL);
          vraw[u] = cache_piece<T, CT>(vn + hidx * D + piece * EPL);
          reinterpret_cast<uint4*>(a.k_c)[at(r) * LPR + piece] = kraw[u];     // Eq. 4: the row joins the cache
          reinterpret_cast<uint4*>(a.v_c)[at(r) * LPR + piece] = vraw[u];
        } else {
          kraw[u] = stream_load16(kc + at(r) * LPR + piece);
          vraw[u] = stream_load16(vc + at(r) * LPR + piece);
        }
      }
    }
    float s[UNROLL][GT];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      float kf[EPL];
      Elems<CT>::unpack(kraw[u], kf);
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) dot = fmaf(qf[g][e], kf[e], dot);
        s[u][g] = row_sum<LPR>(dot);
      }
    }
    float vf[UNROLL][EPL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) Elems<CT>::unpack(vraw[u], vf[u]);
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float mx = m[g];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) mx = valid[u] ? fmaxf(mx, s[u][g]) : mx;
      const float sc = exp2f(m[g] - mx);
      l[g] *= sc;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= sc;
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const float p = valid[u] ? exp2f(s[u][g] - mx) : 0.f;
        l[g] += p;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vf[u][e], acc[g][e]);
      }
      m[g] = mx;
    }
  }

  // merge the RPI row groups of the wave (fixed butterfly), then the NW waves through LDS
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    for (int o = LPR; o < 64; o <<= 1) {
      const float m2 = __shfl_xor(m[g], o, 64), l2 = __shfl_xor(l[g], o, 64);
      const float mx = fmaxf(m[g], m2);
      const float c1 = exp2f(m[g] - mx), c2 = exp2f(m2 - mx);
      l[g] = l[g] * c1 + l2 * c2;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float a2 = __shfl_xor(acc[g][e], o, 64);
        acc[g][e] = acc[g][e] * c1 + a2 * c2;
      }
      m[g] = mx;
    }
    if (sub == 0) {
      if (piece == 0) { s_ml[wave][g][0] = m[g]; s_ml[wave][g][1] = l[g]; }
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_acc[wave][g][piece * EPL + e] = acc[g][e];
    }
  }
  __syncthreads();
  // thread t < D finishes element t of every query head of the group
  const int t = threadIdx.x;
  const long long obase = (lb * a.H + h) * (long long)a.G * D;
  if (t < D) {
    for (int g = 0; g < a.G; ++g) {
      float mx = DNEG_BIG;
      for (int w = 0; w < NW; ++w) mx = fmaxf(mx, s_ml[w][g][0]);
      float ls = 0.f, av = 0.f;
      for (int w = 0; w < NW; ++w) {
        const float c = exp2f(s_ml[w][g][0] - mx);
        ls += s_ml[w][g][1] * c;
        av += s_acc[w][g][t] * c;
      }
      if (nch == 1) {
        store_out<T>(a.out, a.out_fp32, obase + (long long)g * D + t, av / ls);
      } else {
        float* p = a.part + ((hidx * a.max_chunks + chunk) * a.G + g) * (long long)(D + 2);
        p[t] = av;
        if (t == 0) { p[D] = mx; p[D + 1] = ls; }
      }
    }
  }
  // kv_len is read by every chunk of the head: with several chunks per head only the merge
  // kernel, which runs after all of them, may store the new length
  if (a.max_chunks == 1 && can_append && threadIdx.x == 0) a.kv_len[hidx] = len;
}

// ------------------------------------------------------------------------------------
// Grouped-query variant (bf16, G >= 2): both contractions run on the 16x16x32 bf16 MFMA, so
// that the G query heads of a KV head cost no more vector instructions than one.
//   S^T[key][q] = K_tile . Q^T     A = 16 keys x 32 dims read straight from the cache rows
//                                  (a lane takes 16 bytes of "its" key), B = Q, kept in registers
//   O[q][d]    += P . V_tile       contraction over 32 keys.  In S^T a lane holds 4 keys of each
//                                  16-key block for its query; the contraction index is numbered
//                                  so that exactly those 8 keys are the lane's A fragment of P
//                                  (no cross-lane movement); V needs the matching rows per output
//                                  column, read as 2-byte elements from a wave-private LDS tile
//                                  that the V rows were written to with coalesced 16-byte loads.
// P goes through the MFMA as bf16 hi + lo parts (two MFMAs), which keeps fp32-level accuracy.
// The running max / sum live per query in the lanes of S^T; the rescale factors are fetched
// into the O layout with four lane reads per tile.
// ------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 dbf16x8_t;
typedef __attribute__((ext_vector_type(4))) float df32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int du32x4_t;

typedef __attribute__((ext_vector_type(2))) unsigned int du32x2_t;
typedef __attribute__((ext_vector_type(2))) float df32x2_t;

// 4 E4M3 bytes -> 4 bf16 (exact: 3 mantissa bits fit bf16's 7), as two packed dwords
__device__ __forceinline__ du32x2_t e4m3x4_to_bf16x4(uint32_t w) {
  const df32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
  du32x2_t o;
  o[0] = (__float_as_uint(a[0]) >> 16) | (__float_as_uint(a[1]) & 0xffff0000u);
  o[1] = (__float_as_uint(b[0]) >> 16) | (__float_as_uint(b[1]) & 0xffff0000u);
  return o;
}
// 8 bf16 (16 bytes) -> 8 E4M3 bytes
__device__ __forceinline__ du32x2_t bf16x8_to_e4m3x8(const du32x4_t& r) {
  du32x2_t o;
#pragma unroll
  for (int w = 0; w < 2; ++w)
    o[w] = f32_to_e4m3(bf16_lo(r[w * 2])) | (f32_to_e4m3(bf16_hi(r[w * 2])) << 8) |
           (f32_to_e4m3(bf16_lo(r[w * 2 + 1])) << 16) | (f32_to_e4m3(bf16_hi(r[w * 2 + 1])) << 24);
  return o;
}

template <int D, bool FP8>   // FP8: the cache rows are E4M3 bytes, turned into bf16 operands on the fly
__global__ __launch_bounds__(DEC_THREADS) void decode_gqa_kernel(DecodeArgs a) {
  constexpr int GT = 8;                // query heads per KV head supported (rows 8..15 of the MFMA tile are padding)
  constexpr int NW = 4;
  constexpr int KS = D / 32;           // MFMA steps over the head dimension
  constexpr int DB = D / 16;           // 16-column blocks of the output
  constexpr int RS = D + 8;            // bf16 elements per LDS row of the V tile (16 B pad)
  constexpr int CB = FP8 ? 1 : 2;      // bytes per cache element
  constexpr int LPR = D * CB / 16;     // lanes per row in a coalesced 16-byte load
  constexpr int VE = 16 / CB;          // V elements per lane and load
  constexpr int RPI = 64 / LPR;        // rows per load instruction
  constexpr int VL = 32 / RPI;         // load instructions per 32-row V tile
  __shared__ float s_ml[NW][GT][2];
  __shared__ __attribute__((aligned(16))) uint16_t s_v[NW][32][RS];
  // the per-wave results reuse the V tiles once every wave is through with them
  static_assert(sizeof(float) * NW * GT * D <= sizeof(uint16_t) * NW * 32 * RS, "results must fit the V tiles");
  float (*s_acc)[GT][D] = reinterpret_cast<float (*)[GT][D]>(&s_v[0][0][0]);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j16 = lane & 15, c = lane >> 4;
  const long long hidx = blockIdx.x;
  const int chunk = blockIdx.y;
  const int len_old = a.kv_len[hidx];
  const long long off = a.kv_off[hidx];
  const bool can_append = can_append_to(a, off, len_old);
  const int len = len_old + (can_append ? 1 : 0);
  const int nch = max(1, (len + a.chunk_rows - 1) / a.chunk_rows);
  if (chunk >= nch) return;
  const long long lb = hidx / a.H;
  const int h = (int)(hidx % a.H);
  const int r_begin = chunk * a.chunk_rows;
  const int r_end = min(len, r_begin + a.chunk_rows);
  const RowMap at = make_row_map(a, hidx, off, len_old, can_append, r_begin, r_end);

  const unsigned char* kc = reinterpret_cast<const unsigned char*>(a.k_c);   // cache rows of D * CB bytes
  const unsigned char* vc = reinterpret_cast<const unsigned char*>(a.v_c);
  const uint16_t* kn = reinterpret_cast<const uint16_t*>(a.k_new);
  const uint16_t* vn = reinterpret_cast<const uint16_t*>(a.v_new);
  unsigned char* kcw = reinterpret_cast<unsigned char*>(a.k_c);
  unsigned char* vcw = reinterpret_cast<unsigned char*>(a.v_c);

  // Q as the B operand: lane (q = j16, c) holds dims [32 ks + 8 c, +8) of query q
  dbf16x8_t qb[KS];
  const uint16_t* qg = reinterpret_cast<const uint16_t*>(a.q) + (lb * a.H + h) * (long long)a.G * D;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    du32x4_t raw = {0u, 0u, 0u, 0u};
    if (j16 < a.G) raw = *reinterpret_cast<const du32x4_t*>(qg + (long long)j16 * D + ks * 32 + c * 8);
    qb[ks] = __builtin_bit_cast(dbf16x8_t, raw);
  }

  float m_run = DNEG_BIG, l_run = 0.f;       // for query j16 (every lane group c holds a copy of m, a share of l)
  df32x4_t oacc[DB];                         // O[q = 4c + r][d = 16 db + j16]
#pragma unroll
  for (int db = 0; db < DB; ++db) oacc[db] = df32x4_t{0.f, 0.f, 0.f, 0.f};
  uint16_t* vt = &s_v[wave][0][0];
  const int vsub = lane / LPR, vpiece = lane % LPR;

  // Registers hold the K fragments and V rows of the tile being worked on; each set is refilled
  // with the next tile's data as soon as it has been consumed (V: once parked in LDS, K: after
  // the S^T MFMAs), so the loads fly under the softmax and the P.V MFMAs.  Rows past the end of
  // the chunk are clamped to its last row (valid memory) and masked where they are used.
  du32x4_t kraw[2][KS], vraw[VL];            // raw cache bytes (E4M3: 8 bytes of a K piece sit in kraw[..][..].xy)
#define MADAKV_LOAD_V(T0)                                                                          \
  _Pragma("unroll") for (int i = 0; i < VL; ++i) {                                                 \
    const int r = (T0) + i * RPI + vsub;                                                           \
    const int rc = min(r, r_end - 1);                                                              \
    const bool fresh = can_append && rc == len_old;                                                \
    if (!fresh) {                                                                                  \
      vraw[i] = __builtin_nontemporal_load(reinterpret_cast<const du32x4_t*>(vc + (at(rc) * D + vpiece * VE) * CB)); \
    } else {                                                                                       \
      const uint16_t* np_ = vn + hidx * D + vpiece * VE;                                           \
      if (FP8) {                                                                                   \
        const du32x2_t e0 = bf16x8_to_e4m3x8(*reinterpret_cast<const du32x4_t*>(np_));             \
        const du32x2_t e1 = bf16x8_to_e4m3x8(*reinterpret_cast<const du32x4_t*>(np_ + 8));         \
        vraw[i] = du32x4_t{e0[0], e0[1], e1[0], e1[1]};                                            \
      } else {                                                                                     \
        vraw[i] = *reinterpret_cast<const du32x4_t*>(np_);                                         \
      }                                                                                            \
      if (r == rc) *reinterpret_cast<du32x4_t*>(vcw + (at(rc) * D + vpiece * VE) * CB) = vraw[i]; /* Eq. 4 */ \
    }                                                                                              \
  }
#define MADAKV_LOAD_K(T0)                                                                          \
  _Pragma("unroll") for (int blk = 0; blk < 2; ++blk) {                                            \
    const int r = (T0) + blk * 16 + j16;                                                           \
    const int rc = min(r, r_end - 1);                                                              \
    const bool fresh = can_append && rc == len_old;                                                \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                            \
      const long long eo = at(rc) * D + ks * 32 + c * 8;        /* element offset of the piece */ \
      if (!fresh) {                                                                                \
        if (FP8) { const du32x2_t t2 = __builtin_nontemporal_load(reinterpret_cast<const du32x2_t*>(kc + eo)); kraw[blk][ks] = du32x4_t{t2[0], t2[1], 0u, 0u}; } \
        else kraw[blk][ks] = __builtin_nontemporal_load(reinterpret_cast<const du32x4_t*>(kc + eo * 2)); \
      } else {                                                                                     \
        const du32x4_t nb = *reinterpret_cast<const du32x4_t*>(kn + hidx * D + ks * 32 + c * 8);   \
        if (FP8) {                                                                                 \
          const du32x2_t t2 = bf16x8_to_e4m3x8(nb);                                                \
          kraw[blk][ks] = du32x4_t{t2[0], t2[1], 0u, 0u};                                          \
          if (r == rc) *reinterpret_cast<du32x2_t*>(kcw + eo) = t2;                                \
        } else {                                                                                   \
          kraw[blk][ks] = nb;                                                                      \
          if (r == rc) *reinterpret_cast<du32x4_t*>(kcw + eo * 2) = nb;                            \
        }                                                                                          \
      }                                                                                            \
    }                                                                                              \
  }
  const int t_first = r_begin + wave * 32;
  if (t_first < r_end) {
    MADAKV_LOAD_V(t_first)
    MADAKV_LOAD_K(t_first)
  }
  for (int t0 = t_first; t0 < r_end; t0 += NW * 32) {
    const int t_next = t0 + NW * 32;
    // ---- V rows of the tile: parked in the wave's LDS tile, then the registers are refilled
#pragma unroll
    for (int i = 0; i < VL; ++i) {
      if (FP8) {                                           // 16 bytes -> 16 bf16
        const du32x2_t c0 = e4m3x4_to_bf16x4(vraw[i][0]), c1 = e4m3x4_to_bf16x4(vraw[i][1]);
        const du32x2_t c2 = e4m3x4_to_bf16x4(vraw[i][2]), c3 = e4m3x4_to_bf16x4(vraw[i][3]);
        const du32x4_t b0 = {c0[0], c0[1], c1[0], c1[1]}, b1 = {c2[0], c2[1], c3[0], c3[1]};
        *reinterpret_cast<du32x4_t*>(vt + (i * RPI + vsub) * RS + vpiece * 16) = b0;
        *reinterpret_cast<du32x4_t*>(vt + (i * RPI + vsub) * RS + vpiece * 16 + 8) = b1;
      } else {
        *reinterpret_cast<du32x4_t*>(vt + (i * RPI + vsub) * RS + vpiece * 8) = vraw[i];
      }
    }
    MADAKV_LOAD_V(t_next)
    // ---- S^T for the two 16-key blocks
    float p[2][4];
    float tmax = DNEG_BIG;
    df32x4_t sacc[2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      sacc[blk] = df32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        du32x4_t kb = kraw[blk][ks];
        if (FP8) {
          const du32x2_t c0 = e4m3x4_to_bf16x4(kraw[blk][ks][0]), c1 = e4m3x4_to_bf16x4(kraw[blk][ks][1]);
          kb = du32x4_t{c0[0], c0[1], c1[0], c1[1]};
        }
        sacc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(dbf16x8_t, kb), qb[ks], sacc[blk], 0, 0, 0);
      }
    }
    MADAKV_LOAD_K(t_next)
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int key = t0 + blk * 16 + 4 * c + rr;      // in S^T the lane holds keys 4c..4c+3 of the block
        p[blk][rr] = key < r_end ? sacc[blk][rr] * a.scale_log2 : DNEG_BIG;
        tmax = fmaxf(tmax, p[blk][rr]);
      }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    uint32_t hi[4], lo[4];                                // P as bf16 hi + lo, 8 keys per lane: the A fragment
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float pv = exp2f(p[e >> 2][e & 3] - m_new);
      psum += pv;
      const uint32_t hb = f32_to_bf16_rne(pv);
      const uint32_t lb2 = f32_to_bf16_rne(pv - bf16_bits_to_f32(hb));
      if (e & 1) { hi[e >> 1] |= hb << 16; lo[e >> 1] |= lb2 << 16; }
      else { hi[e >> 1] = hb; lo[e >> 1] = lb2; }
    }
    l_run = l_run * alpha + psum;
    const dbf16x8_t pa_hi = __builtin_bit_cast(dbf16x8_t, du32x4_t{hi[0], hi[1], hi[2], hi[3]});
    const dbf16x8_t pa_lo = __builtin_bit_cast(dbf16x8_t, du32x4_t{lo[0], lo[1], lo[2], lo[3]});
    // rescale factors of the queries this lane holds in the O layout (q = 4c + r)
    float al[4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) al[rr] = __shfl(alpha, (c << 4) | (4 * c + rr), 64);
    // the V tile must be complete before it is read with another lane mapping (same wave: in order)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      // B fragment: for output column 16 db + j16 the 8 keys of this lane group (4c..4c+3 of either block)
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = (e >> 2) * 16 + 4 * c + (e & 3);
        const uint32_t x = vt[row * RS + db * 16 + j16];
        if (e & 1) w[e >> 1] |= x << 16; else w[e >> 1] = x;
      }
      const dbf16x8_t vb = __builtin_bit_cast(dbf16x8_t, du32x4_t{w[0], w[1], w[2], w[3]});
      df32x4_t o = oacc[db];
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) o[rr] *= al[rr];
      o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi, vb, o, 0, 0, 0);
      o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo, vb, o, 0, 0, 0);
      oacc[db] = o;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
#undef MADAKV_LOAD_V
#undef MADAKV_LOAD_K

  // ---- per wave: total of the sums over the lane groups, then everything to LDS in [q][d] form
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  __syncthreads();                                   // all V tiles are dead: their space takes the results
  if (c == 0 && j16 < GT) { s_ml[wave][j16][0] = m_run; s_ml[wave][j16][1] = l_run; }
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int q = 4 * c + rr;
      if (q < GT) s_acc[wave][q][db * 16 + j16] = oacc[db][rr];
    }
  __syncthreads();
  const int t = threadIdx.x;
  const long long obase = (lb * a.H + h) * (long long)a.G * D;
  if (t < D) {
    for (int g = 0; g < a.G; ++g) {
      float mx = DNEG_BIG;
      for (int w = 0; w < NW; ++w) mx = fmaxf(mx, s_ml[w][g][0]);
      float ls = 0.f, av = 0.f;
      for (int w = 0; w < NW; ++w) {
        const float cf = exp2f(s_ml[w][g][0] - mx);
        ls += s_ml[w][g][1] * cf;
        av += s_acc[w][g][t] * cf;
      }
      if (nch == 1) {
        store_out<uint16_t>(a.out, a.out_fp32, obase + (long long)g * D + t, av / ls);
      } else {
        float* pp = a.part + ((hidx * a.max_chunks + chunk) * a.G + g) * (long long)(D + 2);
        pp[t] = av;
        if (t == 0) { pp[D] = mx; pp[D + 1] = ls; }
      }
    }
  }
  if (a.max_chunks == 1 && can_append && threadIdx.x == 0) a.kv_len[hidx] = len;
}

// Merges the partial (max, sum, acc) triples of every head that was cut into several chunks,
// in chunk order, and stores the new length.  One workgroup per head, thread t owns element t.
template <typename T>
__global__ __launch_bounds__(1024) void decode_merge_kernel(DecodeArgs a) {
  const long long hidx = blockIdx.x;
  const int D = a.d;
  const int g = min((int)threadIdx.x / D, a.G - 1), t = threadIdx.x % D;   // one thread per (query head of the group, element)
  const long long cstride = (long long)a.G * (D + 2);
  const float* pg = a.part + (hidx * a.max_chunks * a.G + g) * (long long)(D + 2);
  // The first eight chunks' partials are fetched before the head's length is known (slots past the
  // head's last chunk hold old values and are masked below): one round trip to memory instead of two.
  const int lim = a.max_chunks - 1;
  float mc[8], lc[8], ac[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float* p = pg + (long long)min(j, lim) * cstride;
    mc[j] = p[D]; lc[j] = p[D + 1]; ac[j] = p[t];
  }
  const int len_old = a.kv_len[hidx];
  __syncthreads();                                   // every wave has read the length before anyone stores the new one
  const bool can_append = can_append_to(a, a.kv_off[hidx], len_old);
  const int len = len_old + (can_append ? 1 : 0);
  const int nch = max(1, (len + a.chunk_rows - 1) / a.chunk_rows);
  if (can_append && threadIdx.x == 0) a.kv_len[hidx] = len;
  if (nch == 1) return;                              // output already written by the attention kernel
  if ((int)threadIdx.x / D >= a.G) return;
  const long long lb = hidx / a.H;
  const int h = (int)(hidx % a.H);
  const long long obase = (lb * a.H + h) * (long long)a.G * D;
  float m = DNEG_BIG, ls = 0.f, av = 0.f;
  for (int c0 = 0; c0 < nch; c0 += 8) {              // 24 independent loads in flight per batch
    if (c0 > 0) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float* p = pg + (long long)min(c0 + j, lim) * cstride;
        mc[j] = p[D]; lc[j] = p[D + 1]; ac[j] = p[t];
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool ok = c0 + j < nch;
      mc[j] = ok ? mc[j] : DNEG_BIG; lc[j] = ok ? lc[j] : 0.f; ac[j] = ok ? ac[j] : 0.f;
    }
    float bm = m;
#pragma unroll
    for (int j = 0; j < 8; ++j) bm = fmaxf(bm, mc[j]);
    const float sc = exp2f(m - bm);
    ls *= sc; av *= sc;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float w = exp2f(mc[j] - bm);
      ls = fmaf(lc[j], w, ls);
      av = fmaf(ac[j], w, av);
    }
    m = bm;
  }
  store_out<T>(a.out, a.out_fp32, obase + (long long)g * D + t, av / ls);
}

// Rows per workgroup: small for a single layer (many short workgroups balance ragged heads and
// keep every CU streaming), larger when thousands of heads already fill the chip.
DecodePlan decode_plan(const Dims& dm, const madakv_config& c, int longest_rows) {
  DecodePlan p;
  // longest_rows: upper bound on any head's length in this call (the worst case if unknown)
  const int longest = std::max(1, std::min(longest_rows, c.ctx_len + c.max_new_tokens));
  // Measured on MI355X: 256-row chunks for a single layer's ragged heads at a 16K context
  // (smaller chunks lose to per-workgroup start-up cost, one workgroup per head to the imbalance
  // of ragged lengths), growing to 1024 rows when the heads are long (un-evicted cache), so that
  // the chip sees about eight workgroups per CU; 512 rows once a call covers >= 1024 heads.
  int rows = 512;
  if (dm.heads < 1024) {
    const long long typical = std::min(c.budget, c.ctx_len) + c.max_new_tokens;    // rows of an average head
    const long long per = ((long long)dm.heads * typical + 2047) / 2048;
    const long long by_len = typical / 64;                     // a long head is not cut into more than ~64 chunks
    rows = (int)std::min<long long>(1024, std::max<long long>(256, std::max(per, by_len) / 256 * 256));
  }
  p.chunk_rows = rows;
  p.max_chunks = (longest + rows - 1) / rows;
  return p;
}

size_t decode_ws_bytes_for(const Dims& dm, const madakv_config& c, int longest_rows) {
  DecodePlan p = decode_plan(dm, c, longest_rows);
  return (size_t)dm.heads * p.max_chunks * dm.G * (dm.d + 2) * sizeof(float) + 64;
}
size_t decode_ws_bytes(const Dims& dm, const madakv_config& c) { return decode_ws_bytes_for(dm, c, c.ctx_len + c.max_new_tokens); }

template <typename T, typename CT, int LPR>
static hipError_t launch_decode_t(const Dims& dm, DecodeArgs& a, hipStream_t st) {
  dim3 grid(dm.heads, a.max_chunks), block(DEC_THREADS);
  if (sizeof(T) == 2 && dm.G >= 2) {
    // grouped queries in bf16: the MFMA kernel
    constexpr bool F8 = sizeof(CT) == 1;
    if (dm.d == 128) hipLaunchKernelGGL((decode_gqa_kernel<128, F8>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((decode_gqa_kernel<64, F8>), grid, block, 0, st, a);
    if (a.max_chunks > 1) hipLaunchKernelGGL((decode_merge_kernel<T>), dim3(dm.heads), dim3(dm.G * dm.d), 0, st, a);
    return hipGetLastError();
  }
  // (8-bit cache: a lane holds 16 elements per 16-byte load; four rows in flight per lane keep the kernel at 3 waves
  // per SIMD, eight would need 230 registers: 21.2 against 23.3 us per layer call)
  if (dm.G == 1 && sizeof(CT) == 1) hipLaunchKernelGGL((decode_attn_kernel<T, CT, LPR, 1, 4, 4>), grid, block, 0, st, a);
  else if (dm.G == 1) hipLaunchKernelGGL((decode_attn_kernel<T, CT, LPR, 1, 8, 4>), grid, block, 0, st, a);
  else if (dm.G == 2) hipLaunchKernelGGL((decode_attn_kernel<T, CT, LPR, 2, 4, 4>), grid, block, 0, st, a);
  else if (dm.G <= 4) hipLaunchKernelGGL((decode_attn_kernel<T, CT, LPR, 4, 4, 4>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((decode_attn_kernel<T, CT, LPR, 8, 2, 4>), grid, block, 0, st, a);
  if (a.max_chunks > 1) hipLaunchKernelGGL((decode_merge_kernel<T>), dim3(dm.heads), dim3(dm.G * dm.d), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_decode(const Dims& dm, const madakv_config& c, const void* q, const void* k_new,
                         const void* v_new, void* k_c, void* v_c, const int64_t* kv_off, int32_t* kv_len,
                         void* out, void* ws, long long capacity_tokens, int longest_rows, const Paging& pg, int layer0, hipStream_t st) {
  DecodeArgs a;
  a.capacity = capacity_tokens;
  a.page_rows = pg.page_rows; a.tbl_entries = pg.entries; a.page_tbl = pg.table; a.pool_top = pg.pool_top;
  a.page_shift = 0;
  while (pg.page_rows && (1 << a.page_shift) < pg.page_rows) ++a.page_shift;
  a.region_pages = pg.page_rows ? pg.region_tokens / pg.page_rows : 0;
  a.head0 = (long long)layer0 * dm.B * dm.H;
  a.q = q; a.k_new = k_new; a.v_new = v_new; a.k_c = k_c; a.v_c = v_c; a.kv_off = kv_off; a.kv_len = kv_len;
  a.out = out; a.part = reinterpret_cast<float*>(ws);
  DecodePlan p = decode_plan(dm, c, longest_rows);
  a.B = dm.B; a.H = dm.H; a.G = dm.G; a.d = dm.d; a.chunk_rows = p.chunk_rows; a.max_chunks = p.max_chunks;
  a.out_fp32 = c.out_fp32; a.has_new = (k_new != nullptr) ? 1 : 0;
  const float scale = c.softmax_scale > 0.f ? c.softmax_scale : 1.0f / sqrtf((float)dm.d);
  a.scale_log2 = scale * 1.4426950408889634f;
  const int lpr = dm.d * (c.dtype == MADAKV_BF16 ? 2 : 4) / 16;
  if (c.dtype == MADAKV_BF16) {
    if (c.cache_fp8) {                                   // rows of d bytes: d / 16 lanes per row
      if (dm.d == 128) return launch_decode_t<uint16_t, uint8_t, 8>(dm, a, st);
      if (dm.d == 64) return launch_decode_t<uint16_t, uint8_t, 4>(dm, a, st);
    }
    if (lpr == 8) return launch_decode_t<uint16_t, uint16_t, 8>(dm, a, st);
    if (lpr == 16) return launch_decode_t<uint16_t, uint16_t, 16>(dm, a, st);
  } else {
    if (lpr == 16) return launch_decode_t<float, float, 16>(dm, a, st);
    if (lpr == 32) return launch_decode_t<float, float, 32>(dm, a, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace madakv
