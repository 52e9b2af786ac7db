// Builds the reduced KV cache (paper Sec. 3.3: the evicted cache each head keeps):
//   k_c[kv_off + j, :] = k[head, kept_idx[kv_off + j], :]   and the same for v.
// Pure data movement, bound by HBM.  The reduced cache is one flat array of rows; a
// workgroup fills GATHER_ROWS consecutive rows of it, whichever heads they belong to, so
// every workgroup moves the same number of bytes whatever the per-head budgets are.
// A row is d * sizeof(T) bytes = LPR lanes x 16 bytes; a wave moves 64 / LPR rows per
// instruction and keeps UNROLL such loads of K and of V in flight before it stores.
#include "common.h"

#include <algorithm>

namespace madakv {

constexpr size_t GATHER_ROOM_LDS = 36 * 1024;   // four claims fit the 160 KB of a compute unit, five do not

// native vector type: arrays of it stay in registers (the HIP uint4 struct ends up in scratch)
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

struct GatherArgs {
  const void* k; const void* v; const int32_t* kept_idx; const int64_t* kv_off; const int32_t* kv_len;
  void* k_c; void* v_c; const long long* call_range; const int32_t* blk2head;
  int n, B, H, L, blocks_per_batch;
  int li0, li1;          // layers [li0, li1) of the call are gathered by this launch
  long long region_tokens;
};

template <int LPR, bool FP8>   // lanes per source row (row bytes / 16); FP8: bf16 rows are stored as E4M3
__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a) {
  constexpr int RPI = 64 / LPR;                 // rows per wave instruction
  constexpr int ROWS_PER_WAVE = GATHER_ROWS / 4;
  constexpr int ITERS = ROWS_PER_WAVE / RPI;
  const int b = blockIdx.y;
  const long long region = (long long)b * a.region_tokens;
  const long long call_start = a.call_range[b * 2], call_end = a.call_range[b * 2 + 1];
  // rows of the launch's layers: from the first head of layer li0 to the first head of layer li1
  const long long start = a.li0 == 0 ? call_start : a.kv_off[((long long)a.li0 * a.B + b) * a.H] - region;
  const long long end = a.li1 >= a.n ? call_end : a.kv_off[((long long)a.li1 * a.B + b) * a.H] - region;
  const long long blk = start / GATHER_ROWS + blockIdx.x;
  const long long tbl = blk - call_start / GATHER_ROWS;          // the block table is relative to the call's first block
  const long long row0 = blk * GATHER_ROWS;
  if (row0 >= end) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / LPR, piece = lane % LPR;
  const int nh = a.n * a.H;
  int hh = a.blk2head[(long long)b * a.blocks_per_batch + tbl];
  const u32x4_t* kin = reinterpret_cast<const u32x4_t*>(a.k);
  const u32x4_t* vin = reinterpret_cast<const u32x4_t*>(a.v);
  u32x4_t* kout = reinterpret_cast<u32x4_t*>(a.k_c);
  u32x4_t* vout = reinterpret_cast<u32x4_t*>(a.v_c);

  // Phases, so that dependent index loads never sit between the row loads of another row
  // (load counters retire in order: a wait for an index would also wait for every row load
  // issued before it): kept positions + the segment table of the next few heads, then all
  // row loads, then all stores.
  long long dst[ITERS]; int kidx[ITERS]; bool inr[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const long long r = row0 + wave * ROWS_PER_WAVE + it * RPI + sub;     // row relative to the region
    inr[it] = r >= start && r < end;
    dst[it] = region + r;
    kidx[it] = inr[it] ? a.kept_idx[dst[it]] : 0;                          // free slots hold garbage: unused below
  }
  // segments of the first head overlapping the block and its successors (they tile the range)
  constexpr int NC = 4;
  long long coff[NC + 1]; int clen[NC];
#pragma unroll
  for (int c = 0; c <= NC; ++c) {
    const int hc = min(hh + c, nh - 1);
    const long long hidx = ((long long)(hc / a.H) * a.B + b) * a.H + (hc % a.H);
    coff[c] = (hh + c < nh) ? a.kv_off[hidx] - region : end;               // past the last head: the end of the range
    if (c < NC) clen[c] = a.kv_len[hidx];
  }
  long long src[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const long long r = dst[it] - region;
    src[it] = -1;
    if (inr[it]) {
      int hsel = hh; long long hoff = coff[0]; int hlen = clen[0];
#pragma unroll
      for (int c = 1; c < NC; ++c)
        if (hh + c < nh && coff[c] <= r) { hsel = hh + c; hoff = coff[c]; hlen = clen[c]; }
      if (hh + NC < nh && coff[NC] <= r) {
        // more than NC segments start inside this block (very short segments): walk on
        int h2 = hh + NC;
        while (h2 + 1 < nh) {
          const int li = (h2 + 1) / a.H, h = (h2 + 1) % a.H;
          if (a.kv_off[((long long)li * a.B + b) * a.H + h] - region > r) break;
          ++h2;
        }
        const long long hidx = ((long long)(h2 / a.H) * a.B + b) * a.H + (h2 % a.H);
        hsel = h2; hoff = a.kv_off[hidx] - region; hlen = a.kv_len[hidx];
      }
      const long long hidx = ((long long)(hsel / a.H) * a.B + b) * a.H + (hsel % a.H);
      if (r - hoff < hlen)                       // rows past kv_len are the free decode slots
        src[it] = hidx * a.L + kidx[it];
    }
  }
  u32x4_t kv[ITERS], vv[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const long long s0 = src[it] >= 0 ? src[it] : 0;     // an in-bounds dummy keeps the load unconditional
    kv[it] = __builtin_nontemporal_load(kin + s0 * LPR + piece);     // rows are read once: keep them out of the caches
    vv[it] = __builtin_nontemporal_load(vin + s0 * LPR + piece);
  }
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    if (src[it] >= 0) {
      if (FP8) {
        // 8 bf16 -> 8 bytes per lane; a row of the reduced cache is LPR * 8 bytes
        typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
        u32x2_t ko, vo;
#pragma unroll
        for (int w = 0; w < 2; ++w) {
          uint32_t kb = 0, vb = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint32_t kp = kv[it][w * 2 + e / 2], vp = vv[it][w * 2 + e / 2];
            const float kf = (e & 1) ? bf16_hi(kp) : bf16_lo(kp), vf = (e & 1) ? bf16_hi(vp) : bf16_lo(vp);
            kb |= f32_to_e4m3(kf) << (8 * e); vb |= f32_to_e4m3(vf) << (8 * e);
          }
          ko[w] = kb; vo[w] = vb;
        }
        reinterpret_cast<u32x2_t*>(a.k_c)[dst[it] * LPR + piece] = ko;
        reinterpret_cast<u32x2_t*>(a.v_c)[dst[it] * LPR + piece] = vo;
      } else {
        __builtin_nontemporal_store(kv[it], kout + dst[it] * LPR + piece);
        __builtin_nontemporal_store(vv[it], vout + dst[it] * LPR + piece);
      }
    }
  }
}

hipError_t launch_gather(const Dims& dm, const madakv_config& c, int li0, int nli, const void* k, const void* v,
                         const int32_t* kept_idx, const int64_t* kv_off, const int32_t* kv_len,
                         void* k_c, void* v_c, const void* ws, long long region_tokens,
                         int blocks_per_batch, int grid_blocks, hipStream_t st, bool leave_room) {
  GatherArgs a;
  a.k = k; a.v = v; a.kept_idx = kept_idx; a.kv_off = kv_off; a.kv_len = kv_len; a.k_c = k_c; a.v_c = v_c;
  a.call_range = reinterpret_cast<const long long*>(ws);
  a.blk2head = reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(ws) + ((size_t)dm.B * 2 * sizeof(long long) + 63) / 64 * 64);
  a.n = dm.n; a.B = dm.B; a.H = dm.H; a.L = dm.L; a.blocks_per_batch = blocks_per_batch;
  a.region_tokens = region_tokens;
  a.li0 = li0; a.li1 = li0 + nli;
  const int row_bytes = dm.d * (c.dtype == MADAKV_BF16 ? 2 : 4);
  const int lpr = row_bytes / 16;
  dim3 grid(std::min(grid_blocks, blocks_per_batch), dm.B);
  // leave_room: statistics / selection kernels of another layer group run on a second stream meanwhile.
  // Eight of these workgroups fit a compute unit and would keep it full until the grid has drained; the
  // claim of GATHER_ROOM_LDS bytes of (unused) LDS holds them to four, which costs the copy nothing
  // (measured: 2 to 8 workgroups per compute unit move the same bytes per second) and lets the others in.
  const size_t lds = leave_room ? GATHER_ROOM_LDS : 0;
  if (c.cache_fp8) {
    if (lpr == 8) hipLaunchKernelGGL((gather_kernel<8, true>), grid, dim3(256), lds, st, a);
    else if (lpr == 16) hipLaunchKernelGGL((gather_kernel<16, true>), grid, dim3(256), lds, st, a);
    else return hipErrorInvalidValue;
  } else if (lpr == 8) hipLaunchKernelGGL((gather_kernel<8, false>), grid, dim3(256), lds, st, a);
  else if (lpr == 16) hipLaunchKernelGGL((gather_kernel<16, false>), grid, dim3(256), lds, st, a);
  else if (lpr == 32) hipLaunchKernelGGL((gather_kernel<32, false>), grid, dim3(256), lds, st, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace madakv
