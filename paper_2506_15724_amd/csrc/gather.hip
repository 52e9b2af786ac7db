// Builds the reduced KV cache (paper Sec. 3.3: the evicted cache each head keeps):
//   k_c[kv_off + j, :] = k[head, kept_idx[kv_off + j], :]   and the same for v.
// Pure data movement, bound by HBM.  The reduced cache is one flat array of rows; a
// workgroup fills GATHER_ROWS consecutive rows of it, whichever heads they belong to, so
// every workgroup moves the same number of bytes whatever the per-head budgets are.
// A row is d * sizeof(T) bytes = LPR lanes x 16 bytes; a wave moves 64 / LPR rows per
// instruction and keeps UNROLL such loads of K and of V in flight before it stores.
#include "common.h"

namespace madakv {

struct GatherArgs {
  const void* k; const void* v; const int32_t* kept_idx; const int64_t* kv_off; const int32_t* kv_len;
  void* k_c; void* v_c; const long long* call_range; const int32_t* blk2head;
  int n, B, H, L, blocks_per_batch;
  long long region_tokens;
};

template <int LPR>   // lanes per row (row bytes / 16)
__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a) {
  constexpr int RPI = 64 / LPR;                 // rows per wave instruction
  constexpr int ROWS_PER_WAVE = GATHER_ROWS / 4;
  constexpr int ITERS = ROWS_PER_WAVE / RPI;
  const int b = blockIdx.y;
  const long long start = a.call_range[b * 2], end = a.call_range[b * 2 + 1];
  const long long blk = start / GATHER_ROWS + blockIdx.x;
  const long long row0 = blk * GATHER_ROWS;
  if (row0 >= end) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / LPR, piece = lane % LPR;
  const long long region = (long long)b * a.region_tokens;
  const int nh = a.n * a.H;
  int hh = a.blk2head[(long long)b * a.blocks_per_batch + blockIdx.x];
  const uint4* kin = reinterpret_cast<const uint4*>(a.k);
  const uint4* vin = reinterpret_cast<const uint4*>(a.v);
  uint4* kout = reinterpret_cast<uint4*>(a.k_c);
  uint4* vout = reinterpret_cast<uint4*>(a.v_c);

  uint4 kv[ITERS], vv[ITERS];
  long long dst[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const long long r = row0 + wave * ROWS_PER_WAVE + it * RPI + sub;     // row relative to the region
    dst[it] = -1;
    if (r >= start && r < end) {
      // advance to the head whose segment holds row r (segments tile the range without gaps)
      int h2 = hh;
      while (h2 + 1 < nh) {
        const int li = (h2 + 1) / a.H, h = (h2 + 1) % a.H;
        if (a.kv_off[((long long)li * a.B + b) * a.H + h] - region > r) break;
        ++h2;
      }
      const int li = h2 / a.H, h = h2 % a.H;
      const long long hidx = ((long long)li * a.B + b) * a.H + h;
      const long long j = region + r - a.kv_off[hidx];
      if (j < a.kv_len[hidx]) {                 // rows past kv_len are the free decode slots
        const long long src = hidx * a.L + a.kept_idx[region + r];
        kv[it] = kin[src * LPR + piece];
        vv[it] = vin[src * LPR + piece];
        dst[it] = region + r;
      }
    }
  }
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    if (dst[it] >= 0) {
      kout[dst[it] * LPR + piece] = kv[it];
      vout[dst[it] * LPR + piece] = vv[it];
    }
  }
}

hipError_t launch_gather(const Dims& dm, const madakv_config& c, const void* k, const void* v,
                         const int32_t* kept_idx, const int64_t* kv_off, const int32_t* kv_len,
                         void* k_c, void* v_c, const void* ws, long long region_tokens,
                         int blocks_per_batch, hipStream_t st) {
  GatherArgs a;
  a.k = k; a.v = v; a.kept_idx = kept_idx; a.kv_off = kv_off; a.kv_len = kv_len; a.k_c = k_c; a.v_c = v_c;
  a.call_range = reinterpret_cast<const long long*>(ws);
  a.blk2head = reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(ws) + ((size_t)dm.B * 2 * sizeof(long long) + 63) / 64 * 64);
  a.n = dm.n; a.B = dm.B; a.H = dm.H; a.L = dm.L; a.blocks_per_batch = blocks_per_batch;
  a.region_tokens = region_tokens;
  const int row_bytes = dm.d * (c.dtype == MADAKV_BF16 ? 2 : 4);
  const int lpr = row_bytes / 16;
  dim3 grid(blocks_per_batch, dm.B);
  if (lpr == 8) hipLaunchKernelGGL((gather_kernel<8>), grid, dim3(256), 0, st, a);
  else if (lpr == 16) hipLaunchKernelGGL((gather_kernel<16>), grid, dim3(256), 0, st, a);
  else if (lpr == 32) hipLaunchKernelGGL((gather_kernel<32>), grid, dim3(256), 0, st, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace madakv
