// Shared device helpers and the launcher interface between the C ABI and the kernels.
// gfx950 (MI355X) only: 64-lane wavefronts, DPP row operations, bf16 MFMA.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/madakv.h"

namespace madakv {

// Shapes of one call (n layers of the configured model).
struct Dims {
  int n;        // layers in the call
  int B, Hq, H, G;
  int d;        // head_dim
  int L, W;     // context length, proxy-token count
  int M;        // G * W proxy rows per KV head
  int nc;       // L - W candidates
  int heads;    // n * B * H
};

// Paged reduced cache (config.page_rows > 0): a head's kept rows fill whole pages that follow each other
// (so selection and gather see one contiguous segment), the rows decode appends go on into the free
// slots of the last of those pages and then into pages taken, on demand, from the top of the batch
// item's region.  table[head][0] = number of initial pages, table[head][1 + j] = page of the j-th
// page taken later; pool_top[b] = pages taken from the top of batch item b's region so far.
struct Paging {
  int page_rows;              // 0 = contiguous segments with max_new_tokens free rows each
  int entries;                // table entries per head
  int32_t* table;             // [n_layers * B * H][entries], owned by the handle
  unsigned long long* pool_top;   // [B]
  long long region_tokens;    // rows of one batch item's region
  long long init_limit;       // rows of a region the initial segments may fill (the rest is kept for appended pages)
};
long long region_tokens_of(const madakv_config& c);     // rows of the reduced cache one batch item owns
long long init_limit_of(const madakv_config& c);
int page_table_entries(const madakv_config& c);

struct ScorePlan { int nsplit; int chunk; int mpad; int group_heads; };
struct DecodePlan { int chunk_rows; int max_chunks; };

ScorePlan score_plan(const Dims& dm, int dtype);
DecodePlan decode_plan(const Dims& dm, const madakv_config& c, int longest_rows);
size_t score_ws_bytes(const Dims& dm, int dtype);
size_t select_ws_bytes(const Dims& dm, const madakv_config& c);
size_t decode_ws_bytes(const Dims& dm, const madakv_config& c);                             // worst case over head lengths
size_t decode_ws_bytes_for(const Dims& dm, const madakv_config& c, int longest_rows);     // for a known longest head

// Each launcher validates nothing: shapes were checked by the ABI layer.
hipError_t launch_score(const Dims& dm, const madakv_config& c, const void* q_win, const void* k, const float* row_lse,
                        float* psi, void* ws, hipStream_t st);
// Long heads on few heads: statistics and selection give every 16384-candidate chunk of a head a workgroup of its own
// and go through a buffer of split_buffer_bytes (owned by the handle) in several launches; split_chunks = chunks per
// head then, 0 otherwise.
int split_chunks(const Dims& dm);
size_t split_buffer_bytes(int heads, int M, int nchunks);
void launch_split_zero(uint32_t* p, long long words, hipStream_t st);   // a fill kernel (no memset node in captured streams)
hipError_t launch_stats(const Dims& dm, const madakv_config& c, const float* psi, const uint8_t* mask,
                        float* psi_pool, void* stats, int32_t* n_mod, int layer0, hipStream_t st,
                        void* split_buf = nullptr, size_t split_bytes = 0);
hipError_t launch_allocate(const Dims& dm, const madakv_config& c, int layer0, const void* stats,
                           const int32_t* n_mod, int32_t* budgets, long long* pool_state, hipStream_t st);
hipError_t launch_offsets(const Dims& dm, const madakv_config& c, int layer0, const int32_t* budgets,
                          int64_t* kv_off, int32_t* kv_len, long long* cursor_state, int32_t* layer_maxlen, void* ws,
                          const Paging& pg, int blocks_per_batch, hipStream_t st);
hipError_t launch_select(const Dims& dm, const madakv_config& c, const float* psi_pool, const uint8_t* mask,
                         const int32_t* budgets, const int64_t* kv_off, const int32_t* kv_len, int32_t* kept_idx,
                         hipStream_t st, const int32_t* seg_len = nullptr, const uint8_t* rowmod = nullptr,
                         void* split_buf = nullptr, size_t split_bytes = 0);
// re-eviction during generation (reevict.hip, and the one-sweep scoring kernel on ragged segments)
bool score_ragged_supported(const Dims& dm, const madakv_config& c, int longest_rows);
size_t score_ragged_ws_bytes(const Dims& dm, const madakv_config& c, int longest_rows, long long cache_rows);
hipError_t launch_score_ragged(const Dims& dm, const madakv_config& c, const void* q_recent, const void* k_c,
                               const int64_t* seg_off, const int32_t* seg_len, int longest_rows, long long cache_rows,
                               float* psi_c, void* ws, hipStream_t st);
// the last-window prefill attention with the Eq. 7 scores as a by-product
bool window_attn_supported(const Dims& dm, const madakv_config& c);
size_t window_attn_ws_bytes(const Dims& dm, const madakv_config& c);
hipError_t launch_window_attn(const Dims& dm, const madakv_config& c, const void* q_win, const void* k, const void* v,
                              void* out, float* row_lse, float* psi, void* ws, hipStream_t st);
hipError_t launch_restats(const Dims& dm, const madakv_config& c, const float* psi_c, const int32_t* kept_idx, const uint8_t* mask,
                          const int64_t* seg_off, const int32_t* seg_len, int appended, float* pool_c, uint8_t* rowmod,
                          void* stats, int32_t* budgets, hipStream_t st);
hipError_t launch_compact(const Dims& dm, const madakv_config& c, void* k_c, void* v_c, int32_t* kept_idx, const int32_t* sel,
                          const int64_t* seg_off, int32_t* kv_len, const int32_t* budgets, int appended, int gen_base, hipStream_t st);
hipError_t launch_linear_copy(const Dims& dm, const madakv_config& c, void* k_c, void* v_c, int32_t* kept_idx, const int64_t* seg_off,
                              const int32_t* seg_len, const Paging& pg, long long head0, int longest, void* k_lin, void* v_lin,
                              int32_t* kept_lin, int64_t* lin_off, bool back, hipStream_t st);
hipError_t launch_pool_reset(const Paging& pg, int batch, hipStream_t st);
hipError_t launch_gather(const Dims& dm, const madakv_config& c, int li0, int nli, const void* k, const void* v,
                         const int32_t* kept_idx, const int64_t* kv_off, const int32_t* kv_len,
                         void* k_c, void* v_c, const void* ws, long long region_tokens,
                         int blocks_per_batch, int grid_blocks, hipStream_t st, bool leave_room = false);
hipError_t launch_decode(const Dims& dm, const madakv_config& c, const void* q, const void* k_new,
                         const void* v_new, void* k_c, void* v_c, const int64_t* kv_off, int32_t* kv_len,
                         void* out, void* ws, long long capacity_tokens, int longest_rows, const Paging& pg, int layer0, hipStream_t st);

constexpr int GATHER_ROWS = 64;   // rows of the reduced cache one gather workgroup fills

#ifdef __HIPCC__
// ---------------------------------------------------------------- device helpers
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// OCP FP8 E4M3 (1 sign, 4 exponent bits of bias 7, 3 mantissa bits, subnormals, no infinities),
// the element type of the optional 8-bit reduced cache.  Encoding: round to nearest, ties to
// the even mantissa, magnitudes above 448 saturate.  Integer / float bit operations only, so the
// result is the same bit pattern a host implementation of the format's definition gives.
__device__ __forceinline__ uint32_t f32_to_e4m3(float f) {
  const uint32_t u = __float_as_uint(f);
  const uint32_t sign = (u >> 24) & 0x80u;
  const float a = fminf(__uint_as_float(u & 0x7fffffffu), 448.0f);          // NaN falls to 448 as well
  uint32_t code;
  if (a < 0.015625f) {                                                        // below 2^-6: the subnormal grid of 2^-9
    code = (uint32_t)__float2int_rn(a * 512.0f);                              // 0..8, 8 is the first normal code
  } else {
    uint32_t b = __float_as_uint(a);
    b += 0x7ffffu + ((b >> 20) & 1u);                                         // to 3 mantissa bits, ties to even; may carry into the exponent
    code = ((b >> 20) & 0x7ffu) - (120u << 3);                                // exponent re-biased from 127 to 7
  }
  return sign | min(code, 0x7eu);
}
// exact: every E4M3 value is a float.  Normal codes: the 7 magnitude bits become a float's low
// exponent / top mantissa bits with the exponent re-biased (7 -> 127); subnormal codes are m * 2^-9.
__device__ __forceinline__ float e4m3_to_f32(uint32_t c) {
  const float normal = __uint_as_float(((c & 0x7fu) << 20) + (120u << 23));
  const float subnormal = (float)(c & 7u) * 0.001953125f;
  const float mag = (c & 0x78u) ? normal : subnormal;
  return (c & 0x80u) ? -mag : mag;
}

__device__ __forceinline__ float load_elem(const float* p, long long i) { return p[i]; }
__device__ __forceinline__ float load_elem(const uint16_t* p, long long i) { return bf16_bits_to_f32(p[i]); }

// Sum over the 16 lanes of a DPP row; every lane of the row ends with the total.
__device__ __forceinline__ float row16_sum(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // row_half_mirror
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));  // row_mirror
  return x;
}

__device__ __forceinline__ float wave_sum(float x) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ long long shfl_i64(long long v, int src) {
  int lo = __shfl((int)(v & 0xffffffffLL), src, 64);
  int hi = __shfl((int)(v >> 32), src, 64);
  return ((long long)hi << 32) | (unsigned int)lo;
}
__device__ __forceinline__ long long wave_sum_i64(long long v) {
  for (int o = 32; o > 0; o >>= 1) {
    int lo = __shfl_xor((int)(v & 0xffffffffLL), o, 64);
    int hi = __shfl_xor((int)(v >> 32), o, 64);
    v += ((long long)hi << 32) | (unsigned int)lo;
  }
  return v;
}

// Inclusive prefix sum over the 64 lanes (lane 0 first) with DPP row operations: shifts by 1, 2, 4, 8
// inside each row of 16 lanes, then the last lane of row 0 / 2 is added to row 1 / 3 and the last
// lane of row 1 to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t x) {
#define MADAKV_DPP_ADD(ctrl, rmask, bctl) \
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, ctrl, rmask, 0xF, bctl)
  MADAKV_DPP_ADD(0x111, 0xF, true);   // row_shr:1
  MADAKV_DPP_ADD(0x112, 0xF, true);   // row_shr:2
  MADAKV_DPP_ADD(0x114, 0xF, true);   // row_shr:4
  MADAKV_DPP_ADD(0x118, 0xF, true);   // row_shr:8
  MADAKV_DPP_ADD(0x142, 0xA, false);  // row_bcast:15 into rows 1 and 3
  MADAKV_DPP_ADD(0x143, 0xC, false);  // row_bcast:31 into rows 2 and 3
#undef MADAKV_DPP_ADD
  return x;
}
// the same for 64-bit values below 2^63 / 64, as three 21-bit limbs (no carries between lanes' limbs)
__device__ __forceinline__ unsigned long long wave_incl_scan_u63(unsigned long long v) {
  const uint32_t l0 = wave_incl_scan_u32((uint32_t)(v & 0x1fffffULL));
  const uint32_t l1 = wave_incl_scan_u32((uint32_t)((v >> 21) & 0x1fffffULL));
  const uint32_t l2 = wave_incl_scan_u32((uint32_t)(v >> 42));
  return (unsigned long long)l0 + ((unsigned long long)l1 << 21) + ((unsigned long long)l2 << 42);
}

// Order-preserving map float -> uint32 (larger float, larger key); -0 is folded onto +0.
__device__ __forceinline__ uint32_t float_key(float f) {
  f += 0.0f;
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
#endif

}  // namespace madakv
