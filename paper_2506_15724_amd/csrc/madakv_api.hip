// C ABI of the MadaKV hot path: argument validation, the handle, and the order in which
// the kernels of each call are enqueued.  No arithmetic of the method lives here.
#include "common.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace madakv;

constexpr int MAX_GROUPS = 4;      // layer groups a multi-layer call is cut into for the overlap

// Scratch of madakv_decode_attn_static: the partial results of heads that are cut into several
// chunks.  One copy per GPU, at an address of its own on each, held until the process ends.  In
// host code the name below is only a handle for hipGetSymbolAddress; the device address is
// resolved once per device (static_scratch_on_current_device) and passed to the kernels.
constexpr size_t STATIC_SCRATCH_BYTES = MADAKV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES];
static std::mutex g_scratch_mutex;

struct madakv_handle {
  madakv_config cfg;
  int device;
  int32_t last_hip_error;
  long long* d_state;              // [3 * B]: HCC pool, cache cursor, pages taken for appended rows (paged cache), per batch item
  int32_t* d_page_tbl;             // paged cache: [n_layers * B * H][entries] page table (null otherwise)
  void* d_split; size_t split_bytes;   // long contexts: buffer of the chunk-parallel statistics / selection (null otherwise)
  std::vector<int32_t> appended;   // decode rows appended since the last (re-)eviction, per layer
  std::vector<int32_t> gen_base;   // tokens generated before that, per layer (their original positions are ctx_len + 0, 1, ...)
  // Longest head of each layer after eviction: written by the device, copied to pinned host
  // memory asynchronously; decode sizes its grid from it once the copy is known to have landed
  // (event query, never a wait) and from the worst case before that.
  int32_t* d_maxlen;
  int32_t* h_maxlen;
  hipEvent_t maxlen_event;
  // per layer: 0 = nothing known (decode sizes its grid for the worst case), 1 = copy enqueued on
  // maxlen_stream and covered by maxlen_event, 2 = the value in h_maxlen has landed
  std::vector<uint8_t> maxlen_state;
  hipStream_t maxlen_stream;
  void* static_scratch;            // this device's copy of the static scratch array
  // Side stream and events for the overlap of the bandwidth-bound kernels (score sweeps, gather)
  // with the latency-bound per-head kernels (statistics, selection) inside one call.  The side
  // stream forks from and joins the caller's stream through events; default priority.
  hipStream_t side;
  hipEvent_t ev_grp[MAX_GROUPS], ev_sel[MAX_GROUPS], ev_fork, ev_join;
};

namespace madakv {
// Rows of the reduced cache one batch item owns.  Contiguous segments: every head has its kept rows plus
// max_new_tokens free ones.  Paged: the kept rows of all heads in whole pages (the sum of budgets is
// conserved, so at most one partly filled page per head) plus, shared by all heads, the pages
// max_new_tokens appended rows per head can ever need.
int page_table_entries(const madakv_config& c) {
  return c.page_rows ? 2 + (c.max_new_tokens + c.page_rows - 1) / c.page_rows : 0;
}
long long init_limit_of(const madakv_config& c) {
  const long long heads = (long long)c.n_layers * c.n_kv_heads, keep = std::min(c.budget, c.ctx_len);
  if (!c.page_rows) return heads * (keep + c.max_new_tokens);
  return heads * ((keep + c.page_rows - 1) / c.page_rows + 1) * c.page_rows;
}
long long region_tokens_of(const madakv_config& c) {
  if (!c.page_rows) return init_limit_of(c);
  const long long heads = (long long)c.n_layers * c.n_kv_heads;
  return init_limit_of(c) + heads * ((c.max_new_tokens + c.page_rows - 1) / c.page_rows) * c.page_rows;
}
}  // namespace madakv

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool bad_ptr(const void* p) { return p == nullptr || !aligned16(p); }                   // Q/K/V-like tensors: 16-byte vector access
bool bad_ptr(const void* p, size_t align) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) & (align - 1)) != 0; }

Dims make_dims(const madakv_config& c, int n) {
  Dims dm;
  dm.n = n; dm.B = c.batch; dm.Hq = c.n_q_heads; dm.H = c.n_kv_heads; dm.G = c.n_q_heads / c.n_kv_heads;
  dm.d = c.head_dim; dm.L = c.ctx_len; dm.W = c.window; dm.M = dm.G * dm.W; dm.nc = dm.L - dm.W;
  dm.heads = n * c.batch * c.n_kv_heads;
  return dm;
}

long long region_tokens(const madakv_config& c) { return region_tokens_of(c); }

Paging make_paging(const madakv_handle* h) {
  const madakv_config& c = h->cfg;
  Paging pg;
  pg.page_rows = c.page_rows; pg.entries = page_table_entries(c); pg.table = h->d_page_tbl;
  pg.pool_top = reinterpret_cast<unsigned long long*>(h->d_state + 2 * c.batch);
  pg.region_tokens = region_tokens_of(c); pg.init_limit = init_limit_of(c);
  return pg;
}

int blocks_per_batch(const madakv_config& c, int n) {
  long long per_call = (long long)n * c.n_kv_heads * ((long long)c.ctx_len + c.max_new_tokens + 2 * c.page_rows);
  long long tokens = std::min(region_tokens(c), per_call);
  return (int)(tokens / GATHER_ROWS + 2);
}

int32_t check_range(const madakv_handle* h, int layer0, int n) {
  if (!h) return MADAKV_ERR_INVALID_ARG;
  if (layer0 < 0 || n < 1 || layer0 + n > h->cfg.n_layers) return MADAKV_ERR_INVALID_ARG;
  return MADAKV_OK;
}

int32_t hip_fail(madakv_handle* h, hipError_t e) {
  if (e == hipSuccess) return MADAKV_OK;
  h->last_hip_error = (int32_t)e;
  return MADAKV_ERR_HIP;
}

int32_t validate(const madakv_config& c) {
  if (c.n_layers < 1 || c.n_layers > 1024 || c.batch < 1 || c.n_kv_heads < 1 || c.n_kv_heads > 64) return MADAKV_ERR_BAD_SHAPE;
  if (c.n_q_heads < c.n_kv_heads || c.n_q_heads % c.n_kv_heads) return MADAKV_ERR_BAD_SHAPE;
  if (c.n_q_heads / c.n_kv_heads > 8) return MADAKV_ERR_BAD_SHAPE;
  if (c.head_dim != 64 && c.head_dim != 128) return MADAKV_ERR_BAD_SHAPE;
  if (c.dtype != MADAKV_FP32 && c.dtype != MADAKV_BF16) return MADAKV_ERR_UNSUPPORTED_DTYPE;
  if (c.ctx_len < 2 || c.ctx_len > (1 << 20) || c.window < 1 || c.window >= c.ctx_len) return MADAKV_ERR_BAD_SHAPE;
  const int M = c.n_q_heads / c.n_kv_heads * c.window;
  if (M > 256) return MADAKV_ERR_BAD_SHAPE;
  if (c.dtype == MADAKV_FP32 && (long long)M * c.head_dim > 12288) return MADAKV_ERR_BAD_SHAPE;   // Q tile of the FMA path must fit LDS
  if (c.n_modalities < 2 || c.n_modalities > 4) return MADAKV_ERR_BAD_SHAPE;
  if ((c.cache_fp8 | 1) != 1) return MADAKV_ERR_INVALID_ARG;
  if (c.cache_fp8 && c.dtype != MADAKV_BF16) return MADAKV_ERR_UNSUPPORTED_DTYPE;
  if (c.pool_k < 1 || c.pool_k > 63 || (c.pool_k & 1) == 0) return MADAKV_ERR_BAD_SHAPE;
  if (c.budget < 1 || (c.budget < c.ctx_len && c.budget <= c.window)) return MADAKV_ERR_BAD_BUDGET;
  if (c.hcc_rho < 1 || c.hcc_rho > 1024) return MADAKV_ERR_INVALID_ARG;
  if (!(c.theta > 0.f) || c.theta > 1.f) return MADAKV_ERR_INVALID_ARG;
  if (c.softmax_scale < 0.f || c.max_new_tokens < 0) return MADAKV_ERR_INVALID_ARG;
  if (c.mpa_mode < 0 || c.mpa_mode > 3 || c.hcc_mode < 0 || c.hcc_mode > 2 || (c.out_fp32 | 1) != 1) return MADAKV_ERR_INVALID_ARG;
  if (c.page_rows != 0 && c.page_rows != 16 && c.page_rows != 32 && c.page_rows != 64 && c.page_rows != 128 && c.page_rows != 256)
    return MADAKV_ERR_INVALID_ARG;
  if ((c.pool_mode | 1) != 1 || (c.share_mode | 1) != 1 || (c.select_mode | 1) != 1 || c.sink_tokens < 0) return MADAKV_ERR_INVALID_ARG;
  return MADAKV_OK;
}

void destroy_side(madakv_handle* h) {
  if (h->side) { (void)hipStreamSynchronize(h->side); (void)hipStreamDestroy(h->side); }
  if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
  if (h->ev_join) (void)hipEventDestroy(h->ev_join);
  for (int g = 0; g < MAX_GROUPS; ++g) if (h->ev_grp[g]) (void)hipEventDestroy(h->ev_grp[g]);
  for (int g = 0; g < MAX_GROUPS; ++g) if (h->ev_sel[g]) (void)hipEventDestroy(h->ev_sel[g]);
}

// A call over n layers is cut into up to MAX_GROUPS layer groups of (nearly) equal size for the overlap, as many as
// leave a group at least one head per compute unit: the per-head kernels of a group then fill the chip and are worth
// hiding under the next group's sweeps and gathers.  With fewer heads (grouped-query models) only the last group's
// per-head kernels are exposed however the layers are cut, and more groups only add launches: the Qwen-shaped
// eviction takes 1.00-1.05 ms in one or two groups against 1.16 ms in four.
// Fills begin[0 .. groups] and returns the number of groups.
int layer_groups(const madakv_config& c, int n, int* begin) {
  const long long heads = (long long)n * c.batch * c.n_kv_heads;
  int ng = (int)std::max<long long>(1, std::min<long long>(std::min(MAX_GROUPS, n), heads / 256));
  if (const char* e = getenv("MADAKV_LAYER_GROUPS")) ng = std::max(1, std::min(std::min(MAX_GROUPS, n), atoi(e)));   // (tests, measurements)
  for (int g = 0; g <= ng; ++g) begin[g] = (int)((long long)n * g / ng);
  return ng;
}
int largest_group(const madakv_config& c, int n) {
  int b[MAX_GROUPS + 1];
  const int ng = layer_groups(c, n, b);
  int m = 0;
  for (int g = 0; g < ng; ++g) m = std::max(m, b[g + 1] - b[g]);
  return m;
}

size_t window_ws_for_call(const madakv_config& c, int n) {
  int b[MAX_GROUPS + 1];
  const int ng = layer_groups(c, n, b);
  size_t need = 0;
  for (int g = 0; g < ng; ++g) need = std::max(need, window_attn_ws_bytes(make_dims(c, b[g + 1] - b[g]), c));
  return need;
}

size_t score_ws_for_call(const madakv_config& c, int n) {
  int b[MAX_GROUPS + 1];
  const int ng = layer_groups(c, n, b);
  size_t need = 0;
  for (int g = 0; g < ng; ++g) need = std::max(need, score_ws_bytes(make_dims(c, b[g + 1] - b[g]), c.dtype));
  return need;
}

// Hands the longest segment of layers [layer0, layer0 + n) to the host without waiting: an
// asynchronous copy into pinned memory plus an event.  A new pass (layer0 == 0) forgets what was
// known about every layer; a failed enqueue leaves the layers of the call unknown.
hipError_t publish_maxlen(madakv_handle* h, int layer0, int n, hipStream_t st, hipError_t e) {
  const madakv_config& c = h->cfg;
  if (layer0 == 0) std::fill(h->maxlen_state.begin(), h->maxlen_state.end(), (uint8_t)0);
  // copies still in flight on another stream are not covered by the event recorded below
  if (h->maxlen_stream != st)
    for (auto& sflag : h->maxlen_state) if (sflag == 1) sflag = 0;
  for (int l = layer0; l < layer0 + n; ++l) h->maxlen_state[l] = 0;
  if (e == hipSuccess) e = hipMemcpyAsync(h->h_maxlen + (size_t)layer0 * c.batch, h->d_maxlen + (size_t)layer0 * c.batch,
                                             sizeof(int32_t) * n * c.batch, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipEventRecord(h->maxlen_event, st);
  if (e == hipSuccess) {
    for (int l = layer0; l < layer0 + n; ++l) h->maxlen_state[l] = 1;
    h->maxlen_stream = st;
  }
  return e;
}

// Upper bound on the rows of any head of layers [layer0, layer0 + n) after this call's append:
// from the lengths the eviction produced when they are known to have reached the host, the
// worst case otherwise.
// replayed: the launch may run again later without coming through here (a stream under graph capture): the bound
// then covers every row the segments have room for, not only the rows of this step.
int longest_rows(madakv_handle* h, int layer0, int n, bool replayed = false) {
  const madakv_config& c = h->cfg;
  const int worst = c.ctx_len + c.max_new_tokens;
  bool pending = false;
  for (int l = layer0; l < layer0 + n; ++l) pending = pending || h->maxlen_state[l] == 1;
  if (pending && !replayed && hipEventQuery(h->maxlen_event) == hipSuccess)       // (no event query on a capturing stream's behalf)
    for (auto& sflag : h->maxlen_state) if (sflag == 1) sflag = 2;
  int mx = 0;
  for (int l = layer0; l < layer0 + n; ++l) {
    if (h->maxlen_state[l] != 2) return worst;
    const int grown = replayed ? c.max_new_tokens : h->appended[l] + 1;
    for (int b = 0; b < c.batch; ++b) mx = std::max(mx, h->h_maxlen[(size_t)l * c.batch + b] + grown);
  }
  return std::min(worst, mx);
}

// After work was put on the side stream: the caller's stream waits for it, also when an
// enqueue in between failed (the first error is kept).
hipError_t join_side(madakv_handle* h, hipStream_t st, hipError_t e) {
  hipError_t j = hipEventRecord(h->ev_join, h->side);
  if (j == hipSuccess) j = hipStreamWaitEvent(st, h->ev_join, 0);
  return e != hipSuccess ? e : j;
}

// Device address of the static scratch array on the current device (resolved once per device).
hipError_t static_scratch_on_current_device(int device, void** out) {
  if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

int32_t decode_impl(madakv_handle* h, int32_t layer0, int32_t n,
                    const void* q, const void* k_new, const void* v_new,
                    void* k_c, void* v_c, const int64_t* kv_off, int32_t* kv_len,
                    void* out, void* ws, size_t ws_bytes, bool ws_is_static, void* stream) {
  int32_t r = check_range(h, layer0, n);
  if (r != MADAKV_OK) return r;
  if (bad_ptr(q) || bad_ptr(k_c) || bad_ptr(v_c) || bad_ptr(kv_off, 8) || bad_ptr(kv_len, 4) || bad_ptr(out) || bad_ptr(ws))
    return MADAKV_ERR_INVALID_ARG;
  if ((k_new == nullptr) != (v_new == nullptr)) return MADAKV_ERR_INVALID_ARG;
  if (k_new && (!aligned16(k_new) || !aligned16(v_new))) return MADAKV_ERR_INVALID_ARG;
  Dims dm = make_dims(h->cfg, n);
  // Under graph capture the launch is sized once and replayed while the heads grow: the grid (and the share of the
  // workspace) then covers all the rows the segments have room for.
  hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
  const bool replayed = hipStreamIsCapturing(reinterpret_cast<hipStream_t>(stream), &capturing) != hipSuccess ||
                        capturing != hipStreamCaptureStatusNone;
  const int longest = longest_rows(h, layer0, n, replayed);
  // a caller's workspace is sized for the worst case; the static one must hold what this launch uses
  const size_t need = ws_is_static ? decode_ws_bytes_for(dm, h->cfg, longest) : decode_ws_bytes(dm, h->cfg);
  if (ws_bytes < need) return MADAKV_ERR_WORKSPACE_TOO_SMALL;
  if (k_new) {
    for (int l = layer0; l < layer0 + n; ++l)
      if (h->appended[l] >= h->cfg.max_new_tokens) return MADAKV_ERR_INVALID_ARG;
  }
  hipError_t e = launch_decode(dm, h->cfg, q, k_new, v_new, k_c, v_c, kv_off, kv_len, out, ws,
                               region_tokens(h->cfg) * h->cfg.batch, longest, make_paging(h), layer0,
                               reinterpret_cast<hipStream_t>(stream));
  if (e == hipSuccess && k_new) for (int l = layer0; l < layer0 + n; ++l) h->appended[l] += 1;
  return hip_fail(h, e);
}

}  // namespace

extern "C" {

int32_t madakv_create(const madakv_config* cfg, madakv_handle** out) {
  if (!cfg || !out) return MADAKV_ERR_INVALID_ARG;
  int32_t v = validate(*cfg);
  if (v != MADAKV_OK) return v;
  madakv_handle* h = new (std::nothrow) madakv_handle();
  if (!h) return MADAKV_ERR_INVALID_ARG;
  h->cfg = *cfg;
  h->last_hip_error = 0;
  h->d_state = nullptr;
  h->d_maxlen = nullptr; h->h_maxlen = nullptr; h->maxlen_event = nullptr;
  h->maxlen_state.assign(cfg->n_layers, 0); h->maxlen_stream = nullptr;
  h->side = nullptr; h->ev_fork = nullptr; h->ev_join = nullptr;
  for (int g = 0; g < MAX_GROUPS; ++g) { h->ev_grp[g] = nullptr; h->ev_sel[g] = nullptr; }
  h->appended.assign(cfg->n_layers, 0);
  h->gen_base.assign(cfg->n_layers, 0);
  h->static_scratch = nullptr; h->d_page_tbl = nullptr;
  h->d_split = nullptr; h->split_bytes = 0;
  hipError_t e = hipGetDevice(&h->device);
  if (e == hipSuccess) e = static_scratch_on_current_device(h->device, &h->static_scratch);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&h->d_state), sizeof(long long) * 3 * cfg->batch);
  if (e == hipSuccess) e = hipMemset(h->d_state, 0, sizeof(long long) * 3 * cfg->batch);
  if (cfg->page_rows) {
    const size_t tb = sizeof(int32_t) * (size_t)cfg->n_layers * cfg->batch * cfg->n_kv_heads * page_table_entries(*cfg);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&h->d_page_tbl), tb);
    if (e == hipSuccess) e = hipMemset(h->d_page_tbl, 0, tb);
  }
  {
    // long contexts on few heads: room for the largest launch that would use the chunk-parallel statistics / selection
    Dims d1 = make_dims(*cfg, 1);
    if (split_chunks(d1) > 0) {
      const int nchunks = (d1.nc + 16383) / 16384;
      const int heads = std::min(cfg->n_layers * cfg->batch * cfg->n_kv_heads, 128);
      h->split_bytes = split_buffer_bytes(heads, cfg->n_modalities, nchunks);
      if (e == hipSuccess) e = hipMalloc(&h->d_split, h->split_bytes);
    }
  }
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&h->d_maxlen), sizeof(int32_t) * cfg->n_layers * cfg->batch);
  if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&h->h_maxlen), sizeof(int32_t) * cfg->n_layers * cfg->batch, hipHostMallocDefault);
  if (e == hipSuccess) memset(h->h_maxlen, 0, sizeof(int32_t) * cfg->n_layers * cfg->batch);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&h->maxlen_event, hipEventDisableTiming);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&h->ev_join, hipEventDisableTiming);
  for (int g = 0; g < MAX_GROUPS && e == hipSuccess; ++g) e = hipEventCreateWithFlags(&h->ev_grp[g], hipEventDisableTiming);
  for (int g = 0; g < MAX_GROUPS && e == hipSuccess; ++g) e = hipEventCreateWithFlags(&h->ev_sel[g], hipEventDisableTiming);
  if (e != hipSuccess) {
    if (h->d_maxlen) (void)hipFree(h->d_maxlen);
    if (h->d_page_tbl) (void)hipFree(h->d_page_tbl);
    if (h->d_split) (void)hipFree(h->d_split);
    if (h->h_maxlen) (void)hipHostFree(h->h_maxlen);
    if (h->maxlen_event) (void)hipEventDestroy(h->maxlen_event);
    destroy_side(h);
    if (h->d_state) (void)hipFree(h->d_state);
    delete h;
    return MADAKV_ERR_HIP;
  }
  *out = h;
  return MADAKV_OK;
}

int32_t madakv_destroy(madakv_handle* h) {
  if (!h) return MADAKV_ERR_INVALID_ARG;
  hipError_t e = hipFree(h->d_state);
  (void)hipFree(h->d_maxlen);
  if (h->d_page_tbl) (void)hipFree(h->d_page_tbl);
  if (h->d_split) (void)hipFree(h->d_split);
  (void)hipHostFree(h->h_maxlen);
  (void)hipEventDestroy(h->maxlen_event);
  destroy_side(h);
  delete h;
  return e == hipSuccess ? MADAKV_OK : MADAKV_ERR_HIP;
}

int32_t madakv_last_hip_error(const madakv_handle* h) { return h ? h->last_hip_error : 0; }

int32_t madakv_workspace_bytes(const madakv_handle* h, int32_t n_layers_per_call,
                               size_t* score_ws, size_t* select_ws, size_t* decode_ws) {
  if (!h || n_layers_per_call < 1 || n_layers_per_call > h->cfg.n_layers) return MADAKV_ERR_INVALID_ARG;
  Dims dm = make_dims(h->cfg, n_layers_per_call);
  if (score_ws) *score_ws = score_ws_for_call(h->cfg, n_layers_per_call);
  if (select_ws) {
    // enough for madakv_select_gather over n layers and for madakv_evict (one slice per layer group)
    const int gl = largest_group(h->cfg, n_layers_per_call);
    const size_t slices = ((select_ws_bytes(make_dims(h->cfg, gl), h->cfg) + 255) / 256 * 256) * MAX_GROUPS;
    *select_ws = std::max(select_ws_bytes(dm, h->cfg), slices);
  }
  if (decode_ws) *decode_ws = decode_ws_bytes(dm, h->cfg);
  return MADAKV_OK;
}

int32_t madakv_compact_capacity_tokens(const madakv_handle* h, int64_t* tokens) {
  if (!h || !tokens) return MADAKV_ERR_INVALID_ARG;
  *tokens = region_tokens(h->cfg) * h->cfg.batch;
  return MADAKV_OK;
}

// window_attn: v, out (and optionally lse_out) given: the scores come out of the last-window attention kernel
static int32_t score_impl(madakv_handle* h, int32_t layer0, int32_t n,
                          const void* q_win, const void* k, const uint8_t* mask, const float* row_lse,
                          float* psi, float* psi_pool, void* stats, int32_t* n_mod,
                          void* ws, size_t ws_bytes, void* stream,
                          const void* v = nullptr, void* out = nullptr, float* lse_out = nullptr) {
  int32_t r = check_range(h, layer0, n);
  if (r != MADAKV_OK) return r;
  if (bad_ptr(q_win) || bad_ptr(k) || bad_ptr(mask, 1) || bad_ptr(psi, 4) || bad_ptr(psi_pool, 4) || bad_ptr(stats, 4) ||
      bad_ptr(n_mod, 4) || bad_ptr(ws)) return MADAKV_ERR_INVALID_ARG;
  const bool window_attn = v != nullptr;
  if (window_attn) {
    if (!window_attn_supported(make_dims(h->cfg, n), h->cfg)) return MADAKV_ERR_UNIMPLEMENTED;
    if (ws_bytes < window_ws_for_call(h->cfg, n)) return MADAKV_ERR_WORKSPACE_TOO_SMALL;
  } else if (ws_bytes < score_ws_for_call(h->cfg, n)) return MADAKV_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const madakv_config& c = h->cfg;
  // The call is cut into up to MAX_GROUPS layer groups: the score sweeps of a group run on the
  // caller's stream, its statistics on the side stream, under the sweeps of the next group.
  int gb[MAX_GROUPS + 1];
  const int ngroups = layer_groups(c, n, gb);
  const bool overlap = ngroups > 1;
  const size_t es = c.dtype == MADAKV_BF16 ? 2 : 4;
  hipError_t e = hipSuccess;
  for (int gi = 0; gi < ngroups && e == hipSuccess; ++gi) {
    const int g0 = gb[gi];
    Dims dg = make_dims(c, gb[gi + 1] - g0);
    const size_t lb = (size_t)g0 * c.batch;                        // (layer, batch) pairs before the group
    const char* qg = static_cast<const char*>(q_win) + lb * c.n_q_heads * c.window * c.head_dim * es;
    const char* kg = static_cast<const char*>(k) + lb * c.n_kv_heads * (size_t)c.ctx_len * c.head_dim * es;
    float* psi_g = psi + lb * c.n_kv_heads * (size_t)c.ctx_len;
    float* pool_g = psi_pool + lb * c.n_kv_heads * (size_t)(c.ctx_len - c.window);
    const float* lse_g = row_lse ? row_lse + lb * c.n_q_heads * c.window : nullptr;
    if (window_attn) {
      const size_t oes = c.out_fp32 ? 4 : es;
      e = launch_window_attn(dg, c, qg, kg, static_cast<const char*>(v) + lb * c.n_kv_heads * (size_t)c.ctx_len * c.head_dim * es,
                             static_cast<char*>(out) + lb * c.n_q_heads * c.window * c.head_dim * oes,
                             lse_out ? lse_out + lb * c.n_q_heads * c.window : nullptr, psi_g, ws, st);
    } else {
      e = launch_score(dg, c, qg, kg, lse_g, psi_g, ws, st);
    }
    hipStream_t ss = st;
    if (overlap && e == hipSuccess) {
      e = hipEventRecord(h->ev_grp[gi], st);
      if (e == hipSuccess) e = hipStreamWaitEvent(h->side, h->ev_grp[gi], 0);
      ss = h->side;
    }
    if (e == hipSuccess)
      e = launch_stats(dg, c, psi_g, mask, pool_g, static_cast<char*>(stats) + lb * c.n_kv_heads * 8 * (size_t)c.n_modalities,
                       g0 == 0 ? n_mod : nullptr, layer0 + g0, ss, h->d_split, h->split_bytes);
  }
  if (overlap) e = join_side(h, st, e);
  return hip_fail(h, e);
}

int32_t madakv_score(madakv_handle* h, int32_t layer0, int32_t n,
                     const void* q_win, const void* k, const uint8_t* mask,
                     float* psi, float* psi_pool, void* stats, int32_t* n_mod,
                     void* ws, size_t ws_bytes, void* stream) {
  return score_impl(h, layer0, n, q_win, k, mask, nullptr, psi, psi_pool, stats, n_mod, ws, ws_bytes, stream);
}

int32_t madakv_score_lse(madakv_handle* h, int32_t layer0, int32_t n,
                         const void* q_win, const void* k, const uint8_t* mask, const float* row_lse,
                         float* psi, float* psi_pool, void* stats, int32_t* n_mod,
                         void* ws, size_t ws_bytes, void* stream) {
  if (row_lse == nullptr || (reinterpret_cast<uintptr_t>(row_lse) & 3u)) return MADAKV_ERR_INVALID_ARG;
  return score_impl(h, layer0, n, q_win, k, mask, row_lse, psi, psi_pool, stats, n_mod, ws, ws_bytes, stream);
}

int32_t madakv_window_attn_workspace_bytes(const madakv_handle* h, int32_t n_layers_per_call, size_t* bytes) {
  if (!h || !bytes || n_layers_per_call < 1 || n_layers_per_call > h->cfg.n_layers) return MADAKV_ERR_INVALID_ARG;
  *bytes = window_ws_for_call(h->cfg, n_layers_per_call);
  return MADAKV_OK;
}

int32_t madakv_window_attn_score(madakv_handle* h, int32_t layer0, int32_t n,
                                 const void* q_win, const void* k, const void* v, const uint8_t* mask,
                                 void* out, float* row_lse,
                                 float* psi, float* psi_pool, void* stats, int32_t* n_mod,
                                 void* ws, size_t ws_bytes, void* stream) {
  if (bad_ptr(v) || bad_ptr(out) || (row_lse && (reinterpret_cast<uintptr_t>(row_lse) & 3u))) return MADAKV_ERR_INVALID_ARG;
  return score_impl(h, layer0, n, q_win, k, mask, nullptr, psi, psi_pool, stats, n_mod, ws, ws_bytes, stream, v, out, row_lse);
}

int32_t madakv_allocate(madakv_handle* h, int32_t layer0, int32_t n,
                        const void* stats, const int32_t* n_mod,
                        int32_t* budgets, void* stream) {
  int32_t r = check_range(h, layer0, n);
  if (r != MADAKV_OK) return r;
  if (bad_ptr(stats, 4) || bad_ptr(n_mod, 4) || bad_ptr(budgets, 4)) return MADAKV_ERR_INVALID_ARG;
  Dims dm = make_dims(h->cfg, n);
  return hip_fail(h, launch_allocate(dm, h->cfg, layer0, stats, n_mod, budgets, h->d_state,
                                     reinterpret_cast<hipStream_t>(stream)));
}

int32_t madakv_select_gather(madakv_handle* h, int32_t layer0, int32_t n,
                             const float* psi_pool, const uint8_t* mask, const int32_t* budgets,
                             const void* k, const void* v,
                             int32_t* kept_idx, int64_t* kv_off, int32_t* kv_len,
                             void* k_c, void* v_c,
                             void* ws, size_t ws_bytes, void* stream) {
  int32_t r = check_range(h, layer0, n);
  if (r != MADAKV_OK) return r;
  const madakv_config& c = h->cfg;
  const bool keep_all = c.budget >= c.ctx_len;
  if (!keep_all && (bad_ptr(psi_pool, 4) || bad_ptr(budgets, 4))) return MADAKV_ERR_INVALID_ARG;
  if (bad_ptr(mask, 1) || bad_ptr(k) || bad_ptr(v) || bad_ptr(kept_idx, 4) || bad_ptr(kv_off, 8) || bad_ptr(kv_len, 4) ||
      bad_ptr(k_c) || bad_ptr(v_c) || bad_ptr(ws)) return MADAKV_ERR_INVALID_ARG;
  Dims dm = make_dims(c, n);
  if (ws_bytes < select_ws_bytes(dm, c)) return MADAKV_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const long long region = region_tokens(c);
  // Layer groups as in madakv_evict when the workspace has room for a slice per group (what
  // madakv_workspace_bytes reports has): segment layout and selection of a group on the side stream beside
  // the gather of the group before, which leaves them room.  One group otherwise.
  int gb[MAX_GROUPS + 1];
  int ngroups = layer_groups(c, n, gb);
  const size_t sel_slice = (select_ws_bytes(make_dims(c, largest_group(c, n)), c) + 255) / 256 * 256;
  if (ngroups > 1 && ws_bytes < sel_slice * ngroups) { ngroups = 1; gb[0] = 0; gb[1] = n; }
  const bool overlap = ngroups > 1;
  const size_t es = c.dtype == MADAKV_BF16 ? 2 : 4;
  const size_t M = (size_t)c.n_modalities;
  hipError_t e = hipSuccess;
  if (overlap) {
    e = hipEventRecord(h->ev_fork, st);
    if (e == hipSuccess) e = hipStreamWaitEvent(h->side, h->ev_fork, 0);
  }
  hipStream_t ss = overlap ? h->side : st;
  for (int gi = 0; gi < ngroups && e == hipSuccess; ++gi) {
    const int g0 = gb[gi], ng = gb[gi + 1] - g0;
    Dims dg = make_dims(c, ng);
    const size_t heads0 = (size_t)g0 * c.batch * c.n_kv_heads;
    char* ws_g = static_cast<char*>(ws) + (overlap ? sel_slice * gi : 0);
    const float* pool_g = psi_pool ? psi_pool + heads0 * (size_t)(c.ctx_len - c.window) : nullptr;
    const int32_t* bud_g = budgets ? budgets + heads0 * M : nullptr;
    const int bpb = blocks_per_batch(c, ng);
    e = launch_offsets(dg, c, layer0 + g0, bud_g, kv_off + heads0, kv_len + heads0, h->d_state + c.batch,
                       h->d_maxlen + (size_t)(layer0 + g0) * c.batch, ws_g, make_paging(h), bpb, ss);
    if (e == hipSuccess) e = launch_select(dg, c, pool_g, mask, bud_g, kv_off + heads0, kv_len + heads0, kept_idx, ss, nullptr, nullptr, h->d_split, h->split_bytes);
    if (overlap && e == hipSuccess) e = hipEventRecord(h->ev_sel[gi], h->side);
    if (overlap && e == hipSuccess) e = hipStreamWaitEvent(st, h->ev_sel[gi], 0);
    const char* kg = static_cast<const char*>(k) + heads0 * (size_t)c.ctx_len * c.head_dim * es;
    const char* vg = static_cast<const char*>(v) + heads0 * (size_t)c.ctx_len * c.head_dim * es;
    if (e == hipSuccess) e = launch_gather(dg, c, 0, ng, kg, vg, kept_idx, kv_off + heads0, kv_len + heads0, k_c, v_c, ws_g, region, bpb, bpb, st, overlap);
  }
  if (overlap && e != hipSuccess) e = join_side(h, st, e);   // an enqueue failed: whatever did reach the side stream is still joined
  for (int l = layer0; l < layer0 + n; ++l) { h->appended[l] = 0; h->gen_base[l] = 0; }
  e = publish_maxlen(h, layer0, n, st, e);
  return hip_fail(h, e);
}

int32_t madakv_evict(madakv_handle* h, int32_t layer0, int32_t n,
                     const void* q_win, const void* k, const void* v, const uint8_t* mask,
                     float* psi, float* psi_pool, void* stats, int32_t* n_mod, int32_t* budgets,
                     int32_t* kept_idx, int64_t* kv_off, int32_t* kv_len, void* k_c, void* v_c,
                     void* score_ws, size_t score_ws_size, void* select_ws, size_t select_ws_size, void* stream) {
  int32_t r = check_range(h, layer0, n);
  if (r != MADAKV_OK) return r;
  const madakv_config& c = h->cfg;
  if (bad_ptr(q_win) || bad_ptr(k) || bad_ptr(v) || bad_ptr(mask, 1) || bad_ptr(psi, 4) || bad_ptr(psi_pool, 4) ||
      bad_ptr(stats, 4) || bad_ptr(n_mod, 4) || bad_ptr(budgets, 4) || bad_ptr(kept_idx, 4) || bad_ptr(kv_off, 8) ||
      bad_ptr(kv_len, 4) || bad_ptr(k_c) || bad_ptr(v_c) || bad_ptr(score_ws) || bad_ptr(select_ws))
    return MADAKV_ERR_INVALID_ARG;
  int gb[MAX_GROUPS + 1];
  const int ngroups = layer_groups(c, n, gb);
  const int gl = largest_group(c, n);
  // every layer group gets its own slice of the selection workspace (its block table is still in
  // use by its gather while the next group's table is being written)
  const size_t sel_slice = (select_ws_bytes(make_dims(c, gl), c) + 255) / 256 * 256;
  if (score_ws_size < score_ws_for_call(c, n) || select_ws_size < sel_slice * ngroups) return MADAKV_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const bool overlap = ngroups > 1;
  const size_t es = c.dtype == MADAKV_BF16 ? 2 : 4;
  const long long region = region_tokens(c);
  const size_t M = (size_t)c.n_modalities;
  hipError_t e = hipSuccess;
  // Caller's stream: sweeps of group 0, sweeps of group 1, gather of group 0, sweeps of group 2, gather
  // of group 1, ..., gather of the last group.  Side stream: statistics, allocation, segment layout and
  // selection of a group as soon as its sweeps are done.  Only group 0's run beside sweeps (which they
  // slow down by about their own duration); the others run beside the gather of the group before.
  auto gather_group = [&](int gi) {
    const int g0 = gb[gi], ng = gb[gi + 1] - g0;
    Dims dg = make_dims(c, ng);
    const size_t heads0 = (size_t)g0 * c.batch * c.n_kv_heads;
    const char* kg = static_cast<const char*>(k) + heads0 * (size_t)c.ctx_len * c.head_dim * es;
    const char* vg = static_cast<const char*>(v) + heads0 * (size_t)c.ctx_len * c.head_dim * es;
    const char* ws_g = static_cast<const char*>(select_ws) + sel_slice * gi;
    if (overlap) e = hipStreamWaitEvent(st, h->ev_sel[gi], 0);
    const int bpb = blocks_per_batch(c, ng);
    if (e == hipSuccess) e = launch_gather(dg, c, 0, ng, kg, vg, kept_idx, kv_off + heads0, kv_len + heads0, k_c, v_c, ws_g, region, bpb, bpb, st, overlap);
  };
  for (int gi = 0; gi < ngroups && e == hipSuccess; ++gi) {
    const int g0 = gb[gi], ng = gb[gi + 1] - g0;
    Dims dg = make_dims(c, ng);
    const size_t lb = (size_t)g0 * c.batch, heads0 = lb * c.n_kv_heads;
    const char* qg = static_cast<const char*>(q_win) + lb * c.n_q_heads * c.window * c.head_dim * es;
    const char* kg = static_cast<const char*>(k) + heads0 * (size_t)c.ctx_len * c.head_dim * es;
    float* psi_g = psi + heads0 * (size_t)c.ctx_len;
    float* pool_g = psi_pool + heads0 * (size_t)(c.ctx_len - c.window);
    char* stats_g = static_cast<char*>(stats) + heads0 * 8 * M;
    int32_t* bud_g = budgets + heads0 * M;
    char* ws_g = static_cast<char*>(select_ws) + sel_slice * gi;
    e = launch_score(dg, c, qg, kg, nullptr, psi_g, score_ws, st);
    hipStream_t ss = st;
    if (overlap && e == hipSuccess) {
      e = hipEventRecord(h->ev_grp[gi], st);
      if (e == hipSuccess) e = hipStreamWaitEvent(h->side, h->ev_grp[gi], 0);
      ss = h->side;
    }
    if (e == hipSuccess) e = launch_stats(dg, c, psi_g, mask, pool_g, stats_g, g0 == 0 ? n_mod : nullptr, layer0 + g0, ss, h->d_split, h->split_bytes);
    if (e == hipSuccess) e = launch_allocate(dg, c, layer0 + g0, stats_g, n_mod, bud_g, h->d_state, ss);
    if (e == hipSuccess) e = launch_offsets(dg, c, layer0 + g0, bud_g, kv_off + heads0, kv_len + heads0, h->d_state + c.batch,
                                            h->d_maxlen + (size_t)(layer0 + g0) * c.batch, ws_g, make_paging(h), blocks_per_batch(c, ng), ss);
    if (e == hipSuccess) e = launch_select(dg, c, pool_g, mask, bud_g, kv_off + heads0, kv_len + heads0, kept_idx, ss, nullptr, nullptr, h->d_split, h->split_bytes);
    if (overlap && e == hipSuccess) e = hipEventRecord(h->ev_sel[gi], h->side);
    // the gather of the group before goes behind this group's sweeps: this group's statistics and
    // selection then run beside a gather, which leaves them room, and not beside the next sweeps
    if (gi >= 1 && e == hipSuccess) gather_group(gi - 1);
  }
  if (e == hipSuccess) gather_group(ngroups - 1);
  if (overlap && e != hipSuccess) e = join_side(h, st, e);   // an enqueue failed: whatever did reach the side stream is still joined
  for (int l = layer0; l < layer0 + n; ++l) { h->appended[l] = 0; h->gen_base[l] = 0; }
  e = publish_maxlen(h, layer0, n, st, e);
  return hip_fail(h, e);
}

int32_t madakv_decode_attn(madakv_handle* h, int32_t layer0, int32_t n,
                           const void* q, const void* k_new, const void* v_new,
                           void* k_c, void* v_c, const int64_t* kv_off, int32_t* kv_len,
                           void* out, void* ws, size_t ws_bytes, void* stream) {
  return decode_impl(h, layer0, n, q, k_new, v_new, k_c, v_c, kv_off, kv_len, out, ws, ws_bytes, false, stream);
}

int32_t madakv_decode_attn_static(madakv_handle* h, int32_t layer0, int32_t n,
                                  const void* q, const void* k_new, const void* v_new,
                                  void* k_c, void* v_c, const int64_t* kv_off, int32_t* kv_len,
                                  void* out, void* stream) {
  if (!h) return MADAKV_ERR_INVALID_ARG;
  // no allocation on this path: this device's copy of the static array is all it uses beyond the caller's tensors
  return decode_impl(h, layer0, n, q, k_new, v_new, k_c, v_c, kv_off, kv_len, out, h->static_scratch, STATIC_SCRATCH_BYTES,
                     true, stream);
}

namespace {
// workspace of madakv_reevict: per-row arrays over the whole reduced cache (rows are addressed as in k_c),
// the per-head records of the call, the exchange array of the scoring kernel
// (paged cache: the per-row arrays cover the linear copy of the heads' rows, which follows them: K, V, the
// original positions, the heads' offsets in the copy; it has as many rows as the cache)
struct ReevictWs { size_t psi, pool, sel, rowmod, stats, score, lin_k, lin_v, lin_idx, lin_off, total; };
ReevictWs reevict_layout(const madakv_handle* h, int n) {
  const madakv_config& c = h->cfg;
  const Dims dm = make_dims(c, n);
  ReevictWs w;
  const size_t cap = (size_t)(region_tokens(c) * c.batch);
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  w.psi = 0; w.pool = up(cap * 4); w.sel = w.pool + up(cap * 4); w.rowmod = w.sel + up(cap * 4);
  w.stats = w.rowmod + up(cap);
  w.score = w.stats + up((size_t)dm.heads * 8 * c.n_modalities);
  w.lin_k = w.score + up(score_ragged_ws_bytes(dm, c, c.ctx_len + c.max_new_tokens, (long long)cap));
  const size_t row_bytes = (size_t)c.head_dim * (c.cache_fp8 ? 1 : (c.dtype == MADAKV_BF16 ? 2 : 4));
  const size_t lin = c.page_rows ? up(cap * row_bytes) : 0;
  w.lin_v = w.lin_k + lin; w.lin_idx = w.lin_v + lin; w.lin_off = w.lin_idx + (c.page_rows ? up(cap * 4) : 0);
  w.total = w.lin_off + (c.page_rows ? up((size_t)dm.heads * 8) : 0);
  return w;
}
}  // namespace

int32_t madakv_reevict_workspace_bytes(const madakv_handle* h, int32_t n_layers_per_call, size_t* bytes) {
  if (!h || !bytes || n_layers_per_call < 1 || n_layers_per_call > h->cfg.n_layers) return MADAKV_ERR_INVALID_ARG;
  *bytes = reevict_layout(h, n_layers_per_call).total;
  return MADAKV_OK;
}

int32_t madakv_reevict(madakv_handle* h, int32_t layer0, int32_t n,
                       const void* q_recent, const uint8_t* mask,
                       void* k_c, void* v_c, int32_t* kept_idx, const int64_t* kv_off, int32_t* kv_len,
                       int32_t* budgets, void* ws, size_t ws_bytes, void* stream) {
  int32_t r = check_range(h, layer0, n);
  if (r != MADAKV_OK) return r;
  const madakv_config& c = h->cfg;
  if (bad_ptr(q_recent) || bad_ptr(mask, 1) || bad_ptr(k_c) || bad_ptr(v_c) || bad_ptr(kept_idx, 4) || bad_ptr(kv_off, 8) ||
      bad_ptr(kv_len, 4) || bad_ptr(budgets, 4) || bad_ptr(ws)) return MADAKV_ERR_INVALID_ARG;
  if (c.budget >= c.ctx_len) return MADAKV_ERR_BAD_BUDGET;                 // nothing was evicted, nothing to bring back
  // a paged cache hands the pages taken since the eviction back to the pools, which all layers share
  if (c.page_rows && (layer0 != 0 || n != c.n_layers)) return MADAKV_ERR_INVALID_ARG;
  int longest = longest_rows(h, layer0, n);
  if (!score_ragged_supported(make_dims(c, n), c, longest)) {
    // the bound may be the worst case only because the lengths of the eviction have not reached the host
    // yet: this call is rare enough to wait for them once
    bool pending = false;
    for (int l = layer0; l < layer0 + n; ++l) pending = pending || h->maxlen_state[l] == 1;
    if (pending && hipEventSynchronize(h->maxlen_event) == hipSuccess) longest = longest_rows(h, layer0, n);
    if (!score_ragged_supported(make_dims(c, n), c, longest)) return MADAKV_ERR_UNIMPLEMENTED;
  }
  const ReevictWs w = reevict_layout(h, n);
  if (ws_bytes < w.total) return MADAKV_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char* wsb = static_cast<char*>(ws);
  float* psi_c = reinterpret_cast<float*>(wsb + w.psi);
  float* pool_c = reinterpret_cast<float*>(wsb + w.pool);
  int32_t* sel = reinterpret_cast<int32_t*>(wsb + w.sel);
  uint8_t* rowmod = reinterpret_cast<uint8_t*>(wsb + w.rowmod);
  const size_t es = c.dtype == MADAKV_BF16 ? 2 : 4;
  hipError_t e = hipSuccess;
  // paged cache: the kernels below work on a linear copy of the call's heads
  void* k_work = k_c; void* v_work = v_c; int32_t* idx_work = kept_idx; const int64_t* off_work = kv_off;
  const long long cache_rows = region_tokens(c) * c.batch;
  if (c.page_rows) {
    k_work = wsb + w.lin_k; v_work = wsb + w.lin_v; idx_work = reinterpret_cast<int32_t*>(wsb + w.lin_idx);
    off_work = reinterpret_cast<const int64_t*>(wsb + w.lin_off);
    e = launch_linear_copy(make_dims(c, n), c, k_c, v_c, kept_idx, kv_off, kv_len, make_paging(h), (long long)layer0 * c.batch * c.n_kv_heads,
                           longest, k_work, v_work, idx_work, reinterpret_cast<int64_t*>(wsb + w.lin_off), false, st);
  }
  // layers that have appended the same number of rows since their last (re-)eviction go in one set of launches
  for (int l0 = layer0; l0 < layer0 + n && e == hipSuccess;) {
    int l1 = l0 + 1;
    while (l1 < layer0 + n && h->appended[l1] == h->appended[l0] && h->gen_base[l1] == h->gen_base[l0]) ++l1;
    const Dims dr = make_dims(c, l1 - l0);
    const size_t heads0 = (size_t)(l0 - layer0) * c.batch * c.n_kv_heads;
    const char* qr = static_cast<const char*>(q_recent) + (size_t)(l0 - layer0) * c.batch * c.n_q_heads * c.window * c.head_dim * es;
    char* stats_r = wsb + w.stats + heads0 * 8 * c.n_modalities;
    int32_t* bud_r = budgets + heads0 * c.n_modalities;
    e = launch_score_ragged(dr, c, qr, k_work, off_work + heads0, kv_len + heads0, longest, cache_rows, psi_c, wsb + w.score, st);
    if (e == hipSuccess) e = launch_restats(dr, c, psi_c, idx_work, mask, off_work + heads0, kv_len + heads0, h->appended[l0], pool_c, rowmod,
                                            stats_r, bud_r, st);
    if (e == hipSuccess) e = launch_select(dr, c, pool_c, mask, bud_r, off_work + heads0, kv_len + heads0, sel, st, kv_len + heads0, rowmod);
    if (e == hipSuccess) e = launch_compact(dr, c, k_work, v_work, idx_work, sel, off_work + heads0, kv_len + heads0, bud_r, h->appended[l0],
                                            h->gen_base[l0], st);
    if (e == hipSuccess) for (int l = l0; l < l1; ++l) { h->gen_base[l] += h->appended[l]; h->appended[l] = 0; }
    l0 = l1;
  }
  if (c.page_rows && e == hipSuccess) {
    // the survivors go back to the heads' initial pages; every page taken since is free again
    e = launch_linear_copy(make_dims(c, n), c, k_c, v_c, kept_idx, kv_off, kv_len, make_paging(h), (long long)layer0 * c.batch * c.n_kv_heads,
                           longest, k_work, v_work, idx_work, reinterpret_cast<int64_t*>(wsb + w.lin_off), true, st);
    if (e == hipSuccess) e = launch_pool_reset(make_paging(h), c.batch, st);
  }
  return hip_fail(h, e);
}

int32_t madakv_page_table(const madakv_handle* h, const int32_t** table, int32_t* entries_per_head) {
  if (!h || !table || !entries_per_head) return MADAKV_ERR_INVALID_ARG;
  *table = h->d_page_tbl;
  *entries_per_head = page_table_entries(h->cfg);
  return MADAKV_OK;
}

}  // extern "C"
