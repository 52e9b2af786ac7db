// C ABI of the MadaKV hot path: argument validation, the handle, and the order in which
// the kernels of each call are enqueued.  No arithmetic of the method lives here.
#include "common.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

using namespace madakv;

struct madakv_handle {
  madakv_config cfg;
  int device;
  int32_t last_hip_error;
  long long* d_state;              // [2 * B]: HCC pool per batch item, cache cursor per batch item
  std::vector<int32_t> appended;   // decode rows appended so far, per layer
  // Longest head of each layer after eviction: written by the device, copied to pinned host
  // memory asynchronously; decode sizes its grid from it once the copy is known to have landed
  // (event query, never a wait) and from the worst case before that.
  int32_t* d_maxlen;
  int32_t* h_maxlen;
  hipEvent_t maxlen_event;
  bool maxlen_pending;
  int sel_layers_done;             // layers [0, sel_layers_done) have been through select_gather in this pass
};

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

long long region_tokens(const madakv_config& c) {
  return (long long)c.n_layers * c.n_kv_heads * ((long long)std::min(c.budget, c.ctx_len) + c.max_new_tokens);
}

int blocks_per_batch(const madakv_config& c, int n) {
  long long per_call = (long long)n * c.n_kv_heads * ((long long)c.ctx_len + c.max_new_tokens);
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
  if (c.pool_k < 1 || c.pool_k > 63 || (c.pool_k & 1) == 0) return MADAKV_ERR_BAD_SHAPE;
  if (c.budget < 1 || (c.budget < c.ctx_len && c.budget <= c.window)) return MADAKV_ERR_BAD_BUDGET;
  if (c.hcc_rho < 1 || c.hcc_rho > 1024) return MADAKV_ERR_INVALID_ARG;
  if (!(c.theta > 0.f) || c.theta > 1.f) return MADAKV_ERR_INVALID_ARG;
  if (c.softmax_scale < 0.f || c.max_new_tokens < 0) return MADAKV_ERR_INVALID_ARG;
  if ((c.mpa_mode | 1) != 1 || (c.hcc_mode | 1) != 1 || (c.out_fp32 | 1) != 1) return MADAKV_ERR_INVALID_ARG;
  return MADAKV_OK;
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
  h->maxlen_pending = false; h->sel_layers_done = 0;
  h->appended.assign(cfg->n_layers, 0);
  hipError_t e = hipGetDevice(&h->device);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&h->d_state), sizeof(long long) * 2 * cfg->batch);
  if (e == hipSuccess) e = hipMemset(h->d_state, 0, sizeof(long long) * 2 * cfg->batch);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&h->d_maxlen), sizeof(int32_t) * cfg->n_layers);
  if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&h->h_maxlen), sizeof(int32_t) * cfg->n_layers, hipHostMallocDefault);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&h->maxlen_event, hipEventDisableTiming);
  if (e != hipSuccess) {
    if (h->d_maxlen) (void)hipFree(h->d_maxlen);
    if (h->h_maxlen) (void)hipHostFree(h->h_maxlen);
    if (h->maxlen_event) (void)hipEventDestroy(h->maxlen_event);
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
  (void)hipHostFree(h->h_maxlen);
  (void)hipEventDestroy(h->maxlen_event);
  delete h;
  return e == hipSuccess ? MADAKV_OK : MADAKV_ERR_HIP;
}

int32_t madakv_last_hip_error(const madakv_handle* h) { return h ? h->last_hip_error : 0; }

int32_t madakv_workspace_bytes(const madakv_handle* h, int32_t n_layers_per_call,
                               size_t* score_ws, size_t* select_ws, size_t* decode_ws) {
  if (!h || n_layers_per_call < 1 || n_layers_per_call > h->cfg.n_layers) return MADAKV_ERR_INVALID_ARG;
  Dims dm = make_dims(h->cfg, n_layers_per_call);
  if (score_ws) *score_ws = score_ws_bytes(dm, h->cfg.dtype);
  if (select_ws) *select_ws = select_ws_bytes(dm, h->cfg);
  if (decode_ws) *decode_ws = decode_ws_bytes(dm, h->cfg);
  return MADAKV_OK;
}

int32_t madakv_compact_capacity_tokens(const madakv_handle* h, int64_t* tokens) {
  if (!h || !tokens) return MADAKV_ERR_INVALID_ARG;
  *tokens = region_tokens(h->cfg) * h->cfg.batch;
  return MADAKV_OK;
}

int32_t madakv_score(madakv_handle* h, int32_t layer0, int32_t n,
                     const void* q_win, const void* k, const uint8_t* mask,
                     float* psi, float* psi_pool, madakv_head_stats* stats, int32_t* n_mod,
                     void* ws, size_t ws_bytes, void* stream) {
  int32_t r = check_range(h, layer0, n);
  if (r != MADAKV_OK) return r;
  if (bad_ptr(q_win) || bad_ptr(k) || bad_ptr(mask, 1) || bad_ptr(psi, 4) || bad_ptr(psi_pool, 4) || bad_ptr(stats, 4) ||
      bad_ptr(n_mod, 4) || bad_ptr(ws)) return MADAKV_ERR_INVALID_ARG;
  Dims dm = make_dims(h->cfg, n);
  if (ws_bytes < score_ws_bytes(dm, h->cfg.dtype)) return MADAKV_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipError_t e = launch_score(dm, h->cfg, q_win, k, psi, ws, st);
  if (e == hipSuccess) e = launch_stats(dm, h->cfg, psi, mask, psi_pool, stats, n_mod, layer0, st);
  return hip_fail(h, e);
}

int32_t madakv_allocate(madakv_handle* h, int32_t layer0, int32_t n,
                        const madakv_head_stats* stats, const int32_t* n_mod,
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
  const int bpb = blocks_per_batch(c, n);
  hipError_t e = launch_offsets(dm, c, layer0, budgets, kv_off, kv_len, h->d_state + c.batch, h->d_maxlen + layer0, ws, region, bpb, st);
  if (e == hipSuccess) e = launch_select(dm, c, psi_pool, mask, budgets, kv_off, kv_len, kept_idx, st);
  if (e == hipSuccess) e = launch_gather(dm, c, k, v, kept_idx, kv_off, kv_len, k_c, v_c, ws, region, bpb, st);
  for (int l = layer0; l < layer0 + n; ++l) h->appended[l] = 0;
  // hand the per-layer longest length to the host without waiting for it
  if (e == hipSuccess) e = hipMemcpyAsync(h->h_maxlen + layer0, h->d_maxlen + layer0, sizeof(int32_t) * n, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipEventRecord(h->maxlen_event, st);
  h->sel_layers_done = (e == hipSuccess) ? layer0 + n : 0;
  h->maxlen_pending = true;
  return hip_fail(h, e);
}

int32_t madakv_decode_attn(madakv_handle* h, int32_t layer0, int32_t n,
                           const void* q, const void* k_new, const void* v_new,
                           void* k_c, void* v_c, const int64_t* kv_off, int32_t* kv_len,
                           void* out, void* ws, size_t ws_bytes, void* stream) {
  int32_t r = check_range(h, layer0, n);
  if (r != MADAKV_OK) return r;
  if (bad_ptr(q) || bad_ptr(k_c) || bad_ptr(v_c) || bad_ptr(kv_off, 8) || bad_ptr(kv_len, 4) || bad_ptr(out) || bad_ptr(ws))
    return MADAKV_ERR_INVALID_ARG;
  if ((k_new == nullptr) != (v_new == nullptr)) return MADAKV_ERR_INVALID_ARG;
  if (k_new && (!aligned16(k_new) || !aligned16(v_new))) return MADAKV_ERR_INVALID_ARG;
  Dims dm = make_dims(h->cfg, n);
  if (ws_bytes < decode_ws_bytes(dm, h->cfg)) return MADAKV_ERR_WORKSPACE_TOO_SMALL;
  if (k_new) {
    for (int l = layer0; l < layer0 + n; ++l)
      if (h->appended[l] >= h->cfg.max_new_tokens) return MADAKV_ERR_INVALID_ARG;
  }
  // upper bound on the rows of any head in the call (after this call's append)
  int longest = h->cfg.ctx_len + h->cfg.max_new_tokens;
  if (h->maxlen_pending && hipEventQuery(h->maxlen_event) == hipSuccess) h->maxlen_pending = false;
  if (!h->maxlen_pending && layer0 + n <= h->sel_layers_done) {
    int mx = 0;
    for (int l = layer0; l < layer0 + n; ++l) mx = std::max(mx, h->h_maxlen[l] + h->appended[l] + 1);
    longest = std::min(longest, mx);
  }
  hipError_t e = launch_decode(dm, h->cfg, q, k_new, v_new, k_c, v_c, kv_off, kv_len, out, ws,
                               region_tokens(h->cfg) * h->cfg.batch, longest,
                               reinterpret_cast<hipStream_t>(stream));
  if (e == hipSuccess && k_new) for (int l = layer0; l < layer0 + n; ++l) h->appended[l] += 1;
  return hip_fail(h, e);
}

}  // extern "C"
