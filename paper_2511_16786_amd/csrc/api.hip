// C ABI: argument validation, workspace layout and dispatch.  No arithmetic of the method lives here.
#include <math.h>

#include "fc_common.h"

using namespace fc;

namespace {

constexpr int64_t kMaxUnits = 32767;   // grid.y / grid.z limits of the launches below

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

fc_status check_desc(const fc_kv_desc* d) {
  if (!d) return FC_EINVAL;
  if (d->batch < 0 || d->layers < 1 || d->kv_heads < 1 || d->n_tokens < 1 || d->head_dim < 1)
    return FC_EINVAL;
  if (d->dtype != FC_F32 && d->dtype != FC_BF16) return FC_EINVAL;
  const int64_t eb = d->dtype == FC_BF16 ? 2 : 4;
  if ((d->head_dim * eb) % 16 != 0) return FC_EINVAL;
  if (d->stride_n < d->head_dim) return FC_EINVAL;
  if (d->stride_l < 0 || d->stride_b < 0 || d->stride_h < 0) return FC_EINVAL;
  if ((d->stride_n * eb) % 16 || (d->stride_h * eb) % 16 || (d->stride_l * eb) % 16 ||
      (d->stride_b * eb) % 16)
    return FC_EINVAL;
  if ((int64_t)d->batch * d->layers * d->kv_heads > kMaxUnits) return FC_EUNSUPPORTED;
  if (d->layers > 1024) return FC_EUNSUPPORTED;
  return FC_OK;
}

// FC_PATH_DENSE / FC_PATH_FFT, or 0 if unsupported
int32_t resolve(const fc_kv_desc& d, int32_t r, int32_t path) {
  const bool dense_ok = d.head_dim <= 256;     // (rows are multiples of 16 bytes; the kernels pad to 64 columns)
  const bool fft_ok = fft_supported(d, r);
  switch (path) {
    case FC_PATH_AUTO: return fft_ok ? FC_PATH_FFT : (dense_ok ? FC_PATH_DENSE : 0);
    case FC_PATH_DENSE: return dense_ok ? FC_PATH_DENSE : 0;
    case FC_PATH_FFT: return fft_ok ? FC_PATH_FFT : 0;
    default: return 0;
  }
}

}  // namespace

extern "C" {

int32_t flashcache_cutoff_r(int32_t n_tokens, double gamma) {
  if (n_tokens < 1) return 0;
  double w = floor(gamma * (double)n_tokens);
  if (!(w >= 0.0)) w = 0.0;                       // also catches NaN
  if (w > (double)n_tokens) w = (double)n_tokens;
  int64_t r = (int64_t)w + 1;
  if (r > n_tokens) r = n_tokens;
  return (int32_t)r;
}

int64_t flashcache_total_budget(int32_t layers, int32_t n_tokens, double rho) {
  if (layers < 1 || n_tokens < 1) return 0;
  const int64_t full = (int64_t)layers * n_tokens;
  double t = floor(rho * (double)layers * (double)n_tokens);
  if (!(t >= (double)layers)) return layers;      // also catches NaN
  if (t > (double)full) return full;
  return (int64_t)t;
}

int32_t flashcache_resolve_path(const fc_kv_desc* desc, int32_t r, int32_t path) {
  if (check_desc(desc) != FC_OK || r < 1 || r > desc->n_tokens) return 0;
  return resolve(*desc, r, path);
}

size_t flashcache_workspace_bytes(const fc_kv_desc* desc, int32_t r, int32_t path) {
  if (check_desc(desc) != FC_OK || r < 1 || r > desc->n_tokens) return 0;
  switch (resolve(*desc, r, path)) {
    case FC_PATH_DENSE: return dense_layout(*desc, r).total;
    case FC_PATH_FFT: return fft_layout(*desc, r).total;
    default: return 0;
  }
}

size_t flashcache_select_workspace_bytes(const fc_kv_desc* desc) {
  (void)desc;
  return 0;
}

fc_status flashcache_prepare(const fc_kv_desc* desc, int32_t r, int32_t path, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
  fc_status st = check_desc(desc);
  if (st != FC_OK) return st;
  if (r < 1 || r > desc->n_tokens) return FC_EINVAL;
  const int32_t p = resolve(*desc, r, path);
  if (!p) return FC_EUNSUPPORTED;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kWsAlign) != 0) return FC_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (p == FC_PATH_DENSE) {
    DenseLayout lay = dense_layout(*desc, r);
    if (workspace_bytes < lay.total) return FC_EWORKSPACE;
    e = dense_prepare(*desc, r, lay, workspace, s);
  } else {
    FftLayout lay = fft_layout(*desc, r);
    if (workspace_bytes < lay.total) return FC_EWORKSPACE;
    e = fft_prepare(*desc, r, lay, workspace, s);
  }
  return e == hipSuccess ? FC_OK : FC_EHIP;
}

fc_status flashcache_workspace_error(const void* workspace, int32_t* flag_out, void* hip_stream) {
  if (!workspace || !flag_out) return FC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  WsHeader h;
  if (hipMemcpyAsync(&h, workspace, sizeof(h), hipMemcpyDeviceToHost, s) != hipSuccess) return FC_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return FC_EHIP;
  *flag_out = (h.magic != kWsMagic) ? 2 : h.error;
  return FC_OK;
}

static fc_status score_common(const void* K, const void* V, const fc_kv_desc* desc, int32_t r, int32_t path,
                              float* scores, double* energy, void* workspace, size_t workspace_bytes,
                              UnitMap um, void* hip_stream) {
  fc_status st = check_desc(desc);
  if (st != FC_OK) return st;
  if (r < 1 || r > desc->n_tokens) return FC_EINVAL;
  const int32_t p = resolve(*desc, r, path);
  if (!p) return FC_EUNSUPPORTED;
  if (desc->batch == 0) return FC_OK;
  if (!K || !V || !scores || !energy) return FC_EINVAL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(scores) || !aligned16(energy)) return FC_EINVAL;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kWsAlign) != 0) return FC_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (p == FC_PATH_DENSE) {
    DenseLayout lay = dense_layout(*desc, r);
    if (workspace_bytes < lay.total) return FC_EWORKSPACE;
    e = dense_score(K, V, *desc, r, lay, scores, energy, workspace, um, s);
  } else {
    FftLayout lay = fft_layout(*desc, r);
    if (workspace_bytes < lay.total) return FC_EWORKSPACE;
    e = fft_score(K, V, *desc, r, lay, scores, energy, workspace, um, s);
  }
  return e == hipSuccess ? FC_OK : FC_EHIP;
}

fc_status flashcache_score(const void* K, const void* V, const fc_kv_desc* desc, int32_t r, int32_t path,
                           float* scores, double* energy, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
  return score_common(K, V, desc, r, path, scores, energy, workspace, workspace_bytes, UnitMap{0, 0, 0},
                      hip_stream);
}

fc_status flashcache_score_layer(const void* K, const void* V, const fc_kv_desc* desc, int32_t layer,
                                 int32_t total_layers, int32_t r, int32_t path, float* scores,
                                 double* energy, void* workspace, size_t workspace_bytes,
                                 void* hip_stream) {
  if (!desc || desc->layers != 1 || total_layers < 1 || layer < 0 || layer >= total_layers) return FC_EINVAL;
  return score_common(K, V, desc, r, path, scores, energy, workspace, workspace_bytes,
                      UnitMap{desc->kv_heads, total_layers, layer}, hip_stream);
}

fc_status flashcache_lowpass_energy(const fc_kv_desc* desc, int32_t r, int32_t path, void* workspace,
                                    size_t workspace_bytes, double* lowpass_energy, void* hip_stream) {
  fc_status st = check_desc(desc);
  if (st != FC_OK) return st;
  if (r < 1 || r > desc->n_tokens) return FC_EINVAL;
  const int32_t p = resolve(*desc, r, path);
  if (!p) return FC_EUNSUPPORTED;
  if (desc->batch == 0) return FC_OK;
  if (!lowpass_energy || (reinterpret_cast<uintptr_t>(lowpass_energy) & 7u)) return FC_EINVAL;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kWsAlign) != 0) return FC_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (p == FC_PATH_DENSE) {
    DenseLayout lay = dense_layout(*desc, r);
    if (workspace_bytes < lay.total) return FC_EWORKSPACE;
    e = dense_lowpass(*desc, lay, workspace, lowpass_energy, s);
  } else {
    FftLayout lay = fft_layout(*desc, r);
    if (workspace_bytes < lay.total) return FC_EWORKSPACE;
    e = fft_lowpass(*desc, r, lay, workspace, lowpass_energy, s);
  }
  return e == hipSuccess ? FC_OK : FC_EHIP;
}

fc_status flashcache_allocate(const double* energy, int32_t batch, int32_t layers, int32_t kv_heads,
                              int32_t n_tokens, int64_t total_budget, int32_t b_min, int32_t b_max,
                              int32_t* budgets, int64_t* layer_offsets, void* hip_stream) {
  if (batch < 0 || layers < 1 || kv_heads < 1 || n_tokens < 1) return FC_EINVAL;
  if (layers > 1024) return FC_EUNSUPPORTED;
  if (b_min < 1 || b_max < b_min || b_max > n_tokens) return FC_EBUDGET;
  if ((int64_t)layers * b_min > total_budget || (int64_t)layers * b_max < total_budget) return FC_EBUDGET;
  if (batch == 0) return FC_OK;
  if (!energy || !budgets || !layer_offsets) return FC_EINVAL;
  if ((reinterpret_cast<uintptr_t>(energy) & 7u) || (reinterpret_cast<uintptr_t>(layer_offsets) & 7u) ||
      (reinterpret_cast<uintptr_t>(budgets) & 3u))
    return FC_EINVAL;
  hipError_t e = allocate_launch(energy, batch, layers, kv_heads, n_tokens, total_budget, b_min, b_max,
                                 budgets, layer_offsets, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FC_OK : FC_EHIP;
}

static fc_status select_gather_common(const void* K, const void* V, const fc_kv_desc* desc,
                                      const float* scores, const int32_t* budgets,
                                      const int64_t* layer_offsets, int64_t rows_per_seq, bool shared,
                                      int32_t* idx_out, void* K_out, void* V_out,
                                      const int32_t* block_table, int32_t page_size, int32_t max_pages,
                                      int64_t num_pages, void* hip_stream) {
  fc_status st = check_desc(desc);
  if (st != FC_OK) return st;
  if (rows_per_seq < 0 || rows_per_seq > (int64_t)desc->layers * desc->kv_heads * desc->n_tokens)
    return FC_EINVAL;
  if (desc->batch == 0 || rows_per_seq == 0) return FC_OK;
  if (!K || !V || !scores || !budgets || !layer_offsets || !idx_out || !K_out || !V_out) return FC_EINVAL;
  if (!aligned16(K) || !aligned16(V) || !aligned16(K_out) || !aligned16(V_out)) return FC_EINVAL;
  if ((reinterpret_cast<uintptr_t>(scores) & 3u) || (reinterpret_cast<uintptr_t>(budgets) & 3u) ||
      (reinterpret_cast<uintptr_t>(idx_out) & 3u) || (reinterpret_cast<uintptr_t>(layer_offsets) & 7u))
    return FC_EINVAL;
  hipError_t e = select_gather_launch(K, V, *desc, scores, budgets, layer_offsets, rows_per_seq, shared,
                                      idx_out, K_out, V_out, block_table, page_size, max_pages, num_pages,
                                      static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FC_OK : FC_EHIP;
}

fc_status flashcache_select_gather(const void* K, const void* V, const fc_kv_desc* desc, const float* scores,
                                   const int32_t* budgets, const int64_t* layer_offsets,
                                   int64_t rows_per_seq, int32_t* idx_out, void* K_out, void* V_out,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  (void)workspace; (void)workspace_bytes;
  return select_gather_common(K, V, desc, scores, budgets, layer_offsets, rows_per_seq, false, idx_out,
                              K_out, V_out, nullptr, 0, 0, 0, hip_stream);
}

fc_status flashcache_select_gather_shared(const void* K, const void* V, const fc_kv_desc* desc,
                                          const float* scores, const int32_t* budgets,
                                          const int64_t* layer_offsets, int64_t rows_per_seq,
                                          int32_t* idx_out, void* K_out, void* V_out, void* workspace,
                                          size_t workspace_bytes, void* hip_stream) {
  (void)workspace; (void)workspace_bytes;
  return select_gather_common(K, V, desc, scores, budgets, layer_offsets, rows_per_seq, true, idx_out,
                              K_out, V_out, nullptr, 0, 0, 0, hip_stream);
}

fc_status flashcache_select_gather_paged(const void* K, const void* V, const fc_kv_desc* desc,
                                         const float* scores, const int32_t* budgets,
                                         const int64_t* layer_offsets, int64_t rows_per_seq, int32_t shared,
                                         int32_t* idx_out, const int32_t* block_table, int32_t page_size,
                                         int32_t max_pages, int64_t num_pages, void* K_cache, void* V_cache,
                                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  (void)workspace; (void)workspace_bytes;
  if (page_size < 1 || max_pages < 1 || num_pages < 1) return FC_EINVAL;
  if (!block_table || (reinterpret_cast<uintptr_t>(block_table) & 3u)) return FC_EINVAL;
  return select_gather_common(K, V, desc, scores, budgets, layer_offsets, rows_per_seq, shared != 0, idx_out,
                              K_cache, V_cache, block_table, page_size, max_pages, num_pages, hip_stream);
}

size_t flashcache_decode_workspace_bytes(int32_t batch, int32_t layers, int32_t kv_heads, int32_t q_heads,
                                         int32_t head_dim) {
  if (batch < 0 || layers < 1 || kv_heads < 1 || q_heads < kv_heads || q_heads % kv_heads) return 0;
  const int group = q_heads / kv_heads;      // the same size serves both storage types
  if (!decode_supported(group, head_dim, FC_BF16) && !decode_supported(group, head_dim, FC_F32)) return 0;
  if ((int64_t)batch * layers * kv_heads > kMaxUnits) return 0;
  return decode_workspace_bytes(batch, layers, kv_heads, q_heads / kv_heads, head_dim);
}

fc_status flashcache_decode_attention(const void* Q, const void* K_cache, const void* V_cache, int32_t batch,
                                      int32_t layers, int32_t kv_heads, int32_t q_heads, int32_t head_dim,
                                      int32_t dtype, const int32_t* budgets, const int64_t* layer_offsets,
                                      int64_t rows_per_seq, float scale, float* out, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  if (batch < 0 || layers < 1 || kv_heads < 1 || q_heads < kv_heads || q_heads % kv_heads || head_dim < 1)
    return FC_EINVAL;
  if (dtype != FC_F32 && dtype != FC_BF16) return FC_EINVAL;
  if (rows_per_seq < 0 || !(scale == scale)) return FC_EINVAL;
  if (!decode_supported(q_heads / kv_heads, head_dim, dtype)) return FC_EUNSUPPORTED;
  if ((int64_t)batch * layers * kv_heads > kMaxUnits) return FC_EUNSUPPORTED;
  if (batch == 0) return FC_OK;
  if (!Q || !K_cache || !V_cache || !budgets || !layer_offsets || !out) return FC_EINVAL;
  if (!aligned16(Q) || !aligned16(K_cache) || !aligned16(V_cache) || !aligned16(out)) return FC_EINVAL;
  if ((reinterpret_cast<uintptr_t>(budgets) & 3u) || (reinterpret_cast<uintptr_t>(layer_offsets) & 7u))
    return FC_EINVAL;
  const size_t need = decode_workspace_bytes(batch, layers, kv_heads, q_heads / kv_heads, head_dim);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < need)
    return FC_EWORKSPACE;
  hipError_t e = decode_launch(Q, K_cache, V_cache, batch, layers, kv_heads, q_heads / kv_heads, head_dim,
                               dtype, budgets, layer_offsets, rows_per_seq, scale, out, workspace, nullptr, 0, 0,
                               0, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FC_OK : FC_EHIP;
}

size_t flashcache_decode_static_scratch_bytes(void) { return decode_static_scratch_bytes(); }

fc_status flashcache_decode_attention_static(const void* Q, const void* K_cache, const void* V_cache,
                                             int32_t batch, int32_t layers, int32_t kv_heads,
                                             int32_t q_heads, int32_t head_dim, int32_t dtype,
                                             const int32_t* budgets, const int64_t* layer_offsets,
                                             int64_t rows_per_seq, float scale, float* out,
                                             void* hip_stream) {
  if (batch < 0 || layers < 1 || kv_heads < 1 || q_heads < kv_heads || q_heads % kv_heads || head_dim < 1)
    return FC_EINVAL;
  if (dtype != FC_F32 && dtype != FC_BF16) return FC_EINVAL;
  if (rows_per_seq < 0 || !(scale == scale)) return FC_EINVAL;
  if (!decode_supported(q_heads / kv_heads, head_dim, dtype)) return FC_EUNSUPPORTED;
  if ((int64_t)batch * layers * kv_heads > kMaxUnits) return FC_EUNSUPPORTED;
  // the partial results must fit the static array: larger problems need the workspace variant
  if (decode_workspace_bytes(batch, layers, kv_heads, q_heads / kv_heads, head_dim) >
      decode_static_scratch_bytes())
    return FC_EWORKSPACE;
  if (batch == 0) return FC_OK;
  if (!Q || !K_cache || !V_cache || !budgets || !layer_offsets || !out) return FC_EINVAL;
  if (!aligned16(Q) || !aligned16(K_cache) || !aligned16(V_cache) || !aligned16(out)) return FC_EINVAL;
  if ((reinterpret_cast<uintptr_t>(budgets) & 3u) || (reinterpret_cast<uintptr_t>(layer_offsets) & 7u))
    return FC_EINVAL;
  void* scratch_ptr = nullptr;
  if (decode_static_scratch(&scratch_ptr) != hipSuccess) return FC_EHIP;
  hipError_t e = decode_launch(Q, K_cache, V_cache, batch, layers, kv_heads, q_heads / kv_heads, head_dim,
                               dtype, budgets, layer_offsets, rows_per_seq, scale, out, scratch_ptr, nullptr, 0,
                               0, 0, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FC_OK : FC_EHIP;
}

fc_status flashcache_decode_attention_paged(const void* Q, const void* K_pages, const void* V_pages,
                                            const int32_t* block_table, int32_t page_size,
                                            int32_t max_pages, int64_t num_pages, int32_t batch,
                                            int32_t layers, int32_t kv_heads, int32_t q_heads,
                                            int32_t head_dim, int32_t dtype, const int32_t* budgets,
                                            float scale, float* out, void* workspace, size_t workspace_bytes,
                                            void* hip_stream) {
  if (batch < 0 || layers < 1 || kv_heads < 1 || q_heads < kv_heads || q_heads % kv_heads || head_dim < 1)
    return FC_EINVAL;
  if (dtype != FC_F32 && dtype != FC_BF16) return FC_EINVAL;
  if (page_size < 1 || max_pages < 1 || num_pages < 1 || !(scale == scale)) return FC_EINVAL;
  if (!decode_supported(q_heads / kv_heads, head_dim, dtype)) return FC_EUNSUPPORTED;
  if ((int64_t)batch * layers * kv_heads > kMaxUnits) return FC_EUNSUPPORTED;
  if (batch == 0) return FC_OK;
  if (!Q || !K_pages || !V_pages || !block_table || !budgets || !out) return FC_EINVAL;
  if (!aligned16(Q) || !aligned16(K_pages) || !aligned16(V_pages) || !aligned16(out)) return FC_EINVAL;
  if ((reinterpret_cast<uintptr_t>(budgets) & 3u) || (reinterpret_cast<uintptr_t>(block_table) & 3u))
    return FC_EINVAL;
  const size_t need = decode_workspace_bytes(batch, layers, kv_heads, q_heads / kv_heads, head_dim);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < need)
    return FC_EWORKSPACE;
  hipError_t e = decode_launch(Q, K_pages, V_pages, batch, layers, kv_heads, q_heads / kv_heads, head_dim,
                               dtype, budgets, nullptr, 0, scale, out, workspace, block_table, page_size,
                               max_pages, num_pages, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FC_OK : FC_EHIP;
}

const char* flashcache_status_string(int32_t status) {
  switch (status) {
    case FC_OK: return "FC_OK";
    case FC_EINVAL: return "FC_EINVAL: invalid argument";
    case FC_EUNSUPPORTED: return "FC_EUNSUPPORTED: no kernel for this request";
    case FC_EWORKSPACE: return "FC_EWORKSPACE: workspace missing, misaligned or too small";
    case FC_EBUDGET: return "FC_EBUDGET: infeasible budget";
    case FC_EHIP: return "FC_EHIP: HIP error";
    default: return "unknown status";
  }
}

}  // extern "C"
