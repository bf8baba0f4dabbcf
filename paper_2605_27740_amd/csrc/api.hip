// C ABI of the library (declared in include/unique.h): host-side validation, workspace carving and
// kernel dispatch. Nothing here allocates device memory or synchronises.
#include "../../include/unique.h"

#include <algorithm>
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "kernels.hpp"

namespace {

thread_local char g_last_error[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
  va_end(ap);
  return code;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(UNIQUE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

constexpr size_t kAlign = 256;
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Validates the host-visible part of the descriptor and fills the kernel-side view.
int make_view(const unique_cache_desc* d, unique::CacheView* v, bool need_stats, bool need_v) {
  if (!d) return fail(UNIQUE_ERR_INVALID_ARG, "desc is NULL");
  if (d->dtype != UNIQUE_DTYPE_F32 && d->dtype != UNIQUE_DTYPE_BF16)
    return fail(UNIQUE_ERR_INVALID_ARG, "dtype %d is neither fp32 (0) nor bf16 (1)", d->dtype);
  if (d->num_q_heads < 1 || d->num_kv_heads < 1 || d->head_dim < 1 || d->page_size < 1 || d->batch < 1 ||
      d->max_pages_per_seq < 1 || d->num_phys_pages < 1 || d->max_seq_len_hint < 0)
    return fail(UNIQUE_ERR_INVALID_ARG, "non-positive dimension in descriptor (H=%d Hkv=%d D=%d S=%d B=%d "
                "max_pages_per_seq=%d num_phys_pages=%lld hint=%d)", d->num_q_heads, d->num_kv_heads, d->head_dim,
                d->page_size, d->batch, d->max_pages_per_seq, (long long)d->num_phys_pages, d->max_seq_len_hint);
  if (d->num_q_heads % d->num_kv_heads != 0)
    return fail(UNIQUE_ERR_INVALID_ARG, "num_q_heads %d is not a multiple of num_kv_heads %d", d->num_q_heads,
                d->num_kv_heads);
  if (d->batch > 65535 || d->num_kv_heads > 65535)
    return fail(UNIQUE_ERR_UNSUPPORTED, "batch and num_kv_heads are limited to 65535 (grid extent)");
  if ((int64_t)d->max_pages_per_seq * d->page_size > (int64_t)INT32_MAX)
    return fail(UNIQUE_ERR_INVALID_ARG, "max_pages_per_seq * page_size overflows int32 token positions");
  if ((int64_t)d->max_pages_per_seq * d->num_kv_heads > (int64_t)INT32_MAX)
    return fail(UNIQUE_ERR_UNSUPPORTED, "max_pages_per_seq * num_kv_heads overflows int32 (page, head) item indices");
  const int G = d->num_q_heads / d->num_kv_heads;
  if (!unique::stats_supported(d->dtype, d->head_dim, d->page_size) ||
      !unique::score_supported(d->dtype, d->head_dim, G, d->num_kv_heads) ||
      !unique::decode_supported(d->dtype, d->head_dim, d->page_size, G))
    return fail(UNIQUE_ERR_UNSUPPORTED, "shape not compiled: dtype=%d head_dim=%d page_size=%d G=%d num_kv_heads=%d "
                "(supported: head_dim 64|128, page_size 8|16|32, G 1|2|4|8, num_kv_heads 1|2|4|8|16|32)",
                d->dtype, d->head_dim, d->page_size, G, d->num_kv_heads);
  if (!d->k_cache || !d->page_table || !d->seq_lens)
    return fail(UNIQUE_ERR_INVALID_ARG, "k_cache, page_table and seq_lens must be non-NULL");
  if (need_v && !d->v_cache) return fail(UNIQUE_ERR_INVALID_ARG, "v_cache is NULL");
  if (need_stats && !d->page_stats) return fail(UNIQUE_ERR_INVALID_ARG, "page_stats must be non-NULL");
  const uintptr_t misaligned = (uintptr_t)d->k_cache | (uintptr_t)d->v_cache;
  if (misaligned & 15u) return fail(UNIQUE_ERR_INVALID_ARG, "k_cache and v_cache must be 16-byte aligned");
  if ((uintptr_t)d->page_stats & 127u) return fail(UNIQUE_ERR_INVALID_ARG, "page_stats must be 128-byte aligned");
  if (d->stats_dtype != UNIQUE_DTYPE_F32 && d->stats_dtype != UNIQUE_DTYPE_BF16)
    return fail(UNIQUE_ERR_INVALID_ARG, "stats_dtype %d is neither fp32 (0) nor bf16 (1)", d->stats_dtype);
  if (d->force_recent_pages < 0) return fail(UNIQUE_ERR_INVALID_ARG, "force_recent_pages must be >= 0");
  if (d->min_seq_len_hint < 0 || (d->max_seq_len_hint > 0 && d->min_seq_len_hint > d->max_seq_len_hint))
    return fail(UNIQUE_ERR_INVALID_ARG, "min_seq_len_hint %d must lie in [0, max_seq_len_hint %d]", d->min_seq_len_hint,
                d->max_seq_len_hint);
  {
    const int64_t tile = (int64_t)d->page_size * d->head_dim;
    const int64_t hs = d->kv_head_stride ? d->kv_head_stride : tile;
    const int64_t ps = d->kv_page_stride ? d->kv_page_stride : (int64_t)d->num_kv_heads * hs;
    const int64_t vec = d->dtype == UNIQUE_DTYPE_BF16 ? 8 : 4;  // elements per 16-byte load
    if (hs < tile || ps < (int64_t)d->num_kv_heads * hs || hs % vec != 0 || ps % vec != 0)
      return fail(UNIQUE_ERR_INVALID_ARG, "kv_head_stride %lld / kv_page_stride %lld: need head stride >= S*D, page "
                  "stride >= H_kv * head stride, both multiples of 16 bytes", (long long)hs, (long long)ps);
  }

  v->k_cache = d->k_cache;
  v->v_cache = d->v_cache;
  v->page_stats = d->page_stats;
  v->page_table = d->page_table;
  v->seq_lens = d->seq_lens;
  v->H = d->num_q_heads;
  v->Hkv = d->num_kv_heads;
  v->D = d->head_dim;
  v->S = d->page_size;
  v->B = d->batch;
  v->max_pages = d->max_pages_per_seq;
  v->num_phys = d->num_phys_pages;
  v->force_recent = d->force_recent_pages;
  v->dtype = d->dtype;
  int hint_pages = d->max_pages_per_seq;
  if (d->max_seq_len_hint > 0) {
    const int64_t hp = ((int64_t)d->max_seq_len_hint + d->page_size - 1) / d->page_size;
    if (hp < hint_pages) hint_pages = (int)hp;
  }
  v->max_pages_hint = hint_pages;
  v->min_pages_hint = (int)std::min<int64_t>(d->min_seq_len_hint / d->page_size, hint_pages);
  v->stats_bf16 = d->stats_dtype == UNIQUE_DTYPE_BF16;
  v->rec_bytes = unique_page_stats_record_bytes(d);
  v->stream_nt = 0;
  const int64_t tile = (int64_t)d->page_size * d->head_dim;
  v->kv_head_stride = d->kv_head_stride ? d->kv_head_stride : tile;
  v->kv_page_stride = d->kv_page_stride ? d->kv_page_stride : (int64_t)d->num_kv_heads * v->kv_head_stride;
  return UNIQUE_OK;
}

int score_stride_of(const unique::CacheView& v) {
  return (int)round_up((size_t)v.max_pages_hint, unique::kScoreStrideAlign);
}
size_t score_bytes(const unique::CacheView& v) {
  return (size_t)v.B * v.Hkv * score_stride_of(v) * sizeof(float);
}
size_t decode_bytes(const unique::CacheView& v, int max_list_len) {
  return unique::decode_partial_floats(v, max_list_len) * sizeof(float);
}


// Scratch of unique_decode_step_static: score rows, then split-K partials, of one call at a time per GPU. In host
// code the array's name only stands for the symbol; its device address is looked up once per device below and
// that pointer is what kernels and everything else get.
static __device__ __align__(256) unsigned char scratch[UNIQUE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // per device: each GPU holds its own copy of the array at its own address

// Device address of `scratch` on the current device (looked up on the first call per device).
int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(UNIQUE_ERR_UNSUPPORTED, "device ordinal %d beyond %d", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p || ((uintptr_t)p % kAlign)) return fail(UNIQUE_ERR_HIP, "static scratch has no usable device address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return UNIQUE_OK;
}

int check_workspace(const void* ws, size_t have, size_t need) {
  if (!ws) return fail(UNIQUE_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", need);
  if ((uintptr_t)ws % kAlign) return fail(UNIQUE_ERR_WORKSPACE, "workspace must be %zu-byte aligned", kAlign);
  if (have < need) return fail(UNIQUE_ERR_WORKSPACE, "workspace too small: %zu bytes given, %zu needed", have, need);
  return UNIQUE_OK;
}

// Host-side validation shared by the two decode-step entry points; *region = bytes of scratch the step needs.
int decode_step_check(const unique_cache_desc* desc, const void* d_q, int32_t top_k, float lambda, float sm_scale,
                      const int32_t* d_sel_pages, const int32_t* d_sel_count, const void* d_out, unique::CacheView* v,
                      size_t* region) {
  const int rc = make_view(desc, v, true, true);
  if (rc != UNIQUE_OK) return rc;
  if (!d_q || !d_sel_pages || !d_sel_count || !d_out)
    return fail(UNIQUE_ERR_INVALID_ARG, "d_q, d_sel_pages, d_sel_count and d_out must be non-NULL");
  if (((uintptr_t)d_q | (uintptr_t)d_out) & 15u)
    return fail(UNIQUE_ERR_INVALID_ARG, "d_q and d_out must be 16-byte aligned");
  if (top_k < 1) return fail(UNIQUE_ERR_INVALID_ARG, "top_k must be >= 1 (got %d)", top_k);
  if (!(lambda >= 0.f)) return fail(UNIQUE_ERR_INVALID_ARG, "lambda must be >= 0");
  if (!(sm_scale == sm_scale)) return fail(UNIQUE_ERR_INVALID_ARG, "sm_scale is NaN");
  // the decode part is planned like unique_sparse_paged_decode with sel_stride = top_k (same chunks, same bits)
  *region = score_bytes(*v);
  if (decode_bytes(*v, top_k) > *region) *region = decode_bytes(*v, top_k);
  return UNIQUE_OK;
}

// Score -> select -> decode on one buffer: the score rows are consumed by the select kernel before the decode
// kernel reuses the buffer for its partials.
int decode_step_launch(const unique::CacheView& v, const void* d_q, int32_t top_k, float lambda, float sm_scale,
                       int32_t refresh_tail, int32_t* d_sel_pages, int32_t* d_sel_count, void* d_out, float* d_lse_out,
                       float* buf, hipStream_t st) {
  const int stride = score_stride_of(v);
  hipError_t e = unique::launch_score(v, d_q, lambda, buf, stride, nullptr, refresh_tail != 0, st);
  if (e != hipSuccess) return hip_fail(e, "page score launch");
  e = unique::launch_select(v, buf, stride, top_k, d_sel_pages, d_sel_count, st);
  if (e != hipSuccess) return hip_fail(e, "top-k select launch");
  e = unique::launch_decode(v, d_q, d_sel_pages, d_sel_count, top_k, top_k, sm_scale, d_out, d_lse_out, buf, st);
  return e == hipSuccess ? UNIQUE_OK : hip_fail(e, "sparse decode launch");
}

}  // namespace

extern "C" {

int unique_workspace_bytes(const unique_cache_desc* desc, int32_t top_k, size_t* out_bytes) {
  if (!out_bytes) return fail(UNIQUE_ERR_INVALID_ARG, "out_bytes is NULL");
  if (top_k < 1) return fail(UNIQUE_ERR_INVALID_ARG, "top_k must be >= 1 (got %d)", top_k);
  unique_cache_desc d;
  if (!desc) return fail(UNIQUE_ERR_INVALID_ARG, "desc is NULL");
  d = *desc;
  // the size depends on dimensions only; pointers are not needed for this query
  alignas(16) static const int dummy[4] = {0, 0, 0, 0};
  if (!d.k_cache) d.k_cache = dummy;
  if (!d.page_table) d.page_table = dummy;
  if (!d.seq_lens) d.seq_lens = dummy;
  d.v_cache = nullptr;
  d.page_stats = nullptr;
  unique::CacheView v;
  const int rc = make_view(&d, &v, false, false);
  if (rc != UNIQUE_OK) return rc;
  // a caller's list for unique_sparse_paged_decode may be up to top_k entries long whatever the sequence lengths
  size_t need = score_bytes(v);
  const size_t sp = decode_bytes(v, top_k), de = decode_bytes(v, v.max_pages_hint);
  if (sp > need) need = sp;
  if (de > need) need = de;
  *out_bytes = round_up(need, kAlign);
  return UNIQUE_OK;
}

int64_t unique_page_stats_record_bytes(const unique_cache_desc* desc) {
  if (!desc) return 0;
  if (desc->stats_dtype != UNIQUE_DTYPE_F32 && desc->stats_dtype != UNIQUE_DTYPE_BF16) return 0;
  const int64_t elem = desc->stats_dtype == UNIQUE_DTYPE_BF16 ? 2 : 4;
  return (int64_t)desc->num_kv_heads * desc->head_dim * elem + unique::kStdBlockBytes;
}

int unique_update_page_stats(const unique_cache_desc* desc, const int32_t* d_tok_begin, const int32_t* d_tok_end,
                             int32_t max_pages_touched_per_seq, void* stream) {
  unique::CacheView v;
  const int rc = make_view(desc, &v, true, false);
  if (rc != UNIQUE_OK) return rc;
  if ((d_tok_begin == nullptr) != (d_tok_end == nullptr))
    return fail(UNIQUE_ERR_INVALID_ARG, "d_tok_begin and d_tok_end must both be NULL or both be set");
  if (d_tok_begin && max_pages_touched_per_seq < 0)
    return fail(UNIQUE_ERR_INVALID_ARG, "max_pages_touched_per_seq must be >= 0 (got %d)", max_pages_touched_per_seq);
  int touched = max_pages_touched_per_seq;
  if (d_tok_begin && touched > v.max_pages) touched = v.max_pages;
  const hipError_t e = unique::launch_stats(v, d_tok_begin, d_tok_end, touched, (hipStream_t)stream);
  return e == hipSuccess ? UNIQUE_OK : hip_fail(e, "page stats launch");
}

int unique_score_select_topk(const unique_cache_desc* desc, const void* d_q, int32_t top_k, float lambda,
                             int32_t* d_sel_pages, int32_t* d_sel_count, float* d_scores_out, void* d_workspace,
                             size_t workspace_bytes, void* stream) {
  unique::CacheView v;
  int rc = make_view(desc, &v, true, false);
  if (rc != UNIQUE_OK) return rc;
  if (!d_q || !d_sel_pages || !d_sel_count)
    return fail(UNIQUE_ERR_INVALID_ARG, "d_q, d_sel_pages and d_sel_count must be non-NULL");
  if ((uintptr_t)d_q & 15u) return fail(UNIQUE_ERR_INVALID_ARG, "d_q must be 16-byte aligned");
  if (top_k < 1) return fail(UNIQUE_ERR_INVALID_ARG, "top_k must be >= 1 (got %d)", top_k);
  if (!(lambda >= 0.f)) return fail(UNIQUE_ERR_INVALID_ARG, "lambda must be >= 0");
  rc = check_workspace(d_workspace, workspace_bytes, score_bytes(v));
  if (rc != UNIQUE_OK) return rc;
  float* scores = reinterpret_cast<float*>(d_workspace);
  const int stride = score_stride_of(v);
  hipError_t e = unique::launch_score(v, d_q, lambda, scores, stride, d_scores_out, false, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "page score launch");
  e = unique::launch_select(v, scores, stride, top_k, d_sel_pages, d_sel_count, (hipStream_t)stream);
  return e == hipSuccess ? UNIQUE_OK : hip_fail(e, "top-k select launch");
}

int unique_page_scores(const unique_cache_desc* desc, const void* d_q, float lambda, float* d_scores,
                       int32_t score_stride, void* stream) {
  unique::CacheView v;
  const int rc = make_view(desc, &v, true, false);
  if (rc != UNIQUE_OK) return rc;
  if (!d_q || !d_scores) return fail(UNIQUE_ERR_INVALID_ARG, "d_q and d_scores must be non-NULL");
  if (((uintptr_t)d_q | (uintptr_t)d_scores) & 15u)
    return fail(UNIQUE_ERR_INVALID_ARG, "d_q and d_scores must be 16-byte aligned");
  if (!(lambda >= 0.f)) return fail(UNIQUE_ERR_INVALID_ARG, "lambda must be >= 0");
  if (score_stride < v.max_pages_hint || score_stride % 4 != 0)
    return fail(UNIQUE_ERR_INVALID_ARG, "score_stride %d must be a multiple of 4 and >= %d pages", score_stride,
                v.max_pages_hint);
  const hipError_t e = unique::launch_score(v, d_q, lambda, d_scores, score_stride, nullptr, false, (hipStream_t)stream);
  return e == hipSuccess ? UNIQUE_OK : hip_fail(e, "page score launch");
}

int unique_select_topk(const unique_cache_desc* desc, const float* d_scores, int32_t score_stride, int32_t top_k,
                       int32_t* d_sel_pages, int32_t* d_sel_count, void* stream) {
  unique::CacheView v;
  const int rc = make_view(desc, &v, false, false);
  if (rc != UNIQUE_OK) return rc;
  if (!d_scores || !d_sel_pages || !d_sel_count)
    return fail(UNIQUE_ERR_INVALID_ARG, "d_scores, d_sel_pages and d_sel_count must be non-NULL");
  if ((uintptr_t)d_scores & 15u) return fail(UNIQUE_ERR_INVALID_ARG, "d_scores must be 16-byte aligned");
  if (top_k < 1) return fail(UNIQUE_ERR_INVALID_ARG, "top_k must be >= 1 (got %d)", top_k);
  if (score_stride < v.max_pages_hint || score_stride % 4 != 0)
    return fail(UNIQUE_ERR_INVALID_ARG, "score_stride %d must be a multiple of 4 and >= %d pages", score_stride,
                v.max_pages_hint);
  const hipError_t e = unique::launch_select(v, d_scores, score_stride, top_k, d_sel_pages, d_sel_count,
                                             (hipStream_t)stream);
  return e == hipSuccess ? UNIQUE_OK : hip_fail(e, "top-k select launch");
}

int unique_sparse_paged_decode(const unique_cache_desc* desc, const void* d_q, const int32_t* d_sel_pages,
                               const int32_t* d_sel_count, int32_t sel_stride, float sm_scale, void* d_out,
                               float* d_lse_out, void* d_workspace, size_t workspace_bytes, void* stream) {
  unique::CacheView v;
  int rc = make_view(desc, &v, false, true);
  if (rc != UNIQUE_OK) return rc;
  if (!d_q || !d_out || !d_sel_pages || !d_sel_count)
    return fail(UNIQUE_ERR_INVALID_ARG, "d_q, d_out, d_sel_pages and d_sel_count must be non-NULL");
  if (((uintptr_t)d_q | (uintptr_t)d_out) & 15u)
    return fail(UNIQUE_ERR_INVALID_ARG, "d_q and d_out must be 16-byte aligned");
  if (sel_stride < 1) return fail(UNIQUE_ERR_INVALID_ARG, "sel_stride must be >= 1 (got %d)", sel_stride);
  if (!(sm_scale == sm_scale)) return fail(UNIQUE_ERR_INVALID_ARG, "sm_scale is NaN");
  // the split plan covers every entry a row may hold (sel_count <= sel_stride), also when the list is longer than
  // the sequences have pages (padding or foreign entries in between are skipped, valid ones behind them are not lost)
  const int list_len = sel_stride;
  rc = check_workspace(d_workspace, workspace_bytes, decode_bytes(v, list_len));
  if (rc != UNIQUE_OK) return rc;
  const hipError_t e = unique::launch_decode(v, d_q, d_sel_pages, d_sel_count, sel_stride, list_len, sm_scale, d_out,
                                             d_lse_out, reinterpret_cast<float*>(d_workspace), (hipStream_t)stream);
  return e == hipSuccess ? UNIQUE_OK : hip_fail(e, "sparse decode launch");
}

int unique_decode_step(const unique_cache_desc* desc, const void* d_q, int32_t top_k, float lambda, float sm_scale,
                       int32_t refresh_tail, int32_t* d_sel_pages, int32_t* d_sel_count, void* d_out,
                       float* d_lse_out, void* d_workspace, size_t workspace_bytes, void* stream) {
  unique::CacheView v;
  size_t region = 0;
  int rc = decode_step_check(desc, d_q, top_k, lambda, sm_scale, d_sel_pages, d_sel_count, d_out, &v, &region);
  if (rc != UNIQUE_OK) return rc;
  rc = check_workspace(d_workspace, workspace_bytes, region);
  if (rc != UNIQUE_OK) return rc;
  return decode_step_launch(v, d_q, top_k, lambda, sm_scale, refresh_tail, d_sel_pages, d_sel_count, d_out, d_lse_out,
                            reinterpret_cast<float*>(d_workspace), (hipStream_t)stream);
}

int unique_decode_step_static(const unique_cache_desc* desc, const void* d_q, int32_t top_k, float lambda,
                              float sm_scale, int32_t refresh_tail, int32_t* d_sel_pages, int32_t* d_sel_count,
                              void* d_out, float* d_lse_out, void* stream) {
  unique::CacheView v;
  size_t region = 0;
  int rc = decode_step_check(desc, d_q, top_k, lambda, sm_scale, d_sel_pages, d_sel_count, d_out, &v, &region);
  if (rc != UNIQUE_OK) return rc;
  if (region > (size_t)UNIQUE_STATIC_SCRATCH_BYTES)
    return fail(UNIQUE_ERR_WORKSPACE, "this step needs %zu bytes of scratch, the built-in scratch holds %zu: use "
                "unique_decode_step with a caller workspace", region, (size_t)UNIQUE_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != UNIQUE_OK) return rc;
  return decode_step_launch(v, d_q, top_k, lambda, sm_scale, refresh_tail, d_sel_pages, d_sel_count, d_out, d_lse_out,
                            reinterpret_cast<float*>(ws), (hipStream_t)stream);
}

int unique_dense_paged_decode(const unique_cache_desc* desc, const void* d_q, float sm_scale, void* d_out,
                              float* d_lse_out, void* d_workspace, size_t workspace_bytes, void* stream) {
  unique::CacheView v;
  int rc = make_view(desc, &v, false, true);
  if (rc != UNIQUE_OK) return rc;
  if (!d_q || !d_out) return fail(UNIQUE_ERR_INVALID_ARG, "d_q and d_out must be non-NULL");
  if (((uintptr_t)d_q | (uintptr_t)d_out) & 15u)
    return fail(UNIQUE_ERR_INVALID_ARG, "d_q and d_out must be 16-byte aligned");
  if (!(sm_scale == sm_scale)) return fail(UNIQUE_ERR_INVALID_ARG, "sm_scale is NaN");
  rc = check_workspace(d_workspace, workspace_bytes, decode_bytes(v, v.max_pages_hint));
  if (rc != UNIQUE_OK) return rc;
  const hipError_t e = unique::launch_decode(v, d_q, nullptr, nullptr, v.max_pages_hint, v.max_pages_hint, sm_scale,
                                             d_out, d_lse_out, reinterpret_cast<float*>(d_workspace),
                                             (hipStream_t)stream);
  return e == hipSuccess ? UNIQUE_OK : hip_fail(e, "dense decode launch");
}

const char* unique_status_string(int status) {
  switch (status) {
    case UNIQUE_OK: return "ok";
    case UNIQUE_ERR_INVALID_ARG: return "invalid argument";
    case UNIQUE_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case UNIQUE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case UNIQUE_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}

const char* unique_last_error(void) { return g_last_error; }

const char* unique_version(void) { return "unique-gfx950 0.1"; }

}  // extern "C"
