// Internal launch interface between the C ABI (api.hip) and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace unique {

// Device pointers and dimensions of the paged cache, passed by value to every kernel.
struct CacheView {
  const void* k_cache;        // [num_phys][Hkv][S][D]
  const void* v_cache;
  void* page_stats;           // [num_phys] records: Hkv*D means (fp32 or bf16), Hkv fp32 stds, pad to kStdBlockBytes
  const int32_t* page_table;  // [B][max_pages]
  const int32_t* seq_lens;    // [B]
  int32_t H, Hkv, D, S, B, max_pages;
  int64_t num_phys;
  int32_t dtype;              // 0 fp32, 1 bf16
  int32_t max_pages_hint;     // host bound on pages of any sequence (<= max_pages)
  int32_t min_pages_hint;     // host lower bound on full pages of every sequence (0: unknown); sizes tiles only
  int32_t stats_bf16;         // 1: means stored as bf16, 0: fp32
  int64_t rec_bytes;          // bytes per page record of page_stats
  int32_t stream_nt;          // set per launch: read the streamed operand with non-temporal loads
  int64_t kv_page_stride;     // elements between consecutive physical pages of k_cache (and of v_cache)
  int64_t kv_head_stride;     // elements between consecutive KV heads inside a page
  int32_t force_recent;       // the last this-many logical pages of a sequence are always selected (0: none)
};

// Launches that stream more than this many bytes bypass cache allocation (the Infinity Cache holds 256 MB).
constexpr int64_t kStreamNtBytes = 96ll << 20;

// How a decode launch is cut into split-K chunks; computed on the host from bounds only.
struct SplitPlan {
  int32_t pages_per_split;  // list entries handled by one workgroup
  int32_t num_splits;       // grid extent along the split axis (upper bound for every row)
};
SplitPlan plan_splits(int rows, int max_list_len);

constexpr int kStdBlockBytes = 128;     // bytes reserved after the means of a page record (fp32 stds + pad)
constexpr int kScoreStrideAlign = 64;  // score rows in the workspace are padded to this many floats

bool stats_supported(int dtype, int D, int S);
bool score_supported(int dtype, int D, int G, int Hkv);
bool decode_supported(int dtype, int D, int S, int G);

hipError_t launch_stats(const CacheView& c, const int32_t* d_tok_begin, const int32_t* d_tok_end,
                        int max_pages_touched, hipStream_t stream);

// refresh_tail: the workgroup that scores the last page of a sequence first recomputes that page's
// statistics from the keys (the same arithmetic as launch_stats) and stores them.
hipError_t launch_score(const CacheView& c, const void* d_q, float lambda, float* d_scores, int score_stride,
                        float* d_scores_out, bool refresh_tail, hipStream_t stream);

hipError_t launch_select(const CacheView& c, const float* d_scores, int score_stride, int top_k,
                         int32_t* d_sel_pages, int32_t* d_sel_count, hipStream_t stream);

// d_sel_pages == nullptr: attend every page of each sequence (dense).
hipError_t launch_decode(const CacheView& c, const void* d_q, const int32_t* d_sel_pages,
                         const int32_t* d_sel_count, int sel_stride, int max_list_len, float sm_scale,
                         void* d_out, float* d_lse_out, float* d_partials, hipStream_t stream);

// floats of split-K partial storage needed for a list of at most max_list_len pages per row
size_t decode_partial_floats(const CacheView& c, int max_list_len);

}  // namespace unique
