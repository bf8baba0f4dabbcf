/*
 * unique.h -- C ABI of the MI355X (gfx950) library for UNIQUE decode-time top-k sparse attention.
 *
 * The four compute calls follow the paper's statement of the decode step
 * (Section 3.1 and Section 3.2): per-page key statistics (Eq. 1, Eq. 2), the page
 * score (Eq. 3 / its GQA form Eq. 6) with per-(sequence, KV head) top-k page
 * selection, sparse paged attention over the selected pages (Eq. 5), and dense
 * paged attention (Eq. 4) as the in-library comparison point.
 *
 * Conventions
 *   - Every pointer whose name starts with d_ (and every pointer inside
 *     unique_cache_desc) is DEVICE memory owned by the caller. The library never
 *     allocates, frees or keeps device memory and has no global state.
 *   - Every call only enqueues kernels on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and returns without synchronising. Buffers must stay
 *     alive, and must not be written by the caller, until the stream has reached
 *     that point. Nothing else happens on the stream (no allocation, memset, copy or wait), so
 *     a sequence of calls may be captured into a HIP graph and replayed; grid sizes come from
 *     the host-visible bounds in the descriptor, the device arrays are read at replay time.
 *   - Return value: UNIQUE_OK or an error code; unique_last_error() gives a
 *     thread-local description of the last failure. Host-visible arguments are
 *     validated before anything touches the device. The CONTENTS of device arrays
 *     (page ids within the pool, seq_lens within capacity) are the caller's
 *     contract; kernels skip list entries that are out of range instead of
 *     dereferencing them, but do not report them.
 *   - Inputs are assumed finite. A NaN score ranks below every number.
 *
 * Memory layout (row-major, innermost last)
 *   k_cache, v_cache : [num_phys_pages][num_kv_heads][page_size][head_dim]   dtype
 *                      (page and head strides may be widened, see kv_page_stride / kv_head_stride)
 *   page_stats       : one record per physical page, unique_page_stats_record_bytes(desc) bytes each:
 *                      the mean vectors of its KV heads (head h at elements [h*D, (h+1)*D), element type
 *                      float for stats_dtype fp32, bf16 for stats_dtype bf16), then the scalar stds as
 *                      float (head h at float index h after the means), padded by a 128-byte block, so
 *                      that a page's statistics are one contiguous, 128-byte-aligned run:
 *                      record bytes = num_kv_heads*D*sizeof(mean element) + 128. Pad bytes are never
 *                      read or written. The base pointer must be 128-byte aligned.
 *   page_table       : [batch][max_pages_per_seq]  int32, logical page -> physical page
 *   seq_lens         : [batch] int32, tokens cached per sequence INCLUDING the token being
 *                      decoded (the caller appends k_t, v_t first). 0 is tolerated: nothing of that
 *                      sequence is read or refreshed, its rows select nothing (count 0) and its
 *                      output rows are zero with lse = -inf
 *   q, out           : [batch][num_q_heads][head_dim] dtype; query head h uses KV head
 *                      h / (num_q_heads / num_kv_heads)
 *   Logical page p of sequence b holds tokens [p*S, min((p+1)*S, seq_lens[b])); only the
 *   last page may be partial. Slots beyond seq_lens[b] are never read.
 *
 * Supported shapes: dtype fp32 or bf16; head_dim 64 or 128; page_size 8, 16 or 32;
 * group size G = num_q_heads / num_kv_heads in {1, 2, 4, 8}; num_kv_heads in {1, 2, 4, 8, 16, 32}.
 * Anything else returns UNIQUE_ERR_UNSUPPORTED.
 */
#ifndef UNIQUE_H_
#define UNIQUE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  UNIQUE_OK = 0,
  UNIQUE_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, inconsistent dims */
  UNIQUE_ERR_UNSUPPORTED = 2, /* (dtype, head_dim, page_size, G, num_kv_heads) not compiled */
  UNIQUE_ERR_WORKSPACE = 3,   /* workspace missing, misaligned (needs 256 B) or too small */
  UNIQUE_ERR_HIP = 4          /* a kernel launch failed (hipGetLastError) */
};

enum { UNIQUE_DTYPE_F32 = 0, UNIQUE_DTYPE_BF16 = 1 };

typedef struct unique_cache_desc {
  int32_t dtype;             /* UNIQUE_DTYPE_*: element type of q, k_cache, v_cache, out */
  int32_t num_q_heads;       /* H */
  int32_t num_kv_heads;      /* H_kv */
  int32_t head_dim;          /* D */
  int32_t page_size;         /* S */
  int32_t batch;             /* B */
  int32_t max_pages_per_seq; /* row stride of page_table; upper bound on pages of any sequence */
  int32_t max_seq_len_hint;  /* host upper bound on seq_lens[] used to size grids; 0 = max_pages_per_seq*S */
  int64_t num_phys_pages;    /* pages in the pool */
  const void* k_cache;       /* device */
  const void* v_cache;       /* device */
  void* page_stats;          /* device, written by unique_update_page_stats, read by unique_score_select_topk */
  const int32_t* page_table; /* device */
  const int32_t* seq_lens;   /* device */
  int32_t stats_dtype;       /* UNIQUE_DTYPE_F32: means kept in fp32 (selection equals an exact ranking of
                                fp32 scores). UNIQUE_DTYPE_BF16: means rounded to bf16 (the paper's storage
                                format, half the bytes of the score stage); scores and selection are then exact
                                with respect to the STORED statistics. The std is fp32 in both. */
  int32_t force_recent_pages; /* >= 0. n > 0: the last min(n, k, P) logical pages of every sequence are always part of
                                the selection (they take the places of the lowest-ranked of the k); the other
                                places go to the best-scoring remaining pages. 0 = the paper's method, which
                                needs no local window (Section 4.3, long-form speech recognition). A serving safety option, not from the paper. */
  int64_t kv_page_stride;    /* elements between consecutive physical pages of k_cache (the same for v_cache);
                                0 = H_kv*S*D (pages packed) */
  int64_t kv_head_stride;    /* elements between consecutive KV heads inside a page; 0 = S*D (heads packed).
                                The S*D elements of one (page, head) are always contiguous. Setting
                                v_cache = k_cache + S*D, kv_head_stride = 2*S*D and kv_page_stride = H_kv*2*S*D
                                describes a cache that keeps the K and V tiles of a (page, head) side by side. */
  int32_t min_seq_len_hint;  /* host LOWER bound on seq_lens[]; 0 = unknown. A performance hint only: a batch whose
                                sequences are all known to be long lets the page-score launch give each workgroup
                                more pages (fewer prologues) without the risk of starving compute units on a
                                ragged batch. Results never depend on it. Must not exceed max_seq_len_hint when
                                both are given. */
  int32_t reserved0;         /* 0 */
} unique_cache_desc;

/* Bytes of device workspace that any of the calls below may need for this descriptor and top_k
 * (score rows, split-K partial results). Pass a buffer at least this large, 256-byte aligned.
 * The contents need no initialisation and carry nothing between calls; calls that may overlap in time
 * (different streams) need a workspace each. */
int unique_workspace_bytes(const unique_cache_desc* desc, int32_t top_k, size_t* out_bytes);

/* Bytes per page record of page_stats for this descriptor (see the layout above); 0 if desc is NULL or
 * its stats_dtype is not one of the two. */
int64_t unique_page_stats_record_bytes(const unique_cache_desc* desc);

/* Page statistics, Eq. 1 (mean over the page's keys, per dimension) and Eq. 2 (per-dimension
 * population standard deviation collapsed by its l2 norm into one scalar), recomputed from the
 * keys in the cache for every logical page of sequence b that overlaps the token range
 * [d_tok_begin[b], d_tok_end[b]) (clamped to [0, seq_lens[b])), for every KV head. A partial last
 * page uses its valid tokens only. Results go to the page's record in page_stats (PHYSICAL page index).
 *   d_tok_begin, d_tok_end : device int32 [batch], or both NULL = every page of every sequence.
 *   max_pages_touched_per_seq : host upper bound on pages overlapped per sequence (sizes the grid;
 *                               pages beyond it are NOT refreshed); ignored when the ranges are NULL.
 * An empty range refreshes nothing for that sequence. */
int unique_update_page_stats(const unique_cache_desc* desc, const int32_t* d_tok_begin,
                             const int32_t* d_tok_end, int32_t max_pages_touched_per_seq, void* stream);

/* Page scores by Eq. 6 (Eq. 3 when G = 1), score(p) = max_g [ q_g . mean_p + lambda |q_g|_2 std_p ]
 * over the logical pages of each sequence from the cached statistics, then the top-k page set of
 * each (sequence, KV head) (Section 3.2, radix selection; ties go to the lower logical page).
 *   d_q          : [batch][H][D] dtype.
 *   top_k >= 1   : pages to keep; each row keeps k_b = min(top_k, pages of the sequence). No page
 *                  is kept unconditionally unless desc->force_recent_pages asks for it.
 *   lambda >= 0  : weight of the standard-deviation offset (0.5 in the paper).
 *   d_sel_pages  : out, int32 [batch][H_kv][top_k], LOGICAL page indices in ascending order,
 *                  entries at and beyond k_b are -1.
 *   d_sel_count  : out, int32 [batch][H_kv] = k_b.
 *   d_scores_out : optional out (may be NULL), float [batch][H_kv][max_pages_per_seq]; entries at
 *                  and beyond the sequence's page count are left untouched. */
int unique_score_select_topk(const unique_cache_desc* desc, const void* d_q, int32_t top_k, float lambda,
                             int32_t* d_sel_pages, int32_t* d_sel_count, float* d_scores_out,
                             void* d_workspace, size_t workspace_bytes, void* stream);

/* The two halves of unique_score_select_topk as separate calls (same kernels), for callers that keep
 * the score rows or bring their own.
 * unique_page_scores: Eq. 6 scores only. d_scores : out, float, row (b, h_kv) at
 *   d_scores + (b*H_kv + h_kv)*score_stride, entries [0, pages of the sequence) written;
 *   score_stride >= max_pages_per_seq (or the page bound implied by max_seq_len_hint) and a multiple of 4;
 *   d_scores 16-byte aligned.
 * unique_select_topk: top-k page set of each row of d_scores (same layout), outputs as above. */
int unique_page_scores(const unique_cache_desc* desc, const void* d_q, float lambda, float* d_scores,
                       int32_t score_stride, void* stream);
int unique_select_topk(const unique_cache_desc* desc, const float* d_scores, int32_t score_stride, int32_t top_k,
                       int32_t* d_sel_pages, int32_t* d_sel_count, void* stream);

/* Sparse paged decode attention, Eq. 5: for each query head, softmax(q K_T^T * sm_scale) V_T over
 * the valid tokens of the selected pages T of its KV head.
 *   d_sel_pages : int32, row (b, h_kv) starts at d_sel_pages + (b*H_kv + h_kv)*sel_stride and holds
 *                 LOGICAL page indices (any order, distinct); d_sel_count : int32 [batch][H_kv]
 *                 entries used per row (<= sel_stride). Entries that are negative or not a page of
 *                 the sequence are skipped.
 *   sel_stride  : host upper bound on d_sel_count[] and the row stride of d_sel_pages; every one of the first
 *                 d_sel_count entries of a row is visited, also when sel_stride exceeds the pages of the
 *                 sequences. The workspace needs unique_workspace_bytes(desc, sel_stride).
 *   sm_scale    : logit scale; <= 0 selects 1/sqrt(D).
 *   d_out       : [batch][H][D] dtype.  d_lse_out : optional float [batch][H], natural-log
 *                 sum-exp of the scaled logits (-inf and a zero output row if no token was attended). */
int unique_sparse_paged_decode(const unique_cache_desc* desc, const void* d_q, const int32_t* d_sel_pages,
                               const int32_t* d_sel_count, int32_t sel_stride, float sm_scale, void* d_out,
                               float* d_lse_out, void* d_workspace, size_t workspace_bytes, void* stream);

/* One whole decode step in a single call: [refresh of the last page's statistics +] Eq. 6 scores, top-k
 * selection, Eq. 5 sparse attention. The results are bit-identical to unique_update_page_stats (on the last
 * token of every sequence, when refresh_tail != 0) followed by unique_score_select_topk and
 * unique_sparse_paged_decode with sel_stride = top_k; the statistics refresh runs inside the score kernel
 * (the workgroup that scores the last page recomputes its record first, same arithmetic), which saves a launch.
 *   refresh_tail : non-zero = recompute the statistics record of the page holding token seq_lens[b]-1 of every
 *                  sequence before scoring (what a serving loop needs after appending one token).
 *   outputs      : d_sel_pages / d_sel_count as unique_score_select_topk, d_out / d_lse_out as
 *                  unique_sparse_paged_decode. The workspace needs unique_workspace_bytes(desc, top_k). */
int unique_decode_step(const unique_cache_desc* desc, const void* d_q, int32_t top_k, float lambda, float sm_scale,
                       int32_t refresh_tail, int32_t* d_sel_pages, int32_t* d_sel_count, void* d_out,
                       float* d_lse_out, void* d_workspace, size_t workspace_bytes, void* stream);

/* unique_decode_step for callers that cannot allocate device memory or bring a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same results, bit for
 * bit, but the score rows and split-K partials live in a scratch array of UNIQUE_STATIC_SCRATCH_BYTES that is part
 * of the library's device image (each GPU the library runs on holds its own copy until the process ends). The call
 * allocates and frees nothing and calls no allocating routine; inputs and outputs are still the caller's.
 *   - A step that needs more scratch than that (unique_workspace_bytes says how much a descriptor and top_k need)
 *     returns UNIQUE_ERR_WORKSPACE and launches nothing; use unique_decode_step then.
 *   - The device that owns `stream` must be the current device. The first call on a device looks up the array's
 *     address there (no allocation); make that first call outside graph capture.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in time (different streams or threads)
 *     race on it. Nothing in it has to start at zero and nothing is carried from one call to the next. */
#define UNIQUE_STATIC_SCRATCH_BYTES (8u << 20)
int unique_decode_step_static(const unique_cache_desc* desc, const void* d_q, int32_t top_k, float lambda,
                              float sm_scale, int32_t refresh_tail, int32_t* d_sel_pages, int32_t* d_sel_count,
                              void* d_out, float* d_lse_out, void* stream);

/* Dense paged decode attention, Eq. 4: the same kernels with every page of each sequence attended. */
int unique_dense_paged_decode(const unique_cache_desc* desc, const void* d_q, float sm_scale, void* d_out,
                              float* d_lse_out, void* d_workspace, size_t workspace_bytes, void* stream);

/* Static strings; never NULL. */
const char* unique_status_string(int status);
const char* unique_last_error(void); /* thread-local detail of the last non-OK return on this thread */
const char* unique_version(void);

#ifdef __cplusplus
}
#endif
#endif /* UNIQUE_H_ */
