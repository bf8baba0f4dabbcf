// Top-k page selection per (sequence, KV head) row (Section 3.2 of the paper, radix-based top-k).
//
// One workgroup per row; the row's scores are read once and stay in registers as order-preserving
// 32-bit keys. The paper narrows the k-th largest score with two 8-bit radix rounds over bf16 scores;
// here the scores are fp32 and the selected set has to equal an exact ranking, so the search is:
//   1. one histogram pass over 2 * threads buckets that are LINEAR in the score between the row's
//      minimum and maximum (a monotone map, so bucket order never contradicts score order). It finds
//      the bucket holding the k-th largest score; everything in higher buckets is selected. Linear
//      buckets spread page scores far better than the leading bits of a float (which are mostly
//      exponent), so LDS atomics see little same-address contention and the boundary bucket holds
//      only a handful of candidates.
//   2. exact resolution among the candidates of the boundary bucket: by pairwise ranking on
//      (key, page index) when they are few, otherwise by four 8-bit radix rounds over their keys
//      (this also covers degenerate rows such as all scores equal).
//   3. an index-ordered compaction (one workgroup scan) that emits the selected logical pages in
//      ascending order and takes keys tied with the k-th from the lowest page index upward.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace unique {
namespace {

constexpr int kMaxRankCandidates = 512;  // above this the boundary bucket is resolved by radix rounds
constexpr uint32_t kKeyForced = 0xffffffffu;  // key of a page that is selected whatever its score
constexpr uint32_t kKeyNegInf = 0x007fffffu, kKeyPosInf = 0xff800000u;  // keys of -inf and +inf

// Exclusive prefix sums of two counters at once over the threads of a workgroup (thread order). The pair
// travels packed in 64 bits; wave_tot: kThreads / 64 slots of LDS. All threads must call it.
template <int kThreads>
__device__ __forceinline__ unsigned long long block_exclusive_scan(unsigned long long v,
                                                                  unsigned long long* wave_tot /*[kThreads/64]*/) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int lo = (int)(v & 0xffffffffull), hi = (int)(v >> 32);
  const int inc_lo = wave_inclusive_scan(lo), inc_hi = wave_inclusive_scan(hi);
  const unsigned long long inc = (unsigned long long)(uint32_t)inc_lo | ((unsigned long long)(uint32_t)inc_hi << 32);
  if (lane == kWave - 1) wave_tot[wave] = inc;
  __syncthreads();
  unsigned long long base = 0;
#pragma unroll
  for (int w = 0; w < kThreads / kWave; ++w) {  // all totals are read at once, not one dependent read per wave
    const unsigned long long tot = wave_tot[w];
    base += w < wave ? tot : 0ull;
  }
  return base + inc - v;
}

__device__ __forceinline__ float ordered_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Bucket of a key in a histogram of n_buckets buckets that is linear in the score between lo and the row
// maximum (scale = (n_buckets - 1) / range): monotone in the score, so bucket order never contradicts
// score order. -inf and NaN go to the lowest bucket, +inf and always-selected pages to the highest.
__device__ __forceinline__ int linear_bucket(uint32_t k, float lo, float scale, int n_buckets) {
  if (k >= kKeyPosInf) return n_buckets - 1;
  if (k > kKeyNegInf) return min(n_buckets - 1, max(0, (int)((ordered_to_float(k) - lo) * scale)));
  return 0;
}

// One round-set of 8-bit radix selection over the keys accepted by `keep(j)`: returns the exact key of
// the need-th largest accepted key and leaves in `need` how many keys equal to it must be taken.
// hist: 256 ints of LDS; s_prefix / s_need: LDS scalars. All threads of the workgroup must call it.
// kStatic > 0: the per-thread item count is that constant (items live in registers, loops unroll).
template <int kThreads, int kStatic, typename KeyAt, typename Keep>
__device__ __forceinline__ uint32_t radix_threshold(int n_items, KeyAt key_at, Keep keep, int& need, int* hist,
                                                    uint32_t* s_prefix, int* s_need) {
  const int t = threadIdx.x;
  const int n = kStatic > 0 ? kStatic : n_items;
  uint32_t prefix = 0;
#pragma unroll 1
  for (int round = 0; round < 4; ++round) {
    const int shift = 24 - 8 * round;
    __syncthreads();  // everyone is done with the previous contents of hist
    if (t < 256) hist[t] = 0;
    __syncthreads();
    if constexpr (kStatic > 0) {
#pragma unroll
      for (int j = 0; j < n; ++j) {
        if (keep(j)) {
          const uint32_t k = key_at(j);
          if (round == 0 || (k >> (shift + 8)) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
        }
      }
    } else {  // keys come from memory: eight reads are requested before the first one is used
      for (int j0 = 0; j0 < n; j0 += 8) {
        uint32_t kk[8];
        bool kp[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          kp[u] = j0 + u < n && keep(j0 + u);
          kk[u] = kp[u] ? key_at(j0 + u) : 0u;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (kp[u] && (round == 0 || (kk[u] >> (shift + 8)) == prefix)) atomicAdd(&hist[(kk[u] >> shift) & 255u], 1);
      }
    }
    __syncthreads();
    if (t < kWave) {  // the first wave finds the digit that holds the need-th largest key
      int cnt[4];
      int tot = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) { cnt[i] = hist[4 * t + i]; tot += cnt[i]; }
      int suf = tot;  // inclusive suffix sum over lanes: keys in bins >= 4*t
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const int o = __shfl_down(suf, off, kWave);
        if (t + off < kWave) suf += o;
      }
      int above = suf - tot;  // keys in strictly higher bins
#pragma unroll
      for (int i = 3; i >= 0; --i) {
        if (above < need && need <= above + cnt[i]) {
          *s_prefix = (prefix << 8) | (uint32_t)(4 * t + i);
          *s_need = need - above;
        }
        above += cnt[i];
      }
    }
    __syncthreads();
    prefix = *s_prefix;
    need = *s_need;
  }
  return prefix;
}

// kItems keys per thread in registers (blocked: thread t owns pages [t*kItems, (t+1)*kItems)).
template <int kThreads, int kItems>
__global__ __launch_bounds__(kThreads) void topk_select_kernel(CacheView c, const float* __restrict__ scores,
                                                               int score_stride, int top_k,
                                                               int32_t* __restrict__ sel_pages,
                                                               int32_t* __restrict__ sel_count) {
  constexpr int kWaves = kThreads / kWave;
  constexpr int kBuckets = 2 * kThreads;
  constexpr int kMaxRank = kThreads < kMaxRankCandidates ? kThreads : kMaxRankCandidates;
  __shared__ int hist[kBuckets];
  __shared__ unsigned long long wave_tot[kWaves];
  __shared__ uint32_t wave_min[kWaves], wave_max[kWaves];
  __shared__ uint32_t cand_key[kMaxRank];
  __shared__ int cand_idx[kMaxRank];
  __shared__ int s_bucket, s_need, s_ncand;
  __shared__ uint32_t s_prefix;

  const int row = blockIdx.x;
  const int b = row / c.Hkv;
  const int N = c.seq_lens[b];
  int P = min((N + c.S - 1) / c.S, c.max_pages_hint);
  P = min(P, kThreads * kItems);  // a row longer than the host bound is cut, never overrun
  const int kb = min(top_k, P);
  const int t = threadIdx.x, lane = t % kWave, wave = t / kWave;
  int32_t* out = sel_pages + (int64_t)row * top_k;
  const float* srow = scores + (int64_t)row * score_stride;

  for (int i = kb + t; i < top_k; i += kThreads) out[i] = -1;
  if (t == 0) sel_count[row] = kb;
  if (kb == P) {  // everything is selected
    for (int i = t; i < P; i += kThreads) out[i] = i;
    return;
  }

  const int first = t * kItems;
  const int nv = max(0, min(kItems, P - first));  // valid items of this thread
  const int forced_from = P - min(c.force_recent, kb);  // pages from here on are always selected

  uint32_t key[kItems];
  if constexpr (kItems >= 4) {
#pragma unroll
    for (int j = 0; j < kItems; j += 4) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < nv) v = *reinterpret_cast<const float4*>(srow + first + j);  // row stride is padded past P
      key[j] = float_to_ordered(v.x); key[j + 1] = float_to_ordered(v.y);
      key[j + 2] = float_to_ordered(v.z); key[j + 3] = float_to_ordered(v.w);
    }
  } else {
#pragma unroll
    for (int j = 0; j < kItems; ++j) key[j] = j < nv ? float_to_ordered(srow[first + j]) : 0u;
  }
  // an always-selected page takes the largest key there is (above +inf), so it outranks every score
#pragma unroll
  for (int j = 0; j < kItems; ++j)
    if (first + j >= forced_from) key[j] = kKeyForced;

  // ---- 1. linear-bucket histogram between the row's smallest and largest finite score
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    if (j < nv && key[j] > kKeyNegInf && key[j] < kKeyPosInf) { kmin = min(kmin, key[j]); kmax = max(kmax, key[j]); }
  }
  kmin = wave_allreduce_minmax<false>(kmin);
  kmax = wave_allreduce_minmax<true>(kmax);
  if (lane == 0) { wave_min[wave] = kmin; wave_max[wave] = kmax; }
  for (int i = t; i < kBuckets; i += kThreads) hist[i] = 0;
  if (t == 0) s_ncand = 0;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) { kmin = min(kmin, wave_min[w]); kmax = max(kmax, wave_max[w]); }
  float lo = 0.f, scale = 0.f;
  if (kmin < kmax) {  // at least two distinct finite scores
    lo = ordered_to_float(kmin);
    const float range = ordered_to_float(kmax) - lo;
    if (range > 0.f && range < 3.0e38f) scale = (float)(kBuckets - 1) / range;
    if (!(scale < 3.0e38f)) scale = 0.f;  // a denormal range: leave everything in one bucket
  }
  // the bucket of every key is kept in registers, unless the keys alone already take most of them
  constexpr bool kKeepBuckets = kItems <= 32;
  int bucket_reg[kKeepBuckets ? kItems : 1];
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    if (j < nv) {
      const int bk = linear_bucket(key[j], lo, scale, kBuckets);
      atomicAdd(&hist[bk], 1);
      if constexpr (kKeepBuckets) bucket_reg[j] = bk;
    } else if constexpr (kKeepBuckets) {
      bucket_reg[j] = 0;
    }
  }
  auto bucket = [&](int j) {
    if constexpr (kKeepBuckets) return bucket_reg[j];
    else return linear_bucket(key[j], lo, scale, kBuckets);
  };
  __syncthreads();
  {  // suffix scan over the buckets: thread t owns buckets kBuckets-1-2t and kBuckets-2-2t
    const int c_hi = hist[kBuckets - 1 - 2 * t], c_lo = hist[kBuckets - 2 - 2 * t];
    int above = (int)block_exclusive_scan<kThreads>((unsigned long long)(c_hi + c_lo), wave_tot);
    if (above < kb && kb <= above + c_hi) { s_bucket = kBuckets - 1 - 2 * t; s_need = kb - above; }
    above += c_hi;
    if (above < kb && kb <= above + c_lo) { s_bucket = kBuckets - 2 - 2 * t; s_need = kb - above; }
  }
  __syncthreads();
  const int bstar = s_bucket;
  int need = s_need;  // how many of the boundary bucket's keys are selected
  const int ncand = hist[bstar];

  // ---- 2. exact threshold inside the boundary bucket: key T and how many keys equal to T to take
  uint32_t T;
  if (ncand <= kMaxRank) {
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      if (j < nv && bucket(j) == bstar) {
        const int slot = atomicAdd(&s_ncand, 1);
        cand_key[slot] = key[j];
        cand_idx[slot] = first + j;
      }
    }
    __syncthreads();
    if (t < ncand) {
      const uint32_t mk = cand_key[t];
      const int mi = cand_idx[t];
      int rank = 0, greater = 0;
      for (int j = 0; j < ncand; ++j) {
        const uint32_t k = cand_key[j];
        greater += k > mk;
        rank += (k > mk) || (k == mk && cand_idx[j] < mi);
      }
      if (rank == need - 1) { s_prefix = mk; s_need = need - greater; }
    }
    __syncthreads();
    T = s_prefix;
    need = s_need;
  } else {
    T = radix_threshold<kThreads, kItems>(
        kItems, [&](int j) { return key[j]; }, [&](int j) { return j < nv && bucket(j) == bstar; }, need, hist,
        &s_prefix, &s_need);
  }

  // ---- 3. index-ordered compaction. "sure": above the boundary; "tie": equal to the k-th key.
  uint32_t sure = 0, tie = 0;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    if (j < nv) {
      const bool in_b = bucket(j) == bstar;
      sure += (bucket(j) > bstar) || (in_b && key[j] > T);
      tie += in_b && key[j] == T;
    }
  }
  const unsigned long long before =
      block_exclusive_scan<kThreads>((unsigned long long)sure | ((unsigned long long)tie << 32), wave_tot);
  int sure_b = (int)(before & 0xffffffffull), tie_b = (int)(before >> 32);
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    if (j < nv) {
      const bool in_b = bucket(j) == bstar;
      if ((bucket(j) > bstar) || (in_b && key[j] > T)) {
        out[sure_b + min(tie_b, need)] = first + j;
        ++sure_b;
      } else if (in_b && key[j] == T) {
        if (tie_b < need) out[sure_b + tie_b] = first + j;
        ++tie_b;
      }
    }
  }
}

// Rows too long for registers: the same three steps as above, but every pass re-reads the scores (they
// stay in L2). Thread t owns the pages t, t + threads, t + 2*threads, ... so that every read of the row is
// coalesced, and reads are requested eight at a time. The compaction walks the row in blocks of `threads`
// consecutive pages and places each selected page by a ballot prefix inside its wave, the wave totals of
// the block (LDS) and the running totals of the blocks before it, which keeps the output in ascending page
// order and takes keys tied with the k-th from the lowest page upward.
template <int kThreads>
__global__ __launch_bounds__(kThreads) void topk_select_long_kernel(CacheView c, const float* __restrict__ scores,
                                                                    int score_stride, int top_k,
                                                                    int32_t* __restrict__ sel_pages,
                                                                    int32_t* __restrict__ sel_count) {
  constexpr int kWaves = kThreads / kWave;
  constexpr int kBuckets = 2 * kThreads;
  constexpr int kMaxRank = kThreads < kMaxRankCandidates ? kThreads : kMaxRankCandidates;
  __shared__ int hist[kBuckets];
  __shared__ unsigned long long wave_tot[kWaves];
  __shared__ uint32_t wave_min[kWaves], wave_max[kWaves];
  __shared__ uint32_t cand_key[kMaxRank];
  __shared__ int cand_idx[kMaxRank];
  __shared__ int wave_gt[2][kWaves], wave_eq[2][kWaves];
  __shared__ int s_bucket, s_need, s_ncand;
  __shared__ uint32_t s_prefix;

  const int row = blockIdx.x;
  const int b = row / c.Hkv;
  const int N = c.seq_lens[b];
  const int P = min((N + c.S - 1) / c.S, c.max_pages_hint);
  const int kb = min(top_k, P);
  const int t = threadIdx.x, lane = t % kWave, wave = t / kWave;
  int32_t* out = sel_pages + (int64_t)row * top_k;
  const float* srow = scores + (int64_t)row * score_stride;

  for (int i = kb + t; i < top_k; i += kThreads) out[i] = -1;
  if (t == 0) sel_count[row] = kb;
  if (kb == P) {
    for (int i = t; i < P; i += kThreads) out[i] = i;
    return;
  }
  const int forced_from = P - min(c.force_recent, kb);  // pages from here on are always selected
  auto key_of = [&](int page) { return page >= forced_from ? kKeyForced : float_to_ordered(srow[page]); };
  const int ipt = (P + kThreads - 1) / kThreads;  // strided items per thread; the last ones may fall past P
  auto for_each_key = [&](auto f) {               // f(page, key) for every page this thread owns
    for (int j0 = 0; j0 < ipt; j0 += 8) {
      uint32_t kk[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int page = (j0 + u) * kThreads + t;
        kk[u] = page < P ? key_of(page) : 0u;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int page = (j0 + u) * kThreads + t;
        if (page < P) f(page, kk[u]);
      }
    }
  };

  // ---- 1. linear-bucket histogram between the row's smallest and largest finite score
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for_each_key([&](int, uint32_t k) {
    if (k > kKeyNegInf && k < kKeyPosInf) { kmin = min(kmin, k); kmax = max(kmax, k); }
  });
  kmin = wave_allreduce_minmax<false>(kmin);
  kmax = wave_allreduce_minmax<true>(kmax);
  if (lane == 0) { wave_min[wave] = kmin; wave_max[wave] = kmax; }
  for (int i = t; i < kBuckets; i += kThreads) hist[i] = 0;
  if (t == 0) s_ncand = 0;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) { kmin = min(kmin, wave_min[w]); kmax = max(kmax, wave_max[w]); }
  float lo = 0.f, scale = 0.f;
  if (kmin < kmax) {  // at least two distinct finite scores
    lo = ordered_to_float(kmin);
    const float range = ordered_to_float(kmax) - lo;
    if (range > 0.f && range < 3.0e38f) scale = (float)(kBuckets - 1) / range;
    if (!(scale < 3.0e38f)) scale = 0.f;  // a denormal range: leave everything in one bucket
  }
  auto bucket_of = [&](uint32_t k) { return linear_bucket(k, lo, scale, kBuckets); };
  for_each_key([&](int, uint32_t k) { atomicAdd(&hist[bucket_of(k)], 1); });
  __syncthreads();
  {  // suffix scan over the buckets: thread t owns buckets kBuckets-1-2t and kBuckets-2-2t
    const int c_hi = hist[kBuckets - 1 - 2 * t], c_lo = hist[kBuckets - 2 - 2 * t];
    int above = (int)block_exclusive_scan<kThreads>((unsigned long long)(c_hi + c_lo), wave_tot);
    if (above < kb && kb <= above + c_hi) { s_bucket = kBuckets - 1 - 2 * t; s_need = kb - above; }
    above += c_hi;
    if (above < kb && kb <= above + c_lo) { s_bucket = kBuckets - 2 - 2 * t; s_need = kb - above; }
  }
  __syncthreads();
  const int bstar = s_bucket;
  int need = s_need;  // how many of the boundary bucket's keys are selected
  const int ncand = hist[bstar];

  // ---- 2. exact threshold inside the boundary bucket: key T and how many keys equal to T to take
  uint32_t T;
  if (ncand <= kMaxRank) {
    for_each_key([&](int page, uint32_t k) {
      if (bucket_of(k) == bstar) {
        const int slot = atomicAdd(&s_ncand, 1);
        cand_key[slot] = k;
        cand_idx[slot] = page;
      }
    });
    __syncthreads();
    if (t < ncand) {
      const uint32_t mk = cand_key[t];
      const int mi = cand_idx[t];
      int rank = 0, greater = 0;
      for (int j = 0; j < ncand; ++j) {
        const uint32_t k = cand_key[j];
        greater += k > mk;
        rank += (k > mk) || (k == mk && cand_idx[j] < mi);
      }
      if (rank == need - 1) { s_prefix = mk; s_need = need - greater; }
    }
    __syncthreads();
    T = s_prefix;
    need = s_need;
  } else {
    T = radix_threshold<kThreads, 0>(
        ipt, [&](int j) { return key_of(j * kThreads + t); },
        [&](int j) { return j * kThreads + t < P && bucket_of(key_of(j * kThreads + t)) == bstar; }, need, hist,
        &s_prefix, &s_need);
  }

  // ---- 3. compaction in page order. "gt": above the boundary; "eq": equal to the k-th key.
  int gt_run = 0, eq_run = 0;  // such pages in the blocks already walked
  constexpr int kAhead = 8;    // blocks whose keys are read together, ahead of the barriers that walk them
  for (int base0 = 0, it = 0; base0 < P; base0 += kAhead * kThreads) {
    uint32_t kk[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const int page = base0 + u * kThreads + t;
      kk[u] = page < P ? key_of(page) : 0u;
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u, ++it) {
      const int page = base0 + u * kThreads + t;
      if (base0 + u * kThreads >= P) break;  // uniform
      const int bk = page < P ? bucket_of(kk[u]) : -1;
      const bool gt = bk > bstar || (bk == bstar && kk[u] > T), eq = bk == bstar && kk[u] == T;
      const unsigned long long bg = __ballot(gt), be = __ballot(eq);
      const unsigned long long below = (1ull << lane) - 1ull;
      if (lane == 0) { wave_gt[it & 1][wave] = __popcll(bg); wave_eq[it & 1][wave] = __popcll(be); }
      __syncthreads();  // the buffers alternate, so one barrier per block is enough
      int gt_before = gt_run + __popcll(bg & below), eq_before = eq_run + __popcll(be & below);
      int gt_block = 0, eq_block = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const int g = wave_gt[it & 1][w], e = wave_eq[it & 1][w];
        gt_before += w < wave ? g : 0;
        eq_before += w < wave ? e : 0;
        gt_block += g;
        eq_block += e;
      }
      if (gt) out[gt_before + min(eq_before, need)] = page;
      else if (eq && eq_before < need) out[gt_before + eq_before] = page;
      gt_run += gt_block;
      eq_run += eq_block;
    }
  }
}

template <int kThreads, int kItems>
hipError_t launch_t(const CacheView& c, const float* scores, int stride, int top_k, int32_t* sel, int32_t* cnt,
                    hipStream_t st) {
  topk_select_kernel<kThreads, kItems><<<dim3(c.B * c.Hkv), dim3(kThreads), 0, st>>>(c, scores, stride, top_k, sel, cnt);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_select(const CacheView& c, const float* d_scores, int score_stride, int top_k,
                         int32_t* d_sel_pages, int32_t* d_sel_count, hipStream_t stream) {
  const int P = c.max_pages_hint;
  if (P <= 256) return launch_t<256, 1>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 1024) return launch_t<256, 4>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 2048) return launch_t<512, 4>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 4096) return launch_t<1024, 4>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 8192) return launch_t<1024, 8>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 16384) return launch_t<1024, 16>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 32768) return launch_t<1024, 32>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 65536) return launch_t<1024, 64>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  topk_select_long_kernel<1024><<<dim3(c.B * c.Hkv), dim3(1024), 0, stream>>>(c, d_scores, score_stride, top_k,
                                                                              d_sel_pages, d_sel_count);
  return hipGetLastError();
}

}  // namespace unique
