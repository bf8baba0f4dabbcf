// Top-k page selection per (sequence, KV head) row (Section 3.2 of the paper, radix-based top-k).
//
// One workgroup per row. Scores become order-preserving 32-bit keys held in registers (a row of up to
// 32768 pages fits a 1024-thread workgroup at 32 keys per thread); four rounds of 8-bit radix selection
// over an LDS histogram narrow the k-th largest key exactly; a final index-ordered compaction emits
// the selected logical pages in ascending order, taking tied keys from the lowest page index upward.
// The paper selects over bf16 scores in two rounds; fp32 keys in four rounds are used here so that
// the chosen set equals an exact ranking of the fp32 scores.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace unique {
namespace {

template <int kThreads>
__device__ __forceinline__ unsigned long long block_exclusive_scan(unsigned long long v,
                                                                  unsigned long long* wave_tot /*[kThreads/64]*/) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  unsigned long long inc = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const unsigned long long o = __shfl_up(inc, off, kWave);
    if (lane >= off) inc += o;
  }
  if (lane == kWave - 1) wave_tot[wave] = inc;
  __syncthreads();
  unsigned long long base = 0;
  for (int w = 0; w < wave; ++w) base += wave_tot[w];
  return base + inc - v;
}

// kItems > 0: keys of the row live in registers, kItems per thread. kItems == 0: the row is too long
// for that, and every pass re-reads the scores (they stay in L2).
template <int kThreads, int kItems>
__global__ __launch_bounds__(kThreads) void topk_select_kernel(CacheView c, const float* __restrict__ scores,
                                                               int score_stride, int top_k,
                                                               int32_t* __restrict__ sel_pages,
                                                               int32_t* __restrict__ sel_count) {
  __shared__ int hist[256];
  __shared__ unsigned long long wave_tot[kThreads / kWave];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;

  const int row = blockIdx.x;
  const int b = row / c.Hkv;
  const int N = c.seq_lens[b];
  int P = min((N + c.S - 1) / c.S, c.max_pages_hint);
  if (kItems > 0) P = min(P, kThreads * kItems);  // a row longer than the host bound is cut, never overrun
  const int kb = min(top_k, P);
  const int t = threadIdx.x;
  int32_t* out = sel_pages + (int64_t)row * top_k;
  const float* srow = scores + (int64_t)row * score_stride;

  for (int i = kb + t; i < top_k; i += kThreads) out[i] = -1;
  if (t == 0) sel_count[row] = kb;
  if (kb == P) {  // everything is selected
    for (int i = t; i < P; i += kThreads) out[i] = i;
    return;
  }

  const int ipt = kItems > 0 ? kItems : (P + kThreads - 1) / kThreads;
  const int first = t * ipt;
  const int nv = max(0, min(ipt, P - first));  // valid items of this thread

  uint32_t key[kItems > 0 ? kItems : 1];
  if constexpr (kItems >= 4) {
#pragma unroll
    for (int j = 0; j < kItems; j += 4) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < nv) v = *reinterpret_cast<const float4*>(srow + first + j);  // row stride is padded past P
      key[j] = float_to_ordered(v.x); key[j + 1] = float_to_ordered(v.y);
      key[j + 2] = float_to_ordered(v.z); key[j + 3] = float_to_ordered(v.w);
    }
  } else if constexpr (kItems > 0) {
#pragma unroll
    for (int j = 0; j < kItems; ++j) key[j] = j < nv ? float_to_ordered(srow[first + j]) : 0u;
  }
  auto key_at = [&](int j) -> uint32_t {
    if constexpr (kItems > 0) return key[j];
    else return float_to_ordered(srow[first + j]);
  };

  uint32_t prefix = 0;
  int need = kb;
#pragma unroll 1
  for (int round = 0; round < 4; ++round) {
    const int shift = 24 - 8 * round;
    if (t < 256) hist[t] = 0;
    __syncthreads();
    if constexpr (kItems > 0) {
#pragma unroll
      for (int j = 0; j < kItems; ++j) {
        if (j < nv) {
          const uint32_t k = key[j];
          if (round == 0 || (k >> (shift + 8)) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
        }
      }
    } else {
      for (int j = 0; j < nv; ++j) {
        const uint32_t k = key_at(j);
        if (round == 0 || (k >> (shift + 8)) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
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
          s_prefix = (prefix << 8) | (uint32_t)(4 * t + i);
          s_need = need - above;
        }
        above += cnt[i];
      }
    }
    __syncthreads();
    prefix = s_prefix;
    need = s_need;
  }
  // prefix is now the exact key of the kb-th largest score; `need` keys equal to it are taken.
  uint32_t gt = 0, eq = 0;
  if constexpr (kItems > 0) {
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      if (j < nv) { gt += key[j] > prefix; eq += key[j] == prefix; }
    }
  } else {
    for (int j = 0; j < nv; ++j) { const uint32_t k = key_at(j); gt += k > prefix; eq += k == prefix; }
  }
  // one scan carries both counters: keys above the threshold (low half) and keys equal to it (high half)
  const unsigned long long before =
      block_exclusive_scan<kThreads>((unsigned long long)gt | ((unsigned long long)eq << 32), wave_tot);
  int gt_b = (int)(before & 0xffffffffull), eq_b = (int)(before >> 32);
  auto emit = [&](int j) {
    const uint32_t k = key_at(j);
    if (k > prefix) {
      out[gt_b + min(eq_b, need)] = first + j;
      ++gt_b;
    } else if (k == prefix) {
      if (eq_b < need) out[gt_b + eq_b] = first + j;
      ++eq_b;
    }
  };
  if constexpr (kItems > 0) {
#pragma unroll
    for (int j = 0; j < kItems; ++j) if (j < nv) emit(j);
  } else {
    for (int j = 0; j < nv; ++j) emit(j);
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
  if (P <= 2048) return launch_t<256, 8>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 4096) return launch_t<1024, 4>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 8192) return launch_t<1024, 8>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 16384) return launch_t<1024, 16>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  if (P <= 32768) return launch_t<1024, 32>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
  // longer rows do not fit in registers: every pass re-reads the scores
  return launch_t<1024, 0>(c, d_scores, score_stride, top_k, d_sel_pages, d_sel_count, stream);
}

}  // namespace unique
