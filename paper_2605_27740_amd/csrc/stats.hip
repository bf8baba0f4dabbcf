// Page statistics kernel (Eq. 1 and Eq. 2 of the paper): per (physical page, KV head) the mean key
// and the scalar standard deviation (l2 norm of the per-dimension population std), written into the
// page's record of the statistics cache (means of all heads, then their stds, contiguous per page).
//
// One wavefront owns a run of consecutive logical pages of one sequence, all KV heads of each. A
// (page, head) item's S x D keys are one contiguous block; each lane reads 16-byte chunks so that every
// load instruction of the wave covers a contiguous 1 KiB. Items are taken a few at a time, the next
// batch's loads in flight while the current one is reduced; each item stays in registers for both
// passes (mean, then squared deviations from it). A page's record is written by one wave, its stds
// in one store. Accumulation is fp32.
#include <algorithm>

#include "device_utils.hpp"
#include "kernels.hpp"

namespace unique {
namespace {

constexpr int kStatsWaves = 4;
constexpr int kStatsMaxPagesPerWave = 32;  // <= wavefront size: lane l keeps the id of the wave's l-th page
#ifndef UNIQUE_STATS_TARGET_WAVES
#define UNIQUE_STATS_TARGET_WAVES 65536
#endif

// (page, head) items per batch: about 8 16-byte loads per lane and batch; two batches are in flight per
// wave. Larger batches cost registers and with them resident waves (16 loads per batch measured 9 % slower
// on the 128K bulk build).
template <typename T, int D, int S>
struct StatsShape {
  static constexpr int kVec = Elem<T>::kVec;
  static constexpr int kLanesPerTok = D / kVec;            // lanes covering one key
  static constexpr int kTokPerLoad = kWave / kLanesPerTok;  // keys covered by one wave-wide load
  static constexpr int kLoads = (S + kTokPerLoad - 1) / kTokPerLoad;
  static constexpr int kItems = kLoads >= 8 ? 1 : (kLoads >= 4 ? 2 : 4);
};

template <typename T, int D, int S>
__global__ __launch_bounds__(kStatsWaves* kWave) void page_stats_kernel(CacheView c, const int32_t* tok_begin,
                                                                        const int32_t* tok_end, int pages_per_seq,
                                                                        int items_per_wave) {
  using Sh = StatsShape<T, D, S>;
  constexpr int kVec = Sh::kVec, kLanesPerTok = Sh::kLanesPerTok, kTokPerLoad = Sh::kTokPerLoad;
  constexpr int kLoads = Sh::kLoads, kItems = Sh::kItems;
  static_assert(kLanesPerTok >= 8 && kLanesPerTok <= 32, "unsupported head_dim for this element type");

  const int b = blockIdx.y;
  const int lane = threadIdx.x % kWave;
  const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * kStatsWaves + threadIdx.x / kWave);
  const int hshift = __ffs(c.Hkv) - 1;  // the number of KV heads is a power of two
  // (page offset, head) items, heads of one page adjacent; this wave owns items [i0, i0 + items)
  const int i0 = w * items_per_wave;
  if (i0 >= (pages_per_seq << hshift)) return;

  const int N = c.seq_lens[b];
  const int P = min((N + S - 1) / S, c.max_pages_hint);  // pages beyond the host bound are ignored
  int p_first = 0, p_last = P - 1;
  if (tok_begin != nullptr) {
    const int t0 = max(tok_begin[b], 0), t1 = min(tok_end[b], N);
    if (t0 >= t1) return;
    p_first = t0 / S;
    p_last = min(p_last, (t1 - 1) / S);
  }
  const int pages_here = min(pages_per_seq, p_last - p_first + 1);
  const int items = min(items_per_wave, (pages_here << hshift) - i0);
  if (items <= 0) return;
  const int po0 = i0 >> hshift;                         // first page offset of this wave
  const int np = ((i0 + items - 1) >> hshift) - po0 + 1;  // pages it touches (<= kStatsMaxPagesPerWave)
  const int p0 = p_first + po0;
  const int span = min(items_per_wave, (int)c.Hkv);     // heads of one page owned by one wave (power of two)

  // lane l keeps the physical id of the wave's l-th page (-1: nothing to do for it)
  int my_phys = -1;
  if (lane < np) {
    const int ph = c.page_table[(int64_t)b * c.max_pages + p0 + lane];
    if (ph >= 0 && (int64_t)ph < c.num_phys) my_phys = ph;
  }
  const int batches = (items + kItems - 1) / kItems;

  const int tr = lane / kLanesPerTok;  // key row inside one load
  const int ch = lane % kLanesPerTok;  // 16-byte chunk of the key
  const int64_t mean_bytes = (int64_t)c.Hkv * D * (c.stats_bf16 ? 2 : 4);
  float my_std = 0.f;  // lane h collects the std of head h until the page's record is complete

  struct Item { int phys, n, hkv; };
  auto resolve = [&](int item) {  // item: index inside this wave's run
    Item r;
    const int pl = min(((i0 + item) >> hshift) - po0, kWave - 1);
    r.hkv = (i0 + item) & (c.Hkv - 1);
    r.phys = item < items ? __builtin_amdgcn_readlane(my_phys, pl) : -1;
    r.n = r.phys >= 0 ? min(S, N - (p0 + pl) * S) : 0;
    return r;
  };
  // Loads are unconditional (rows past the page's keys re-read its last key, items past the wave's
  // range read the cache's first bytes; neither is used), so the pipeline below is straight-line code
  // and every wait names the exact number of requests that may stay in flight.
  auto load_batch = [&](int t, Raw16(&raw)[kItems][kLoads]) {
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
      const Item m = resolve(t * kItems + it);
      const T* page = reinterpret_cast<const T*>(c.k_cache) + (int64_t)max(m.phys, 0) * c.kv_page_stride +
                      m.hkv * c.kv_head_stride + ch * kVec;
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        const int tok = min(j * kTokPerLoad + tr, m.n - 1);
        const T* src = m.phys >= 0 ? page + (int64_t)tok * D : reinterpret_cast<const T*>(c.k_cache);
        raw[it][j] = load_raw_stream(src, true);
      }
    }
  };
  auto reduce_batch = [&](int t, const Raw16(&raw)[kItems][kLoads]) {
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
      const Item m = resolve(t * kItems + it);
      if (m.phys < 0) continue;  // wave-uniform
      float x[kLoads][kVec];
      float sum[kVec];
#pragma unroll
      for (int i = 0; i < kVec; ++i) sum[i] = 0.f;
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        const int tok = j * kTokPerLoad + tr;
        unpack_raw(raw[it][j], x[j], (const T*)nullptr);
        if (tok < m.n) {
#pragma unroll
          for (int i = 0; i < kVec; ++i) sum[i] += x[j][i];
        }
      }
      const float inv_n = 1.0f / (float)m.n;
      float mean[kVec];
#pragma unroll
      for (int i = 0; i < kVec; ++i) mean[i] = cross_group_allreduce<kLanesPerTok>(sum[i], OpSum()) * inv_n;

      float ss = 0.f;
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        const int tok = j * kTokPerLoad + tr;
        if (tok < m.n) {
#pragma unroll
          for (int i = 0; i < kVec; ++i) {
            const float dev = x[j][i] - mean[i];
            ss = fmaf(dev, dev, ss);  // explicit: both statistics paths must round identically
          }
        }
      }
      ss = group_allreduce<kWave>(ss, OpSum());

      char* rec = reinterpret_cast<char*>(c.page_stats) + (int64_t)m.phys * c.rec_bytes;  // this page's record
      if (tr == 0) {
        if (c.stats_bf16) {  // means rounded to bf16 (nearest even); the std above is about the unrounded mean
          bf16_t* mp = reinterpret_cast<bf16_t*>(rec) + m.hkv * D + ch * kVec;
          uint32_t wd[kVec / 2];
#pragma unroll
          for (int i = 0; i < kVec; i += 2)
            wd[i / 2] = (uint32_t)float_to_bf16(mean[i]) | ((uint32_t)float_to_bf16(mean[i + 1]) << 16);
          if constexpr (kVec == 8) *reinterpret_cast<uint4*>(mp) = make_uint4(wd[0], wd[1], wd[2], wd[3]);
          else *reinterpret_cast<uint2*>(mp) = make_uint2(wd[0], wd[1]);
        } else {
          float* mp = reinterpret_cast<float*>(rec) + m.hkv * D + ch * kVec;
#pragma unroll
          for (int i = 0; i < kVec; i += 4)
            *reinterpret_cast<float4*>(mp + i) = make_float4(mean[i], mean[i + 1], mean[i + 2], mean[i + 3]);
        }
      }
      if (lane == m.hkv) my_std = sqrtf(ss * inv_n);
      // the stds of the heads this wave owns in the page leave as one contiguous store
      if (((m.hkv + 1) & (span - 1)) == 0 && lane <= m.hkv && lane > m.hkv - span)
        reinterpret_cast<float*>(rec + mean_bytes)[lane] = my_std;
    }
  };

  // Two register buffers: the next batch is requested before the current one is reduced. The steady-state
  // loop has no branches (both following batches exist); the last one or two batches are peeled off.
  Raw16 buf_a[kItems][kLoads], buf_b[kItems][kLoads];
  load_batch(0, buf_a);
  int t = 0;
  for (; t + 2 < batches; t += 2) {
    load_batch(t + 1, buf_b);
    reduce_batch(t, buf_a);
    load_batch(t + 2, buf_a);
    reduce_batch(t + 1, buf_b);
  }
  if (t + 1 < batches) {
    load_batch(t + 1, buf_b);
    reduce_batch(t, buf_a);
    reduce_batch(t + 1, buf_b);
  } else {
    reduce_batch(t, buf_a);
  }
}

template <typename T, int D>
hipError_t dispatch_s(const CacheView& cv, const int32_t* tb, const int32_t* te, int pages_per_seq, hipStream_t st) {
  CacheView c = cv;
  // Enough waves to fill the chip many times over (ragged batches then balance), each with a run of
  // items that amortises its prologue. The run is a power of two, so it is a multiple or a divisor of
  // the (power-of-two) head count: a wave owns whole pages, or an aligned group of heads of one page.
  auto launch = [&](auto kernel, int k_items) {
    const int64_t total = (int64_t)pages_per_seq * c.Hkv;
    // a launch with very few items (the tail-page refresh) gives every item its own wave; otherwise a wave
    // takes at least one full batch
    int64_t ipw = total * c.B <= 4096 ? 1 : k_items;
    while (ipw * UNIQUE_STATS_TARGET_WAVES < total * c.B && ipw < (int64_t)kStatsMaxPagesPerWave * c.Hkv) ipw *= 2;
    const int64_t waves = (total + ipw - 1) / ipw;
    const dim3 grid((unsigned)((waves + kStatsWaves - 1) / kStatsWaves), c.B), block(kStatsWaves * kWave);
    kernel<<<grid, block, 0, st>>>(c, tb, te, pages_per_seq, (int)ipw);
  };
  switch (c.S) {
    case 8: launch(page_stats_kernel<T, D, 8>, StatsShape<T, D, 8>::kItems); break;
    case 16: launch(page_stats_kernel<T, D, 16>, StatsShape<T, D, 16>::kItems); break;
    case 32: launch(page_stats_kernel<T, D, 32>, StatsShape<T, D, 32>::kItems); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

bool stats_supported(int dtype, int D, int S) {
  return (dtype == 0 || dtype == 1) && (D == 64 || D == 128) && (S == 8 || S == 16 || S == 32);
}

hipError_t launch_stats(const CacheView& c, const int32_t* d_tok_begin, const int32_t* d_tok_end,
                        int max_pages_touched, hipStream_t stream) {
  const int pages_per_seq = d_tok_begin ? max_pages_touched : c.max_pages_hint;
  if (pages_per_seq <= 0) return hipSuccess;
  if (c.dtype == 0) {
    return c.D == 64 ? dispatch_s<float, 64>(c, d_tok_begin, d_tok_end, pages_per_seq, stream)
                     : dispatch_s<float, 128>(c, d_tok_begin, d_tok_end, pages_per_seq, stream);
  }
  return c.D == 64 ? dispatch_s<bf16_t, 64>(c, d_tok_begin, d_tok_end, pages_per_seq, stream)
                   : dispatch_s<bf16_t, 128>(c, d_tok_begin, d_tok_end, pages_per_seq, stream);
}

}  // namespace unique
