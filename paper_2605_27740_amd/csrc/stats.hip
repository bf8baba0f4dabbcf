// Page statistics kernel (Eq. 1 and Eq. 2 of the paper): per (physical page, KV head) the mean key
// and the scalar standard deviation (l2 norm of the per-dimension population std), written into the
// page's record of the statistics cache (means of all heads, then their stds, contiguous per page).
//
// One wavefront owns one (sequence, logical page, KV head). The page's S x D keys are one contiguous
// block; each lane reads 16-byte chunks so that every load instruction of the wave covers a
// contiguous 1 KiB, the whole page stays in registers, and both passes (mean, then squared
// deviations from it) run without touching memory again. Accumulation is fp32.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace unique {
namespace {

constexpr int kStatsWaves = 4;

template <typename T, int D, int S>
__global__ __launch_bounds__(kStatsWaves* kWave) void page_stats_kernel(CacheView c, const int32_t* tok_begin,
                                                                        const int32_t* tok_end, int pages_per_seq) {
  constexpr int kVec = Elem<T>::kVec;
  constexpr int kLanesPerTok = D / kVec;            // lanes covering one key
  constexpr int kTokPerLoad = kWave / kLanesPerTok;  // keys covered by one wave-wide load
  constexpr int kLoads = (S + kTokPerLoad - 1) / kTokPerLoad;
  static_assert(kLanesPerTok >= 8 && kLanesPerTok <= 32, "unsupported head_dim for this element type");

  const int b = blockIdx.y;
  const int lane = threadIdx.x % kWave;
  const int item = blockIdx.x * kStatsWaves + threadIdx.x / kWave;  // (page offset, kv head) of this wave
  const int hkv = item % c.Hkv;
  const int page_off = item / c.Hkv;
  if (page_off >= pages_per_seq) return;

  const int N = c.seq_lens[b];
  const int P = min((N + S - 1) / S, c.max_pages_hint);  // pages beyond the host bound are ignored
  int p = page_off;
  if (tok_begin != nullptr) {
    int t0 = max(tok_begin[b], 0), t1 = min(tok_end[b], N);
    if (t0 >= t1) return;
    p = t0 / S + page_off;
    if (p > (t1 - 1) / S) return;
  }
  if (p >= P) return;
  const int n = min(S, N - p * S);
  const int64_t phys = c.page_table[(int64_t)b * c.max_pages + p];
  if (phys < 0 || phys >= c.num_phys) return;

  const int tr = lane / kLanesPerTok;  // key row inside one load
  const int ch = lane % kLanesPerTok;  // 16-byte chunk of the key
  const T* base = reinterpret_cast<const T*>(c.k_cache) + phys * c.kv_page_stride + hkv * c.kv_head_stride + ch * kVec;

  float x[kLoads][kVec];
  float sum[kVec];
#pragma unroll
  for (int i = 0; i < kVec; ++i) sum[i] = 0.f;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    const int tok = j * kTokPerLoad + tr;
    if (tok < n) {
      unpack_raw(load_raw_stream(base + (int64_t)tok * D, c.stream_nt), x[j], (const T*)nullptr);
#pragma unroll
      for (int i = 0; i < kVec; ++i) sum[i] += x[j][i];
    } else {
#pragma unroll
      for (int i = 0; i < kVec; ++i) x[j][i] = 0.f;
    }
  }
  const float inv_n = 1.0f / (float)n;
  float mean[kVec];
#pragma unroll
  for (int i = 0; i < kVec; ++i) mean[i] = cross_group_allreduce<kLanesPerTok>(sum[i], OpSum()) * inv_n;

  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    const int tok = j * kTokPerLoad + tr;
    if (tok < n) {
#pragma unroll
      for (int i = 0; i < kVec; ++i) {
        const float dev = x[j][i] - mean[i];
        ss = fmaf(dev, dev, ss);  // explicit: both statistics paths must round identically
      }
    }
  }
  ss = group_allreduce<kWave>(ss, OpSum());

  char* rec = reinterpret_cast<char*>(c.page_stats) + phys * c.rec_bytes;  // this page's record
  if (tr == 0) {
    if (c.stats_bf16) {  // means rounded to bf16 (nearest even); the std above is about the unrounded mean
      bf16_t* m = reinterpret_cast<bf16_t*>(rec) + hkv * D + ch * kVec;
      uint32_t w[kVec / 2];
#pragma unroll
      for (int i = 0; i < kVec; i += 2)
        w[i / 2] = (uint32_t)float_to_bf16(mean[i]) | ((uint32_t)float_to_bf16(mean[i + 1]) << 16);
      if constexpr (kVec == 8) *reinterpret_cast<uint4*>(m) = make_uint4(w[0], w[1], w[2], w[3]);
      else *reinterpret_cast<uint2*>(m) = make_uint2(w[0], w[1]);
    } else {
      float* m = reinterpret_cast<float*>(rec) + hkv * D + ch * kVec;
#pragma unroll
      for (int i = 0; i < kVec; i += 4)
        *reinterpret_cast<float4*>(m + i) = make_float4(mean[i], mean[i + 1], mean[i + 2], mean[i + 3]);
    }
  }
  if (lane == 0) {
    const int64_t mean_bytes = (int64_t)c.Hkv * D * (c.stats_bf16 ? 2 : 4);
    reinterpret_cast<float*>(rec + mean_bytes)[hkv] = sqrtf(ss * inv_n);
  }
}

template <typename T, int D>
hipError_t dispatch_s(const CacheView& cv, const int32_t* tb, const int32_t* te, int pages_per_seq, hipStream_t st) {
  CacheView c = cv;
  const int items = pages_per_seq * c.Hkv;
  c.stream_nt = (int64_t)c.B * items * c.S * D * (int64_t)sizeof(T) > kStreamNtBytes;
  dim3 grid((items + kStatsWaves - 1) / kStatsWaves, c.B), block(kStatsWaves * kWave);
  switch (c.S) {
    case 8: page_stats_kernel<T, D, 8><<<grid, block, 0, st>>>(c, tb, te, pages_per_seq); break;
    case 16: page_stats_kernel<T, D, 16><<<grid, block, 0, st>>>(c, tb, te, pages_per_seq); break;
    case 32: page_stats_kernel<T, D, 32><<<grid, block, 0, st>>>(c, tb, te, pages_per_seq); break;
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
