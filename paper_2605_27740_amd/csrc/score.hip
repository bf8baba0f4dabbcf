// Fused page-score kernel (Eq. 6 of the paper; Eq. 3 when G = 1):
//   score(p) = max_g [ q_g . mean_p + lambda * |q_g|_2 * std_p ]   per (sequence, KV head, logical page).
// The G x P intermediate never exists in memory: each group of D/4 lanes holds one page-head mean
// (one 16-byte chunk per lane), keeps its G query slices in registers for the whole kernel,
// reduces the G dot products across the lane group, applies the offset and the max, and writes one float.
//
// A workgroup of 4 waves walks a tile of consecutive logical pages of one sequence. The lane groups
// of the workgroup are laid over (page, KV head) so that, for one page, all KV heads are read as one
// contiguous Hkv*D*4-byte block even when the page table scatters pages over the pool. Page-table
// entries for several iterations are fetched ahead of the mean loads that depend on them.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace unique {
namespace {

constexpr int kScoreWaves = 4;
#ifndef UNIQUE_SCORE_TILE
#define UNIQUE_SCORE_TILE 64
#endif
#ifndef UNIQUE_SCORE_UNROLL
#define UNIQUE_SCORE_UNROLL 8
#endif
constexpr int kTilePages = UNIQUE_SCORE_TILE;  // logical pages per workgroup
constexpr int kUnroll = UNIQUE_SCORE_UNROLL;   // iterations whose loads are issued together

__device__ __forceinline__ void load_q4(const float* p, float (&out)[4]) { load_vec(p, out); }
__device__ __forceinline__ void load_q4(const bf16_t* p, float (&out)[4]) {
  const uint2 v = *reinterpret_cast<const uint2*>(p);
  out[0] = bits_to_float(v.x << 16); out[1] = bits_to_float(v.x & 0xffff0000u);
  out[2] = bits_to_float(v.y << 16); out[3] = bits_to_float(v.y & 0xffff0000u);
}

template <typename T, int D, int G>
__global__ __launch_bounds__(kScoreWaves* kWave) void page_score_kernel(CacheView c, const T* __restrict__ q,
                                                                        float lambda, float* __restrict__ scores,
                                                                        int score_stride,
                                                                        float* __restrict__ scores_out) {
  constexpr int kLanesPerHead = D / 4;                  // lanes covering one fp32 mean vector
  constexpr int kSlotsPerWave = kWave / kLanesPerHead;  // (page, head) items per wave-wide load
  constexpr int kSlots = kScoreWaves * kSlotsPerWave;   // items per workgroup iteration

  const int b = blockIdx.y;
  const int N = c.seq_lens[b];
  const int P = min((N + c.S - 1) / c.S, c.max_pages_hint);  // pages beyond the host bound are ignored
  const int tile0 = blockIdx.x * kTilePages;
  if (tile0 >= P) return;

  const int lane = threadIdx.x % kWave;
  const int dl = lane % kLanesPerHead;
  const int slot = (threadIdx.x / kWave) * kSlotsPerWave + lane / kLanesPerHead;
  const int hkv = slot % c.Hkv;        // fixed for the whole kernel because kSlots % Hkv == 0
  const int page_in_iter = slot / c.Hkv;
  const int pages_per_iter = kSlots / c.Hkv;

  // this lane's slice of the G queries of its KV head, and lambda * |q_g|
  float qv[G][4];
  float off[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    load_q4(q + ((int64_t)b * c.H + hkv * G + g) * D + dl * 4, qv[g]);
    float qq = qv[g][0] * qv[g][0] + qv[g][1] * qv[g][1] + qv[g][2] * qv[g][2] + qv[g][3] * qv[g][3];
    qq = group_allreduce<kLanesPerHead>(qq, OpSum());
    off[g] = lambda * sqrtf(qq);
  }

  const int32_t* pt = c.page_table + (int64_t)b * c.max_pages;
  const int tile_end = min(tile0 + kTilePages, P);
  for (int p0 = tile0 + page_in_iter; p0 < tile_end + page_in_iter; p0 += pages_per_iter * kUnroll) {
    int64_t item[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int p = p0 + u * pages_per_iter;
      int64_t phys = -1;
      if (p < tile_end) phys = pt[p];
      item[u] = (phys >= 0 && phys < c.num_phys) ? phys * c.Hkv + hkv : -1;
    }
    float4 m[kUnroll];
    float sd[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      if (item[u] >= 0) {
        m[u] = *reinterpret_cast<const float4*>(c.page_mean + item[u] * D + dl * 4);
#ifdef EXP_NO_STD
        sd[u] = 1.0f;
#else
        sd[u] = c.page_std[item[u]];
#endif
      } else {
        m[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        sd[u] = 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      float best = 0.f;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float dot = qv[g][0] * m[u].x;
        dot = fmaf(qv[g][1], m[u].y, dot);
        dot = fmaf(qv[g][2], m[u].z, dot);
        dot = fmaf(qv[g][3], m[u].w, dot);
        dot = group_allreduce<kLanesPerHead>(dot, OpSum());
        const float s = fmaf(off[g], sd[u], dot);
        best = (g == 0) ? s : fmaxf(best, s);
      }
      const int p = p0 + u * pages_per_iter;
      if (dl == 0 && item[u] >= 0) {
        scores[((int64_t)b * c.Hkv + hkv) * score_stride + p] = best;
        if (scores_out) scores_out[((int64_t)b * c.Hkv + hkv) * c.max_pages + p] = best;
      }
    }
  }
}

template <typename T, int D, int G>
hipError_t launch_t(const CacheView& c, const void* q, float lambda, float* scores, int stride, float* out,
                    hipStream_t st) {
  dim3 grid((c.max_pages_hint + kTilePages - 1) / kTilePages, c.B), block(kScoreWaves * kWave);
  page_score_kernel<T, D, G><<<grid, block, 0, st>>>(c, reinterpret_cast<const T*>(q), lambda, scores, stride, out);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t dispatch_g(const CacheView& c, const void* q, float lambda, float* scores, int stride, float* out,
                      hipStream_t st) {
  switch (c.H / c.Hkv) {
    case 1: return launch_t<T, D, 1>(c, q, lambda, scores, stride, out, st);
    case 2: return launch_t<T, D, 2>(c, q, lambda, scores, stride, out, st);
    case 4: return launch_t<T, D, 4>(c, q, lambda, scores, stride, out, st);
    case 8: return launch_t<T, D, 8>(c, q, lambda, scores, stride, out, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool score_supported(int dtype, int D, int G, int Hkv) {
  if (!(dtype == 0 || dtype == 1) || !(D == 64 || D == 128)) return false;
  if (!(G == 1 || G == 2 || G == 4 || G == 8)) return false;
  const int slots = kScoreWaves * (kWave / (D / 4));
  return Hkv >= 1 && Hkv <= slots && slots % Hkv == 0;
}

hipError_t launch_score(const CacheView& c, const void* d_q, float lambda, float* d_scores, int score_stride,
                        float* d_scores_out, hipStream_t stream) {
  if (c.dtype == 0) {
    return c.D == 64 ? dispatch_g<float, 64>(c, d_q, lambda, d_scores, score_stride, d_scores_out, stream)
                     : dispatch_g<float, 128>(c, d_q, lambda, d_scores, score_stride, d_scores_out, stream);
  }
  return c.D == 64 ? dispatch_g<bf16_t, 64>(c, d_q, lambda, d_scores, score_stride, d_scores_out, stream)
                   : dispatch_g<bf16_t, 128>(c, d_q, lambda, d_scores, score_stride, d_scores_out, stream);
}

}  // namespace unique
