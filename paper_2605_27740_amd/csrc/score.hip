// Fused page-score kernel (Eq. 6 of the paper; Eq. 3 when G = 1):
//   score(p) = max_g [ q_g . mean_p + lambda * |q_g|_2 * std_p ]   per (sequence, KV head, logical page).
// The G x P intermediate never exists in memory: the G dot products, the rank-one offset and the max
// over the group are all formed in registers and one float per (KV head, page) is written.
//
// Layout of the work: 8 lanes own one (page, KV head) mean row and read it as 16-byte chunks (D/32
// of them for fp32 means, D/64 for bf16 means) each, so a wave covers 8 consecutive head rows per step -- with 8 KV heads that is exactly one
// page record, read as one contiguous block whatever the page table does to page placement, with
// the page's stds taken from the tail of the same record. Every lane keeps its slices of the G
// queries of its (fixed) KV head in registers for the whole kernel. The G partial dot products are
// reduced over the 8 lanes with three DPP steps. The page-table entries of all of a wave's steps are
// fetched up front (together with the sequence length and the queries, so the prologue is two memory
// round trips); two records are in flight per wave, requested with unconditional loads so that the
// loop is straight-line code with exact waits. Scores of a tile are staged in LDS and written as one
// contiguous run per KV head (4-byte scattered stores cost a tenth of the kernel otherwise).
#include "device_utils.hpp"
#include "kernels.hpp"

namespace unique {
namespace {

constexpr int kScoreWaves = 4;
#ifndef UNIQUE_SCORE_DEPTH
#define UNIQUE_SCORE_DEPTH 2
#endif
#ifndef UNIQUE_SCORE_FULL_TILES
#define UNIQUE_SCORE_FULL_TILES 512  // full tiles (two per CU) a batch of known-long sequences must supply for the next larger tile
#endif
#ifndef UNIQUE_SCORE_FAT_GRID
#define UNIQUE_SCORE_FAT_GRID 4096  // workgroups above which a launch can afford the next larger tile
#endif
constexpr int kRowLanes = 8;                   // lanes per (page, head) row
constexpr int kRowsPerWave = kWave / kRowLanes;
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// kE consecutive query elements, loaded as raw 32-bit words, as floats (kE = 4 or 8)
template <int kE>
__device__ __forceinline__ void unpack_q(const uint32_t (&w)[kE], float (&out)[kE], const float*) {
#pragma unroll
  for (int i = 0; i < kE; ++i) out[i] = bits_to_float(w[i]);
}
template <int kE>
__device__ __forceinline__ void unpack_q(const uint32_t (&w)[kE / 2], float (&out)[kE], const bf16_t*) {
#pragma unroll
  for (int i = 0; i < kE / 2; ++i) {
    out[2 * i] = bits_to_float(w[i] << 16);
    out[2 * i + 1] = bits_to_float(w[i] & 0xffff0000u);
  }
}

// Statistics of the last (possibly partial) page of sequence b, recomputed from the keys by the whole
// workgroup: wave w takes KV heads w, w+4, ... The lane layout, the order of every sum and the
// cross-lane reductions are those of the bulk statistics kernel, so the stored record is bit-identical
// to what unique_update_page_stats writes. The page size is a run-time value here, so the loads are
// predicated up to the largest supported page (32 tokens).
template <typename T, int D>
__device__ __forceinline__ void refresh_tail_record(const CacheView& c, int b, int N, int P) {
  constexpr int kVec = Elem<T>::kVec;
  constexpr int kLanesPerTok = D / kVec;
  constexpr int kTokPerLoad = kWave / kLanesPerTok;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;  // wave: scalar
  const int tr = lane / kLanesPerTok, ch = lane % kLanesPerTok;
  const int p = P - 1, S = c.S;
  const int n = min(S, N - p * S);
  const int64_t phys = c.page_table[(int64_t)b * c.max_pages + p];
  if (phys < 0 || phys >= c.num_phys || n < 1) return;
  char* rec = reinterpret_cast<char*>(c.page_stats) + phys * c.rec_bytes;
  const int64_t mean_bytes = (int64_t)c.Hkv * D * (c.stats_bf16 ? 2 : 4);
  const float inv_n = 1.0f / (float)n;
  constexpr int kMaxLoads = 32 / kTokPerLoad;  // page_size <= 32
  for (int hkv = wave; hkv < c.Hkv; hkv += kScoreWaves) {
    const T* base = reinterpret_cast<const T*>(c.k_cache) + phys * c.kv_page_stride + hkv * c.kv_head_stride + ch * kVec;
    // the page is read once and kept as raw 16-byte chunks; both passes unpack from registers
    Raw16 raw[kMaxLoads];
#pragma unroll
    for (int j = 0; j < kMaxLoads; ++j) {
      const int tok = j * kTokPerLoad + tr;
      raw[j] = tok < n ? load_raw(base + (int64_t)tok * D) : zero_raw();
    }
    float sum[kVec];
#pragma unroll
    for (int i = 0; i < kVec; ++i) sum[i] = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxLoads; ++j) {
      if (j * kTokPerLoad + tr < n) {
        float x[kVec];
        unpack_raw(raw[j], x, (const T*)nullptr);
#pragma unroll
        for (int i = 0; i < kVec; ++i) sum[i] += x[i];
      }
    }
    float mean[kVec];
#pragma unroll
    for (int i = 0; i < kVec; ++i) mean[i] = cross_group_allreduce<kLanesPerTok>(sum[i], OpSum()) * inv_n;
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxLoads; ++j) {
      if (j * kTokPerLoad + tr < n) {
        float x[kVec];
        unpack_raw(raw[j], x, (const T*)nullptr);
#pragma unroll
        for (int i = 0; i < kVec; ++i) {
          const float dev = x[i] - mean[i];
          ss = fmaf(dev, dev, ss);  // explicit: both statistics paths must round identically
        }
      }
    }
    ss = group_allreduce<kWave>(ss, OpSum());
    if (tr == 0) {
      if (c.stats_bf16) {
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
    if (lane == 0) reinterpret_cast<float*>(rec + mean_bytes)[hkv] = sqrtf(ss * inv_n);
  }
}

// T: element type of q; TS: element type of the stored means (float, or bf16_t for bf16 statistics).
// kNT: the records are read with non-temporal loads (a launch that streams more than the caches hold).
template <typename T, typename TS, int D, int G, bool kNT>
__global__ __launch_bounds__(kScoreWaves* kWave) void page_score_kernel(CacheView c, const T* __restrict__ q,
                                                                        float lambda, float* __restrict__ scores,
                                                                        int score_stride,
                                                                        float* __restrict__ scores_out,
                                                                        int refresh_tail, int tile_pages) {
  constexpr int kE = Elem<TS>::kVec;                 // mean elements per 16-byte load
  constexpr int kChunks = D / (kE * kRowLanes);      // 16-byte loads per lane per row
  constexpr int kDepth = UNIQUE_SCORE_DEPTH;          // records in flight per wave (deeper rings measured no faster)

  const int b = blockIdx.y;
  const int tile0 = blockIdx.x * tile_pages;  // tile_pages logical pages per workgroup (a power of two, 8..256)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;  // wave: scalar
  const int row8 = lane / kRowLanes, cl = lane % kRowLanes;
  // which head and which page of a step this lane's row is; both fixed for the whole kernel
  int hkv, page_in_step, pages_per_step, wave_slot, wave_slots;
  if (c.Hkv >= kRowsPerWave) {
    const int slots_per_page = c.Hkv / kRowsPerWave;  // a page record spans this many wave steps
    hkv = (wave % slots_per_page) * kRowsPerWave + row8;
    page_in_step = 0;
    pages_per_step = 1;
    wave_slot = wave / slots_per_page;
    wave_slots = kScoreWaves / slots_per_page;
  } else {
    pages_per_step = kRowsPerWave / c.Hkv;
    hkv = row8 % c.Hkv;
    page_in_step = row8 / c.Hkv;
    wave_slot = wave;
    wave_slots = kScoreWaves;
  }
  const int step_pages = wave_slots * pages_per_step;  // pages the workgroup advances per step

  // The sequence length, the page ids of all of this wave's steps (lane L holds entry L = step *
  // pages_per_step + page_in_step) and the queries are requested together; the page-table row always has
  // max_pages readable entries, so its load does not have to wait for the page count.
  const int32_t* pt = c.page_table + (int64_t)b * c.max_pages;
  int my_page, my_phys_raw = -1;
  {
    const int st = lane / pages_per_step, po = lane % pages_per_step;
    my_page = tile0 + (wave_slot + st * wave_slots) * pages_per_step + po;
    if (my_page < min(tile0 + tile_pages, c.max_pages_hint)) my_phys_raw = pt[my_page];
  }
  const int N = c.seq_lens[b];
  // raw query words of this lane's row: kE elements per chunk, for each of the G heads of the group
  constexpr int kQWords = kE * (int)sizeof(T) / 4;
  uint32_t qraw[G][kChunks][kQWords];
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int j = 0; j < kChunks; ++j) {
      const uint32_t* qsrc = reinterpret_cast<const uint32_t*>(q + ((int64_t)b * c.H + hkv * G + g) * D +
                                                               j * (kE * kRowLanes) + cl * kE);
      if constexpr (kQWords == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(qsrc);
        qraw[g][j][0] = v.x; qraw[g][j][1] = v.y;
      } else {
#pragma unroll
        for (int w = 0; w < kQWords; w += 4) {
          const uint4 v = *reinterpret_cast<const uint4*>(qsrc + w);
          qraw[g][j][w] = v.x; qraw[g][j][w + 1] = v.y; qraw[g][j][w + 2] = v.z; qraw[g][j][w + 3] = v.w;
        }
      }
    }
  }
  const int P = min((N + c.S - 1) / c.S, c.max_pages_hint);  // pages beyond the host bound are ignored
  if (tile0 >= P) return;
  const int tile_end = min(tile0 + tile_pages, P);
  if (refresh_tail && tile_end == P) {  // this workgroup scores the last page: bring its record up to date first
    refresh_tail_record<T, D>(c, b, N, P);
    __threadfence_block();
    __syncthreads();
  }

  // bf16 queries against bf16 means: packed bf16 pairs go straight into v_dot2_f32_bf16 (two products
  // per instruction accumulated in fp32, no unpacking); every other combination multiplies in fp32.
  constexpr bool kDot2 = sizeof(T) == 2 && sizeof(TS) == 2;
  float qv[kDot2 ? 1 : G][kChunks][kE];
  uint32_t qp[kDot2 ? G : 1][kChunks][kE / 2];
  float off[G];

  const char* stats = reinterpret_cast<const char*>(c.page_stats);
  const int64_t std_off = (int64_t)c.Hkv * D * (int64_t)sizeof(TS);  // byte offset of the stds inside a record
  extern __shared__ float tile_scores[];  // [Hkv][tile_pages]

  const int n_steps = (tile_end - (tile0 + wave_slot * pages_per_step) + step_pages - 1) / step_pages;  // may be <= 0
  const int my_phys = (my_page < tile_end && my_phys_raw >= 0 && (int64_t)my_phys_raw < c.num_phys) ? my_phys_raw : -1;

  // A ring of kDepth records is in flight per wave. The loads are unconditional -- a step past the end
  // of the tile, or one whose page id is invalid, reads the first bytes of the statistics instead, which
  // costs no memory traffic -- so the loop is straight-line code and every wait names the exact number of
  // requests that may stay outstanding.
  Raw16 ring[kDepth][kChunks];
  float ring_sd[kDepth];
  int ring_phys[kDepth];
  auto issue = [&](int st, Raw16(&md)[kChunks], float& sd, int& phys) {
    const int src_lane = min(st * pages_per_step + page_in_step, kWave - 1);
    const int ph = pages_per_step == 1 ? __builtin_amdgcn_readlane(my_phys, min(st, kWave - 1))
                                       : __shfl(my_phys, src_lane, kWave);
    phys = st < n_steps ? ph : -1;
    const char* rec = stats + (int64_t)max(phys, 0) * c.rec_bytes;
    const TS* row = phys >= 0 ? reinterpret_cast<const TS*>(rec) + hkv * D + cl * kE : reinterpret_cast<const TS*>(stats);
#pragma unroll
    for (int j = 0; j < kChunks; ++j) md[j] = load_raw_stream(row + j * (kE * kRowLanes), kNT);
    sd = reinterpret_cast<const float*>(rec + std_off)[hkv];
  };
  auto consume = [&](int st, const Raw16(&mc)[kChunks], float sd_cur, int phys_cur) {
    float mf[kDot2 ? 1 : kChunks][kE];
    if constexpr (!kDot2) {
#pragma unroll
      for (int j = 0; j < kChunks; ++j) unpack_raw(mc[j], mf[j], (const TS*)nullptr);
    }
    float best = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float dot = 0.f;
      if constexpr (kDot2) {
#pragma unroll
        for (int j = 0; j < kChunks; ++j) {
          const uint32_t mw[4] = {mc[j].v.x, mc[j].v.y, mc[j].v.z, mc[j].v.w};
#pragma unroll
          for (int i = 0; i < 4; ++i)
            dot = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, qp[g][j][i]),
                                                  __builtin_bit_cast(bf16x2_t, mw[i]), dot, false);
        }
      } else {
#pragma unroll
        for (int j = 0; j < kChunks; ++j)
#pragma unroll
          for (int i = 0; i < kE; ++i) dot = fmaf(qv[g][j][i], mf[j][i], dot);
      }
      dot = group_allreduce<kRowLanes>(dot, OpSum());
      const float sc = fmaf(off[g], sd_cur, dot);
      best = (g == 0) ? sc : fmaxf(best, sc);
    }
    const int p = tile0 + (wave_slot + st * wave_slots) * pages_per_step + page_in_step;
    // a page whose table entry points outside the pool gets NaN, which ranks below every score
    if (cl == 0 && p < tile_end) tile_scores[hkv * tile_pages + p - tile0] = phys_cur >= 0 ? best : __uint_as_float(0x7fc00000u);
  };
#pragma unroll
  for (int u = 0; u < kDepth; ++u) issue(u, ring[u], ring_sd[u], ring_phys[u]);
  // the queries arrived with the page ids; they are unpacked while the first records are on their way
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float qq = 0.f;
#pragma unroll
    for (int j = 0; j < kChunks; ++j) {
      float qf[kE];
      unpack_q<kE>(qraw[g][j], qf, (const T*)nullptr);
#pragma unroll
      for (int i = 0; i < kE; ++i) qq = fmaf(qf[i], qf[i], qq);
      if constexpr (kDot2) {
#pragma unroll
        for (int i = 0; i < kE / 2; ++i) qp[g][j][i] = qraw[g][j][i];
      } else {
#pragma unroll
        for (int i = 0; i < kE; ++i) qv[g][j][i] = qf[i];
      }
    }
    qq = group_allreduce<kRowLanes>(qq, OpSum());
    off[g] = lambda * sqrtf(qq);
  }
  for (int st0 = 0; st0 < n_steps; st0 += kDepth) {
#pragma unroll
    for (int u = 0; u < kDepth; ++u) {
      consume(st0 + u, ring[u], ring_sd[u], ring_phys[u]);
      issue(st0 + u + kDepth, ring[u], ring_sd[u], ring_phys[u]);
    }
  }
  __syncthreads();
  // the tile's scores leave as one contiguous run per KV head
  const int tile_len = tile_end - tile0;
  const int tshift = __ffs(tile_pages) - 1;  // the tile is a power of two
  for (int idx = threadIdx.x; idx < c.Hkv * tile_pages; idx += kScoreWaves * kWave) {
    const int h = idx >> tshift, pp = idx & (tile_pages - 1);
    if (pp < tile_len) {
      const float v = tile_scores[idx];
      scores[((int64_t)b * c.Hkv + h) * score_stride + tile0 + pp] = v;
      if (scores_out) scores_out[((int64_t)b * c.Hkv + h) * c.max_pages + tile0 + pp] = v;
    }
  }
}

template <typename T, int D, int G>
hipError_t launch_t(const CacheView& cv, const void* q, float lambda, float* scores, int stride, float* out,
                    bool refresh_tail, hipStream_t st) {
  const CacheView& c = cv;
  const bool nt = (int64_t)c.B * c.max_pages_hint * c.rec_bytes > kStreamNtBytes;
  // Small tiles balance ragged batches and small launches over the 256 CUs; larger ones save prologues
  // (fewer, longer streams). A tile is doubled while the batch is known to fill the chip with FULL tiles
  // of the larger size: either every sequence is long enough by the host's lower bound (at least two
  // workgroups of equal work per CU), or the launch has workgroups to spare whatever the lengths are.
  // A wave keeps the page ids of all its steps in its 64 lanes, which caps the tile at 64 pages per wave
  // slot (4 slots up to 8 KV heads, 2 at 16, 1 when one wave steps through all 32 heads of a page alone).
  const int wave_slots = c.Hkv <= 8 ? kScoreWaves : kScoreWaves * kRowsPerWave / c.Hkv;
  const int max_tile = 64 * wave_slots;
  constexpr int kMinTile = 8, kNumCUs = 256;
  int tile = 32;
  while (2 * tile <= max_tile &&
         ((int64_t)c.B * (c.min_pages_hint / (2 * tile)) >= UNIQUE_SCORE_FULL_TILES ||
          (int64_t)c.B * ((c.max_pages_hint + 2 * tile - 1) / (2 * tile)) >= UNIQUE_SCORE_FAT_GRID))
    tile *= 2;
  // a launch too small to give every CU a workgroup is all latency: shorter tiles spread it over more CUs
  // (one sequence of 32K tokens: 10.7 us with 32-page tiles, 8.7 us with 8-page tiles)
  while (tile > kMinTile && (int64_t)c.B * ((c.max_pages_hint + tile - 1) / tile) < kNumCUs) tile /= 2;
  dim3 grid((c.max_pages_hint + tile - 1) / tile, c.B), block(kScoreWaves * kWave);
  const size_t lds = (size_t)c.Hkv * tile * sizeof(float);
  auto go = [&](auto kernel) {
    kernel<<<grid, block, lds, st>>>(c, reinterpret_cast<const T*>(q), lambda, scores, stride, out, refresh_tail,
                                     tile);
  };
  if (c.stats_bf16) {
    if (nt) go(page_score_kernel<T, bf16_t, D, G, true>);
    else go(page_score_kernel<T, bf16_t, D, G, false>);
  } else {
    if (nt) go(page_score_kernel<T, float, D, G, true>);
    else go(page_score_kernel<T, float, D, G, false>);
  }
  return hipGetLastError();
}

template <typename T, int D>
hipError_t dispatch_g(const CacheView& c, const void* q, float lambda, float* scores, int stride, float* out,
                      bool refresh_tail, hipStream_t st) {
  switch (c.H / c.Hkv) {
    case 1: return launch_t<T, D, 1>(c, q, lambda, scores, stride, out, refresh_tail, st);
    case 2: return launch_t<T, D, 2>(c, q, lambda, scores, stride, out, refresh_tail, st);
    case 4: return launch_t<T, D, 4>(c, q, lambda, scores, stride, out, refresh_tail, st);
    case 8: return launch_t<T, D, 8>(c, q, lambda, scores, stride, out, refresh_tail, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool score_supported(int dtype, int D, int G, int Hkv) {
  if (!(dtype == 0 || dtype == 1) || !(D == 64 || D == 128)) return false;
  if (!(G == 1 || G == 2 || G == 4 || G == 8)) return false;
  // a wave covers 8 head rows per step; the 4 waves of a workgroup must tile whole page records
  return Hkv == 1 || Hkv == 2 || Hkv == 4 || Hkv == 8 || Hkv == 16 || Hkv == 32;
}

hipError_t launch_score(const CacheView& c, const void* d_q, float lambda, float* d_scores, int score_stride,
                        float* d_scores_out, bool refresh_tail, hipStream_t stream) {
  if (c.dtype == 0) {
    return c.D == 64 ? dispatch_g<float, 64>(c, d_q, lambda, d_scores, score_stride, d_scores_out, refresh_tail, stream)
                     : dispatch_g<float, 128>(c, d_q, lambda, d_scores, score_stride, d_scores_out, refresh_tail, stream);
  }
  return c.D == 64 ? dispatch_g<bf16_t, 64>(c, d_q, lambda, d_scores, score_stride, d_scores_out, refresh_tail, stream)
                   : dispatch_g<bf16_t, 128>(c, d_q, lambda, d_scores, score_stride, d_scores_out, refresh_tail, stream);
}

}  // namespace unique
