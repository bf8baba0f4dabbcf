// Ceiling probe of the profiling build for the page-score kernel: the kernel's memory access with everything else
// taken away. Workgroups of 4 waves take tiles of consecutive logical pages of one sequence, look their physical
// pages up in the page table (lane i of a wave holds the id of the wave's i-th page, as in the score kernel) and
// stream the mean block of every page record -- 16-byte non-temporal loads, each load instruction of a wave
// covering a contiguous 1 KiB -- with kDepth records in flight per wave. No queries, no arithmetic but an xor, no
// scores written. Only bench.py --record-probe calls it; the product library does not contain it.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kWave = 64;
constexpr int kProbeWaves = 4;
typedef unsigned int probe_u32x4 __attribute__((ext_vector_type(4)));

template <int kLoads, int kDepth>
__global__ __launch_bounds__(kProbeWaves* kWave) void record_probe_kernel(const char* __restrict__ stats, int64_t rec_bytes,
                                                                          const int32_t* __restrict__ page_table,
                                                                          int max_pages, int pages, int tile,
                                                                          probe_u32x4* __restrict__ sink) {
  const int b = blockIdx.y, tile0 = blockIdx.x * tile;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
  const int tile_end = min(tile0 + tile, pages);
  const int my_page = tile0 + wave + kProbeWaves * lane;  // wave w takes pages tile0 + w, + 4, + 8, ...
  int my_phys = 0;
  if (my_page < tile_end) my_phys = page_table[(int64_t)b * max_pages + my_page];
  const int n = (tile_end - tile0 - wave + kProbeWaves - 1) / kProbeWaves;  // pages of this wave (<= 64)
  probe_u32x4 acc = {0, 0, 0, 0};
  probe_u32x4 buf[kDepth][kLoads];
  auto issue = [&](int i, probe_u32x4(&bb)[kLoads]) {  // past the wave's last page: that page again (straight-line code)
    const int phys = __builtin_amdgcn_readlane(my_phys, max(min(i, n - 1), 0));
    const char* rec = stats + (int64_t)phys * rec_bytes + lane * 16;
#pragma unroll
    for (int j = 0; j < kLoads; ++j)
      bb[j] = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4*>(rec + j * 1024));
  };
#pragma unroll
  for (int d = 0; d < kDepth; ++d) issue(d, buf[d]);
  for (int i = 0; i < n; i += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
#pragma unroll
      for (int j = 0; j < kLoads; ++j) acc ^= buf[d][j];
      issue(i + d + kDepth, buf[d]);
    }
  }
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) sink[threadIdx.x] = acc;  // never true in practice; keeps the loads alive
}

}  // namespace

// stats: device, num_phys records of rec_bytes each, of which the first loads_per_record KiB are read (2 or 4);
// page_table: device int32 [batch][max_pages], every entry of the first `pages` columns in [0, num_phys);
// tile: pages per workgroup, a power of two in 32..256; depth: records in flight per wave, 2, 4 or 8;
// sink: device, 4 KiB, never written in practice. Returns 0, or a hipError_t (hipErrorInvalidValue for bad arguments).
extern "C" int unique_debug_record_probe(const void* stats, int64_t rec_bytes, int loads_per_record,
                                         const int32_t* page_table, int max_pages, int pages, int batch, int tile,
                                         int depth, void* sink, void* stream) {
  if (!stats || !page_table || !sink || batch < 1 || batch > 65535 || pages < 1 || pages > max_pages) return (int)hipErrorInvalidValue;
  if (!(loads_per_record == 2 || loads_per_record == 4) || rec_bytes < (int64_t)loads_per_record * 1024 || rec_bytes % 16 != 0)
    return (int)hipErrorInvalidValue;
  if (tile < 32 || tile > 256 || (tile & (tile - 1)) != 0) return (int)hipErrorInvalidValue;
  const dim3 grid((pages + tile - 1) / tile, batch), block(kProbeWaves * kWave);
  auto go = [&](auto kernel) {
    kernel<<<grid, block, 0, (hipStream_t)stream>>>(reinterpret_cast<const char*>(stats), rec_bytes, page_table, max_pages,
                                                    pages, tile, reinterpret_cast<probe_u32x4*>(sink));
  };
  if (loads_per_record == 4 && depth == 2) go(record_probe_kernel<4, 2>);
  else if (loads_per_record == 4 && depth == 4) go(record_probe_kernel<4, 4>);
  else if (loads_per_record == 4 && depth == 8) go(record_probe_kernel<4, 8>);
  else if (loads_per_record == 2 && depth == 2) go(record_probe_kernel<2, 2>);
  else if (loads_per_record == 2 && depth == 4) go(record_probe_kernel<2, 4>);
  else if (loads_per_record == 2 && depth == 8) go(record_probe_kernel<2, 8>);
  else return (int)hipErrorInvalidValue;
  return (int)hipGetLastError();
}
