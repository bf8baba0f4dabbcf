/* Plain C99 client of include/unique.h: proves that the header is C, that the library links from C without
 * any C++ or torch in sight, and that host-side validation answers before anything touches a device.
 * Built and run by tests/test_boundary_cpu.py (no GPU needed). */
#include <stdio.h>
#include <string.h>

#include "unique.h"

int main(void) {
  unique_cache_desc d;
  size_t bytes = 0;
  memset(&d, 0, sizeof d);
  if (strncmp(unique_version(), "unique-gfx950", 13) != 0) return 1;
  if (unique_workspace_bytes(NULL, 16, &bytes) != UNIQUE_ERR_INVALID_ARG) return 2;
  if (unique_dense_paged_decode(&d, NULL, 0.0f, NULL, NULL, NULL, 0, NULL) != UNIQUE_ERR_INVALID_ARG) return 3;
  if (strlen(unique_last_error()) == 0) return 4;
  d.dtype = UNIQUE_DTYPE_BF16; d.num_q_heads = 32; d.num_kv_heads = 8; d.head_dim = 128; d.page_size = 16; d.batch = 2;
  d.max_pages_per_seq = 64; d.num_phys_pages = 128; d.stats_dtype = UNIQUE_DTYPE_F32;
  if (unique_page_stats_record_bytes(&d) != 8 * 128 * 4 + 128) return 5;
  d.head_dim = 96; /* not compiled */
  d.k_cache = (const void*)0x1000; d.v_cache = (const void*)0x2000; d.page_table = (const int32_t*)0x3000;
  d.seq_lens = (const int32_t*)0x4000;
  if (unique_dense_paged_decode(&d, (const void*)0x5000, 0.0f, (void*)0x6000, NULL, (void*)0x7000, 1u << 20, NULL) !=
      UNIQUE_ERR_UNSUPPORTED)
    return 6;
  printf("%s: %s / %s\n", unique_version(), unique_status_string(UNIQUE_ERR_UNSUPPORTED), unique_last_error());
  return 0;
}
