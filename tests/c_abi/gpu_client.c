/* A C client that runs the whole path on the GPU through include/unique.h with nothing but the HIP runtime's
 * C API around it (no Python, no torch): bulk statistics, one decode step (scores, top-k, sparse attention)
 * and the dense comparison on a small fp32 problem, each checked against the definitions evaluated on the host
 * in double precision (Eq. 1, 2, 6, 5 and 4 of the paper, written out below for this one case).
 * Built by __graft_entry__.build(); run by the GPU tests. Exit code 0 = all checks passed. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "unique.h"

enum { B = 2, H = 4, HKV = 2, G = 2, D = 64, S = 8, MAXP = 4, POOL = 8, TOPK = 2 };
static const int kSeqLens[B] = {29, 8};
static const int kPageTable[B][MAXP] = {{5, 2, 7, 0}, {3, 0, 0, 0}};

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 10; } } while (0)
#define LIB_OK(x) do { int s_ = (x); if (s_ != UNIQUE_OK) { printf("library error %d (%s) at line %d\n", s_, unique_last_error(), __LINE__); return 11; } } while (0)

static unsigned lcg_state = 12345u;
static float lcg(void) {  /* deterministic values in [-1, 1) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return (float)((lcg_state >> 8) & 0xffffu) / 32768.0f - 1.0f;
}

static float k_host[POOL][HKV][S][D], v_host[POOL][HKV][S][D], q_host[B][H][D];

static int pages_of(int b) { return (kSeqLens[b] + S - 1) / S; }
static int tokens_in(int b, int p) { int n = kSeqLens[b] - p * S; return n < S ? n : S; }

/* Eq. 5 / Eq. 4 over the given logical pages, in double */
static void attend(int b, int h, const int* pages, int np, double* out, double* lse) {
  const int hkv = h / G;
  double m = -INFINITY, l = 0.0, acc[D];
  int i, t, d;
  memset(acc, 0, sizeof acc);
  for (i = 0; i < np; ++i)
    for (t = 0; t < tokens_in(b, pages[i]); ++t) {
      const float* kr = k_host[kPageTable[b][pages[i]]][hkv][t];
      double s = 0.0;
      for (d = 0; d < D; ++d) s += (double)q_host[b][h][d] * kr[d];
      s /= sqrt((double)D);
      if (s > m) { const double sc = exp(m - s); l *= sc; for (d = 0; d < D; ++d) acc[d] *= sc; m = s; }
      { const double w = exp(s - m); const float* vr = v_host[kPageTable[b][pages[i]]][hkv][t];
        l += w; for (d = 0; d < D; ++d) acc[d] += w * vr[d]; }
    }
  for (d = 0; d < D; ++d) out[d] = acc[d] / l;
  *lse = m + log(l);
}

int main(void) {
  unique_cache_desc desc;
  void *d_k, *d_v, *d_q, *d_stats, *d_pt, *d_len, *d_sel, *d_cnt, *d_out, *d_lse, *d_ws, *d_outd, *d_lsed;
  static float out_gpu[B][H][D], lse_gpu[B][H], outd_gpu[B][H][D], lsed_gpu[B][H];
  int sel_gpu[B][HKV][TOPK], cnt_gpu[B][HKV];
  size_t ws_bytes = 0;
  int64_t rec;
  int b, h, p, t, d, g, n_dev = 0, bad = 0;

  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1) { printf("no GPU\n"); return 77; }
  for (p = 0; p < POOL; ++p) for (h = 0; h < HKV; ++h) for (t = 0; t < S; ++t) for (d = 0; d < D; ++d) {
    k_host[p][h][t][d] = lcg() + 0.25f * (float)((p * 3 + h) % 5 - 2);   /* a per-(page, head) shift, so pages differ */
    v_host[p][h][t][d] = lcg();
  }
  for (b = 0; b < B; ++b) for (h = 0; h < H; ++h) for (d = 0; d < D; ++d) q_host[b][h][d] = lcg();

  memset(&desc, 0, sizeof desc);
  desc.dtype = UNIQUE_DTYPE_F32; desc.num_q_heads = H; desc.num_kv_heads = HKV; desc.head_dim = D; desc.page_size = S;
  desc.batch = B; desc.max_pages_per_seq = MAXP; desc.num_phys_pages = POOL; desc.stats_dtype = UNIQUE_DTYPE_F32;
  rec = unique_page_stats_record_bytes(&desc);
  HIP_OK(hipMalloc(&d_k, sizeof k_host)); HIP_OK(hipMalloc(&d_v, sizeof v_host)); HIP_OK(hipMalloc(&d_q, sizeof q_host));
  HIP_OK(hipMalloc(&d_stats, (size_t)rec * POOL)); HIP_OK(hipMalloc(&d_pt, sizeof kPageTable)); HIP_OK(hipMalloc(&d_len, sizeof kSeqLens));
  HIP_OK(hipMalloc(&d_sel, sizeof sel_gpu)); HIP_OK(hipMalloc(&d_cnt, sizeof cnt_gpu));
  HIP_OK(hipMalloc(&d_out, sizeof out_gpu)); HIP_OK(hipMalloc(&d_lse, sizeof lse_gpu));
  HIP_OK(hipMalloc(&d_outd, sizeof outd_gpu)); HIP_OK(hipMalloc(&d_lsed, sizeof lsed_gpu));
  HIP_OK(hipMemcpy(d_k, k_host, sizeof k_host, hipMemcpyHostToDevice)); HIP_OK(hipMemcpy(d_v, v_host, sizeof v_host, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_q, q_host, sizeof q_host, hipMemcpyHostToDevice)); HIP_OK(hipMemcpy(d_pt, kPageTable, sizeof kPageTable, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_len, kSeqLens, sizeof kSeqLens, hipMemcpyHostToDevice));
  desc.k_cache = d_k; desc.v_cache = d_v; desc.page_stats = d_stats; desc.page_table = (const int32_t*)d_pt; desc.seq_lens = (const int32_t*)d_len;
  LIB_OK(unique_workspace_bytes(&desc, TOPK, &ws_bytes));
  HIP_OK(hipMalloc(&d_ws, ws_bytes ? ws_bytes : 256));

  LIB_OK(unique_update_page_stats(&desc, NULL, NULL, 0, NULL));
  LIB_OK(unique_decode_step(&desc, d_q, TOPK, 0.5f, 0.0f, 1, (int32_t*)d_sel, (int32_t*)d_cnt, d_out, (float*)d_lse, d_ws, ws_bytes, NULL));
  LIB_OK(unique_dense_paged_decode(&desc, d_q, 0.0f, d_outd, (float*)d_lsed, d_ws, ws_bytes, NULL));
  HIP_OK(hipDeviceSynchronize());
  HIP_OK(hipMemcpy(sel_gpu, d_sel, sizeof sel_gpu, hipMemcpyDeviceToHost)); HIP_OK(hipMemcpy(cnt_gpu, d_cnt, sizeof cnt_gpu, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(out_gpu, d_out, sizeof out_gpu, hipMemcpyDeviceToHost)); HIP_OK(hipMemcpy(lse_gpu, d_lse, sizeof lse_gpu, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(outd_gpu, d_outd, sizeof outd_gpu, hipMemcpyDeviceToHost)); HIP_OK(hipMemcpy(lsed_gpu, d_lsed, sizeof lsed_gpu, hipMemcpyDeviceToHost));

  for (b = 0; b < B; ++b) for (h = 0; h < HKV; ++h) {
    const int P = pages_of(b), kb = TOPK < P ? TOPK : P;
    double score[MAXP];
    int order[MAXP], i, j, all[MAXP];
    for (p = 0; p < P; ++p) {  /* Eq. 1, Eq. 2, Eq. 6 for page p */
      const int n = tokens_in(b, p);
      double mean[D], var = 0.0, best = -INFINITY;
      for (d = 0; d < D; ++d) {
        double s1 = 0.0, s2 = 0.0;
        for (t = 0; t < n; ++t) s1 += k_host[kPageTable[b][p]][h][t][d];
        mean[d] = s1 / n;
        for (t = 0; t < n; ++t) { const double dv = k_host[kPageTable[b][p]][h][t][d] - mean[d]; s2 += dv * dv; }
        var += s2 / n;
      }
      for (g = 0; g < G; ++g) {
        double dot = 0.0, qq = 0.0;
        for (d = 0; d < D; ++d) { const double qd = q_host[b][h * G + g][d]; dot += qd * mean[d]; qq += qd * qd; }
        dot += 0.5 * sqrt(qq) * sqrt(var);
        if (dot > best) best = dot;
      }
      score[p] = best; order[p] = p; all[p] = p;
    }
    for (i = 0; i < P; ++i) for (j = i + 1; j < P; ++j)   /* (score desc, page asc) */
      if (score[order[j]] > score[order[i]] || (score[order[j]] == score[order[i]] && order[j] < order[i])) { const int x = order[i]; order[i] = order[j]; order[j] = x; }
    if (kb > 1 && order[0] > order[1]) { const int x = order[0]; order[0] = order[1]; order[1] = x; }  /* ascending set of 2 */
    if (cnt_gpu[b][h] != kb) { printf("count (%d,%d): %d != %d\n", b, h, cnt_gpu[b][h], kb); ++bad; }
    for (i = 0; i < TOPK; ++i) {
      const int want = i < kb ? order[i] : -1;
      if (sel_gpu[b][h][i] != want) { printf("selection (%d,%d)[%d]: %d != %d\n", b, h, i, sel_gpu[b][h][i], want); ++bad; }
    }
    for (g = 0; g < G; ++g) {
      double o[D], lse;
      attend(b, h * G + g, order, kb, o, &lse);
      for (d = 0; d < D; ++d) if (fabs(out_gpu[b][h * G + g][d] - o[d]) > 1e-4) { if (bad < 20) printf("sparse out (%d,%d,%d)\n", b, h * G + g, d); ++bad; }
      if (fabs(lse_gpu[b][h * G + g] - lse) > 1e-4 * fmax(1.0, fabs(lse))) { printf("sparse lse (%d,%d)\n", b, h * G + g); ++bad; }
      attend(b, h * G + g, all, P, o, &lse);
      for (d = 0; d < D; ++d) if (fabs(outd_gpu[b][h * G + g][d] - o[d]) > 1e-4) { if (bad < 20) printf("dense out (%d,%d,%d)\n", b, h * G + g, d); ++bad; }
      if (fabs(lsed_gpu[b][h * G + g] - lse) > 1e-4 * fmax(1.0, fabs(lse))) { printf("dense lse (%d,%d)\n", b, h * G + g); ++bad; }
    }
  }
  printf("%s: %d mismatches\n", unique_version(), bad);
  return bad ? 1 : 0;
}
