// Paged decode attention over a list of logical pages per (sequence, KV head):
//   Eq. 5 of the paper when the list is the selected top-k set, Eq. 4 when it is every page.
//
// Split-K: the page list of a row is cut into chunks; one workgroup (4 waves) handles one chunk for all
// G query heads of the KV head at once, so every K/V byte is read exactly once per step. Inside a wave
// each lane reads 16-byte chunks of K and V rows (a wave-wide load covers a contiguous 1 KiB of the
// page), the q.k dot products are reduced across the D/vec lanes that share a token with DPP row
// operations, and each group of lanes that shares a token row keeps its own online-softmax state, so
// the inner loop has no cross-row communication. States are merged (log-sum-exp) across lane groups,
// then across the 4 waves through LDS, and the chunk's partial (o, m, l) goes to the workspace; a
// second small kernel merges the chunks of a row and writes the output in the cache dtype (a row with
// a single chunk is written by the first kernel itself and the second is not launched).
// Logits are kept in the log2 domain (q is pre-multiplied by sm_scale * log2 e) so exp is one v_exp_f32.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace unique {
namespace {

#ifndef UNIQUE_DEC_WAVES
#define UNIQUE_DEC_WAVES 4
#endif
constexpr int kDecWaves = UNIQUE_DEC_WAVES;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for "no logit seen yet"
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// With a single chunk per row there is nothing to merge: the partial kernel writes the attention output
// itself, with the arithmetic of the merge kernel (a scale of exp2(0) = 1), so the result is the same bits.
template <typename T>
__device__ __forceinline__ void write_final(const CacheView& c, T* out, float* lse_out, int b, int h, int d, int D,
                                            float o, float M, float L) {
  const bool any = L > 0.f;
  store_elem(out + ((int64_t)b * c.H + h) * D + d, any ? o / L : 0.f);
  if (lse_out && d == 0) lse_out[(int64_t)b * c.H + h] = any ? (M + log2f(L)) * kLn2 : -INFINITY;
}

template <typename T, int D, int S, int G>
__global__ __launch_bounds__(kDecWaves* kWave) void paged_decode_partial_kernel(
    CacheView c, const T* __restrict__ q, const int32_t* __restrict__ sel_pages,
    const int32_t* __restrict__ sel_count, int sel_stride, int pages_per_split, int num_splits, float scale_log2,
    float* __restrict__ part_o /*[rows][num_splits][G][D]*/, float* __restrict__ part_ml /*[rows][num_splits][G][2]*/,
    T* __restrict__ out, float* __restrict__ lse_out /* written directly when num_splits == 1 */) {
  constexpr int kVec = Elem<T>::kVec;
  constexpr int kLanesPerTok = D / kVec;
  constexpr int kTokPerLoad = kWave / kLanesPerTok;
  constexpr int kLoads = S / kTokPerLoad;                       // wave-wide loads per page (K or V)
  constexpr int kTileLoads = kLoads < 4 ? kLoads : 4;           // loads handled per pipeline stage
  constexpr int kTilesPerPage = kLoads / kTileLoads;
  static_assert(S % kTokPerLoad == 0 && kLoads % kTileLoads == 0, "page size / element type combination");

  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  const int row = b * c.Hkv + hkv;
  const int N = c.seq_lens[b];
  const int P = min((N + S - 1) / S, c.max_pages_hint);
  const int cnt = sel_pages ? min(sel_count[row], sel_stride) : P;
  const int begin = split * pages_per_split;
  if (begin >= cnt) {
    if (num_splits == 1) {  // an empty list: the output is defined as zero, the lse as -inf
      for (int idx = threadIdx.x; idx < G * D; idx += kDecWaves * kWave)
        write_final(c, out, lse_out, b, hkv * G + idx / D, idx % D, D, 0.f, 0.f, 0.f);
    }
    return;
  }
  const int end = min(begin + pages_per_split, cnt);

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;  // wave: scalar
  const int tr = lane / kLanesPerTok, ch = lane % kLanesPerTok;

  float qv[G][kVec];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    load_vec(q + ((int64_t)b * c.H + hkv * G + g) * D + ch * kVec, qv[g]);
#pragma unroll
    for (int i = 0; i < kVec; ++i) qv[g][i] *= scale_log2;
  }

  float m[G], l[G], acc[G][kVec];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = kNegBig;
    l[g] = 0.f;
#pragma unroll
    for (int i = 0; i < kVec; ++i) acc[g][i] = 0.f;
  }

  const T* kc = reinterpret_cast<const T*>(c.k_cache);
  const T* vc = reinterpret_cast<const T*>(c.v_cache);
  const int64_t lane_off = ch * kVec;

  // entries of this chunk are dealt to the waves round-robin; a wave looks up 64 of them at a time
  for (int e0 = begin + wave; e0 < end; e0 += kDecWaves * kWave) {
    int my_phys = 0, my_ntok = 0;
    {
      const int e = e0 + lane * kDecWaves;
      if (e < end) {
        const int lp = sel_pages ? sel_pages[(int64_t)row * sel_stride + e] : e;
        if (lp >= 0 && lp < P) {
          const int ph = c.page_table[(int64_t)b * c.max_pages + lp];
          if (ph >= 0 && (int64_t)ph < c.num_phys) {
            my_phys = ph;
            my_ntok = min(S, N - lp * S);
          }
        }
      }
    }
    const int n_ent = min(kWave, (end - e0 + kDecWaves - 1) / kDecWaves);
    const int n_tiles = n_ent * kTilesPerPage;

    Raw16 kr[kTileLoads], vr[kTileLoads], kn[kTileLoads], vn[kTileLoads];
    int ntok_cur = 0, ntok_nxt = 0, tbase_cur = 0, tbase_nxt = 0;
    auto issue = [&](int it, Raw16(&kd)[kTileLoads], Raw16(&vd)[kTileLoads], int& ntok, int& tbase) {
      const int ent = it / kTilesPerPage;
      const int phys = __builtin_amdgcn_readlane(my_phys, ent);
      ntok = __builtin_amdgcn_readlane(my_ntok, ent);
      tbase = (it % kTilesPerPage) * kTileLoads * kTokPerLoad;
      const int64_t page_off = (int64_t)phys * c.kv_page_stride + (int64_t)hkv * c.kv_head_stride + lane_off;
#pragma unroll
      for (int j = 0; j < kTileLoads; ++j) {
        const int tok = tbase + j * kTokPerLoad + tr;
        if (tok < ntok) {
          kd[j] = load_raw_stream(kc + page_off + (int64_t)tok * D, c.stream_nt);
          vd[j] = load_raw_stream(vc + page_off + (int64_t)tok * D, c.stream_nt);
        } else {
          kd[j] = zero_raw();
          vd[j] = zero_raw();
        }
      }
    };

    issue(0, kr, vr, ntok_cur, tbase_cur);
    for (int it = 0; it < n_tiles; ++it) {
      if (it + 1 < n_tiles) issue(it + 1, kn, vn, ntok_nxt, tbase_nxt);

      // logits of this lane group's tokens for the G heads
      float s[kTileLoads][G];
#pragma unroll
      for (int j = 0; j < kTileLoads; ++j) {
        float kf[kVec];
        unpack_raw(kr[j], kf, (const T*)nullptr);
        const bool valid = (tbase_cur + j * kTokPerLoad + tr) < ntok_cur;
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float d = qv[g][0] * kf[0];
#pragma unroll
          for (int i = 1; i < kVec; ++i) d = fmaf(qv[g][i], kf[i], d);
          d = group_allreduce<kLanesPerTok>(d, OpSum());
          s[j][g] = valid ? d : -INFINITY;
        }
      }
      // online softmax update, one state per lane group
      float p[kTileLoads][G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float mx = s[0][g];
#pragma unroll
        for (int j = 1; j < kTileLoads; ++j) mx = fmaxf(mx, s[j][g]);
        const float mnew = fmaxf(m[g], mx);
        const float alpha = fast_exp2(m[g] - mnew);
        m[g] = mnew;
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < kTileLoads; ++j) {
          p[j][g] = fast_exp2(s[j][g] - mnew);
          psum += p[j][g];
        }
        l[g] = fmaf(l[g], alpha, psum);
#pragma unroll
        for (int i = 0; i < kVec; ++i) acc[g][i] *= alpha;
      }
#pragma unroll
      for (int j = 0; j < kTileLoads; ++j) {
        float vf[kVec];
        unpack_raw(vr[j], vf, (const T*)nullptr);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int i = 0; i < kVec; ++i) acc[g][i] = fmaf(p[j][g], vf[i], acc[g][i]);
      }

#pragma unroll
      for (int j = 0; j < kTileLoads; ++j) { kr[j] = kn[j]; vr[j] = vn[j]; }
      ntok_cur = ntok_nxt;
      tbase_cur = tbase_nxt;
    }
  }

  // merge the lane groups of the wave (they hold disjoint token subsets)
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float M = cross_group_allreduce<kLanesPerTok>(m[g], OpMax());
    const float sc = fast_exp2(m[g] - M);
    m[g] = M;
    l[g] = cross_group_allreduce<kLanesPerTok>(l[g] * sc, OpSum());
#pragma unroll
    for (int i = 0; i < kVec; ++i) acc[g][i] = cross_group_allreduce<kLanesPerTok>(acc[g][i] * sc, OpSum());
  }

  // merge the waves of the workgroup through LDS
  __shared__ float sm_acc[kDecWaves][G][D];
  __shared__ float sm_m[kDecWaves][G], sm_l[kDecWaves][G];
  if (tr == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int i = 0; i < kVec; ++i) sm_acc[wave][g][ch * kVec + i] = acc[g][i];
  }
  if (lane == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) { sm_m[wave][g] = m[g]; sm_l[wave][g] = l[g]; }
  }
  __syncthreads();
  const int64_t pbase = (int64_t)row * num_splits + split;
  for (int idx = threadIdx.x; idx < G * D; idx += kDecWaves * kWave) {
    const int g = idx / D, d = idx % D;
    float M = sm_m[0][g];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) M = fmaxf(M, sm_m[w][g]);
    float o = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float sc = fast_exp2(sm_m[w][g] - M);
      o = fmaf(sm_acc[w][g][d], sc, o);
      L = fmaf(sm_l[w][g], sc, L);
    }
    if (num_splits == 1) {
      write_final(c, out, lse_out, b, hkv * G + g, d, D, o, M, L);
    } else {
      part_o[(pbase * G + g) * D + d] = o;
      if (d == 0) {
        part_ml[(pbase * G + g) * 2 + 0] = M;
        part_ml[(pbase * G + g) * 2 + 1] = L;
      }
    }
  }
}


// ---- bf16 caches: the q.k products of a tile of 16 tokens run on the matrix cores ----
// v_mfma_f32_16x16x32_bf16 computes D[m][n] += sum_k A[m][k] B[k][n] with A rows m = lane % 16, B columns
// n = lane % 16, each lane supplying 8 consecutive k of its 16-lane group, and the result held as
// D[4*(lane/16) + i][lane % 16] in register i. With A = the G query heads (rows >= G are zero) and
// B = the keys of 16 token slots, lanes 0..15 end up with the logits of one token each for heads 0..3
// (lanes 16..31 for heads 4..7). A lane reads, for MFMA step s, the 16-byte chunk 4*s + lane/16 of
// its token's key, so the contraction order inside a step is whatever the hardware pairs up -- the
// same for A and B. Softmax runs on those lanes (one token per lane, tokens reduced across the 16
// lanes with DPP), the probabilities go through 1 KiB of LDS per wave to the row layout in which V
// was loaded (a lane owns a 16-byte chunk of a token's value), and the PV products stay on the
// vector ALUs. This removes the unpack + FMA + lane-reduction work of the q.k stage, which made the
// all-VALU kernel issue-bound (VALU busy 67 % on the dense stream).
// Profiling build (-DUNIQUE_DEC_STAMPS, a second library next to the product one): every wave of the matrix-core
// kernel records the 100 MHz wall clock at kernel entry, once its page ids are resolved, after its first tile, at
// the end of its loop and after its stores, after every tile, and the compute unit it ran on, into a device array
// that unique_debug_dec_stamps() hands out; unique_debug_gather_probe() (bottom of this file) is the bare memory
// access of the kernel. The product build has none of it.
#ifdef UNIQUE_DEC_STAMPS
constexpr int kStampSlots = 32, kStampWaves = 1 << 14;
__device__ unsigned long long g_dec_stamps[kStampWaves][kStampSlots];
#define DEC_STAMP(slot)                                                                                         \
  do {                                                                                                          \
    const int sw_ = ((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * kDecWaves + wave;          \
    if (lane == 0 && sw_ < kStampWaves) g_dec_stamps[sw_][slot] = wall_clock64();                               \
  } while (0)
// the stamp is taken only once `value` (a 32-bit register) has been produced
#define DEC_STAMP_AFTER(slot, value)                 \
  do {                                               \
    asm volatile("" ::"v"(value) : "memory");        \
    DEC_STAMP(slot);                                 \
  } while (0)
#else
#define DEC_STAMP(slot) do {} while (0)
#define DEC_STAMP_AFTER(slot, value) do {} while (0)
#endif

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8_t as_bf16x8(const Raw16& r) {
  return __builtin_bit_cast(bf16x8_t, r.v);
}

#ifndef UNIQUE_DEC_BUFFERS
#define UNIQUE_DEC_BUFFERS 2
#endif
constexpr int kDecBuffers = UNIQUE_DEC_BUFFERS;  // register tiles per wave: one being consumed, the others in flight

// kNT: K and V are read with non-temporal loads (a launch that streams more than the caches hold).
template <int D, int S, int G, bool kNT>
__global__ __launch_bounds__(kDecWaves* kWave) void paged_decode_partial_mfma_kernel(
    CacheView c, const bf16_t* __restrict__ q, const int32_t* __restrict__ sel_pages,
    const int32_t* __restrict__ sel_count, int sel_stride, int pages_per_split, int num_splits, float scale_log2,
    float* __restrict__ part_o, float* __restrict__ part_ml, bf16_t* __restrict__ out, float* __restrict__ lse_out) {
  constexpr int kVec = 8;
  constexpr int kTile = 16;                          // token slots per MFMA tile
  constexpr int kSteps = D / 32;                     // MFMA steps (and K loads per lane) per tile
  constexpr int kLanesPerTok = D / kVec;             // V row layout: lanes covering one value row
  constexpr int kTokPerLoad = kWave / kLanesPerTok;
  constexpr int kVLoads = kTile / kTokPerLoad;       // V loads per lane per tile
  constexpr int kGPad = G < 4 ? 4 : G;               // floats per token slot in the LDS exchange
  constexpr int kGroups = (G + 3) / 4;               // 16-lane groups that hold real heads
  static_assert(G <= 8, "at most 8 query heads per KV head");

  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  const int row = b * c.Hkv + hkv;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;  // wave: scalar
  const int begin = split * pages_per_split;
  DEC_STAMP(0);  // kernel entry
  // the first list entry of this lane is requested together with the lengths (row storage is sel_stride
  // entries long, so the load does not have to wait for the count)
  int first_lp = -1;
  {
    const int e = begin + wave + lane * kDecWaves;
    if (sel_pages && e < min(begin + pages_per_split, sel_stride)) first_lp = sel_pages[(int64_t)row * sel_stride + e];
  }
  const int N = c.seq_lens[b];
  const int P = min((N + S - 1) / S, c.max_pages_hint);
  const int cnt = sel_pages ? min(sel_count[row], sel_stride) : P;
  if (begin >= cnt) {
    if (num_splits == 1) {  // an empty list: the output is defined as zero, the lse as -inf
      for (int idx = threadIdx.x; idx < G * D; idx += kDecWaves * kWave)
        write_final(c, out, lse_out, b, hkv * G + idx / D, idx % D, D, 0.f, 0.f, 0.f);
    }
    return;
  }
  const int end = min(begin + pages_per_split, cnt);

  const int kt = lane % 16, kg = lane / 16;                       // K / logit layout: token slot, lane group
  const int vr_ = lane / kLanesPerTok, vc_ = lane % kLanesPerTok;  // V layout: token row inside a load, chunk

  __shared__ float p_lds[kDecWaves][kTile][kGPad];
  __shared__ float sm_acc[kDecWaves][G][D];
  __shared__ float sm_m[kDecWaves][G], sm_l[kDecWaves][G];

  // A operand: query head kt (zero rows beyond G), the 8 elements of chunk 4*s + kg
  const bf16_t* q_row = q + ((int64_t)b * c.H + hkv * G) * D;  // first query row of the group
  bf16x8_t qa[kSteps];
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    Raw16 r = zero_raw();
    if (kt < G) r = load_raw(q_row + (int64_t)kt * D + (4 * s + kg) * kVec);
    qa[s] = as_bf16x8(r);
  }

  float m[4], l[4];     // softmax state of heads 4*kg + i: m replicated over the 16 lanes, l a per-lane partial sum
#pragma unroll
  for (int i = 0; i < 4; ++i) { m[i] = kNegBig; l[i] = 0.f; }
  float acc[G][kVec];   // this lane's chunk of the output rows, summed over its token rows
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int i = 0; i < kVec; ++i) acc[g][i] = 0.f;

  const bf16_t* kc = reinterpret_cast<const bf16_t*>(c.k_cache);
  const bf16_t* vc = reinterpret_cast<const bf16_t*>(c.v_cache);
  const int64_t head_off = (int64_t)hkv * c.kv_head_stride;
  const int64_t page_stride = c.kv_page_stride;

  for (int e0 = begin + wave; e0 < end; e0 += kDecWaves * kWave) {
    int my_phys = 0, my_ntok = 0;
    {
      const int e = e0 + lane * kDecWaves;
      if (e < end) {
        const int lp = !sel_pages ? e : (e0 == begin + wave ? first_lp : sel_pages[(int64_t)row * sel_stride + e]);
        if (lp >= 0 && lp < P) {
          const int ph = c.page_table[(int64_t)b * c.max_pages + lp];
          if (ph >= 0 && (int64_t)ph < c.num_phys) {
            my_phys = ph;
            my_ntok = min(S, N - lp * S);
          }
        }
      }
    }
    const int n_ent = min(kWave, (end - e0 + kDecWaves - 1) / kDecWaves);
    const int n_tiles = (n_ent * S + kTile - 1) / kTile;
    DEC_STAMP_AFTER(1, my_phys);  // page ids resolved (list entry and page-table entry arrived)

    // slot gs (counted over the wave's entries) -> entry gs / S, token gs % S. Entries at or beyond n_ent
    // were never looked up and carry ntok = 0; so does every slot of a tile at or beyond n_tiles.
    auto slot_info = [&](int tile, int slot, int& phys, int& ntok, int& tok) {
      const int gs = tile * kTile + slot;
      tok = gs % S;
      if constexpr (S >= kTile) {  // one entry per tile: uniform, scalar broadcast
        const int ent = min(tile / (S / kTile), kWave - 1);
        phys = __builtin_amdgcn_readlane(my_phys, ent);
        ntok = tile < n_tiles ? __builtin_amdgcn_readlane(my_ntok, ent) : 0;
      } else {                     // two pages share a tile: per-lane lookup
        const int ent = min(gs / S, kWave - 1);
        phys = __shfl(my_phys, ent, kWave);
        ntok = tile < n_tiles ? __shfl(my_ntok, ent, kWave) : 0;
      }
    };

    // kDecBuffers register tiles: while one is consumed, the loads of the following kDecBuffers - 1 are in flight,
    // so a wave is not paced by one memory round trip per tile. Every load is issued unconditionally -- a slot
    // that has no token (beyond a partial page, an invalid list entry, a tile past the wave's last) reads the
    // group's first query row instead, which is always cached, finite and never attended (its probability is
    // zero) -- so the pipeline is straight-line code and every wait names exactly the requests that may stay in
    // flight; with predicated loads the compiler waited for ALL outstanding loads before each tile, prefetched
    // ones included. Slots beyond a sequence's length are still never read.
    Raw16 kb[kDecBuffers][kSteps], vb[kDecBuffers][kVLoads];
    bool kv[kDecBuffers];
    auto issue = [&](int tile, Raw16(&kd)[kSteps], Raw16(&vd)[kVLoads], bool& kvalid) {
      int phys, ntok, tok;
      slot_info(tile, kt, phys, ntok, tok);
      kvalid = tok < ntok;
      const bf16_t* kp = kvalid ? kc + phys * page_stride + head_off + (int64_t)tok * D + kg * kVec : q_row;
#pragma unroll
      for (int s = 0; s < kSteps; ++s) kd[s] = load_raw_stream(kp + s * (4 * kVec), kNT);
#pragma unroll
      for (int j = 0; j < kVLoads; ++j) {
        slot_info(tile, j * kTokPerLoad + vr_, phys, ntok, tok);
        const bf16_t* vp = tok < ntok ? vc + phys * page_stride + head_off + (int64_t)tok * D + vc_ * kVec : q_row;
        vd[j] = load_raw_stream(vp, kNT);
      }
    };
    auto consume = [&](const Raw16(&kr)[kSteps], const Raw16(&vr)[kVLoads], bool kvalid_cur) {
      f32x4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < kSteps; ++s)
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[s], as_bf16x8(kr[s]), sacc, 0, 0, 0);

      float alpha[4], pr[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float sv = kvalid_cur ? sacc[i] * scale_log2 : -INFINITY;
        const float mx = group_allreduce<16>(sv, OpMax());
        const float mnew = fmaxf(m[i], mx);
        alpha[i] = fast_exp2(m[i] - mnew);
        m[i] = mnew;
        pr[i] = fast_exp2(sv - mnew);
        l[i] = fmaf(l[i], alpha[i], pr[i]);
      }
      // probabilities of the 16 token slots to LDS, [slot][head]
      if (kg < kGroups) *reinterpret_cast<float4*>(&p_lds[wave][kt][4 * kg]) = make_float4(pr[0], pr[1], pr[2], pr[3]);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

      // rescale the running output by alpha of each head (held by lane group g / 4, register g % 4)
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, alpha[g % 4]), 16 * (g / 4)));
#pragma unroll
        for (int i = 0; i < kVec; ++i) acc[g][i] *= a;
      }
#pragma unroll
      for (int j = 0; j < kVLoads; ++j) {
        float vf[kVec];
        unpack_bf16x8(vr[j].v, vf);
        const int ts = j * kTokPerLoad + vr_;
        float pg[kGPad];
#pragma unroll
        for (int g4 = 0; g4 < kGPad; g4 += 4) {
          const float4 t = *reinterpret_cast<const float4*>(&p_lds[wave][ts][g4]);
          pg[g4] = t.x; pg[g4 + 1] = t.y; pg[g4 + 2] = t.z; pg[g4 + 3] = t.w;
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int i = 0; i < kVec; ++i) acc[g][i] = fmaf(pg[g], vf[i], acc[g][i]);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    };

#pragma unroll
    for (int u = 0; u < kDecBuffers - 1; ++u) issue(u, kb[u], vb[u], kv[u]);
    for (int t0 = 0; t0 < n_tiles; t0 += kDecBuffers) {
#pragma unroll
      for (int u = 0; u < kDecBuffers; ++u) {
        constexpr int kAhead = kDecBuffers - 1;
        issue(t0 + u + kAhead, kb[(u + kAhead) % kDecBuffers], vb[(u + kAhead) % kDecBuffers], kv[(u + kAhead) % kDecBuffers]);
        if (u == 0 || t0 + u < n_tiles) consume(kb[u], vb[u], kv[u]);  // uniform
        if (t0 + u == 0) DEC_STAMP_AFTER(2, acc[0][0]);  // first tile consumed (first K/V data arrived)
#ifdef UNIQUE_DEC_STAMPS
        if (t0 + u < n_tiles && t0 + u < kStampSlots - 6) DEC_STAMP_AFTER(6 + t0 + u, acc[0][0]);  // tile t0 + u consumed
        if (t0 + u == 0) {  // which compute unit this wave runs on (HW_ID: bits 8-11 CU, 13-15 SE; XCC_ID register)
          const int sw_ = ((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * kDecWaves + wave;
          if (lane == 0 && sw_ < kStampWaves)
            g_dec_stamps[sw_][5] = ((unsigned long long)__builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (31 << 11)) << 32) |
                                   (unsigned)__builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (3 << 11));
        }
#endif
      }
    }
  }

  DEC_STAMP_AFTER(3, acc[0][0]);  // streaming loop done
  // the wave's result: sum the per-lane l over the 16 token lanes, and acc over the token rows of the V layout
#pragma unroll
  for (int i = 0; i < 4; ++i) l[i] = group_allreduce<16>(l[i], OpSum());
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int i = 0; i < kVec; ++i) acc[g][i] = cross_group_allreduce<kLanesPerTok>(acc[g][i], OpSum());

  if (vr_ == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int i = 0; i < kVec; ++i) sm_acc[wave][g][vc_ * kVec + i] = acc[g][i];
  }
  if (kt == 0 && kg < kGroups) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (4 * kg + i < G) { sm_m[wave][4 * kg + i] = m[i]; sm_l[wave][4 * kg + i] = l[i]; }
  }
  __syncthreads();
  const int64_t pbase = (int64_t)row * num_splits + split;
  for (int idx = threadIdx.x; idx < G * D; idx += kDecWaves * kWave) {
    const int g = idx / D, d = idx % D;
    float M = sm_m[0][g];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) M = fmaxf(M, sm_m[w][g]);
    float o = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float sc = fast_exp2(sm_m[w][g] - M);
      o = fmaf(sm_acc[w][g][d], sc, o);
      L = fmaf(sm_l[w][g], sc, L);
    }
    if (num_splits == 1) {
      write_final(c, out, lse_out, b, hkv * G + g, d, D, o, M, L);
    } else {
      part_o[(pbase * G + g) * D + d] = o;
      if (d == 0) {
        part_ml[(pbase * G + g) * 2 + 0] = M;
        part_ml[(pbase * G + g) * 2 + 1] = L;
      }
    }
  }
  DEC_STAMP(4);  // partial results stored
}

// Log-sum-exp merge of the chunk partials of one (sequence, query head); writes out (and lse).
// One wave per head. Lane s takes the (m, l) pair of chunk s, so the maximum, the per-chunk scales and the
// normaliser come from two wave reductions instead of a serial pass; the output rows of the chunks are then
// accumulated with the scale of chunk s broadcast from lane s, eight independent loads in flight at a time
// (a thread per element walking the chunks one dependent load after the other took 8 us for 32 chunks).
template <typename T, int D, int G>
__global__ __launch_bounds__(kWave) void paged_decode_merge_kernel(CacheView c, const int32_t* __restrict__ sel_count,
                                                                   int sel_stride, bool dense, int pages_per_split,
                                                                   int num_splits, const float* __restrict__ part_o,
                                                                   const float* __restrict__ part_ml,
                                                                   T* __restrict__ out, float* __restrict__ lse_out) {
  constexpr int kPer = D / kWave;  // output elements per lane (1 or 2)
  static_assert(kPer == 1 || kPer == 2, "head_dim 64 or 128");
  const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  const int hkv = h / G, g = h % G;
  const int row = b * c.Hkv + hkv;
  const int N = c.seq_lens[b];
  const int P = min((N + c.S - 1) / c.S, c.max_pages_hint);
  const int cnt = dense ? P : min(sel_count[row], sel_stride);
  const int ns = min(num_splits, (cnt + pages_per_split - 1) / pages_per_split);
  const int64_t base = (int64_t)row * num_splits;
  const float2* ml = reinterpret_cast<const float2*>(part_ml);  // (m, l) per (row, chunk, head)

  float M = kNegBig;
  for (int s0 = 0; s0 < ns; s0 += kWave)
    if (s0 + lane < ns) M = fmaxf(M, ml[(base + s0 + lane) * G + g].x);
  M = group_allreduce<kWave>(M, OpMax());

  float L = 0.f, o[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) o[i] = 0.f;
  for (int s0 = 0; s0 < ns; s0 += kWave) {
    float sc = 0.f;
    if (s0 + lane < ns) {
      const float2 v = ml[(base + s0 + lane) * G + g];
      sc = fast_exp2(v.x - M);
      L = fmaf(v.y, sc, L);
    }
    const int n = min(kWave, ns - s0);
    const float* po = part_o + ((base + s0) * G + g) * D + lane * kPer;
    // blocks of eight chunks; a slot past the last chunk re-reads that chunk with the zero scale of its lane
    for (int j0 = 0; j0 < n; j0 += 8) {
      float2 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float* src = po + (int64_t)min(j0 + u, n - 1) * G * D;
        if constexpr (kPer == 2) v[u] = *reinterpret_cast<const float2*>(src);
        else v[u] = make_float2(src[0], 0.f);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float scj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sc), j0 + u));
        o[0] = fmaf(v[u].x, scj, o[0]);
        if constexpr (kPer == 2) o[1] = fmaf(v[u].y, scj, o[1]);
      }
    }
  }
  L = group_allreduce<kWave>(L, OpSum());
  const bool any = L > 0.f;
  T* dst = out + ((int64_t)b * c.H + h) * D + lane * kPer;
#pragma unroll
  for (int i = 0; i < kPer; ++i) store_elem(dst + i, any ? o[i] / L : 0.f);
  if (lse_out && lane == 0) lse_out[(int64_t)b * c.H + h] = any ? (M + log2f(L)) * kLn2 : -INFINITY;
}

template <typename T, int D, int S, int G>
hipError_t launch_t(const CacheView& cv, const void* q, const int32_t* sel, const int32_t* cnt, int sel_stride,
                    int max_list_len, float sm_scale, void* out, float* lse, float* partials, hipStream_t st) {
  CacheView c = cv;
  const int rows = c.B * c.Hkv;
  c.stream_nt = (int64_t)rows * max_list_len * S * D * 2 * (int64_t)sizeof(T) > kStreamNtBytes;
  const SplitPlan plan = plan_splits(rows, max_list_len);
  float* part_o = partials;
  float* part_ml = partials + (size_t)rows * plan.num_splits * G * D;
  const float scale_log2 = (sm_scale > 0.f ? sm_scale : 1.0f / sqrtf((float)D)) * kLog2e;
#ifndef UNIQUE_DEC_NO_MFMA
  if constexpr (sizeof(T) == 2) {
    auto go = [&](auto kernel) {
      kernel<<<dim3(plan.num_splits, c.Hkv, c.B), dim3(kDecWaves * kWave), 0, st>>>(
          c, reinterpret_cast<const bf16_t*>(q), sel, cnt, sel_stride, plan.pages_per_split, plan.num_splits,
          scale_log2, part_o, part_ml, reinterpret_cast<bf16_t*>(out), lse);
    };
    if (c.stream_nt) go(paged_decode_partial_mfma_kernel<D, S, G, true>);
    else go(paged_decode_partial_mfma_kernel<D, S, G, false>);
  } else
#endif
    paged_decode_partial_kernel<T, D, S, G><<<dim3(plan.num_splits, c.Hkv, c.B), dim3(kDecWaves * kWave), 0, st>>>(
        c, reinterpret_cast<const T*>(q), sel, cnt, sel_stride, plan.pages_per_split, plan.num_splits, scale_log2,
        part_o, part_ml, reinterpret_cast<T*>(out), lse);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || plan.num_splits == 1) return e;  // one chunk per row: the partial kernel wrote the output
  paged_decode_merge_kernel<T, D, G><<<dim3(c.H, c.B), dim3(kWave), 0, st>>>(
      c, cnt, sel_stride, sel == nullptr, plan.pages_per_split, plan.num_splits, part_o, part_ml,
      reinterpret_cast<T*>(out), lse);
  return hipGetLastError();
}

template <typename T, int D, int S>
hipError_t dispatch_g(const CacheView& c, const void* q, const int32_t* sel, const int32_t* cnt, int sel_stride,
                      int max_list_len, float sm_scale, void* out, float* lse, float* partials, hipStream_t st) {
  switch (c.H / c.Hkv) {
    case 1: return launch_t<T, D, S, 1>(c, q, sel, cnt, sel_stride, max_list_len, sm_scale, out, lse, partials, st);
    case 2: return launch_t<T, D, S, 2>(c, q, sel, cnt, sel_stride, max_list_len, sm_scale, out, lse, partials, st);
    case 4: return launch_t<T, D, S, 4>(c, q, sel, cnt, sel_stride, max_list_len, sm_scale, out, lse, partials, st);
    case 8: return launch_t<T, D, S, 8>(c, q, sel, cnt, sel_stride, max_list_len, sm_scale, out, lse, partials, st);
    default: return hipErrorInvalidValue;
  }
}

template <typename T, int D>
hipError_t dispatch_s(const CacheView& c, const void* q, const int32_t* sel, const int32_t* cnt, int sel_stride,
                      int max_list_len, float sm_scale, void* out, float* lse, float* partials, hipStream_t st) {
  switch (c.S) {
    case 8: return dispatch_g<T, D, 8>(c, q, sel, cnt, sel_stride, max_list_len, sm_scale, out, lse, partials, st);
    case 16: return dispatch_g<T, D, 16>(c, q, sel, cnt, sel_stride, max_list_len, sm_scale, out, lse, partials, st);
    case 32: return dispatch_g<T, D, 32>(c, q, sel, cnt, sel_stride, max_list_len, sm_scale, out, lse, partials, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

#ifdef UNIQUE_DEC_STAMPS
extern "C" int unique_debug_dec_stamps(void** ptr, int* waves, int* slots) {
  *waves = kStampWaves;
  *slots = kStampSlots;
  return (int)hipGetSymbolAddress(ptr, HIP_SYMBOL(g_dec_stamps));
}

// Ceiling probe of the profiling build: the memory access of the sparse decode with everything else taken away.
// One wave fetches the 4 KiB K tile and the 4 KiB V tile of each of its (physical page, head) entries -- page ids
// straight from `list`, no page table, no arithmetic but an xor -- with kDepth tiles in flight. kPattern 0: every
// load instruction covers a contiguous 1 KiB; 1: K in the operand layout of the matrix-core q.k stage (64-byte
// pieces of 16 rows); 2: contiguous loads that go straight into LDS (second kernel below). Geometry as the decode kernel: rows x ceil(k / pages_per_wg) workgroups of `waves` waves.
namespace {
typedef unsigned int probe_u32x4 __attribute__((ext_vector_type(4)));
template <int kPattern, int kDepth>
__global__ __launch_bounds__(1024) void gather_probe_kernel(const char* __restrict__ kpool, const char* __restrict__ vpool,
                                                             const int32_t* __restrict__ list, int k, int pages_per_wg,
                                                             int waves, int heads, probe_u32x4* __restrict__ sink) {
  const int row = blockIdx.y, split = blockIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
  const int begin = split * pages_per_wg, end = min(begin + pages_per_wg, k);
  const int hkv = row % heads;
  const int n = min(kWave, (end - begin - wave + waves - 1) / waves);  // entries of this wave (lane i holds the i-th)
  int my_phys = 0;
  if (lane < n) my_phys = list[(size_t)row * k + begin + wave + lane * waves];
  probe_u32x4 acc = {0, 0, 0, 0};
  probe_u32x4 buf[kDepth][8];
  const int koff = kPattern == 0 ? lane * 16 : (lane % 16) * 256 + (lane / 16) * 16;
  const int kstep = kPattern == 0 ? 1024 : 64;
  auto issue = [&](int i, probe_u32x4(&b)[8]) {  // past the wave's last entry: its last page again (keeps the code straight-line)
    const int phys = __builtin_amdgcn_readlane(my_phys, max(min(i, n - 1), 0));
    const size_t base = ((size_t)phys * heads + hkv) * 4096;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      b[j] = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4*>(kpool + base + koff + j * kstep));
#pragma unroll
    for (int j = 0; j < 4; ++j)
      b[4 + j] = __builtin_nontemporal_load(reinterpret_cast<const probe_u32x4*>(vpool + base + lane * 16 + j * 1024));
  };
#pragma unroll
  for (int d = 0; d < kDepth; ++d) issue(d, buf[d]);
  for (int i = 0; i < n; i += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc ^= buf[d][j];
      issue(i + d + kDepth, buf[d]);
    }
  }
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) sink[threadIdx.x] = acc;  // never true in practice; keeps the loads alive
}

// The same gather with the tiles sent straight into LDS (global_load_lds_dwordx4, no register between memory and
// LDS): a ring of kDepth tiles of 8 KiB per wave, each tile waited for with an explicit vmcnt and read back with
// ds_read_b128. Dynamic LDS: waves * kDepth * 8 KiB.
template <int kN>
__device__ __forceinline__ void probe_wait_vmcnt() {  // s_waitcnt vmcnt(kN) alone (expcnt and lgkmcnt fields left at their maximum)
  __builtin_amdgcn_s_waitcnt((kN & 0xF) | ((kN >> 4) << 14) | 0x0F70);
}
template <int kDepth>
__global__ __launch_bounds__(1024) void gather_probe_lds_kernel(const char* __restrict__ kpool,
                                                                 const char* __restrict__ vpool,
                                                                 const int32_t* __restrict__ list, int k, int pages_per_wg,
                                                                 int waves, int heads, probe_u32x4* __restrict__ sink) {
  extern __shared__ __attribute__((aligned(16))) char probe_lds[];
  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  const int row = blockIdx.y, split = blockIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = threadIdx.x % kWave;
  const int begin = split * pages_per_wg, end = min(begin + pages_per_wg, k);
  const int hkv = row % heads;
  const int n = min(kWave, (end - begin - wave + waves - 1) / waves);
  int my_phys = 0;
  if (lane < n) my_phys = list[(size_t)row * k + begin + wave + lane * waves];
  char* ring = probe_lds + (size_t)wave * kDepth * 8192;  // wave-uniform
  probe_u32x4 acc = {0, 0, 0, 0};
  auto issue = [&](int i, int d) {
    const int phys = __builtin_amdgcn_readlane(my_phys, max(min(i, n - 1), 0));
    const size_t base = ((size_t)phys * heads + hkv) * 4096 + lane * 16;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      __builtin_amdgcn_global_load_lds((gptr_t)(kpool + base + j * 1024), (lptr_t)(ring + d * 8192 + j * 1024), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      __builtin_amdgcn_global_load_lds((gptr_t)(vpool + base + j * 1024), (lptr_t)(ring + d * 8192 + 4096 + j * 1024), 16, 0, 0);
  };
#pragma unroll
  for (int d = 0; d < kDepth; ++d) issue(d, d);
  for (int i = 0; i < n; i += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      probe_wait_vmcnt<(kDepth - 1) * 8>();  // the oldest tile has landed; the younger ones may still be on their way
      asm volatile("" ::: "memory");
#pragma unroll
      for (int j = 0; j < 8; ++j) acc ^= *reinterpret_cast<const probe_u32x4*>(ring + d * 8192 + j * 1024 + lane * 16);
      asm volatile("" ::"v"(acc.x), "v"(acc.y), "v"(acc.z), "v"(acc.w) : "memory");  // the reads are done before the slot is refilled
      issue(i + d + kDepth, d);
    }
  }
  probe_wait_vmcnt<0>();
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) sink[threadIdx.x] = acc;
}
}  // namespace

// k_pool / v_pool: [num_pages][heads][4096 bytes]; list: int32 [rows][k] physical page ids (all < num_pages, which the
// caller guarantees); sink: 16 KiB of device memory. Returns a hipError_t.
extern "C" int unique_debug_gather_probe(const void* k_pool, const void* v_pool, const int32_t* list, int rows, int k,
                                         int heads, int pages_per_wg, int waves, int depth, int pattern, void* sink,
                                         void* stream) {
  if (rows < 1 || k < 1 || heads < 1 || waves < 1 || waves > 16 || pages_per_wg < waves || pages_per_wg > 64 * waves)
    return (int)hipErrorInvalidValue;
  const dim3 grid((k + pages_per_wg - 1) / pages_per_wg, rows), block(waves * kWave);
  auto go = [&](auto kernel) {
    kernel<<<grid, block, 0, (hipStream_t)stream>>>((const char*)k_pool, (const char*)v_pool, list, k, pages_per_wg,
                                                    waves, heads, (probe_u32x4*)sink);
  };
  if (pattern == 2) {  // through LDS
    const size_t lds = (size_t)waves * depth * 8192;
    if (lds > 160 * 1024 || (depth != 2 && depth != 4)) return (int)hipErrorInvalidValue;
    auto go_lds = [&](auto kernel) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return (int)e;
      kernel<<<grid, block, lds, (hipStream_t)stream>>>((const char*)k_pool, (const char*)v_pool, list, k, pages_per_wg,
                                                        waves, heads, (probe_u32x4*)sink);
      return (int)hipGetLastError();
    };
    return depth == 2 ? go_lds(gather_probe_lds_kernel<2>) : go_lds(gather_probe_lds_kernel<4>);
  }
  if (pattern == 0 && depth == 2) go(gather_probe_kernel<0, 2>);
  else if (pattern == 0 && depth == 4) go(gather_probe_kernel<0, 4>);
  else if (pattern == 1 && depth == 2) go(gather_probe_kernel<1, 2>);
  else if (pattern == 1 && depth == 4) go(gather_probe_kernel<1, 4>);
  else return (int)hipErrorInvalidValue;
  return (int)hipGetLastError();
}
#endif

bool decode_supported(int dtype, int D, int S, int G) {
  return (dtype == 0 || dtype == 1) && (D == 64 || D == 128) && (S == 8 || S == 16 || S == 32) &&
         (G == 1 || G == 2 || G == 4 || G == 8);
}

SplitPlan plan_splits(int rows, int max_list_len) {
  // aim at ~2 workgroups (8 waves) per CU of a 256-CU device, with at least 1 page per wave; from 256 rows on one
  // workgroup per row already fills the device, the row is not cut and no merge launch is needed (lists of up to
  // UNIQUE_DEC_MAX_PPS pages)
#ifndef UNIQUE_DEC_TARGET_GROUPS
#define UNIQUE_DEC_TARGET_GROUPS 512
#endif
  constexpr int kTargetGroups = UNIQUE_DEC_TARGET_GROUPS;
#ifndef UNIQUE_DEC_MAX_PPS
#define UNIQUE_DEC_MAX_PPS 256
#endif
  if (rows < 1) rows = 1;
  if (max_list_len < 1) max_list_len = 1;
  const int wanted = rows >= 256 ? 1 : (kTargetGroups + rows - 1) / rows;
  int pps = (max_list_len + wanted - 1) / wanted;
#ifndef UNIQUE_DEC_MIN_PAGES_PER_WAVE
#define UNIQUE_DEC_MIN_PAGES_PER_WAVE 1
#endif
  if (pps < UNIQUE_DEC_MIN_PAGES_PER_WAVE * kDecWaves) pps = UNIQUE_DEC_MIN_PAGES_PER_WAVE * kDecWaves;
  // long lists are cut into many equal chunks so that ragged batches balance across the CUs
  if (pps > UNIQUE_DEC_MAX_PPS) pps = UNIQUE_DEC_MAX_PPS;
  pps = (pps + kDecWaves - 1) / kDecWaves * kDecWaves;
  SplitPlan p;
  p.pages_per_split = pps;
  p.num_splits = (max_list_len + pps - 1) / pps;
  return p;
}

size_t decode_partial_floats(const CacheView& c, int max_list_len) {
  const int rows = c.B * c.Hkv;
  const SplitPlan plan = plan_splits(rows, max_list_len);
  return (size_t)rows * plan.num_splits * (size_t)(c.H / c.Hkv) * (size_t)(c.D + 2);
}

hipError_t launch_decode(const CacheView& c, const void* d_q, const int32_t* d_sel_pages,
                         const int32_t* d_sel_count, int sel_stride, int max_list_len, float sm_scale,
                         void* d_out, float* d_lse_out, float* d_partials, hipStream_t stream) {
  if (c.dtype == 0) {
    return c.D == 64 ? dispatch_s<float, 64>(c, d_q, d_sel_pages, d_sel_count, sel_stride, max_list_len, sm_scale,
                                             d_out, d_lse_out, d_partials, stream)
                     : dispatch_s<float, 128>(c, d_q, d_sel_pages, d_sel_count, sel_stride, max_list_len, sm_scale,
                                              d_out, d_lse_out, d_partials, stream);
  }
  return c.D == 64 ? dispatch_s<bf16_t, 64>(c, d_q, d_sel_pages, d_sel_count, sel_stride, max_list_len, sm_scale,
                                            d_out, d_lse_out, d_partials, stream)
                   : dispatch_s<bf16_t, 128>(c, d_q, d_sel_pages, d_sel_count, sel_stride, max_list_len, sm_scale,
                                             d_out, d_lse_out, d_partials, stream);
}

}  // namespace unique
