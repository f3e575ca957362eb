// lsp_commit: stability mask, longest stable prefix L'(tau), snap to the last
// delimiter inside the look-back window, L_min / fallback, token commit and the
// contiguous KV-cache append (Section 3.2 of the paper; Algorithm 1 lines 7-10).
//
// Two kernels.  The boundary kernel runs one workgroup per sequence: every
// wave ballots "unstable" over its 64 positions, the first set bit of the first
// non-empty ballot is that wave's candidate, and an LDS minimum across waves
// gives L'.  The same pass ballots "predicts a delimiter" per position into
// LDS words, so the search for the last delimiter inside the window is a scan
// of a few words (one thread per word, highest set bit, LDS maximum); margins,
// ids, lengths and bitmap words are all requested up front, which leaves two
// dependent trips to memory on the critical path.  The append kernel then
// copies, per (layer, K|V, sequence), the single contiguous block of
// L * Hkv * D elements from the suffix buffer to cache row P with 16-byte
// loads and stores; the block length is read from device memory, so the host
// never learns L and the grid is sized for the worst case with early exit.
#include <limits.h>

#include "lsp_common.h"

namespace lsp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kScanThreads = 256;
constexpr int kMaxScanRows = 65536;  // S at most this (one delimiter ballot bit per row in LDS)

__global__ __launch_bounds__(kScanThreads) void boundary_kernel(
    const float *__restrict__ margin, const int32_t *__restrict__ top1_id,
    const uint32_t *__restrict__ bitmap, int S, int V, int C, int T, float tau, int window,
    int min_commit, int snap_enabled, int adaptive, float alpha, float beta, int max_commit,
    int32_t *__restrict__ tokens,
    int32_t *__restrict__ prefix_len, int32_t *__restrict__ suffix_len,
    uint8_t *__restrict__ stable_mask, int32_t *__restrict__ raw_boundary,
    int32_t *__restrict__ snapped_boundary, int32_t *__restrict__ commit_len,
    int32_t *__restrict__ status_flags, float *__restrict__ tau_used) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  __shared__ int s_first, s_snap, s_lo_hit, s_hi_hit;
  __shared__ float s_min[kScanThreads];
  __shared__ unsigned long long s_delim[kMaxScanRows / 64];  // bit i%64 of word i/64: position i predicts a delimiter
  const float *mg = margin + int64_t(b) * S;
  const int32_t *id = top1_id + int64_t(b) * S;
  uint8_t *mk = stable_mask + int64_t(b) * S;
  // Everything the scan needs is requested before anything is waited for: the
  // lengths, and this thread's margins and ids (in bounds for every i < S,
  // whatever N turns out to be).  The delimiter bit of every position is looked
  // up right away as well, so that the snap search further down is a scan over
  // ballot words in LDS instead of two more dependent trips to memory.
  const int nraw = suffix_len[b], praw = prefix_len[b];
  constexpr int kKeep = 4;  // ids of the first kKeep rounds stay in registers for the token commit
  int32_t idr[kKeep];
  float mgr[kKeep];
#pragma unroll
  for (int k = 0; k < kKeep; ++k) {
    const int i = k * kScanThreads + tid;
    idr[k] = i < S ? id[i] : 0;
    mgr[k] = i < S ? mg[i] : 0.f;
  }
  const int N = min(max(nraw, 0), S);
  const int P = max(praw, 0);
  if (tid == 0) {
    s_first = N;
    s_snap = 0;
    s_lo_hit = INT_MAX;
    s_hi_hit = -1;
  }
  __syncthreads();

  // mask + first unstable position + delimiter ballots
  int first = N;
  for (int base = 0, k = 0; base < S; base += kScanThreads, ++k) {
    const int i = base + tid;
    const bool in = i < N;
    float x;
    int32_t v;
    if (k < kKeep) {
      x = mgr[k < kKeep ? k : 0];
      v = idr[k < kKeep ? k : 0];
    } else {
      x = i < S ? mg[i] : 0.f;
      v = i < S ? id[i] : 0;
    }
    const bool stable = in && x > tau;
    if (i < S) mk[i] = stable ? 1 : 0;
    const unsigned long long bal = __ballot(in && !stable);
    if (bal != 0ull && first == N) first = i - lane + __builtin_ctzll(bal);
    if (snap_enabled) {
      const bool d = in && unsigned(v) < unsigned(V) && ((bitmap[v >> 5] >> (v & 31)) & 1u);
      const unsigned long long dbal = __ballot(d);
      if (lane == 0) s_delim[(base + tid) >> 6] = dbal;
    }
  }
  if (lane == 0 && first < N) atomicMin(&s_first, first);
  __syncthreads();
  int Lp = s_first;
  float tk = tau;
  int flag = 0;

  // Adaptive threshold (Eq. 2): a length a in [1, N) is produced by some threshold
  // exactly when margin[a] is a strict new minimum of margin[0..a].  Every thread
  // owns a contiguous chunk of positions: chunk minima, an exclusive prefix
  // minimum across threads in LDS, then a walk over the chunk that keeps the
  // first and the last such length inside [lo, hi].
  if (adaptive && N > 0) {
    int lo = int(ceilf(__fmul_rn(alpha, float(N))));
    int hi = int(floorf(__fmul_rn(beta, float(N))));
    lo = min(max(lo, 0), N);
    hi = max(min(hi, N), lo);
    if (Lp < lo || Lp > hi) {  // uniform over the workgroup
      const int chunk = (N + kScanThreads - 1) / kScanThreads;
      const int i0 = min(tid * chunk, N), i1 = min(i0 + chunk, N);
      float m = INFINITY;
      for (int i = i0; i < i1; ++i) m = fminf(m, mg[i]);
      s_min[tid] = m;
      __syncthreads();
      for (int d = 1; d < kScanThreads; d <<= 1) {  // inclusive prefix minimum over threads
        const float other = tid >= d ? s_min[tid - d] : INFINITY;
        __syncthreads();
        s_min[tid] = fminf(s_min[tid], other);
        __syncthreads();
      }
      float pm = tid > 0 ? s_min[tid - 1] : INFINITY;  // minimum of everything before this chunk
      int first = INT_MAX, last = -1;
      for (int i = i0; i < i1; ++i) {
        const float x = mg[i];
        if (x < pm) {
          if (i >= lo && i <= hi && i >= 1) {
            first = min(first, i);
            last = i;
          }
          pm = x;
        }
      }
      if (lo == 0 && tid == 0) first = 0;  // length 0 is produced by any threshold >= margin[0]
      if (first != INT_MAX) atomicMin(&s_lo_hit, first);
      if (last >= 0) atomicMax(&s_hi_hit, last);
      if (tid == 0 && hi == N) atomicMax(&s_hi_hit, N), atomicMin(&s_lo_hit, N);  // N: any threshold below every margin
      __syncthreads();
      const int fst = s_lo_hit, lst = s_hi_hit;
      if (lst < 0) {  // no threshold satisfies Eq. 2
        flag |= LSP_FLAG_NO_THRESHOLD;
        tk = __int_as_float(0x7fc00000);
        Lp = Lp < lo ? lo : hi;
      } else {
        Lp = Lp < lo ? fst : lst;
        tk = Lp == N ? -INFINITY : mg[Lp];
      }
    }
  }

  // last delimiter inside the window: candidate lengths j = lo .. Lp are positions
  // lo-1 .. Lp-1 of the ballot words; one thread per word, highest set bit wins
  if (snap_enabled && Lp > 0) {
    const int lo = window < 0 ? 1 : max(1, Lp - window);
    const int w0 = (lo - 1) >> 6, w1 = (Lp - 1) >> 6;
    for (int w = w0 + tid; w <= w1; w += kScanThreads) {
      const int lowbit = max(lo - 1, 64 * w) - 64 * w, highbit = min(Lp - 1, 64 * w + 63) - 64 * w;
      const unsigned long long m = s_delim[w] & (~0ull << lowbit) & (~0ull >> (63 - highbit));
      if (m != 0ull) atomicMax(&s_snap, 64 * w + 64 - __builtin_clzll(m));
    }
  }
  __syncthreads();
  const int Ls = s_snap > 0 ? s_snap : Lp;
  int L = min(N, max(Ls, min_commit));
  if (max_commit > 0) L = min(L, max_commit);
  if (L > C - P) {
    L = max(C - P, 0);
    flag |= LSP_FLAG_CACHE_FULL;
  }
  if (tokens != nullptr && L > T - P) {
    L = max(T - P, 0);
    flag |= LSP_FLAG_TOKENS_FULL;
  }
  if (tokens != nullptr) {
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
      const int i = k * kScanThreads + tid;
      if (i < L) tokens[int64_t(b) * T + P + i] = idr[k];
    }
    for (int i = kKeep * kScanThreads + tid; i < L; i += kScanThreads) tokens[int64_t(b) * T + P + i] = id[i];
  }
  if (tid == 0) {
    raw_boundary[b] = Lp;
    snapped_boundary[b] = Ls;
    commit_len[b] = L;
    if (status_flags != nullptr) status_flags[b] = flag;
    if (tau_used != nullptr) tau_used[b] = tk;
    prefix_len[b] = P + L;
    suffix_len[b] = N - L;
  }
}

constexpr int kMaxLayersPerLaunch = 32;
struct LayerPtrs {
  const char *src[2 * kMaxLayersPerLaunch];  // K then V per layer
  char *dst[2 * kMaxLayersPerLaunch];
};

// grid: (workgroups per block copy, B, 2 * layers in this launch); a workgroup walks the
// block in chunks of NT*VECS*16 bytes with stride gridDim.x chunks.  (The commit length is
// only known on the device; a grid sized for S rows per copy costs a quarter of a
// millisecond in launch-and-exit alone when a decode step commits a few rows.)
// prefix_len already holds P + L; the block starts at row P = prefix_len - L.
template <int NT, int VECS>
__global__ __launch_bounds__(NT) void append_kernel(
    LayerPtrs ptrs, int64_t row_bytes, int64_t suf_batch_bytes, int64_t cache_batch_bytes,
    const int32_t *__restrict__ prefix_len, const int32_t *__restrict__ commit_len) {
  constexpr int kBytes = NT * VECS * 16;
  const int b = blockIdx.y;
  const int L = commit_len[b];
  const int64_t total = int64_t(L) * row_bytes;
  if (int64_t(blockIdx.x) * kBytes >= total) return;
  const int P = prefix_len[b] - L;
  const char *src = ptrs.src[blockIdx.z] + int64_t(b) * suf_batch_bytes;
  char *dst = ptrs.dst[blockIdx.z] + int64_t(b) * cache_batch_bytes + int64_t(P) * row_bytes;
  for (int64_t off0 = int64_t(blockIdx.x) * kBytes; off0 < total; off0 += int64_t(gridDim.x) * kBytes) {
    u32x4 v[VECS];
#pragma unroll
    for (int k = 0; k < VECS; ++k) {
      const int64_t o = off0 + (int64_t(k) * NT + threadIdx.x) * 16;
      if (o < total) v[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
    }
#pragma unroll
    for (int k = 0; k < VECS; ++k) {
      const int64_t o = off0 + (int64_t(k) * NT + threadIdx.x) * 16;
      if (o < total) __builtin_nontemporal_store(v[k], reinterpret_cast<u32x4 *>(dst + o));
    }
  }
}

template <int NT, int VECS>
void launch_append(const LayerPtrs &p, int64_t max_bytes, int B, int nl, hipStream_t st, int64_t row_bytes,
                   int64_t suf_bb, int64_t cache_bb, const int32_t *prefix_len, const int32_t *commit_len) {
  constexpr int kBytes = NT * VECS * 16;
  // enough workgroups to fill the chip when whole suffixes are committed (about 64 K in all), never more
  // than the block has chunks
  const int64_t all_chunks = (max_bytes + kBytes - 1) / kBytes;
  const int64_t copies = int64_t(B) * 2 * nl;
  int64_t per_copy = (65536 + copies - 1) / copies;
  if (per_copy > all_chunks) per_copy = all_chunks;
  if (per_copy < 1) per_copy = 1;
  const unsigned chunks = unsigned(per_copy);
  append_kernel<NT, VECS><<<dim3(chunks, B, 2 * nl), NT, 0, st>>>(p, row_bytes, suf_bb, cache_bb, prefix_len, commit_len);
}

}  // namespace
}  // namespace lsp

extern "C" size_t lsp_commit_workspace_bytes(const lsp_commit_desc *) { return 0; }

extern "C" int32_t lsp_commit(const lsp_commit_desc *d, const float *margin, const int32_t *top1_id,
                              const uint32_t *delimiter_bitmap,
                              const void *const *k_suf_layers, const void *const *v_suf_layers,
                              void *const *k_cache_layers, void *const *v_cache_layers,
                              int32_t *tokens, int32_t *prefix_len, int32_t *suffix_len,
                              uint8_t *stable_mask, int32_t *raw_boundary,
                              int32_t *snapped_boundary, int32_t *commit_len,
                              int32_t *status_flags, float *tau_used, void *workspace, size_t workspace_bytes,
                              void *stream) {
  using namespace lsp;
  (void)workspace;
  (void)workspace_bytes;
  LSP_CHECK_ARG(d != nullptr, "lsp_commit: null descriptor");
  LSP_CHECK_ARG(margin && top1_id && prefix_len && suffix_len && stable_mask && raw_boundary &&
                    snapped_boundary && commit_len,
                "lsp_commit: null pointer");
  LSP_CHECK_ARG(d->B > 0 && d->S > 0 && d->V >= 2 && d->C > 0, "lsp_commit: bad B/S/V/C");
  LSP_CHECK_ARG(d->B <= 65535 && d->S <= kMaxScanRows, "lsp_commit: B must be <= 65535 and S <= 65536");
  LSP_CHECK_ARG(d->min_commit >= 0, "lsp_commit: min_commit must be >= 0");
  LSP_CHECK_ARG(d->tau == d->tau, "lsp_commit: tau is NaN");
  LSP_CHECK_ARG(!d->snap_enabled || delimiter_bitmap, "lsp_commit: snapping needs a delimiter bitmap");
  LSP_CHECK_ARG(tokens == nullptr || d->T > 0, "lsp_commit: token buffer needs T > 0");
  LSP_CHECK_ARG(d->num_layers >= 0, "lsp_commit: num_layers < 0");
  LSP_CHECK_ARG(d->max_commit >= 0, "lsp_commit: max_commit must be >= 0");
  LSP_CHECK_ARG(!d->adaptive || (d->alpha > 0.f && d->alpha <= d->beta && d->beta <= 1.f),
                "lsp_commit: adaptive sizing needs 0 < alpha <= beta <= 1 (got %g, %g)", double(d->alpha), double(d->beta));
  int64_t row_bytes = 0, suf_bb = 0, cache_bb = 0;
  if (d->num_layers > 0) {
    LSP_CHECK_ARG(d->kv_dtype == LSP_F32 || d->kv_dtype == LSP_BF16, "lsp_commit: unknown kv_dtype");
    LSP_CHECK_ARG(d->Hkv > 0 && d->D > 0, "lsp_commit: bad Hkv/D");
    LSP_CHECK_ARG(k_suf_layers && v_suf_layers && k_cache_layers && v_cache_layers,
                  "lsp_commit: null layer pointer table");
    const int64_t es = int64_t(elem_size(d->kv_dtype));
    row_bytes = int64_t(d->Hkv) * d->D * es;
    LSP_CHECK_ARG(row_bytes % 16 == 0, "lsp_commit: K/V row of %lld bytes is not a multiple of 16", (long long)row_bytes);
    suf_bb = (d->suf_batch_stride ? d->suf_batch_stride : int64_t(d->S) * d->Hkv * d->D) * es;
    cache_bb = (d->cache_batch_stride ? d->cache_batch_stride : int64_t(d->C) * d->Hkv * d->D) * es;
    LSP_CHECK_ARG(suf_bb % 16 == 0 && cache_bb % 16 == 0 && suf_bb >= int64_t(d->S) * row_bytes &&
                      cache_bb >= int64_t(d->C) * row_bytes,
                  "lsp_commit: bad batch strides");
    for (int l = 0; l < d->num_layers; ++l) {
      LSP_CHECK_ARG(k_suf_layers[l] && v_suf_layers[l] && k_cache_layers[l] && v_cache_layers[l],
                    "lsp_commit: null K/V pointer in layer %d", l);
      LSP_CHECK_ARG(aligned16(k_suf_layers[l]) && aligned16(v_suf_layers[l]) &&
                        aligned16(k_cache_layers[l]) && aligned16(v_cache_layers[l]),
                    "lsp_commit: K/V pointer of layer %d is not 16-byte aligned", l);
    }
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  boundary_kernel<<<d->B, kScanThreads, 0, st>>>(
      margin, top1_id, delimiter_bitmap, d->S, d->V, d->C, d->T, d->tau, d->window, d->min_commit,
      d->snap_enabled, d->adaptive, d->alpha, d->beta, d->max_commit, tokens, prefix_len, suffix_len,
      stable_mask, raw_boundary, snapped_boundary, commit_len, status_flags, tau_used);
  LSP_CHECK_LAUNCH("lsp_commit: boundary launch");
  if (d->num_layers > 0) {
    const int64_t max_bytes = int64_t(d->S) * row_bytes;
    for (int l0 = 0; l0 < d->num_layers; l0 += kMaxLayersPerLaunch) {
      const int nl = d->num_layers - l0 < kMaxLayersPerLaunch ? d->num_layers - l0 : kMaxLayersPerLaunch;
      LayerPtrs p;
      for (int l = 0; l < nl; ++l) {
        p.src[2 * l] = static_cast<const char *>(k_suf_layers[l0 + l]);
        p.src[2 * l + 1] = static_cast<const char *>(v_suf_layers[l0 + l]);
        p.dst[2 * l] = static_cast<char *>(k_cache_layers[l0 + l]);
        p.dst[2 * l + 1] = static_cast<char *>(v_cache_layers[l0 + l]);
      }
      for (int l = 2 * nl; l < 2 * kMaxLayersPerLaunch; ++l) {
        p.src[l] = nullptr;
        p.dst[l] = nullptr;
      }
      // 256 threads x two 16-byte vectors per thread: the fastest of the shapes
      // measured (1..8 vectors, 256..1024 threads) when only the first rows of
      // every block are live, and within 3 % of the best for full blocks
      launch_append<256, 2>(p, max_bytes, d->B, nl, st, row_bytes, suf_bb, cache_bb, prefix_len, commit_len);
      LSP_CHECK_LAUNCH("lsp_commit: append launch");
    }
  }
  return LSP_OK;
}
