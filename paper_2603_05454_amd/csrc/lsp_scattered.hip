// Scattered-Margin baseline of Section 4.3.3 (same block size as LSP, positions
// taken from anywhere in the active sequence) and the cache update it implies.
// These entry points exist to MEASURE what the paper's prefix-first topology
// saves: selection, a gathered append, and (in lsp_attn.hip) attention over a
// cache addressed through a row index.
//
// Selection: every position is ranked by counting
// (rank_i = #{j : m_j > m_i} + #{j < i : m_j = m_i}, so equal margins are
// ordered by position) against the sequence's margins held in LDS, and is
// selected when its rank is below the requested count; a second kernel writes
// the selected positions in ascending order.
#include "lsp_common.h"

namespace lsp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSelThreads = 256;
constexpr int kSelMaxS = 8192;  // margins of one sequence live in LDS

typedef float f32x4 __attribute__((ext_vector_type(4)));

// grid (ceil(S / 256), B): every workgroup ranks 256 positions of one sequence
// against all of its active margins (copied to LDS, padded with -inf to a
// multiple of 4 so that the scan reads 16 bytes per LDS broadcast).
__global__ __launch_bounds__(kSelThreads) void rank_kernel(
    const float *__restrict__ margin, int S, const int32_t *__restrict__ suffix_len,
    const int32_t *__restrict__ count, uint8_t *__restrict__ sel_mask) {
  extern __shared__ __attribute__((aligned(16))) float s_m[];
  const int b = blockIdx.y, tid = threadIdx.x;
  const int N = min(max(suffix_len[b], 0), S);
  const int k = min(max(count[b], 0), N);
  const float *mg = margin + int64_t(b) * S;
  const int i = blockIdx.x * kSelThreads + tid;
  if (k == 0 || blockIdx.x * kSelThreads >= N) {  // uniform: nothing to rank here
    if (i < S) sel_mask[int64_t(b) * S + i] = 0;
    return;
  }
  const int N4 = (N + 3) & ~3;
  for (int j = tid; j < N4; j += kSelThreads) s_m[j] = j < N ? mg[j] : -INFINITY;
  __syncthreads();
  bool sel = false;
  if (i < N) {
    const float mi = s_m[i];
    int rank = 0;
    for (int j = 0; j < N4; j += 4) {
      const f32x4 m = *reinterpret_cast<const f32x4 *>(s_m + j);
      rank += (m.x > mi) || (m.x == mi && j < i);
      rank += (m.y > mi) || (m.y == mi && j + 1 < i);
      rank += (m.z > mi) || (m.z == mi && j + 2 < i);
      rank += (m.w > mi) || (m.w == mi && j + 3 < i);
    }
    sel = rank < k;
  }
  if (i < S) sel_mask[int64_t(b) * S + i] = sel ? 1 : 0;
}

// One workgroup per sequence writes the selected positions in ascending order:
// wave ballots give the in-wave offsets, an LDS prefix over the waves the rest.
__global__ __launch_bounds__(kSelThreads) void compact_kernel(
    int S, const int32_t *__restrict__ suffix_len, const int32_t *__restrict__ count,
    const uint8_t *__restrict__ sel_mask, int32_t *__restrict__ sel_index) {
  __shared__ int s_wave[kSelThreads / kWave];
  __shared__ int s_base;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int N = min(max(suffix_len[b], 0), S);
  const int k = min(max(count[b], 0), N);
  int32_t *ix = sel_index + int64_t(b) * S;
  const uint8_t *mk = sel_mask + int64_t(b) * S;
  if (tid == 0) s_base = 0;
  __syncthreads();
  for (int base = 0; base < N; base += kSelThreads) {
    const int i = base + tid;
    const bool sel = i < N && mk[i] != 0;
    const unsigned long long bal = __ballot(sel);
    if (lane == 0) s_wave[wave] = __popcll(bal);
    __syncthreads();
    int off = s_base;
    for (int w2 = 0; w2 < wave; ++w2) off += s_wave[w2];
    if (sel) ix[off + __popcll(bal & ((1ull << lane) - 1ull))] = i;
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
      for (int w2 = 0; w2 < kSelThreads / kWave; ++w2) tot += s_wave[w2];
      s_base += tot;
    }
    __syncthreads();
  }
  for (int i = k + tid; i < S; i += kSelThreads) ix[i] = -1;  // exactly k positions were selected
}

constexpr int kMaxLayersPerLaunch = 32;
struct LayerPtrs {
  const char *src[2 * kMaxLayersPerLaunch];  // K then V per layer
  char *dst[2 * kMaxLayersPerLaunch];
};

constexpr int kRowThreads = 256;

// Rows to append per sequence: count[b], cut to the cache room and to the length
// of the list (it ends at its first negative entry: lsp_select_scattered pads
// with -1 when fewer positions than count[b] are active).  One workgroup per
// sequence.
__global__ __launch_bounds__(256) void gather_count_kernel(int S, int C, const int32_t *__restrict__ sel_index,
                                                           const int32_t *__restrict__ count,
                                                           const int32_t *__restrict__ prefix_len,
                                                           int32_t *__restrict__ appended) {
  __shared__ int first_bad;
  const int b = blockIdx.x;
  const int P = max(prefix_len[b], 0);
  const int k = min(min(max(count[b], 0), max(C - P, 0)), S);
  if (threadIdx.x == 0) first_bad = k;
  __syncthreads();
  int mine = k;
  for (int j = threadIdx.x; j < k; j += blockDim.x)
    if (sel_index[int64_t(b) * S + j] < 0) mine = min(mine, j);
  if (mine < k) atomicMin(&first_bad, mine);
  __syncthreads();
  if (threadIdx.x == 0) appended[b] = first_bad;
}

// grid: (S candidate rows, B, 2 * layers in this launch); row j of sequence b is
// live when j < appended[b].  One workgroup copies one K or V row.
__global__ __launch_bounds__(kRowThreads) void gather_append_kernel(
    LayerPtrs ptrs, int S, int64_t row_bytes, int64_t suf_batch_bytes,
    int64_t cache_batch_bytes, const int32_t *__restrict__ sel_index,
    const int32_t *__restrict__ appended, const int32_t *__restrict__ prefix_len) {
  const int j = blockIdx.x, b = blockIdx.y;
  if (j >= appended[b]) return;
  const int P = max(prefix_len[b], 0);
  const int src_row = min(sel_index[int64_t(b) * S + j], S - 1);  // a bad index must not leave the buffer (>= 0 here)
  const char *src = ptrs.src[blockIdx.z] + int64_t(b) * suf_batch_bytes + int64_t(src_row) * row_bytes;
  char *dst = ptrs.dst[blockIdx.z] + int64_t(b) * cache_batch_bytes + int64_t(P + j) * row_bytes;
  for (int64_t o = int64_t(threadIdx.x) * 16; o < row_bytes; o += int64_t(kRowThreads) * 16) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(dst + o));
  }
}

__global__ void advance_prefix_kernel(int B, const int32_t *__restrict__ appended, int32_t *__restrict__ prefix_len) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  prefix_len[b] = max(prefix_len[b], 0) + appended[b];
}

}  // namespace
}  // namespace lsp

extern "C" int32_t lsp_select_scattered(const float *margin, int32_t B, int32_t S,
                                        const int32_t *suffix_len, const int32_t *count,
                                        int32_t *sel_index, uint8_t *sel_mask, void *stream) {
  using namespace lsp;
  LSP_CHECK_ARG(margin && suffix_len && count && sel_index && sel_mask, "lsp_select_scattered: null pointer");
  LSP_CHECK_ARG(B > 0 && S > 0, "lsp_select_scattered: bad B/S");
  if (S > kSelMaxS) {
    set_error("lsp_select_scattered: S = %d exceeds the %d positions one workgroup ranks", S, kSelMaxS);
    return LSP_ERR_UNSUPPORTED;
  }
  LSP_CHECK_ARG(B <= 65535, "lsp_select_scattered: B must be <= 65535");
  hipStream_t st = static_cast<hipStream_t>(stream);
  rank_kernel<<<dim3((S + kSelThreads - 1) / kSelThreads, B), kSelThreads, size_t(S + 4) * sizeof(float), st>>>(
      margin, S, suffix_len, count, sel_mask);
  LSP_CHECK_LAUNCH("lsp_select_scattered: rank launch");
  compact_kernel<<<B, kSelThreads, 0, st>>>(S, suffix_len, count, sel_mask, sel_index);
  LSP_CHECK_LAUNCH("lsp_select_scattered: compact launch");
  return LSP_OK;
}

extern "C" int32_t lsp_kv_gather_append(int32_t kv_dtype, int32_t B, int32_t S, int32_t Hkv, int32_t D,
                                        int32_t C, int32_t num_layers, int64_t suf_batch_stride,
                                        int64_t cache_batch_stride, const int32_t *sel_index,
                                        const int32_t *count, const void *const *k_suf_layers,
                                        const void *const *v_suf_layers, void *const *k_cache_layers,
                                        void *const *v_cache_layers, int32_t *prefix_len,
                                        int32_t *appended, void *stream) {
  using namespace lsp;
  LSP_CHECK_ARG(sel_index && count && prefix_len && appended, "lsp_kv_gather_append: null pointer");
  LSP_CHECK_ARG(kv_dtype == LSP_F32 || kv_dtype == LSP_BF16, "lsp_kv_gather_append: unknown kv_dtype");
  LSP_CHECK_ARG(B > 0 && B <= 65535 && S > 0 && Hkv > 0 && D > 0 && C > 0 && num_layers > 0,
                "lsp_kv_gather_append: bad dimension");
  LSP_CHECK_ARG(k_suf_layers && v_suf_layers && k_cache_layers && v_cache_layers,
                "lsp_kv_gather_append: null layer pointer table");
  const int64_t es = int64_t(elem_size(kv_dtype));
  const int64_t row_bytes = int64_t(Hkv) * D * es;
  LSP_CHECK_ARG(row_bytes % 16 == 0, "lsp_kv_gather_append: K/V row of %lld bytes is not a multiple of 16", (long long)row_bytes);
  const int64_t suf_bb = (suf_batch_stride ? suf_batch_stride : int64_t(S) * Hkv * D) * es;
  const int64_t cache_bb = (cache_batch_stride ? cache_batch_stride : int64_t(C) * Hkv * D) * es;
  LSP_CHECK_ARG(suf_bb % 16 == 0 && cache_bb % 16 == 0 && suf_bb >= int64_t(S) * row_bytes &&
                    cache_bb >= int64_t(C) * row_bytes,
                "lsp_kv_gather_append: bad batch strides");
  for (int l = 0; l < num_layers; ++l) {
    LSP_CHECK_ARG(k_suf_layers[l] && v_suf_layers[l] && k_cache_layers[l] && v_cache_layers[l],
                  "lsp_kv_gather_append: null K/V pointer in layer %d", l);
    LSP_CHECK_ARG(aligned16(k_suf_layers[l]) && aligned16(v_suf_layers[l]) && aligned16(k_cache_layers[l]) &&
                      aligned16(v_cache_layers[l]),
                  "lsp_kv_gather_append: K/V pointer of layer %d is not 16-byte aligned", l);
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  gather_count_kernel<<<B, 256, 0, st>>>(S, C, sel_index, count, prefix_len, appended);
  LSP_CHECK_LAUNCH("lsp_kv_gather_append: count launch");
  for (int l0 = 0; l0 < num_layers; l0 += kMaxLayersPerLaunch) {
    const int nl = num_layers - l0 < kMaxLayersPerLaunch ? num_layers - l0 : kMaxLayersPerLaunch;
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
    gather_append_kernel<<<dim3(S, B, 2 * nl), kRowThreads, 0, st>>>(p, S, row_bytes, suf_bb, cache_bb,
                                                                     sel_index, appended, prefix_len);
    LSP_CHECK_LAUNCH("lsp_kv_gather_append: copy launch");
  }
  advance_prefix_kernel<<<(B + 255) / 256, 256, 0, st>>>(B, appended, prefix_len);
  LSP_CHECK_LAUNCH("lsp_kv_gather_append: prefix launch");
  return LSP_OK;
}
