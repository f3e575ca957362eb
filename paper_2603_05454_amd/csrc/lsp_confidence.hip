// lsp_confidence: per-position top-1 id, logit margin (Eq. 1 of the paper;
// Algorithm 1 line 5) and top-1 soft-max probability, as one streaming pass
// over the logits.
//
// The kernel is bound by HBM reads (V * sizeof(elem) bytes per active row, each
// byte read once), so the design goal is: 16-byte coalesced loads with several
// in flight per lane, and few enough VALU operations per element that the
// arithmetic hides under the stream:
//   - top-2 tracking costs two operations per element: m2 = med3(m1, x, m2),
//     m1 = max(m1, x) (valid because m2 <= m1 always);
//   - the arg-max index is not tracked per element.  A lane only remembers in
//     which 16-byte vector its running maximum last rose strictly; since a lane
//     visits its elements in increasing index order, that vector holds the
//     lane's first occurrence of its maximum, and it is re-read once at the end;
//   - the soft-max sum uses one exp2 per element against a lagging per-lane
//     reference r (log2 domain) which is only moved when the lane maximum has
//     run more than 32 octaves ahead of it, so the rescale branch is cold.
// Lane results are merged with an associative (max1, idx, max2, sum@ref)
// operator in which the lower index wins on equal maxima, first across the
// wave by shuffles, then across waves through LDS, and - when one row is split
// over several workgroups because there are too few rows to fill the chip -
// across workgroups by a second tiny kernel.
#include <float.h>
#include <limits.h>

#include "lsp_common.h"

namespace lsp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLagOctaves = 32.0f;

struct Top {
  float m1, m2;  // largest and second largest value seen (duplicates count)
  float s;       // sum of exp2(x*log2e - r)
  float r;       // reference exponent (log2 domain)
  int idx;       // >= 0: element index of the first maximum; < 0: ~(start of the vector holding it)
};

__device__ __forceinline__ void top_init(Top &t) {
  t.m1 = -INFINITY;
  t.m2 = -INFINITY;
  t.s = 0.f;
  t.r = -FLT_MAX;
  t.idx = INT_MAX;
}

template <int N>
__device__ __forceinline__ void absorb(Top &t, const float (&x)[N], int tag) {
  const float old = t.m1;
#pragma unroll
  for (int j = 0; j < N; ++j) {
    t.m2 = __builtin_amdgcn_fmed3f(t.m1, x[j], t.m2);
    t.m1 = __builtin_fmaxf(t.m1, x[j]);
  }
  t.idx = t.m1 > old ? tag : t.idx;
  const float mc = t.m1 * kLog2e;
  if (mc - t.r > kLagOctaves) {
    t.s *= __builtin_amdgcn_exp2f(t.r - mc);
    t.r = mc;
  }
  const float nr = -t.r;
#pragma unroll
  for (int j = 0; j < N; ++j) t.s += __builtin_amdgcn_exp2f(__builtin_fmaf(x[j], kLog2e, nr));
}

__device__ __forceinline__ Top merge(const Top &a, const Top &b) {
  Top o;
  o.m1 = __builtin_fmaxf(a.m1, b.m1);
  o.idx = a.m1 > b.m1 ? a.idx : (b.m1 > a.m1 ? b.idx : (a.idx < b.idx ? a.idx : b.idx));
  o.m2 = __builtin_fmaxf(__builtin_fminf(a.m1, b.m1), __builtin_fmaxf(a.m2, b.m2));
  o.r = __builtin_fmaxf(a.r, b.r);
  o.s = a.s * __builtin_amdgcn_exp2f(a.r - o.r) + b.s * __builtin_amdgcn_exp2f(b.r - o.r);
  return o;
}

__device__ __forceinline__ Top shfl_xor(const Top &t, int mask) {
  Top o;
  o.m1 = __shfl_xor(t.m1, mask);
  o.m2 = __shfl_xor(t.m2, mask);
  o.s = __shfl_xor(t.s, mask);
  o.r = __shfl_xor(t.r, mask);
  o.idx = __shfl_xor(t.idx, mask);
  return o;
}

template <typename T>
struct Vec;
template <>
struct Vec<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const u32x4 &w, float (&x)[4]) {
    x[0] = __uint_as_float(w.x);
    x[1] = __uint_as_float(w.y);
    x[2] = __uint_as_float(w.z);
    x[3] = __uint_as_float(w.w);
  }
  static __device__ __forceinline__ float scalar(const float *p) { return *p; }
};
template <>
struct Vec<uint16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const u32x4 &w, float (&x)[8]) {
    x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x);
    x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
    x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z);
    x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
  }
  static __device__ __forceinline__ float scalar(const uint16_t *p) { return bf16_to_f32(*p); }
};

struct Partial {  // one row segment, normalised: s = sum exp(x - m1) over the segment
  float m1, m2, s;
  int idx;
};

// One workgroup reduces elements [c0, c1) of one row.  NT threads, U vectors
// per lane in flight per buffer, two buffers.
template <typename T, int NT, int U>
__global__ __launch_bounds__(NT) void confidence_kernel(
    const T *__restrict__ logits, int S, int V, int64_t row_stride, int64_t batch_stride,
    const int32_t *__restrict__ suffix_len, int splits, int seg_elems,
    int32_t *__restrict__ top1_id, float *__restrict__ top1_prob, float *__restrict__ margin,
    Partial *__restrict__ partials) {
  constexpr int N = Vec<T>::N;
  const int split = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
  if (suffix_len != nullptr && i >= suffix_len[b]) return;
  const int tid = threadIdx.x;
  const int c0 = split * seg_elems;
  const int c1 = min(V, c0 + seg_elems);
  const T *row = logits + int64_t(b) * batch_stride + int64_t(i) * row_stride;

  Top t;
  top_init(t);

  // split [c0,c1) into an unaligned head, 16-byte vectors, and a tail
  const int len = c1 - c0;
  int head = int(((16u - (unsigned(reinterpret_cast<uintptr_t>(row + c0)) & 15u)) & 15u) / sizeof(T));
  head = min(head, len);
  const int nvec = (len - head) / N;
  const int tail0 = c0 + head + nvec * N;

  if (tid < head) {
    float x[1] = {Vec<T>::scalar(row + c0 + tid)};
    absorb<1>(t, x, c0 + tid);
  }

  const u32x4 *vp = reinterpret_cast<const u32x4 *>(row + c0 + head);
  const int vbase = c0 + head;  // element index of vector 0
  constexpr int G = NT * U;     // vectors per full group
  const int ngroups = nvec / G;
  if (ngroups > 0) {
    u32x4 cur[U], nxt[U];
#pragma unroll
    for (int u = 0; u < U; ++u) cur[u] = __builtin_nontemporal_load(vp + u * NT + tid);
    for (int g = 0; g < ngroups; ++g) {
      const int v0 = g * G + tid;
      if (g + 1 < ngroups) {
#pragma unroll
        for (int u = 0; u < U; ++u) nxt[u] = __builtin_nontemporal_load(vp + v0 + G + u * NT);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float x[N];
        Vec<T>::unpack(cur[u], x);
        absorb<N>(t, x, ~(vbase + (v0 + u * NT) * N));
      }
#pragma unroll
      for (int u = 0; u < U; ++u) cur[u] = nxt[u];
    }
  }
  for (int v = ngroups * G + tid; v < nvec; v += NT) {
    const u32x4 w = __builtin_nontemporal_load(vp + v);
    float x[N];
    Vec<T>::unpack(w, x);
    absorb<N>(t, x, ~(vbase + v * N));
  }
  if (tid < c1 - tail0) {
    float x[1] = {Vec<T>::scalar(row + tail0 + tid)};
    absorb<1>(t, x, tail0 + tid);
  }

  // resolve the lane's arg-max inside its remembered vector
  if (t.idx < 0) {
    const int e0 = ~t.idx;
    const u32x4 w = *reinterpret_cast<const u32x4 *>(row + e0);
    float x[N];
    Vec<T>::unpack(w, x);
    int j = N - 1;
#pragma unroll
    for (int k = N - 2; k >= 0; --k) j = (x[k] == t.m1) ? k : j;
    t.idx = e0 + j;
  }

#pragma unroll
  for (int m = 1; m < kWave; m <<= 1) t = merge(t, shfl_xor(t, m));

  constexpr int NW = NT / kWave;
  __shared__ Top lds[NW];
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  if (NW > 1) {
    if (lane == 0) lds[wave] = t;
    __syncthreads();
    if (wave != 0) return;
    if (lane < NW) t = lds[lane]; else top_init(t);
#pragma unroll
    for (int m = 1; m < NW; m <<= 1) t = merge(t, shfl_xor(t, m));
  }
  if (tid != 0) return;
  // an all -inf segment has an empty sum
  const float s = t.m1 == -INFINITY ? 0.f : t.s * __builtin_amdgcn_exp2f(t.r - t.m1 * kLog2e);
  const int64_t o = int64_t(b) * S + i;
  if (splits == 1) {
    top1_id[o] = t.idx;
    margin[o] = t.m1 - t.m2;
    top1_prob[o] = 1.0f / s;
  } else {
    Partial p;
    p.m1 = t.m1; p.m2 = t.m2; p.s = s; p.idx = t.idx;
    partials[o * splits + split] = p;
  }
}

// One thread per row folds the row's `splits` segment results, in index order.
__global__ void confidence_finish_kernel(const Partial *__restrict__ partials, int rows, int S,
                                         int splits, const int32_t *__restrict__ suffix_len,
                                         int32_t *__restrict__ top1_id,
                                         float *__restrict__ top1_prob,
                                         float *__restrict__ margin) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= rows) return;
  if (suffix_len != nullptr && (o % S) >= suffix_len[o / S]) return;
  Partial a = partials[int64_t(o) * splits];
  for (int k = 1; k < splits; ++k) {
    const Partial p = partials[int64_t(o) * splits + k];
    const float M = __builtin_fmaxf(a.m1, p.m1);
    const float m2 = __builtin_fmaxf(__builtin_fminf(a.m1, p.m1), __builtin_fmaxf(a.m2, p.m2));
    const float wa = a.m1 == M ? 1.f : __builtin_amdgcn_exp2f((a.m1 - M) * kLog2e);
    const float wp = p.m1 == M ? 1.f : __builtin_amdgcn_exp2f((p.m1 - M) * kLog2e);
    const float s = a.s * wa + p.s * wp;
    a.idx = p.m1 > a.m1 ? p.idx : a.idx;  // earlier segment keeps an equal maximum
    a.m1 = M; a.m2 = m2; a.s = s;
  }
  top1_id[o] = a.idx;
  margin[o] = a.m1 - a.m2;
  top1_prob[o] = 1.0f / a.s;
}

// Rows are split only when there are too few of them to occupy the chip.
struct Plan {
  int splits, seg_elems;
};
inline Plan plan(int64_t rows, int V) {
  Plan p;
  int splits = 1;
  if (rows < 192) {
    splits = int((512 + rows - 1) / rows);
    const int max_by_len = (V + 8191) / 8192;  // keep segments >= 8192 elements
    if (splits > max_by_len) splits = max_by_len;
    if (splits > 32) splits = 32;
    if (splits < 1) splits = 1;
  }
  int seg = (V + splits - 1) / splits;
  seg = (seg + 63) / 64 * 64;
  p.seg_elems = seg;
  p.splits = (V + seg - 1) / seg;
  return p;
}

}  // namespace
}  // namespace lsp

extern "C" size_t lsp_confidence_workspace_bytes(int32_t B, int32_t S, int32_t V) {
  if (B <= 0 || S <= 0 || V <= 0) return 0;
  const lsp::Plan p = lsp::plan(int64_t(B) * S, V);
  return p.splits > 1 ? size_t(B) * S * p.splits * sizeof(lsp::Partial) : 0;
}

extern "C" int32_t lsp_confidence(int32_t dtype, const void *logits, int32_t B, int32_t S, int32_t V,
                                  int64_t row_stride, int64_t batch_stride,
                                  const int32_t *suffix_len, int32_t *top1_id, float *top1_prob,
                                  float *margin, void *workspace, size_t workspace_bytes,
                                  void *stream) {
  using namespace lsp;
  LSP_CHECK_ARG(dtype == LSP_F32 || dtype == LSP_BF16, "lsp_confidence: unknown dtype %d", dtype);
  LSP_CHECK_ARG(logits && top1_id && top1_prob && margin, "lsp_confidence: null pointer");
  LSP_CHECK_ARG(B > 0 && S > 0 && V >= 2, "lsp_confidence: need B>0, S>0, V>=2 (got %d %d %d)", B, S, V);
  LSP_CHECK_ARG(B <= 65535 && S <= 65535, "lsp_confidence: B and S must be <= 65535");
  if (row_stride == 0) row_stride = V;
  if (batch_stride == 0) batch_stride = int64_t(S) * row_stride;
  LSP_CHECK_ARG(row_stride >= V && batch_stride >= 0, "lsp_confidence: bad strides");
  const size_t es = elem_size(dtype);
  LSP_CHECK_ARG((reinterpret_cast<uintptr_t>(logits) & (es - 1)) == 0, "lsp_confidence: logits misaligned");
  const Plan p = plan(int64_t(B) * S, V);
  const size_t need = p.splits > 1 ? size_t(B) * S * p.splits * sizeof(Partial) : 0;
  if (need > 0 && (workspace == nullptr || workspace_bytes < need ||
                   (reinterpret_cast<uintptr_t>(workspace) & 15u))) {
    set_error("lsp_confidence: workspace of %zu bytes (16-byte aligned) required, got %zu", need, workspace_bytes);
    return LSP_ERR_WORKSPACE;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid(p.splits, S, B);
  Partial *parts = static_cast<Partial *>(workspace);
  const int64_t seg_bytes = int64_t(p.seg_elems) * es;
  // big segments: 1024 threads, 4 vectors in flight per lane per buffer; small ones: 256 threads
  if (dtype == LSP_BF16) {
    const uint16_t *z = static_cast<const uint16_t *>(logits);
    if (seg_bytes >= 128 * 1024)
      confidence_kernel<uint16_t, 1024, 4><<<grid, 1024, 0, st>>>(z, S, V, row_stride, batch_stride, suffix_len, p.splits, p.seg_elems, top1_id, top1_prob, margin, parts);
    else
      confidence_kernel<uint16_t, 256, 4><<<grid, 256, 0, st>>>(z, S, V, row_stride, batch_stride, suffix_len, p.splits, p.seg_elems, top1_id, top1_prob, margin, parts);
  } else {
    const float *z = static_cast<const float *>(logits);
    if (seg_bytes >= 128 * 1024)
      confidence_kernel<float, 1024, 4><<<grid, 1024, 0, st>>>(z, S, V, row_stride, batch_stride, suffix_len, p.splits, p.seg_elems, top1_id, top1_prob, margin, parts);
    else
      confidence_kernel<float, 256, 4><<<grid, 256, 0, st>>>(z, S, V, row_stride, batch_stride, suffix_len, p.splits, p.seg_elems, top1_id, top1_prob, margin, parts);
  }
  LSP_CHECK_LAUNCH("lsp_confidence: launch");
  if (p.splits > 1) {
    const int rows = B * S;
    confidence_finish_kernel<<<(rows + 255) / 256, 256, 0, st>>>(parts, rows, S, p.splits, suffix_len, top1_id, top1_prob, margin);
    LSP_CHECK_LAUNCH("lsp_confidence: finish launch");
  }
  return LSP_OK;
}
