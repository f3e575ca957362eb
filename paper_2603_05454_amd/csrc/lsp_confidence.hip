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
//     which group of its 16-byte vectors its running maximum last rose
//     strictly; since a lane visits its elements in increasing index order,
//     that group holds the lane's first occurrence of its maximum, and it is
//     re-read once at the end - by the lanes that hold the wave's maximum only
//     (every lane doing so would add 16 KB of scattered cache lines per wave);
//   - the soft-max sum uses one exp2 per element against a lagging per-lane
//     reference r (log2 domain) which is only moved when the lane maximum has
//     run more than 32 octaves ahead of it, so the rescale branch is cold.  A
//     group's top-2 pass runs before its sum pass, so the reference always
//     covers the values being exponentiated.
// Lane results are merged in two steps: the maximum first (DPP reduction), then
// each lane rescales its sum to it and the runner-up, the sum and the lowest
// index among the lanes holding the maximum are plain max / add / min
// reductions.  The same merge runs across the waves of a workgroup through
// LDS and - when one row is split over several workgroups because there are
// too few rows to fill the chip - across workgroups in a second tiny kernel.
#include <float.h>
#include <limits.h>

#include <mutex>
#include <type_traits>

#include "lsp_common.h"

namespace lsp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLagOctaves = 32.0f;  // the reference may lag the maximum by this much

struct Top {
  float m1, m2;  // largest and second largest value seen (duplicates count)
  float s;       // sum of exp2(x*log2e - r)
  float r;       // reference exponent (log2 domain): some earlier maximum times log2e, ROUNDED
  int idx;       // >= 0: element index of the first maximum; < 0: ~(first element of the lane's group holding it)
};

__device__ __forceinline__ void top_init(Top &t) {
  t.m1 = -INFINITY;
  t.m2 = -INFINITY;
  t.s = 0.f;
  t.r = -FLT_MAX;
  t.idx = INT_MAX;
}

// max as exactly one v_max_f32.  fmaxf() costs two here: the kernel runs in IEEE
// mode, where the compiler first quiets a possible signalling NaN in each
// operand; the precondition excludes NaN, so the bare instruction is enough.
__device__ __forceinline__ float fmax_raw(float a, float b) {
  float d;
  asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
  return d;
}

// Top-2 update over N values; `tag` is recorded when the maximum rose strictly.
template <int N>
__device__ __forceinline__ void absorb_top2(Top &t, const float (&x)[N]) {
#pragma unroll
  for (int j = 0; j < N; ++j) {
    t.m2 = __builtin_amdgcn_fmed3f(t.m1, x[j], t.m2);
    t.m1 = fmax_raw(t.m1, x[j]);
  }
}

// Move the reference up when the maximum has run ahead of it (cold branch).
__device__ __forceinline__ void settle_reference(Top &t) {
  const float mc = t.m1 * kLog2e;
  if (mc - t.r > kLagOctaves) {
    t.s *= __builtin_amdgcn_exp2f(t.r - mc);
    t.r = mc;
  }
}

// Soft-max sum over N values that are already covered by t.m1 / t.r.
template <int N>
__device__ __forceinline__ void absorb_sum(Top &t, const float (&x)[N]) {
  // One fma + exp2 per element.  r is a ROUNDED product, so every term is off by
  // the same factor 2^(m*log2e - r) (up to 2e-5 for logits around 500); the fold
  // in wave_combine takes the sum off this reference with an fma of its own,
  // which removes that factor exactly.
  const float nr = -t.r;
#pragma unroll
  for (int j = 0; j < N; ++j) t.s += __builtin_amdgcn_exp2f(__builtin_fmaf(x[j], kLog2e, nr));
}

template <int N>
__device__ __forceinline__ void absorb(Top &t, const float (&x)[N], int tag) {
  const float old = t.m1;
  absorb_top2<N>(t, x);
  t.idx = t.m1 > old ? tag : t.idx;
  settle_reference(t);
  absorb_sum<N>(t, x);
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

// ---- cross-lane reductions on the DPP network (no LDS traffic) ---------------
// Classic GCN reduction: two quad permutes, row shifts by 4 and 8, then the row
// broadcasts 15 and 31; lane 63 ends up holding the reduction of all 64 lanes.
// Lanes without a source keep op(v, v), which never feeds lane 63.
template <typename Op>
__device__ __forceinline__ float wave_reduce(float v, Op op) {
#define LSP_DPP_STEP(ctrl)                                                                    \
  v = op(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), \
                                                       ctrl, 0xf, 0xf, false)))
  LSP_DPP_STEP(0xb1);   // quad_perm [1,0,3,2]
  LSP_DPP_STEP(0x4e);   // quad_perm [2,3,0,1]
  LSP_DPP_STEP(0x114);  // row_shr:4
  LSP_DPP_STEP(0x118);  // row_shr:8
  LSP_DPP_STEP(0x142);  // row_bcast:15
  LSP_DPP_STEP(0x143);  // row_bcast:31
#undef LSP_DPP_STEP
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmax_raw(a, b); } };
struct OpAdd { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
// min over non-negative ints: their float bit patterns order the same way
struct OpMinI {
  __device__ __forceinline__ float operator()(float a, float b) const {
    return __int_as_float(min(__float_as_int(a), __float_as_int(b)));
  }
};

struct RowStat {  // wave-uniform: maximum, second, sum of exp(x - m1), first index of the maximum
  float m1, m2, s;
  int idx;
};

// Combine the 64 lane states of a wave, given the maximum over the lanes and the
// factor w that takes this lane's sum from its own reference to that maximum.
// The remaining reductions are plain max/add/min.  A lane's idx is only read
// when the lane holds the maximum.
__device__ __forceinline__ RowStat wave_combine(const Top &t, float wave_max, float w) {
  RowStat o;
  o.m1 = wave_max;
  const bool top = t.m1 == o.m1;
  const int ntop = __popcll(__ballot(top));
  const float second = wave_reduce(top ? t.m2 : t.m1, OpMax());
  o.m2 = ntop >= 2 ? o.m1 : second;  // the maximum held by two lanes is its own runner-up
  o.idx = __float_as_int(wave_reduce(__int_as_float(top ? t.idx : INT_MAX), OpMinI()));
  const float sum = wave_reduce(t.s * w, OpAdd());
  o.s = o.m1 == -INFINITY ? 0.f : sum;  // an all -inf segment has an empty sum
  return o;
}

// One workgroup reduces elements [c0, c1) of one row.  NT threads; U vectors per
// lane per group; two groups of loads in flight (ping-pong register buffers).
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
  constexpr int G = NT * U;     // vectors per group
  const int ngroups = (nvec + G - 1) / G;  // the last one may be partial

  // Lanes past the end of the last, partial group re-read the row's last vector
  // (their values are replaced by -inf below), so that group is one burst of
  // loads like every other.
  auto load_group = [&](u32x4 (&buf)[U], int g, auto last) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int v = g * G + u * NT + tid;
      buf[u] = __builtin_nontemporal_load(vp + (decltype(last)::value ? min(v, nvec - 1) : v));
    }
  };
  // phase 1: top-2 over the whole group, one index tag and one reference check per
  // group; phase 2: the soft-max sum.  (The tag names the lane's first vector of the
  // group; the lane keeps a copy of its U vectors of that group, eight selects per
  // group, and scans the copy at the end.  Re-reading them from memory instead put
  // a dependent round trip at the end of every row.)
  u32x4 kept[U];
#pragma unroll
  for (int u = 0; u < U; ++u) kept[u] = u32x4{0, 0, 0, 0};
  auto process_group = [&](const u32x4 (&buf)[U], int g, auto last) {
    float x[U][N];
    const float old = t.m1;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      Vec<T>::unpack(buf[u], x[u]);
      if (decltype(last)::value && g * G + u * NT + tid >= nvec) {
#pragma unroll
        for (int k = 0; k < N; ++k) x[u][k] = -INFINITY;  // never the maximum, adds 0 to the sum
      }
      absorb_top2<N>(t, x[u]);
    }
    const bool rose = t.m1 > old;
    t.idx = rose ? ~(vbase + (g * G + tid) * N) : t.idx;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      kept[u].x = rose ? buf[u].x : kept[u].x;
      kept[u].y = rose ? buf[u].y : kept[u].y;
      kept[u].z = rose ? buf[u].z : kept[u].z;
      kept[u].w = rose ? buf[u].w : kept[u].w;
    }
    settle_reference(t);
#pragma unroll
    for (int u = 0; u < U; ++u) absorb_sum<N>(t, x[u]);
  };
  if (ngroups > 0) {
    const std::false_type full;
    const std::true_type maybe_partial;
    u32x4 ping[U], pong[U];
    if (ngroups == 1) load_group(ping, 0, maybe_partial); else load_group(ping, 0, full);
    int g = 0;
    for (; g + 3 < ngroups; g += 2) {  // groups g+1 and g+2 are full
      load_group(pong, g + 1, full);
      process_group(ping, g, full);
      load_group(ping, g + 2, full);
      process_group(pong, g + 1, full);
    }
    // one to three groups left; only the very last may be partial
    if (g + 2 < ngroups) {
      load_group(pong, g + 1, full);
      process_group(ping, g, full);
      load_group(ping, g + 2, maybe_partial);
      process_group(pong, g + 1, full);
      process_group(ping, g + 2, maybe_partial);
    } else if (g + 1 < ngroups) {
      load_group(pong, g + 1, maybe_partial);
      process_group(ping, g, full);
      process_group(pong, g + 1, maybe_partial);
    } else {
      process_group(ping, g, maybe_partial);
    }
  }
  if (tid < c1 - tail0) {
    float x[1] = {Vec<T>::scalar(row + tail0 + tid)};
    absorb<1>(t, x, tail0 + tid);
  }

  // A lane whose maximum came from a group scans its copy of that group, from the
  // last vector to the first so that the lowest index wins.
  const float wave_max = wave_reduce(t.m1, OpMax());
  if (t.idx < 0) {
    const int e0 = ~t.idx;
    int found = INT_MAX;
#pragma unroll
    for (int u = U - 1; u >= 0; --u) {
      const int eb = e0 + u * NT * N;
      if (eb >= tail0) continue;  // past the end of a partial group (the copy holds a repeat of the last vector)
      float x[N];
      Vec<T>::unpack(kept[u], x);
#pragma unroll
      for (int k = N - 1; k >= 0; --k) found = (x[k] == t.m1) ? eb + k : found;
    }
    t.idx = found;
  }

  // exp2(r - max*log2e) with the product unrounded inside the fma; 0 for an empty lane (r = -FLT_MAX)
  RowStat r = wave_combine(t, wave_max, __builtin_amdgcn_exp2f(__builtin_fmaf(-wave_max, kLog2e, t.r)));
  constexpr int NW = NT / kWave;
  if (NW > 1) {
    __shared__ RowStat lds[NW];
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    if (lane == 0) lds[wave] = r;
    __syncthreads();
    if (wave != 0) return;
    top_init(t);
    if (lane < NW) {
      const RowStat w = lds[lane];
      t.m1 = w.m1; t.m2 = w.m2; t.s = w.s; t.idx = w.idx;
    }
    // a wave's sum is relative to that wave's own maximum: exp((m1 - max)), 0 for the lanes beyond NW
    const float all_max = wave_reduce(t.m1, OpMax());
    r = wave_combine(t, all_max, __builtin_amdgcn_exp2f((t.m1 - all_max) * kLog2e));
  }
  if (tid != 0) return;
  const int64_t o = int64_t(b) * S + i;
  if (splits == 1) {
    top1_id[o] = r.idx;
    margin[o] = r.m1 - r.m2;
    top1_prob[o] = 1.0f / r.s;
  } else {
    Partial p;
    p.m1 = r.m1; p.m2 = r.m2; p.s = r.s; p.idx = r.idx;
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

// Launch shape (measured on MI355X).  A workgroup takes a row; it is as wide as
// leaves each lane about 64 vectors of 16 bytes (one wave for rows of a few
// thousand entries, four waves for a 126 464-entry bf16 row: 2-7 % faster there
// than one wave per row, and a 512-thread workgroup is 3x slower on 4 096-entry
// rows); with few rows it widens further so that at least 2048 waves are in
// flight, and below that rows are also cut into segments reduced by separate
// workgroups.  Per element the kernel issues about nine VALU cycles (the
// exponential counts four), which at these sizes is as long as the memory time
// itself.
struct Plan {
  int nt, splits, seg_elems;
};
inline Plan plan(int64_t rows, int V, int elem_bytes) {
  Plan p;
  int nt = 64;
  const int64_t nvec = int64_t(V) * elem_bytes / 16;
  while (nt < 512 && nvec / nt >= 96) nt *= 2;
  while (nt < 512 && rows * (nt / 64) < 2048) nt *= 2;
  int splits = 1;
  const int64_t waves = rows * (nt / 64);
  if (waves < 1024) {
    splits = int((2048 + waves - 1) / waves);
    const int max_by_len = (V + 16383) / 16384;  // keep segments >= 16384 elements
    if (splits > max_by_len) splits = max_by_len;
    if (splits > 32) splits = 32;
    if (splits < 1) splits = 1;
  }
  int seg = (V + splits - 1) / splits;
  seg = (seg + 63) / 64 * 64;
  p.nt = nt;
  p.seg_elems = seg;
  p.splits = (V + seg - 1) / seg;
  return p;
}

template <typename T, int NT, int U>
void launch_one(const Plan &p, dim3 grid, hipStream_t st, const T *z, int S, int V,
                int64_t row_stride, int64_t batch_stride, const int32_t *suffix_len,
                int32_t *top1_id, float *top1_prob, float *margin, Partial *parts) {
  confidence_kernel<T, NT, U><<<grid, NT, 0, st>>>(z, S, V, row_stride, batch_stride, suffix_len,
                                                   p.splits, p.seg_elems, top1_id, top1_prob,
                                                   margin, parts);
}

template <typename T>
void launch_confidence(const Plan &p, dim3 grid, hipStream_t st, const T *z, int S, int V,
                       int64_t row_stride, int64_t batch_stride, const int32_t *suffix_len,
                       int32_t *top1_id, float *top1_prob, float *margin, Partial *parts) {
#define LSP_CONF_CASE(NT_)                                                                      \
  if (p.nt == NT_)                                                                              \
    return launch_one<T, NT_, 2>(p, grid, st, z, S, V, row_stride, batch_stride, suffix_len,    \
                                 top1_id, top1_prob, margin, parts)
  LSP_CONF_CASE(64);
  LSP_CONF_CASE(128);
  LSP_CONF_CASE(256);
  LSP_CONF_CASE(512);
#undef LSP_CONF_CASE
}

}  // namespace
}  // namespace lsp

extern "C" size_t lsp_confidence_workspace_bytes(int32_t B, int32_t S, int32_t V) {
  if (B <= 0 || S <= 0 || V <= 0) return 0;
  // the dtype is not an argument here: enough for either
  const int s2 = lsp::plan(int64_t(B) * S, V, 2).splits, s4 = lsp::plan(int64_t(B) * S, V, 4).splits;
  const int splits = s2 > s4 ? s2 : s4;
  return splits > 1 ? size_t(B) * S * splits * sizeof(lsp::Partial) : 0;
}

namespace lsp {
namespace {

int32_t scratch_address(void **out);  // device address of the library's own scratch buffer (defined below)

// Host side shared by both entry points: validation, launch plan, launches.
// `parts` is where split rows leave their per-segment results (`parts_bytes`
// available); `who` names the entry point in error texts and `fixed_scratch`
// says that the buffer is the library's own (a different error then).
int32_t confidence_run(const char *who, bool fixed_scratch, int32_t dtype, const void *logits, int32_t B,
                       int32_t S, int32_t V, int64_t row_stride, int64_t batch_stride,
                       const int32_t *suffix_len, int32_t *top1_id, float *top1_prob, float *margin,
                       void *parts_mem, size_t parts_bytes, void *stream) {
  LSP_CHECK_ARG(dtype == LSP_F32 || dtype == LSP_BF16, "%s: unknown dtype %d", who, dtype);
  LSP_CHECK_ARG(logits && top1_id && top1_prob && margin, "%s: null pointer", who);
  LSP_CHECK_ARG(B > 0 && S > 0 && V >= 2, "%s: need B>0, S>0, V>=2 (got %d %d %d)", who, B, S, V);
  LSP_CHECK_ARG(B <= 65535 && S <= 65535, "%s: B and S must be <= 65535", who);
  if (row_stride == 0) row_stride = V;
  if (batch_stride == 0) batch_stride = int64_t(S) * row_stride;
  LSP_CHECK_ARG(row_stride >= V && batch_stride >= 0, "%s: bad strides", who);
  const size_t es = elem_size(dtype);
  LSP_CHECK_ARG((reinterpret_cast<uintptr_t>(logits) & (es - 1)) == 0, "%s: logits misaligned", who);
  const Plan p = plan(int64_t(B) * S, V, int(es));
  const size_t need = p.splits > 1 ? size_t(B) * S * p.splits * sizeof(Partial) : 0;
  if (need > 0 && fixed_scratch && parts_bytes < need) {
    set_error("%s: this shape needs %zu bytes of scratch, the built-in buffer holds %zu; use lsp_confidence "
              "with a workspace", who, need, parts_bytes);
    return LSP_ERR_UNSUPPORTED;
  }
  if (fixed_scratch) {  // looked up only after the arguments have passed validation
    const int32_t rc = scratch_address(&parts_mem);
    if (rc != LSP_OK) return rc;
  }
  if (need > 0 && (parts_mem == nullptr || parts_bytes < need || (reinterpret_cast<uintptr_t>(parts_mem) & 15u))) {
    set_error("%s: workspace of %zu bytes (16-byte aligned) required, got %zu", who, need, parts_bytes);
    return LSP_ERR_WORKSPACE;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid(p.splits, S, B);
  Partial *parts = static_cast<Partial *>(parts_mem);
  if (dtype == LSP_BF16)
    launch_confidence<uint16_t>(p, grid, st, static_cast<const uint16_t *>(logits), S, V, row_stride,
                                batch_stride, suffix_len, top1_id, top1_prob, margin, parts);
  else
    launch_confidence<float>(p, grid, st, static_cast<const float *>(logits), S, V, row_stride,
                             batch_stride, suffix_len, top1_id, top1_prob, margin, parts);
  LSP_CHECK_LAUNCH("lsp_confidence: launch");
  if (p.splits > 1) {
    const int rows = B * S;
    confidence_finish_kernel<<<(rows + 255) / 256, 256, 0, st>>>(parts, rows, S, p.splits, suffix_len, top1_id, top1_prob, margin);
    LSP_CHECK_LAUNCH("lsp_confidence: finish launch");
  }
  return LSP_OK;
}

}  // namespace
}  // namespace lsp

extern "C" int32_t lsp_confidence(int32_t dtype, const void *logits, int32_t B, int32_t S, int32_t V,
                                  int64_t row_stride, int64_t batch_stride,
                                  const int32_t *suffix_len, int32_t *top1_id, float *top1_prob,
                                  float *margin, void *workspace, size_t workspace_bytes,
                                  void *stream) {
  return lsp::confidence_run("lsp_confidence", false, dtype, logits, B, S, V, row_stride, batch_stride,
                             suffix_len, top1_id, top1_prob, margin, workspace, workspace_bytes, stream);
}

// ---- the same call for callers that cannot allocate ----------------------------
// The per-segment results of split rows go to a buffer that is part of the
// library's device image instead of a caller-provided workspace.  Rows are only
// split when there are fewer than 128 of them, into at most 32 segments of 16
// bytes each, so 64 KB cover every shape the launch plan can produce.
#define LSP_CONF_SCRATCH_BYTES 65536
static __device__ __align__(256) unsigned char scratch[LSP_CONF_SCRATCH_BYTES];

namespace lsp {
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU (every GPU has its own copy)

// Device address of the scratch array on the current GPU, looked up once per GPU.
int32_t scratch_address(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "lsp_confidence_static: hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) {
    set_error("lsp_confidence_static: device ordinal %d not supported (< %d)", dev, kMaxDevices);
    return LSP_ERR_UNSUPPORTED;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) return hip_fail(e, "lsp_confidence_static: hipGetSymbolAddress");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LSP_OK;
}
}  // namespace
}  // namespace lsp

extern "C" size_t lsp_confidence_static_scratch_bytes(void) { return LSP_CONF_SCRATCH_BYTES; }

extern "C" int32_t lsp_confidence_static(int32_t dtype, const void *logits, int32_t B, int32_t S, int32_t V,
                                         int64_t row_stride, int64_t batch_stride,
                                         const int32_t *suffix_len, int32_t *top1_id, float *top1_prob,
                                         float *margin, void *stream) {
  // Every segment result that the second kernel reads is written by the first
  // kernel of the same call, so nothing has to be cleared between calls.
  return lsp::confidence_run("lsp_confidence_static", true, dtype, logits, B, S, V, row_stride, batch_stride,
                             suffix_len, top1_id, top1_prob, margin, nullptr, LSP_CONF_SCRATCH_BYTES, stream);
}
