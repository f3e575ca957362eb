// Library-wide pieces of liblsp: error text, version, flip bookkeeping.
#include <stdarg.h>

#include "lsp_common.h"

namespace lsp {

static thread_local char g_error[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}

namespace {

// Section 4.3.4 flip bookkeeping: one workgroup per sequence; a position counts
// when it already had a prediction at the previous step.  The sequence's counts
// also go to the mid-generation window when the number of its positions already
// committed lies in [window_lo, window_hi].
__global__ __launch_bounds__(256) void flip_kernel(
    const int32_t *__restrict__ top1_id, int S, int G, const int32_t *__restrict__ prefix_len,
    const int32_t *__restrict__ suffix_len, const int32_t *__restrict__ base_prefix_len,
    int32_t *__restrict__ last_id, unsigned long long *__restrict__ counters, int window_lo,
    int window_hi, int32_t *__restrict__ step_counts) {
  __shared__ int total[2];
  const int b = blockIdx.x;
  const int N = min(max(suffix_len[b], 0), S);
  const int done = prefix_len[b] - base_prefix_len[b];
  if (threadIdx.x < 2) total[threadIdx.x] = 0;
  __syncthreads();
  int flips = 0, seen = 0;
  for (int u = threadIdx.x; u < N; u += blockDim.x) {
    const int j = done + u;
    if (j < 0 || j >= G) continue;
    const int32_t cur = top1_id[int64_t(b) * S + u];
    const int32_t old = last_id[int64_t(b) * G + j];
    if (old >= 0) {
      ++seen;
      flips += (old != cur);
    }
    last_id[int64_t(b) * G + j] = cur;
  }
#pragma unroll
  for (int m = 1; m < kWave; m <<= 1) {
    flips += __shfl_xor(flips, m);
    seen += __shfl_xor(seen, m);
  }
  if ((threadIdx.x & (kWave - 1)) == 0 && seen > 0) {
    atomicAdd(&total[0], flips);
    atomicAdd(&total[1], seen);
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  if (step_counts != nullptr) {
    step_counts[2 * b] = total[0];
    step_counts[2 * b + 1] = total[1];
  }
  if (total[1] > 0) {
    atomicAdd(&counters[0], (unsigned long long)total[0]);
    atomicAdd(&counters[1], (unsigned long long)total[1]);
    if (done >= window_lo && done <= window_hi) {
      atomicAdd(&counters[2], (unsigned long long)total[0]);
      atomicAdd(&counters[3], (unsigned long long)total[1]);
    }
  }
}

// Measurement helper: a bare streaming read.  Workgroup w reads segment w of the buffer
// with 16-byte non-temporal loads, four in flight per lane, and folds them with XOR; one
// word per workgroup is written.  This is the floor under any kernel that has to read a
// buffer of that size once (launch, first loads, drain included).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(512) void read_kernel(const u32x4 *__restrict__ p, int64_t vec_per_wg,
                                                   uint32_t *__restrict__ out) {
  const u32x4 *q = p + int64_t(blockIdx.x) * vec_per_wg;
  u32x4 acc = {0, 0, 0, 0};
  int64_t i = threadIdx.x;
  for (; i + 3 * 512 < vec_per_wg; i += 4 * 512) {
    const u32x4 a = __builtin_nontemporal_load(q + i), b = __builtin_nontemporal_load(q + i + 512);
    const u32x4 c = __builtin_nontemporal_load(q + i + 1024), d = __builtin_nontemporal_load(q + i + 1536);
    acc ^= a ^ b ^ c ^ d;
  }
  for (; i < vec_per_wg; i += 512) acc ^= __builtin_nontemporal_load(q + i);
  uint32_t v = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
  for (int m = 1; m < kWave; m <<= 1) v ^= __shfl_xor(v, m);
  if ((threadIdx.x & (kWave - 1)) == 0) atomicXor(&out[blockIdx.x], v);
}

// Measurement helper: a bare matrix-instruction loop (no memory traffic inside the loop).
// Every lane loads 8 A and 8 B fragments (16 bytes each) once, then issues
// v_mfma_f32_32x32x16_bf16 over them round robin into four accumulators.  What it sustains
// depends on the operand VALUES: with random operands the chip lowers its clock to stay inside
// its power limit, so this is the matrix ceiling a kernel working on such data can be held to.
typedef float f32x16 __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(512) void mfma_kernel(const u32x4 *__restrict__ operands, int32_t iters,
                                                   float *__restrict__ out) {
  u32x4 A[8], B[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    A[s] = operands[s * 512 + threadIdx.x];
    B[s] = operands[(8 + s) * 512 + threadIdx.x];
  }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 8; ++s)
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[s & 3]) : "v"(A[s]), "v"(B[(s * 3 + 1) & 7]));
  }
  float t = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) t += acc[n][r];
  out[blockIdx.x * 512 + threadIdx.x] = t;
}

}  // namespace
}  // namespace lsp

extern "C" int32_t lsp_bench_mfma(const void *operands, int32_t iters, int32_t workgroups, float *out, void *stream) {
  using namespace lsp;
  LSP_CHECK_ARG(operands && out && iters > 0 && workgroups > 0, "lsp_bench_mfma: bad argument");
  LSP_CHECK_ARG(aligned16(operands), "lsp_bench_mfma: operands must be 16-byte aligned");
  mfma_kernel<<<workgroups, 512, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const u32x4 *>(operands), iters, out);
  LSP_CHECK_LAUNCH("lsp_bench_mfma: launch");
  return LSP_OK;
}

extern "C" int32_t lsp_bench_read(const void *buffer, int64_t bytes, int32_t workgroups, uint32_t *out, void *stream) {
  using namespace lsp;
  LSP_CHECK_ARG(buffer && out && bytes > 0 && workgroups > 0, "lsp_bench_read: bad argument");
  LSP_CHECK_ARG(aligned16(buffer) && bytes % (int64_t(workgroups) * 16) == 0,
                "lsp_bench_read: buffer must be 16-byte aligned and split evenly into 16-byte vectors per workgroup");
  read_kernel<<<workgroups, 512, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const u32x4 *>(buffer),
                                                                         bytes / (int64_t(workgroups) * 16), out);
  LSP_CHECK_LAUNCH("lsp_bench_read: launch");
  return LSP_OK;
}

extern "C" const char *lsp_version(void) { return "liblsp 0.1 (gfx950)"; }
extern "C" const char *lsp_last_error(void) { return lsp::g_error; }

extern "C" int32_t lsp_flip_update(const int32_t *top1_id, int32_t B, int32_t S, int32_t G,
                                   const int32_t *prefix_len, const int32_t *suffix_len,
                                   const int32_t *base_prefix_len, int32_t *last_id,
                                   int64_t *counters, int32_t window_lo, int32_t window_hi,
                                   int32_t *step_counts, void *stream) {
  using namespace lsp;
  LSP_CHECK_ARG(top1_id && prefix_len && suffix_len && base_prefix_len && last_id && counters,
                "lsp_flip_update: null pointer");
  LSP_CHECK_ARG(B > 0 && S > 0 && G > 0, "lsp_flip_update: bad B/S/G");
  flip_kernel<<<B, 256, 0, static_cast<hipStream_t>(stream)>>>(
      top1_id, S, G, prefix_len, suffix_len, base_prefix_len, last_id,
      reinterpret_cast<unsigned long long *>(counters), window_lo, window_hi, step_counts);
  LSP_CHECK_LAUNCH("lsp_flip_update: launch");
  return LSP_OK;
}
