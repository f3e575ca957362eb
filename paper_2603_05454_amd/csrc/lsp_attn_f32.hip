// fp32 variant of the suffix attention (Algorithm 1 line 4; Section 3.2): plain
// FMA arithmetic, one query row per lane, K/V tiles staged in LDS and read as
// wave-wide broadcasts.  It exists for full-precision callers and checks (the
// bf16 MFMA kernel in lsp_attn_bf16.hip is the throughput path).
#include "lsp_attn.h"

namespace lsp {
namespace {

constexpr int kQ = 64;   // query rows per workgroup (one per lane)
constexpr int kKT = 32;  // keys per LDS tile
constexpr int kKC = 8;   // keys per soft-max update

template <int D>
__global__ __launch_bounds__(kQ) void attn_f32_kernel(AttnArgs a) {
  const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * kQ;
  const int N = min(max(a.suffix_len[b], 0), a.S);
  if (q0 >= N) return;
  const int P = min(max(a.prefix_len[b], 0), a.C);
  const int g = h / (a.Hq / a.Hkv);
  const int tid = threadIdx.x;
  const int i = min(q0 + tid, N - 1);
  const float *q = static_cast<const float *>(a.q) + b * a.qs[0] + i * a.qs[1] + h * a.qs[2];
  const float *kc = static_cast<const float *>(a.k_cache) + b * a.cs[0] + g * a.cs[2];
  const float *vc = static_cast<const float *>(a.v_cache) + b * a.cs[0] + g * a.cs[2];
  const float *ks = static_cast<const float *>(a.k_suf) + b * a.ks[0] + g * a.ks[2];
  const float *vs = static_cast<const float *>(a.v_suf) + b * a.ks[0] + g * a.ks[2];

  __shared__ float sK[kKT][D];
  __shared__ float sV[kKT][D];

  float qr[D], o[D];
  const float sc = a.scale * 1.4426950408889634f;
#pragma unroll
  for (int d = 0; d < D; d += 4) {
    const float4 v = *reinterpret_cast<const float4 *>(q + d);
    qr[d] = v.x * sc; qr[d + 1] = v.y * sc; qr[d + 2] = v.z * sc; qr[d + 3] = v.w * sc;
  }
#pragma unroll
  for (int d = 0; d < D; ++d) o[d] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int T = P + N;
  for (int t0 = 0; t0 < T; t0 += kKT) {
    const int nt = min(kKT, T - t0);
    __syncthreads();
    // stage nt rows of K and V: (row, 16-byte column) pairs spread over the 64 lanes
    for (int e = tid; e < nt * (D / 4); e += kQ) {
      const int r = e / (D / 4), c = (e % (D / 4)) * 4;
      const int t = t0 + r;
      const int64_t crow = t < P ? (a.cache_rows ? cache_row<true>(a, b, t) : t) : 0;
      const float *kp = t < P ? kc + crow * a.cs[1] : ks + int64_t(t - P) * a.ks[1];
      const float *vp = t < P ? vc + crow * a.cs[1] : vs + int64_t(t - P) * a.ks[1];
      *reinterpret_cast<float4 *>(&sK[r][c]) = *reinterpret_cast<const float4 *>(kp + c);
      *reinterpret_cast<float4 *>(&sV[r][c]) = *reinterpret_cast<const float4 *>(vp + c);
    }
    __syncthreads();
    for (int c0 = 0; c0 < nt; c0 += kKC) {
      float s[kKC];
      float cm = m;
#pragma unroll
      for (int k = 0; k < kKC; ++k) {
        float acc = 0.f;
        if (c0 + k < nt) {
#pragma unroll
          for (int d = 0; d < D; ++d) acc = __builtin_fmaf(qr[d], sK[c0 + k][d], acc);
        } else {
          acc = -INFINITY;
        }
        s[k] = acc;
        cm = __builtin_fmaxf(cm, acc);
      }
      const float alpha = __builtin_amdgcn_exp2f(m - cm);  // m = -inf on the first chunk: alpha = 0
      l *= alpha;
#pragma unroll
      for (int d = 0; d < D; ++d) o[d] *= alpha;
      m = cm;
#pragma unroll
      for (int k = 0; k < kKC; ++k) {
        if (c0 + k < nt) {
          const float p = __builtin_amdgcn_exp2f(s[k] - m);
          l += p;
#pragma unroll
          for (int d = 0; d < D; ++d) o[d] = __builtin_fmaf(p, sV[c0 + k][d], o[d]);
        }
      }
    }
  }
  if (q0 + tid < N) {
    float *out = static_cast<float *>(a.out) + b * a.os[0] + i * a.os[1] + h * a.os[2];
    const float inv = 1.0f / l;
#pragma unroll
    for (int d = 0; d < D; d += 4) {
      float4 v;
      v.x = o[d] * inv; v.y = o[d + 1] * inv; v.z = o[d + 2] * inv; v.w = o[d + 3] * inv;
      *reinterpret_cast<float4 *>(out + d) = v;
    }
  }
}

}  // namespace

int32_t launch_attn_f32(const AttnArgs &a, hipStream_t st) {
  const dim3 grid((a.S + kQ - 1) / kQ, a.Hq, a.B);
  if (a.D == 64)
    attn_f32_kernel<64><<<grid, kQ, 0, st>>>(a);
  else if (a.D == 128)
    attn_f32_kernel<128><<<grid, kQ, 0, st>>>(a);
  else {
    set_error("lsp_attn_step: fp32 head_dim %d not built (64, 128)", a.D);
    return LSP_ERR_UNSUPPORTED;
  }
  LSP_CHECK_LAUNCH("lsp_attn_step: fp32 launch");
  return LSP_OK;
}

}  // namespace lsp
