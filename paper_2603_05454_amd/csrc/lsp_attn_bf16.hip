// bf16 suffix attention on the CDNA4 matrix cores (Algorithm 1 line 4; Section
// 3.2): active-suffix queries over [cached prefix K/V || suffix K/V], no mask.
//
// Formulation.  Each wave owns 32 query columns and works on the TRANSPOSED
// score tile  S^T[key, query] = K . Q^T  with v_mfma_f32_32x32x16_bf16, so that
//   - a lane holds scores of ONE query (its accumulator column): the online
//     soft-max needs one exchange with the lane 32 away and its rescale factor
//     is a per-lane scalar for every output accumulator;
//   - the probabilities, once rounded to bf16, already sit in the B-operand
//     layout of the second product  O^T[d, query] = V^T . P^T  (the contraction
//     order over keys is the accumulator's row order, and V^T is read from LDS
//     in that same order), so P never goes through LDS.
// K tiles are staged row-major in LDS (A operand = 16-byte row reads), V tiles
// are staged transposed ([d][key]) so that the A operand of the second product
// is two 8-byte reads.  The next tile's global loads are issued before the
// current tile's arithmetic.
#include "lsp_attn.h"

namespace lsp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBM = 128;      // queries per workgroup (32 per wave)
constexpr int kBN = 64;       // keys per tile
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return uint32_t(f32_to_bf16(lo)) | (uint32_t(f32_to_bf16(hi)) << 16);
}

template <int D>
__global__ __launch_bounds__(kThreads) void attn_bf16_kernel(AttnArgs a) {
  constexpr int KP = D + 8;      // sK row pitch (elements)
  constexpr int VP = kBN + 8;    // sVt row pitch (elements)
  constexpr int CPR = D / 8;     // 16-byte columns per K/V row
  constexpr int RPT = kThreads / CPR;          // rows covered per pass of the loader
  constexpr int NLD = kBN / RPT;               // loader passes per tile
  __shared__ __attribute__((aligned(16))) uint16_t sK[kBN * KP];
  __shared__ __attribute__((aligned(16))) uint16_t sVt[D * VP];

  const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * kBM;
  const int N = min(max(a.suffix_len[b], 0), a.S);
  if (q0 >= N) return;
  const int P = min(max(a.prefix_len[b], 0), a.C);
  const int T = P + N;
  const int g = h / (a.Hq / a.Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, hf = lane >> 5;

  const uint16_t *kc = static_cast<const uint16_t *>(a.k_cache) + b * a.cs[0] + g * a.cs[2];
  const uint16_t *vc = static_cast<const uint16_t *>(a.v_cache) + b * a.cs[0] + g * a.cs[2];
  const uint16_t *ks = static_cast<const uint16_t *>(a.k_suf) + b * a.ks[0] + g * a.ks[2];
  const uint16_t *vs = static_cast<const uint16_t *>(a.v_suf) + b * a.ks[0] + g * a.ks[2];

  // Q fragments (B operand of S^T = K.Q^T): query lq of this wave, d = 16*kk + 8*hf + 0..7
  const int qi = q0 + wave * 32 + lq;
  const uint16_t *qp = static_cast<const uint16_t *>(a.q) + b * a.qs[0] + int64_t(min(qi, N - 1)) * a.qs[1] + h * a.qs[2];
  bf16x8 qf[D / 16];
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk)
    qf[kk] = *reinterpret_cast<const bf16x8 *>(qp + 16 * kk + 8 * hf);

  f32x16 oacc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m = -INFINITY, lsum = 0.f;
  const float sc = a.scale * kLog2e;

  // loader: thread covers column lc of rows lr + RPT*k
  const int lc = tid % CPR, lr = tid / CPR;
  u32x4 kreg[NLD], vreg[NLD];
  auto load_tile = [&](int t0) {
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
      const int t = t0 + lr + RPT * k;
      u32x4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
      if (t < T) {
        const uint16_t *kp = t < P ? kc + int64_t(t) * a.cs[1] : ks + int64_t(t - P) * a.ks[1];
        const uint16_t *vp = t < P ? vc + int64_t(t) * a.cs[1] : vs + int64_t(t - P) * a.ks[1];
        kv = *reinterpret_cast<const u32x4 *>(kp + 8 * lc);
        vv = *reinterpret_cast<const u32x4 *>(vp + 8 * lc);
      }
      kreg[k] = kv;
      vreg[k] = vv;
    }
  };
  load_tile(0);

  for (int t0 = 0; t0 < T; t0 += kBN) {
    __syncthreads();  // every wave is done reading the previous tile
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
      const int r = lr + RPT * k;
      *reinterpret_cast<u32x4 *>(&sK[r * KP + 8 * lc]) = kreg[k];
      const uint32_t w[4] = {vreg[k].x, vreg[k].y, vreg[k].z, vreg[k].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sVt[(8 * lc + 2 * e) * VP + r] = uint16_t(w[e] & 0xffffu);
        sVt[(8 * lc + 2 * e + 1) * VP + r] = uint16_t(w[e] >> 16);
      }
    }
    __syncthreads();
    if (t0 + kBN < T) load_tile(t0 + kBN);

    // S^T blocks: keys 32*kb + .., this wave's 32 queries
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&sK[(32 * kb + lq) * KP + 16 * kk + 8 * hf]);
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[kb], 0, 0, 0);
      }
    }
    // scale to the log2 domain, mask keys beyond T, tile maximum for this query
    float tmax = -INFINITY;
    const bool ragged = t0 + kBN > T;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float s = sacc[kb][r] * sc;
        if (ragged) {
          const int key = t0 + 32 * kb + 8 * (r >> 2) + 4 * hf + (r & 3);
          s = key < T ? s : -INFINITY;
        }
        sacc[kb][r] = s;
        tmax = __builtin_fmaxf(tmax, s);
      }
    tmax = __builtin_fmaxf(tmax, __shfl_xor(tmax, 32));
    const float mn = __builtin_fmaxf(m, tmax);  // finite: every tile holds at least one valid key
    const float alpha = __builtin_amdgcn_exp2f(m - mn);
    m = mn;
    lsum *= alpha;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;

    // probabilities -> bf16 B operands; contraction slot (8*hf + e) of step (kb,k2)
    // is key 32*kb + 16*k2 + 8*(e/4) + 4*hf + e%4
    bf16x8 pf[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2) {
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          p[e] = __builtin_amdgcn_exp2f(sacc[kb][8 * k2 + e] - mn);
          lsum += p[e];
        }
        u32x4 w;
        w.x = pack_bf16(p[0], p[1]);
        w.y = pack_bf16(p[2], p[3]);
        w.z = pack_bf16(p[4], p[5]);
        w.w = pack_bf16(p[6], p[7]);
        pf[kb][k2] = __builtin_bit_cast(bf16x8, w);
      }
    // O^T[d, query] += V^T[d, key] . P^T[key, query]
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          const uint16_t *vrow = &sVt[(32 * db + lq) * VP + 32 * kb + 16 * k2 + 4 * hf];
          const u32x2 lo = *reinterpret_cast<const u32x2 *>(vrow);
          const u32x2 hi = *reinterpret_cast<const u32x2 *>(vrow + 8);
          const u32x4 w = {lo.x, lo.y, hi.x, hi.y};
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), pf[kb][k2], oacc[db], 0, 0, 0);
        }
  }

  lsum += __shfl_xor(lsum, 32);
  if (qi < N) {
    const float inv = 1.0f / lsum;
    uint16_t *op = static_cast<uint16_t *>(a.out) + b * a.os[0] + int64_t(qi) * a.os[1] + h * a.os[2];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 w;
        w.x = pack_bf16(oacc[db][4 * r4] * inv, oacc[db][4 * r4 + 1] * inv);
        w.y = pack_bf16(oacc[db][4 * r4 + 2] * inv, oacc[db][4 * r4 + 3] * inv);
        *reinterpret_cast<u32x2 *>(op + 32 * db + 8 * r4 + 4 * hf) = w;
      }
  }
}

}  // namespace

size_t attn_bf16_workspace_bytes(int32_t, int32_t, int32_t, int32_t) { return 0; }

int32_t launch_attn_bf16(const AttnArgs &a, hipStream_t st) {
  const dim3 grid((a.S + kBM - 1) / kBM, a.Hq, a.B);
  if (a.D == 128)
    attn_bf16_kernel<128><<<grid, kThreads, 0, st>>>(a);
  else if (a.D == 64)
    attn_bf16_kernel<64><<<grid, kThreads, 0, st>>>(a);
  else {
    set_error("lsp_attn_step: bf16 head_dim %d not built (64, 128)", a.D);
    return LSP_ERR_UNSUPPORTED;
  }
  LSP_CHECK_LAUNCH("lsp_attn_step: bf16 launch");
  return LSP_OK;
}

}  // namespace lsp
