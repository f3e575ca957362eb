// bf16 suffix attention on the CDNA4 matrix cores (Algorithm 1 line 4; Section
// 3.2): active-suffix queries over [cached prefix K/V || suffix K/V], no mask.
//
// Formulation.  Each wave owns 32 query columns and works on the TRANSPOSED
// score block  S^T[key, query] = K . Q^T  with v_mfma_f32_32x32x16_bf16, so that
//   - a lane holds scores of ONE query (its accumulator column): the online
//     soft-max needs one exchange with the lane 32 away and its rescale factor
//     is a per-lane scalar for every output accumulator;
//   - the probabilities, once rounded to bf16, already sit in the B-operand
//     layout of the second product  O^T[d, query] = V^T . P^T  (the contraction
//     order over keys is the accumulator's row order, and V^T is read in that
//     same order), so P never goes through LDS.
// K blocks (32 keys) go from global memory straight into the A-operand
// registers (a lane reads 16 bytes of its key's row per 16-wide d-step); V
// blocks are staged row-major in a wave-private LDS region and read back with
// the LDS transpose load (ds_read_tr16_b64), which hands each lane four keys
// of its d column.  Waves never synchronise inside the key loop; block j+1's
// global loads are in flight while block j goes through the soft-max and the
// second product, and two waves per SIMD cover each other's waits.
//
// The soft-max reference m only moves when a block maximum exceeds it by more
// than 8 octaves, so the accumulator rescale is a cold, wave-uniform branch;
// probabilities are then at most 2^8, which bf16 and the fp32 sums hold
// without loss, and the final division by the row sum removes the offset.
//
// A workgroup is WM x WK waves: WM blocks of 32 queries, and WK-way split of
// the key range between waves of the same query block (merged through LDS at
// the end).  Few active rows => small WM, large WK, so that short suffixes
// still fill 256 compute units.
#include "lsp_attn.h"

namespace lsp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLagOctaves = 8.0f;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// two fp32 -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// One-instruction maxima (fmaxf would first quiet possible signalling NaNs of
// each operand, doubling the cost; scores are finite or -inf here).
__device__ __forceinline__ float fmax_raw(float a, float b) {
  float d;
  asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
  return d;
}
__device__ __forceinline__ float fmax3_raw(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

// value held by the lane 32 away
__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32); }

template <int D>
struct Geo {
  static constexpr int VPITCH = D * 2 + 64;   // bytes per staged V row: 64 mod 256 keeps the transpose reads conflict-free
  static constexpr int OPITCH = D * 4 + 16;   // bytes per merged O row (fp32): 16 mod 256 for 16-byte column writes
  static constexpr int VBYTES = 32 * VPITCH;
  static constexpr int OBYTES = 32 * OPITCH + 2 * 32 * 4;  // O^T block + m[32] + l[32]
  static constexpr int WAVE_LDS = VBYTES > OBYTES ? VBYTES : OBYTES;
};

template <int D, int WM, int WK>
__global__ __launch_bounds__(64 * WM * WK, 2) void attn_bf16_kernel(AttnArgs a) {
  using G = Geo<D>;
  constexpr int KK = D / 16;  // d-steps of the first product
  constexpr int DB = D / 32;  // 32-row blocks of O^T
  constexpr int VL = D / 16;  // 16-byte V loads per lane per block (32 rows * D*2 bytes / 64 lanes / 16)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  // XCD-aware placement.  Workgroups are handed to the 8 XCDs round-robin by
  // linear id, and each XCD has its own L2.  All workgroups that read the same
  // K/V stream - the query tiles of every query head of one (sequence, KV head)
  // unit - are therefore given ids that are congruent modulo 8, so the stream
  // is fetched into one L2 instead of eight.
  const int QT = (a.S + 32 * WM - 1) / (32 * WM);
  const int rep = a.Hq / a.Hkv;
  const int per_unit = rep * QT;
  const int n = blockIdx.x;
  const int m8 = n >> 3;
  const int unit = (m8 / per_unit) * 8 + (n & 7);
  if (unit >= a.B * a.Hkv) return;
  const int wu = m8 % per_unit;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const int h = g * rep + wu / QT;
  const int q0 = (wu % QT) * (32 * WM);
  const int N = min(max(a.suffix_len[b], 0), a.S);
  if (q0 >= N) return;
  const int P = min(max(a.prefix_len[b], 0), a.C);
  const int T = P + N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WK, wk = wave % WK;
  const int lq = lane & 31, hf = lane >> 5;
  unsigned char *wlds = smem + wave * G::WAVE_LDS;

  const uint16_t *kc = static_cast<const uint16_t *>(a.k_cache) + b * a.cs[0] + g * a.cs[2];
  const uint16_t *vc = static_cast<const uint16_t *>(a.v_cache) + b * a.cs[0] + g * a.cs[2];
  const uint16_t *ks = static_cast<const uint16_t *>(a.k_suf) + b * a.ks[0] + g * a.ks[2];
  const uint16_t *vs = static_cast<const uint16_t *>(a.v_suf) + b * a.ks[0] + g * a.ks[2];

  // Q fragments (B operand of S^T = K.Q^T): query lq of this wave, d = 16*kk + 8*hf + 0..7
  const int qi = q0 + wm * 32 + lq;
  const uint16_t *qp = static_cast<const uint16_t *>(a.q) + b * a.qs[0] + int64_t(min(qi, N - 1)) * a.qs[1] + h * a.qs[2];
  bf16x8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8 *>(qp + 16 * kk + 8 * hf);

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float mref = -INFINITY, lsum = 0.f;
  const float sc = a.scale * kLog2e;

  const int NB = (T + 31) >> 5;  // 32-key blocks; this wave takes wk, wk+WK, ...

  auto krow = [&](int t) -> const uint16_t * {
    t = min(t, T - 1);
    return t < P ? kc + int64_t(t) * a.cs[1] : ks + int64_t(t - P) * a.ks[1];
  };
  auto vrow = [&](int t) -> const uint16_t * {
    t = min(t, T - 1);
    return t < P ? vc + int64_t(t) * a.cs[1] : vs + int64_t(t - P) * a.ks[1];
  };
  auto load_k = [&](int jb, bf16x8 (&kf)[KK]) {
    const uint16_t *p = krow(32 * jb + lq) + 8 * hf;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = *reinterpret_cast<const bf16x8 *>(p + 16 * kk);
  };
  // V block: load i covers rows 4*i*(16/VCOL).. ; lane -> (row, 16-byte column)
  constexpr int VCOL = D / 8;          // 16-byte columns per row
  constexpr int RPL = 64 / VCOL;       // rows covered by one wave-wide load
  const int vcol = lane % VCOL, vr0 = lane / VCOL;
  u32x4 vreg[VL];
  auto load_v = [&](int jb) {
#pragma unroll
    for (int i = 0; i < VL; ++i)
      vreg[i] = *reinterpret_cast<const u32x4 *>(vrow(32 * jb + RPL * i + vr0) + 8 * vcol);
  };
  auto stage_v = [&](int jb) {
#pragma unroll
    for (int i = 0; i < VL; ++i) {
      const int r = RPL * i + vr0;
      u32x4 v = vreg[i];
      if (32 * jb + r >= T) v = u32x4{0, 0, 0, 0};  // keys beyond T contribute exact zeros
      *reinterpret_cast<u32x4 *>(wlds + r * G::VPITCH + 16 * vcol) = v;
    }
  };

  bf16x8 kf[KK];
  auto block = [&](int jb) {
    stage_v(jb);
    const int jn = jb + WK;
    if (jn < NB) load_v(jn);
    // S^T block
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], s, 0, 0, 0);
    // the K registers are free again: fetch the next block's rows while this
    // block goes through the soft-max and the second product
    if (jn < NB) load_k(jn, kf);
    if (32 * jb + 32 > T) {  // ragged last block: keys >= T get -inf
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = 32 * jb + 8 * (r >> 2) + 4 * hf + (r & 3);
        s[r] = key < T ? s[r] : -INFINITY;
      }
    }
    float bm = fmax_raw(s[0], s[1]);
#pragma unroll
    for (int r = 2; r < 16; r += 2) bm = fmax3_raw(bm, s[r], s[r + 1]);
    bm = fmax_raw(bm, other_half(bm)) * sc;  // finite: key 32*jb < T is valid
    if (__any(bm > mref + kLagOctaves)) {
      const float mn = bm > mref + kLagOctaves ? bm : mref;
      const float alpha = __builtin_amdgcn_exp2f(mref - mn);  // 0 on the first block (mref = -inf)
      mref = mn;
      lsum *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    const float nm = -mref;
    bf16x8 pf[2];
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
      float p[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * k2 + e], sc, nm));
        lsum += p[e];
      }
      u32x4 w;
      w.x = pack_bf16(p[0], p[1]);
      w.y = pack_bf16(p[2], p[3]);
      w.z = pack_bf16(p[4], p[5]);
      w.w = pack_bf16(p[6], p[7]);
      pf[k2] = __builtin_bit_cast(bf16x8, w);
    }
    // O^T[d, query] += V^T[d, key] . P^T[key, query]; contraction slot 8*hf+e of
    // step k2 is key 16*k2 + 8*(e/4) + 4*hf + e%4 (the accumulator row order).
    // Transpose load: within 16 lanes, lane s addresses row (s/4), columns 4*(s%4)..+3
    // and receives column s of the 4 rows.
    const int s16 = lane & 15;
    const unsigned char *vbase = wlds + (4 * hf + (s16 >> 2)) * G::VPITCH + (16 * ((lane >> 4) & 1) + 4 * (s16 & 3)) * 2;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2) {
        const unsigned char *ap = vbase + (16 * k2) * G::VPITCH + 64 * db;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(ap));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(ap + 8 * G::VPITCH));
        const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
        const u32x4 w = {l2.x, l2.y, h2.x, h2.y};
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), pf[k2], oacc[db], 0, 0, 0);
      }
  };

  if (wk < NB) {
    load_k(wk, kf);
    load_v(wk);
  }
  for (int jb = wk; jb < NB; jb += WK) block(jb);

  // ---- merge the WK partial results of each query block and store ----------------
  lsum += other_half(lsum);
  __syncthreads();  // all waves are done with their V staging area
  float *ob = reinterpret_cast<float *>(wlds);
  float *ml = reinterpret_cast<float *>(wlds + 32 * G::OPITCH);
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const f32x4 v = {oacc[db][4 * r4], oacc[db][4 * r4 + 1], oacc[db][4 * r4 + 2], oacc[db][4 * r4 + 3]};
      *reinterpret_cast<f32x4 *>(reinterpret_cast<unsigned char *>(ob) + lq * G::OPITCH + (32 * db + 8 * r4 + 4 * hf) * 4) = v;
    }
  if (hf == 0) {
    ml[lq] = mref;
    ml[32 + lq] = lsum;
  }
  __syncthreads();
  // wave (wm, wk) finishes d-range [wk*D/WK, (wk+1)*D/WK) of its query block: items = (query, 8 d)
  constexpr int DW = D / WK;            // d columns per wave
  constexpr int CH = DW / 8;            // 16-byte output chunks per query
  for (int it = lane; it < 32 * CH; it += 64) {
    const int qq = it / CH, dd = wk * DW + 8 * (it % CH);
    const int qrow = q0 + wm * 32 + qq;
    float M = -INFINITY;
#pragma unroll
    for (int w2 = 0; w2 < WK; ++w2) {
      const float *ml2 = reinterpret_cast<const float *>(smem + (wm * WK + w2) * G::WAVE_LDS + 32 * G::OPITCH);
      M = fmax_raw(M, ml2[qq]);
    }
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    float den = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < WK; ++w2) {
      const unsigned char *base = smem + (wm * WK + w2) * G::WAVE_LDS;
      const float *ml2 = reinterpret_cast<const float *>(base + 32 * G::OPITCH);
      const float wgt = __builtin_amdgcn_exp2f(ml2[qq] - M);  // 0 for a wave that saw no key
      den += ml2[32 + qq] * wgt;
      const f32x4 x0 = *reinterpret_cast<const f32x4 *>(base + qq * G::OPITCH + dd * 4);
      const f32x4 x1 = *reinterpret_cast<const f32x4 *>(base + qq * G::OPITCH + dd * 4 + 16);
      acc[0] += x0.x * wgt; acc[1] += x0.y * wgt; acc[2] += x0.z * wgt; acc[3] += x0.w * wgt;
      acc[4] += x1.x * wgt; acc[5] += x1.y * wgt; acc[6] += x1.z * wgt; acc[7] += x1.w * wgt;
    }
    if (qrow < N) {
      const float inv = 1.0f / den;
      u32x4 w;
      w.x = pack_bf16(acc[0] * inv, acc[1] * inv);
      w.y = pack_bf16(acc[2] * inv, acc[3] * inv);
      w.z = pack_bf16(acc[4] * inv, acc[5] * inv);
      w.w = pack_bf16(acc[6] * inv, acc[7] * inv);
      uint16_t *op = static_cast<uint16_t *>(a.out) + b * a.os[0] + int64_t(qrow) * a.os[1] + h * a.os[2];
      *reinterpret_cast<u32x4 *>(op + dd) = w;
    }
  }
}

template <int D, int WM, int WK>
int32_t launch(const AttnArgs &a, hipStream_t st) {
  const int64_t QT = (a.S + 32 * WM - 1) / (32 * WM);
  const int64_t units = int64_t(a.B) * a.Hkv;
  const int64_t nwg = (units + 7) / 8 * 8 * (a.Hq / a.Hkv) * QT;
  if (nwg > 0x7fffffff) {
    set_error("lsp_attn_step: launch of %lld workgroups is too large", (long long)nwg);
    return LSP_ERR_UNSUPPORTED;
  }
  const dim3 grid(static_cast<unsigned>(nwg), 1, 1);
  const size_t lds = size_t(WM * WK) * Geo<D>::WAVE_LDS;
  auto kern = attn_bf16_kernel<D, WM, WK>;
  static bool configured = false;  // per instantiation
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
    if (e != hipSuccess) return hip_fail(e, "lsp_attn_step: hipFuncSetAttribute");
    configured = true;
  }
  kern<<<grid, 64 * WM * WK, lds, st>>>(a);
  LSP_CHECK_LAUNCH("lsp_attn_step: bf16 launch");
  return LSP_OK;
}

template <int D>
int32_t dispatch(const AttnArgs &a, hipStream_t st) {
  // Pick the widest query tile that still gives every compute unit work.
  const int64_t rows = int64_t(a.B) * a.Hq * a.S;  // upper bound on (b,h,row) triples
  if (rows / 128 >= 512) return launch<D, 4, 1>(a, st);
  if (rows / 64 >= 512) return launch<D, 2, 2>(a, st);
  if (rows / 32 >= 512) return launch<D, 1, 4>(a, st);
  return launch<D, 1, 8>(a, st);
}

}  // namespace

size_t attn_bf16_workspace_bytes(int32_t, int32_t, int32_t, int32_t) { return 0; }

int32_t launch_attn_bf16(const AttnArgs &a, hipStream_t st) {
  if (a.D == 128) return dispatch<128>(a, st);
  if (a.D == 64) return dispatch<64>(a, st);
  set_error("lsp_attn_step: bf16 head_dim %d not built (64, 128)", a.D);
  return LSP_ERR_UNSUPPORTED;
}

}  // namespace lsp
