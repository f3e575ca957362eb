// Output head fused with the per-position confidence (Algorithm 1 lines 4-5):
// logits z = hidden . weight^T on the CDNA4 matrix cores, reduced inside the
// same kernel to top-1 id, logit margin (Eq. 1) and top-1 probability, so the
// [rows x V] logits never reach memory.
//
// Formulation.  A workgroup owns a tile of TV = 256 vocabulary entries x TR =
// 256 rows and walks K in steps of 64.  It computes the TRANSPOSED logits tile
//   Z^T[v, row] = W[v, :] . H[row, :]      (A operand = weight, B = hidden)
// with v_mfma_f32_32x32x16_bf16, so that a lane's accumulator registers hold
// 16 vocabulary entries of ONE row per 32x32 block: the running (max, runner-up,
// arg-max, sum of exponentials) of Eq. 1 is per-lane state, updated in
// increasing vocabulary order, and only the last combine crosses lanes (the two
// half-columns of a block, then the waves that share the rows).  Every
// (row, vocabulary tile) leaves one 16-byte partial; a second, tiny kernel
// folds a row's partials.
//
// Tiles go to the 8 XCDs round-robin by workgroup id; ids are laid out so that
// the 32 workgroups an XCD runs at a time form a block of VB vocabulary tiles x
// RB row tiles: each weight slice is then read by RB and each hidden slice by
// VB workgroups out of the same L2.
#include <float.h>

#include "lsp_common.h"

namespace lsp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

constexpr int TV = 256;          // vocabulary entries per tile
constexpr int TR = 256;          // rows per tile
constexpr int BK = 64;           // K step
constexpr int PITCH = BK * 2 + 16;  // bytes per staged row: 144 = 9 * 16, so 16 consecutive rows hit 16 distinct 16-byte slots of a 256-byte bank line
constexpr int TILE_BYTES = 256 * PITCH;
constexpr int STAGE = 2 * TILE_BYTES;  // weight tile, then hidden tile
constexpr int NT = 512;          // 8 waves: 2 along the vocabulary x 4 along the rows
constexpr int WV = 2, WR = 4;
constexpr int MV = TV / WV / 32;  // 32x32 blocks per wave along the vocabulary (4)
constexpr int MR = TR / WR / 32;  // ... along the rows (2)
constexpr int PIECES = 256 * (BK / 8) / NT;  // 16-byte pieces per thread per operand tile and K step (4)

struct Partial {
  float m1, m2, s;
  int32_t idx;
};

struct LmArgs {
  const uint16_t *hidden, *weight;
  int32_t B, S, K, V;
  int64_t hrs, hbs, wrs;  // element strides
  const int32_t *suffix_len;
  Partial *partials;
  int32_t VT, RT, VB, RB;  // tile counts, XCD block shape
};

__device__ __forceinline__ float fmax_raw(float a, float b) {
  float d;
  asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
  return d;
}
__device__ __forceinline__ float fmin_raw(float a, float b) {
  float d;
  asm("v_min_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
  return d;
}
__device__ __forceinline__ float fmed3_raw(float a, float b, float c) {
  float d;
  asm("v_med3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

// Fold of two partial results of one row; ties on the maximum keep the lower index.
__device__ __forceinline__ Partial fold(Partial a, Partial b) {
  const float am = a.m1, bm = b.m1;
  const int ai = a.idx, bi = b.idx;
  const float M = fmax_raw(am, bm);
  const float wa = am == M ? 1.f : __builtin_amdgcn_exp2f((am - M) * kLog2e);
  const float wb = bm == M ? 1.f : __builtin_amdgcn_exp2f((bm - M) * kLog2e);
  const bool take_b = bm > am || (bm == am && bi < ai);
  Partial r;
  r.m1 = M;
  r.m2 = fmax_raw(fmin_raw(am, bm), fmax_raw(a.m2, b.m2));
  r.s = a.s * wa + b.s * wb;
  r.idx = take_b ? bi : ai;
  return r;
}

// Tile coordinates of this workgroup (vt, rt) or vt = -1 for a padding id.
__device__ __forceinline__ void tile_of(const LmArgs &a, int &vt, int &rt) {
  const int n = blockIdx.x;
  const int x = n & 7, m = n >> 3;
  const int per = a.VB * a.RB;
  const int sb = m / per, loc = m % per;
  const int RG = (a.RT + a.RB - 1) / a.RB;
  const int vgroup = sb / RG, rgroup = sb % RG;
  vt = (vgroup * a.VB + loc % a.VB) * 8 + x;
  rt = rgroup * a.RB + loc / a.VB;
  if (vt >= a.VT || rt >= a.RT) vt = -1;
}

__global__ __launch_bounds__(NT, 2) void lm_head_kernel(LmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_any;
  int vt, rt;
  tile_of(a, vt, rt);
  if (vt < 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wv = wave % WV, wr = wave / WV;
  const int lq = lane & 31, hf = lane >> 5;
  const int rows = a.B * a.S;
  const int v0 = vt * TV, r0 = rt * TR;

  // a tile none of whose rows is active does nothing
  if (a.suffix_len != nullptr) {
    if (tid == 0) s_any = 0;
    __syncthreads();
    bool act = false;
    if (tid < TR) {
      const int r = r0 + tid;
      if (r < rows) act = (r % a.S) < a.suffix_len[r / a.S];
    }
    if (act) s_any = 1;
    __syncthreads();
    if (!s_any) return;
  }

  // loader: piece i of this thread is (tile row, 16-byte column) = ((tid + NT*i) / 8, (tid + NT*i) % 8)
  const char *wp[PIECES], *hp[PIECES];
  int lds_off[PIECES];
  const int pcol = tid & 7;
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    const int prow = (tid + NT * i) >> 3;
    const int v = min(v0 + prow, a.V - 1);     // rows beyond V or the row count repeat the last valid one
    const int r = min(r0 + prow, rows - 1);    // (their results are masked or never written)
    wp[i] = reinterpret_cast<const char *>(a.weight + int64_t(v) * a.wrs) + 16 * pcol;
    hp[i] = reinterpret_cast<const char *>(a.hidden + int64_t(r / a.S) * a.hbs + int64_t(r % a.S) * a.hrs) + 16 * pcol;
    lds_off[i] = prow * PITCH + 16 * pcol;
  }
  const int KS = (a.K + BK - 1) / BK;
  u32x4 wreg[PIECES], hreg[PIECES];
  auto load_stage = [&](int ks) {
    const int kbyte = ks * BK * 2;
    const bool in = (ks * BK + 8 * pcol) < a.K;  // K tail: pieces beyond K are zeros
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      wreg[i] = in ? *reinterpret_cast<const u32x4 *>(wp[i] + kbyte) : u32x4{0, 0, 0, 0};
      hreg[i] = in ? *reinterpret_cast<const u32x4 *>(hp[i] + kbyte) : u32x4{0, 0, 0, 0};
    }
  };
  auto store_stage = [&](int ks) {
    unsigned char *st = smem + (ks & 1) * STAGE;
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      *reinterpret_cast<u32x4 *>(st + lds_off[i]) = wreg[i];
      *reinterpret_cast<u32x4 *>(st + TILE_BYTES + lds_off[i]) = hreg[i];
    }
  };

  f32x16 acc[MV][MR];
#pragma unroll
  for (int i = 0; i < MV; ++i)
#pragma unroll
    for (int j = 0; j < MR; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  load_stage(0);
  store_stage(0);
  if (KS > 1) load_stage(1);
  __syncthreads();
  const int a_off = (wv * (TV / WV) + lq) * PITCH + 16 * hf;
  const int b_off = TILE_BYTES + (wr * (TR / WR) + lq) * PITCH + 16 * hf;
  for (int ks = 0; ks < KS; ++ks) {
    // stage ks+1 goes into the buffer every wave finished reading before the last barrier
    if (ks + 1 < KS) store_stage(ks + 1);
    if (ks + 2 < KS) load_stage(ks + 2);
    const unsigned char *st = smem + (ks & 1) * STAGE;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[MV], bf[MR];
#pragma unroll
      for (int i = 0; i < MV; ++i) af[i] = *reinterpret_cast<const bf16x8 *>(st + a_off + i * 32 * PITCH + kk * 32);
#pragma unroll
      for (int j = 0; j < MR; ++j) bf[j] = *reinterpret_cast<const bf16x8 *>(st + b_off + j * 32 * PITCH + kk * 32);
#pragma unroll
      for (int i = 0; i < MV; ++i)
#pragma unroll
        for (int j = 0; j < MR; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // ---- Eq. 1 on the accumulators ------------------------------------------------
  // acc[i][j][r] = z[v][row] with v = v0 + wv*128 + 32 i + 8 (r/4) + 4 hf + r%4 (increasing
  // in (i, r)) and row = r0 + wr*64 + 32 j + lq.
  const int vbase = v0 + wv * (TV / WV) + 4 * hf;
  const bool ragged = v0 + TV > a.V;
  Partial *lds_part = reinterpret_cast<Partial *>(smem);  // [WR][MR][WV][32] after the last barrier
#pragma unroll
  for (int j = 0; j < MR; ++j) {
    float m1 = -INFINITY, m2 = -INFINITY;
    int code = 0;
#pragma unroll
    for (int i = 0; i < MV; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float x = acc[i][j][r];
        if (ragged && vbase + 32 * i + 8 * (r >> 2) + (r & 3) >= a.V) x = acc[i][j][r] = -INFINITY;
        code = x > m1 ? 16 * i + r : code;
        m2 = fmed3_raw(m1, m2, x);
        m1 = fmax_raw(m1, x);
      }
    const float ref = m1 == -INFINITY ? 0.f : m1;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MV; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += __builtin_amdgcn_exp2f((acc[i][j][r] - ref) * kLog2e);
    Partial p;
    p.m1 = m1; p.m2 = m2; p.s = s;
    p.idx = vbase + 32 * (code >> 4) + 8 * ((code & 15) >> 2) + (code & 3);
    // the other half-column of the 32x32 blocks (lane +-32) holds the rows' other vocabulary entries
    Partial o;
    o.m1 = __shfl_xor(p.m1, 32); o.m2 = __shfl_xor(p.m2, 32); o.s = __shfl_xor(p.s, 32); o.idx = __shfl_xor(p.idx, 32);
    p = fold(p, o);
    if (hf == 0) lds_part[((wr * MR + j) * WV + wv) * 32 + lq] = p;
  }
  __syncthreads();
  // one thread per row of the tile folds the WV waves' results and writes the partial
  if (tid < TR) {
    const int w = tid >> 6, j = (tid >> 5) & 1, q = tid & 31;  // tid = w*64 + j*32 + q = row within the tile
    Partial p = lds_part[((w * MR + j) * WV + 0) * 32 + q];
#pragma unroll
    for (int u = 1; u < WV; ++u) p = fold(p, lds_part[((w * MR + j) * WV + u) * 32 + q]);
    const int r = r0 + tid;
    if (r < rows) a.partials[int64_t(r) * a.VT + vt] = p;
  }
}

// One wave per row folds the row's VT partials and writes the three results.
__global__ __launch_bounds__(256) void lm_head_finish_kernel(const Partial *__restrict__ partials, int rows, int S, int VT,
                                                             const int32_t *__restrict__ suffix_len,
                                                             int32_t *__restrict__ top1_id,
                                                             float *__restrict__ top1_prob,
                                                             float *__restrict__ margin) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (r >= rows) return;
  if (suffix_len != nullptr && (r % S) >= suffix_len[r / S]) return;
  Partial p;
  p.m1 = -INFINITY; p.m2 = -INFINITY; p.s = 0.f; p.idx = 0x7fffffff;
  for (int t = lane; t < VT; t += 64) p = fold(p, partials[int64_t(r) * VT + t]);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    Partial o;
    o.m1 = __shfl_xor(p.m1, d); o.m2 = __shfl_xor(p.m2, d); o.s = __shfl_xor(p.s, d); o.idx = __shfl_xor(p.idx, d);
    p = fold(p, o);
  }
  if (lane == 0) {
    top1_id[r] = p.idx;
    margin[r] = p.m1 - p.m2;
    top1_prob[r] = 1.0f / p.s;
  }
}

}  // namespace
}  // namespace lsp

extern "C" size_t lsp_lm_head_confidence_workspace_bytes(int32_t B, int32_t S, int32_t V) {
  if (B <= 0 || S <= 0 || V <= 0) return 0;
  const size_t VT = (size_t(V) + lsp::TV - 1) / lsp::TV;
  return size_t(B) * S * VT * sizeof(lsp::Partial);
}

extern "C" int32_t lsp_lm_head_confidence(int32_t dtype, const void *hidden, const void *weight, int32_t B,
                                          int32_t S, int32_t K, int32_t V, int64_t hidden_row_stride,
                                          int64_t hidden_batch_stride, int64_t weight_row_stride,
                                          const int32_t *suffix_len, int32_t *top1_id, float *top1_prob,
                                          float *margin, void *workspace, size_t workspace_bytes,
                                          void *stream) {
  using namespace lsp;
  LSP_CHECK_ARG(dtype == LSP_F32 || dtype == LSP_BF16, "lsp_lm_head_confidence: unknown dtype %d", dtype);
  if (dtype != LSP_BF16) {
    set_error("lsp_lm_head_confidence: only bf16 operands are built");
    return LSP_ERR_UNSUPPORTED;
  }
  LSP_CHECK_ARG(hidden && weight && top1_id && top1_prob && margin, "lsp_lm_head_confidence: null pointer");
  LSP_CHECK_ARG(B > 0 && S > 0 && V >= 2 && K > 0, "lsp_lm_head_confidence: need B>0, S>0, K>0, V>=2 (got %d %d %d %d)", B, S, K, V);
  LSP_CHECK_ARG(K % 8 == 0, "lsp_lm_head_confidence: K must be a multiple of 8 (got %d)", K);
  LSP_CHECK_ARG(int64_t(B) * S <= 0x3fffffff, "lsp_lm_head_confidence: B*S too large");
  if (hidden_row_stride == 0) hidden_row_stride = K;
  if (hidden_batch_stride == 0) hidden_batch_stride = int64_t(S) * hidden_row_stride;
  if (weight_row_stride == 0) weight_row_stride = K;
  LSP_CHECK_ARG(hidden_row_stride >= K && weight_row_stride >= K && hidden_batch_stride >= 0 &&
                    hidden_row_stride % 8 == 0 && hidden_batch_stride % 8 == 0 && weight_row_stride % 8 == 0,
                "lsp_lm_head_confidence: strides must be >= K and multiples of 8 elements");
  LSP_CHECK_ARG(aligned16(hidden) && aligned16(weight), "lsp_lm_head_confidence: hidden and weight must be 16-byte aligned");
  const size_t need = lsp_lm_head_confidence_workspace_bytes(B, S, V);
  if (workspace == nullptr || workspace_bytes < need || !aligned16(workspace)) {
    set_error("lsp_lm_head_confidence: workspace of %zu bytes (16-byte aligned) required, got %zu", need, workspace_bytes);
    return LSP_ERR_WORKSPACE;
  }
  LmArgs a;
  a.hidden = static_cast<const uint16_t *>(hidden);
  a.weight = static_cast<const uint16_t *>(weight);
  a.B = B; a.S = S; a.K = K; a.V = V;
  a.hrs = hidden_row_stride; a.hbs = hidden_batch_stride; a.wrs = weight_row_stride;
  a.suffix_len = suffix_len;
  a.partials = static_cast<Partial *>(workspace);
  const int64_t rows = int64_t(B) * S;
  a.VT = (V + TV - 1) / TV;
  a.RT = int32_t((rows + TR - 1) / TR);
  a.RB = a.RT < 4 ? a.RT : 4;
  a.VB = 32 / a.RB;
  const int64_t RG = (a.RT + a.RB - 1) / a.RB;
  const int64_t per_xcd_vt = (a.VT + 7) / 8;                    // vocabulary tiles an XCD owns
  const int64_t VG = (per_xcd_vt + a.VB - 1) / a.VB;
  const int64_t nwg = VG * RG * a.VB * a.RB * 8;
  if (nwg > 0x7fffffff) {
    set_error("lsp_lm_head_confidence: launch of %lld workgroups is too large", (long long)nwg);
    return LSP_ERR_UNSUPPORTED;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t lds = 2 * size_t(STAGE);
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(lm_head_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
    if (e != hipSuccess) return hip_fail(e, "lsp_lm_head_confidence: hipFuncSetAttribute");
    configured = true;
  }
  lm_head_kernel<<<dim3(static_cast<unsigned>(nwg)), NT, lds, st>>>(a);
  LSP_CHECK_LAUNCH("lsp_lm_head_confidence: launch");
  lm_head_finish_kernel<<<dim3(static_cast<unsigned>((rows + 3) / 4)), 256, 0, st>>>(
      a.partials, int(rows), S, a.VT, suffix_len, top1_id, top1_prob, margin);
  LSP_CHECK_LAUNCH("lsp_lm_head_confidence: finish launch");
  return LSP_OK;
}
