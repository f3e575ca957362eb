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
// Main loop.  Both operand tiles of a K step go from global memory straight
// into LDS (no registers, no LDS store instructions), one step ahead of the
// products, into the buffer freed at the last barrier.  Fragments of k-step
// kk+1 are read while the matrix instructions of kk run, and the issue order
// of a whole step is pinned: one LDS read or one global load after each matrix
// instruction, global loads first.
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
constexpr int TILE_BYTES = 256 * BK * 2;  // one operand tile of a K step in LDS: 256 rows of 128 bytes
constexpr int STAGE = 2 * TILE_BYTES;     // weight tile, then hidden tile

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

// One wave-wide load from global memory straight into LDS: lane l fetches 16
// bytes at its own address g and they land at lds_base + 16 l (lds_base is
// wave-uniform; the counter to wait on is vmcnt).
__device__ __forceinline__ void load_to_lds(const char *g, unsigned char *lds_base) {
  __builtin_amdgcn_global_load_lds(g, (__attribute__((address_space(3))) void *)lds_base, 16, 0, 0);
}

// WV x WR waves: WV along the vocabulary, WR along the rows.
template <int WV, int WR>
__global__ __launch_bounds__(64 * WV * WR, 512 / (64 * WV * WR) >= 2 ? 1 : 2) void lm_head_kernel(LmArgs a) {
  constexpr int NT = 64 * WV * WR;
  constexpr int MV = TV / WV / 32;  // 32x32 blocks per wave along the vocabulary
  constexpr int MR = TR / WR / 32;  // ... along the rows
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
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
    for (int t = tid; t < TR; t += NT) {
      const int r = r0 + t;
      if (r < rows) act |= (r % a.S) < a.suffix_len[r / a.S];
    }
    if (act) s_any = 1;
    __syncthreads();
    if (!s_any) return;
  }

  // Loader.  Operand tiles go from global memory straight into LDS
  // (global_load_lds_dwordx4: lane l of a wave-wide load deposits its 16 bytes at
  // LDS base + 16 l, so one load fills 1 KB = 8 tile rows of 128 bytes).  Rows
  // are stored unpadded; to keep the fragment reads (16 consecutive rows, one
  // 16-byte chunk each) on distinct banks, chunk c of row r is kept at chunk
  // position c ^ ((r >> 1) & 7), which the loading lane applies to its GLOBAL
  // address.  Wave w issues loads w, w + NW, ... of the tile's 32.
  constexpr int NW = NT / 64;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);  // wave-uniform, for the scalar LDS base
  constexpr int LPW = 32 / NW;  // wave-wide loads per wave, per operand tile and K step
  const char *wp[LPW], *hp[LPW];
  int chunk[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int row = 8 * (wave + NW * i) + (lane >> 3);
    chunk[i] = (lane & 7) ^ ((row >> 1) & 7);
    const int v = min(v0 + row, a.V - 1);     // rows beyond V or the row count repeat the last valid one
    const int r = min(r0 + row, rows - 1);    // (their results are masked or never written)
    wp[i] = reinterpret_cast<const char *>(a.weight + int64_t(v) * a.wrs) + 16 * chunk[i];
    hp[i] = reinterpret_cast<const char *>(a.hidden + int64_t(r / a.S) * a.hbs + int64_t(r % a.S) * a.hrs) + 16 * chunk[i];
  }
  const int KS = (a.K + BK - 1) / BK;
  const int tail_chunks = (a.K % BK) / 8;  // valid 16-byte chunks of a ragged last step (0 = none ragged)
  auto issue = [&](int ks, int buf, int i) {
    unsigned char *st = smem + buf * STAGE + 1024 * (wave_s + NW * i);
    int back = 0;  // a lane whose chunk lies beyond K fetches the row's chunk 0 of this step instead (zeroed below)
    if (tail_chunks != 0 && ks == KS - 1 && chunk[i] >= tail_chunks) back = 16 * chunk[i];
    const int kbyte = ks * BK * 2 - back;
    load_to_lds(wp[i] + kbyte, st);
    load_to_lds(hp[i] + kbyte, st + TILE_BYTES);
  };
  // after the loads of a ragged last step have landed: the lanes that fetched a
  // stand-in overwrite their own LDS slots with zeros
  auto zero_tail = [&](int ks) {
    if (tail_chunks == 0 || ks != KS - 1) return;
#pragma unroll
    for (int i = 0; i < LPW; ++i)
      if (chunk[i] >= tail_chunks) {
        unsigned char *st = smem + (ks & 1) * STAGE + 1024 * (wave + NW * i) + 16 * lane;
        *reinterpret_cast<u32x4 *>(st) = u32x4{0, 0, 0, 0};
        *reinterpret_cast<u32x4 *>(st + TILE_BYTES) = u32x4{0, 0, 0, 0};
      }
  };

  f32x16 acc[MV][MR];
#pragma unroll
  for (int i = 0; i < MV; ++i)
#pragma unroll
    for (int j = 0; j < MR; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

#pragma unroll
  for (int i = 0; i < LPW; ++i) issue(0, 0, i);
  __builtin_amdgcn_s_waitcnt(0);  // vmcnt = 0: the loads have written LDS
  zero_tail(0);
  __syncthreads();
  // fragment of 32x32 block i at k-step kk: row (block base + lq), chunk 2 kk + hf, swizzled
  const int y16 = 16 * (hf ^ ((lq >> 1) & 7));
  const int a_row = (wv * (TV / WV) + lq) * 128;
  const int b_row = TILE_BYTES + (wr * (TR / WR) + lq) * 128;
  auto read_frags = [&](const unsigned char *st, int kk, bf16x8 (&af)[MV], bf16x8 (&bf)[MR]) {
    const int off = (32 * kk) ^ y16;
#pragma unroll
    for (int i = 0; i < MV; ++i) af[i] = *reinterpret_cast<const bf16x8 *>(st + a_row + i * 32 * 128 + off);
#pragma unroll
    for (int j = 0; j < MR; ++j) bf[j] = *reinterpret_cast<const bf16x8 *>(st + b_row + j * 32 * 128 + off);
  };
  constexpr int KSTEPS = BK / 16;
  for (int ks = 0; ks < KS; ++ks) {
    // Step ks+1 is fetched into the buffer every wave finished reading before the
    // last barrier (the last step fetches itself again, into the idle buffer, so
    // that the loop body stays free of branches).  Within a k-step the
    // fragments of the NEXT k-step are read and a share of the global loads is
    // issued between the matrix instructions of this one.
    const int kn = min(ks + 1, KS - 1);
    const unsigned char *st = smem + (ks & 1) * STAGE;
    bf16x8 af[2][MV], bf[2][MR];
    read_frags(st, 0, af[0], bf[0]);
    constexpr int NREAD = MV + MR, NMFMA = MV * MR;
    constexpr int LOADS_PER_K = (NMFMA - NREAD) / 2 > 0 ? (NMFMA - NREAD) / 2 : 1;  // operand-pair loads per k-step, earliest first
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      const int cur = kk & 1;
      if (kk + 1 < KSTEPS) read_frags(st, kk + 1, af[cur ^ 1], bf[cur ^ 1]);
#pragma unroll
      for (int i = kk * LOADS_PER_K; i < (kk + 1) * LOADS_PER_K && i < LPW; ++i) issue(kn, (ks + 1) & 1, i);
#pragma unroll
      for (int i = 0; i < MV; ++i)
#pragma unroll
        for (int j = 0; j < MR; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cur][i], bf[cur][j], acc[i][j], 0, 0, 0);
    }
    // Issue order of the whole step (one scheduling region): the first k-step's
    // fragment reads; then, per k-step, after each matrix instruction one LDS read
    // (fragments of the next k-step) or one global load.  The global loads all go
    // out in the first k-steps so that they have the rest of the step to land.
    {
      static_assert(KSTEPS * LOADS_PER_K >= LPW, "all loads of a step fit into its k-steps");
      __builtin_amdgcn_sched_group_barrier(0x100, NREAD, 0);
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        const bool reads = kk + 1 < KSTEPS;
        const int first = kk * LOADS_PER_K;
        const int nl = first >= LPW ? 0 : (LPW - first < LOADS_PER_K ? LPW - first : LOADS_PER_K);
        if (reads) {
#pragma unroll
          for (int q = 0; q < NREAD; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          }
        }
#pragma unroll
        for (int q = 0; q < 2 * nl; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        // the remaining matrix instructions of the k-step, one group each (sizes must be literals)
#pragma unroll
        for (int q = (reads ? NREAD : 0) + 2 * nl; q < NMFMA; ++q) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      }
    }
    __builtin_amdgcn_s_waitcnt(0);  // this wave's share of step ks+1 is in LDS
    zero_tail(ks + 1);
    __syncthreads();
  }

  // ---- Eq. 1 on the accumulators ------------------------------------------------
  // acc[i][j][r] = z[v][row] with v = v0 + wv*(TV/WV) + 32 i + 8 (r/4) + 4 hf + r%4
  // (increasing in (i, r)) and row = r0 + wr*(TR/WR) + 32 j + lq.
  const int vbase = v0 + wv * (TV / WV) + 4 * hf;
  const bool ragged = v0 + TV > a.V;
  Partial *lds_part = reinterpret_cast<Partial *>(smem);  // [TR][WV] after the last barrier
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
    // sum of exp2(z*log2e - rc) against the ROUNDED product rc = m1*log2e (one fma +
    // exp2 per logit), then taken off that reference with an fma of its own, which
    // cancels the rounding of rc exactly
    const float ref = m1 == -INFINITY ? 0.f : m1;
    const float rc = ref * kLog2e;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MV; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i][j][r], kLog2e, -rc));
    s *= __builtin_amdgcn_exp2f(__builtin_fmaf(-ref, kLog2e, rc));
    Partial p;
    p.m1 = m1; p.m2 = m2; p.s = s;
    p.idx = vbase + 32 * (code >> 4) + 8 * ((code & 15) >> 2) + (code & 3);
    // the other half-column of the 32x32 blocks (lane +-32) holds the rows' other vocabulary entries
    Partial o;
    o.m1 = __shfl_xor(p.m1, 32); o.m2 = __shfl_xor(p.m2, 32); o.s = __shfl_xor(p.s, 32); o.idx = __shfl_xor(p.idx, 32);
    p = fold(p, o);
    if (hf == 0) lds_part[(wr * (TR / WR) + 32 * j + lq) * WV + wv] = p;
  }
  __syncthreads();
  // one thread per row of the tile folds the WV waves' results and writes the partial
  for (int t = tid; t < TR; t += NT) {
    Partial p = lds_part[t * WV];
#pragma unroll
    for (int u = 1; u < WV; ++u) p = fold(p, lds_part[t * WV + u]);
    const int r = r0 + t;
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

template <int WV, int WR>
int32_t launch_lm_head_t(const LmArgs &a, int64_t nwg, hipStream_t st) {
  const size_t lds = 2 * size_t(STAGE);  // two K steps in LDS
  auto kern = lm_head_kernel<WV, WR>;
  static std::atomic<uint64_t> configured{0};  // per instantiation, one bit per device
  if (const int32_t rc = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, configured, "lsp_lm_head_confidence: hipFuncSetAttribute")) return rc;
  kern<<<dim3(static_cast<unsigned>(nwg)), 64 * WV * WR, lds, st>>>(a);
  LSP_CHECK_LAUNCH("lsp_lm_head_confidence: launch");
  return LSP_OK;
}

int32_t launch_lm_head(const LmArgs &a, int64_t nwg, hipStream_t st) {
  // Four waves of 128 x 128 outputs each need the fewest LDS reads per matrix
  // instruction (8 fragment reads feed 16 instructions; eight waves of 128 x 64
  // need 6 for 8) and win once several row tiles share every weight tile.  With
  // few rows the weight matrix streams from HBM once and nothing is re-used: two
  // waves per SIMD then cover the longer load latency better (measured).
  if (a.RT >= 4) return launch_lm_head_t<2, 2>(a, nwg, st);
  return launch_lm_head_t<2, 4>(a, nwg, st);
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
  const int32_t rc = launch_lm_head(a, nwg, st);
  if (rc != LSP_OK) return rc;
  lm_head_finish_kernel<<<dim3(static_cast<unsigned>((rows + 3) / 4)), 256, 0, st>>>(
      a.partials, int(rows), S, a.VT, suffix_len, top1_id, top1_prob, margin);
  LSP_CHECK_LAUNCH("lsp_lm_head_confidence: finish launch");
  return LSP_OK;
}
