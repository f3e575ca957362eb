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
// K and V blocks (32 keys) are fetched with coalesced 16-byte loads and staged
// row-major in LDS; K fragments are read back as 16-byte row pieces, V^T
// fragments with the LDS transpose load (ds_read_tr16_b64), which hands each
// lane four keys of its d column.  Block j+1's global loads are in flight while
// block j goes through the products and the soft-max, and two waves per SIMD
// cover each other's waits.
//
// The soft-max reference m only moves when a block maximum exceeds it by more
// than 8 octaves, so the accumulator rescale is a cold, wave-uniform branch;
// probabilities are then at most 2^8, which bf16 and the fp32 sums hold
// without loss, and the final division by the row sum removes the offset.
//
// Four kernels share that arithmetic:
//  * attn_bf16_kernel (short suffixes): a workgroup is WM x WK waves, WM blocks
//    of 32 queries and a WK-way split of the key range between waves of the
//    same query block (merged through LDS at the end).  Every wave streams its
//    own K/V blocks and never waits for another wave, so a step with few
//    active rows still fills 256 compute units and runs at memory latency.
//    With head_dim 128 its K/V rows go from global memory straight into the
//    wave's LDS region (global_load_lds_dwordx4, rows unpadded and swizzled).
//  * attn_bf16_tile_kernel (long suffixes): the WM waves of a workgroup share
//    each K/V block through a two-stage LDS ring (every wave fetches 1/WM of
//    the block), one barrier per block; L1/L2 traffic per flop drops WM-fold,
//    which is what the matrix cores need once the problem is compute bound.
//  * attn_bf16_ring_kernel (long suffixes at head_dim 128 with suffix buffers of
//    more than 128 rows, cache rows addressed through an index list): eight
//    waves, K/V straight from global memory into an eight-stage LDS ring, one
//    barrier every four blocks; described where it is defined.
//  * attn_bf16_pipe_kernel (the same shapes with a contiguous cache, i.e. the
//    long-context and decode-loop configurations): the same ring, but the block
//    loop is a generated, hand-scheduled inline-asm statement
//    (gen_attn_pipe.py -> lsp_attn_pipe_loop.inc) in which the first product of
//    block j+1, the soft-max of block j and the second product of block j are
//    interleaved instruction by instruction; ragged first/last blocks and
//    short sequences are handled in C++ around it.  A wave with no active
//    query (last tile of a ragged suffix) runs lsp_attn_pipe_idle_loop.inc:
//    its loads, waits and barriers only.
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

// Reductions over the two lanes l and l+32 (the two halves of an accumulator
// column), result in both lanes.  v_permlane32_swap with both operands equal
// hands every lane the lower-half value and the upper-half value of its column
// as a register pair: one VALU instruction instead of a trip through LDS.
__device__ __forceinline__ float half_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmax_raw(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int D>
struct Geo {
  static constexpr int KPITCH = D * 2 + 16;   // bytes per staged K row: 16 mod 256 keeps 16-byte column reads conflict-free
  static constexpr int VPITCH = D * 2 + 64;   // bytes per staged V row: 64 mod 256 keeps the transpose reads conflict-free
  static constexpr int OPITCH = D * 4 + 16;   // bytes per merged O row (fp32): 16 mod 256 for 16-byte column writes
  static constexpr int KBYTES = 32 * KPITCH;
  static constexpr int VBYTES = 32 * VPITCH;
  static constexpr int OBYTES = 32 * OPITCH + 2 * 32 * 4;  // O^T block + m[32] + l[32]
  static constexpr int WAVE_LDS = KBYTES + VBYTES > OBYTES ? KBYTES + VBYTES : OBYTES;
};

// V^T fragments of a 32-key block for O^T += V^T . P^T, read from an LDS tile of
// 32 rows (pitch VPITCH) with the transpose load: within 16 lanes, lane s
// addresses row (s/4), columns 4*(s%4)..+3 and receives column s of the 4 rows.
// Contraction slot 8*hf+e of step k2 is key 16*k2 + 8*(e/4) + 4*hf + e%4 (the
// accumulator row order of the first product).
// SWZ selects the tile layout: false = rows of pitch Geo<D>::VPITCH (padded);
// true = unpadded rows of D*2 bytes whose 64-byte chunk c sits at chunk position
// c ^ (row & 3), which is what loads that go from global memory straight into
// LDS produce (they cannot pad, so they permute).
// One V^T fragment: two transpose loads, rows r..r+3 and r+8..r+11 of a tile with
// PITCH bytes per row, at the address of this lane's piece of row r.
// The pointer is declared restrict for the sake of the compiler's wait-count
// tracking: without alias scope information every transpose load is made to
// wait for ALL outstanding global -> LDS loads (vmcnt(0)), also those that fill
// other rows; the waits that order these reads after the loads they do depend
// on are written out where the kernels issue such loads.
template <int PITCH>
__device__ __forceinline__ bf16x8 vt_read(const unsigned char *__restrict__ ap) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(ap));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(ap + 8 * PITCH));
  const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
  const u32x4 w = {l2.x, l2.y, h2.x, h2.y};
  return __builtin_bit_cast(bf16x8, w);
}
template <int D, bool SWZ = false>
__device__ __forceinline__ void load_v_frags(bf16x8 (&vf)[D / 32][2], int lane, const unsigned char *vtile) {
  constexpr int VPITCH = SWZ ? D * 2 : Geo<D>::VPITCH;
  const int hf = lane >> 5, s16 = lane & 15;
  const unsigned char *vbase = vtile + (4 * hf + (s16 >> 2)) * VPITCH + (16 * ((lane >> 4) & 1) + 4 * (s16 & 3)) * 2;
  const int r3 = (s16 >> 2) & 3;  // row & 3 of every row this lane addresses
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2)
      vf[db][k2] = vt_read<VPITCH>(vbase + (16 * k2) * VPITCH + 64 * (SWZ ? (db ^ r3) : db));
}

// Second half of a 32-key block, shared by both kernels: soft-max of the score
// block s (keys key0.., this wave's 32 queries) against the lagging reference,
// then O^T += V^T . P^T with the V^T fragments vf.
template <int D>
__device__ __forceinline__ void softmax_pv(f32x16 &s, f32x16 (&oacc)[D / 32], float &mref, float &lsum,
                                           int key0, int T, float sc, int lane,
                                           const bf16x8 (&vf)[D / 32][2]) {
  constexpr int DB = D / 32;
  const int hf = lane >> 5;
  if (key0 + 32 > T) {  // ragged last block: keys >= T get -inf
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = key0 + 8 * (r >> 2) + 4 * hf + (r & 3);
      s[r] = key < T ? s[r] : -INFINITY;
    }
  }
  float bm = fmax_raw(s[0], s[1]);
#pragma unroll
  for (int r = 2; r < 16; r += 2) bm = fmax3_raw(bm, s[r], s[r + 1]);
  bm = half_max(bm) * sc;  // finite: key0 < T is a valid key
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
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2)
      oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][k2], pf[k2], oacc[db], 0, 0, 0);
}

// Workgroup placement shared by both kernels.  Workgroups are handed to the 8
// XCDs round-robin by linear id, and each XCD has its own L2.  All workgroups
// that read the same K/V stream - the query tiles of every query head of one
// (sequence, KV head) unit - are therefore given ids that are congruent modulo
// 8, so the stream is fetched into one L2 instead of eight.
// Within an XCD the order is: groups of kUnitGroup units; inside a group the
// query tile is the slow index and the unit the fast one.  Tiles at or beyond
// the active length exit at once, and in a decode loop that is most tiles of
// every unit: with the tile as the fast index the surviving workgroups would sit
// at a fixed stride of the dispatch order, which the hardware maps onto a fixed
// subset of the compute units (measured: the time did not drop at all when the
// active length fell from 1024 to 256).  Runs of kUnitGroup live workgroups
// spread over all of them, and the tiles of one unit still run close enough
// together to share its K/V stream in L2.
constexpr int kUnitGroup = 8;
constexpr int kShortSuffix = 64;  // sequences with at most this many active rows take the key-split kernel
// (the hand-scheduled kernel decides per TILE and at 32 rows: with its loader-only loop for waves
// without a query, a tile with two active waves is faster than two key-split workgroups - 38 against
// 50 us per C5 layer - while a tile with one active wave is slower than one key-split workgroup)
constexpr int kShortSuffixPipe = 32;
struct Place {
  int b, g, h, q0;
  bool valid;
};
__device__ __forceinline__ Place place(const AttnArgs &a, int qtile) {
  Place p;
  const int QT = (a.S + qtile - 1) / qtile;
  const int rep = a.Hq / a.Hkv;
  const int per_unit = rep * QT;
  const int n = blockIdx.x;
  const int m8 = n >> 3;
  const int G = a.unit_group;
  const int grp = m8 / (G * per_unit), r = m8 % (G * per_unit);
  const int wu = r / G;
  const int unit = (grp * G + r % G) * 8 + (n & 7);
  p.valid = unit < a.B * a.Hkv;
  p.b = unit / a.Hkv;
  p.g = unit % a.Hkv;
  p.h = p.g * rep + wu / QT;
  p.q0 = (wu % QT) * qtile;
  return p;
}
// group size (stored in a.unit_group) and number of workgroups of that placement
inline int64_t place_grid(AttnArgs &a, int qtile) {
  const int64_t QT = (a.S + qtile - 1) / qtile;
  const int64_t units8 = (int64_t(a.B) * a.Hkv + 7) / 8;  // units per XCD
  int64_t G = units8 < kUnitGroup ? units8 : kUnitGroup;
  a.unit_group = int32_t(G);
  const int64_t groups = (units8 + G - 1) / G;
  return groups * G * (a.Hq / a.Hkv) * QT * 8;
}

// Final step shared by both kernels: the WK partial results of every query
// block are combined through LDS (each wave's region holds O^T as [query][d]
// fp32 plus m and l), normalised and stored as 16-byte bf16 chunks.
template <int D, int WM, int WK>
__device__ __forceinline__ void merge_store(const AttnArgs &a, const f32x16 (&oacc)[D / 32], float mref,
                                            float lsum, unsigned char *smem, int b, int h, int q0,
                                            int N) {
  using G = Geo<D>;
  constexpr int DB = D / 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WK, wk = wave % WK;
  const int lq = lane & 31, hf = lane >> 5;
  unsigned char *wlds = smem + wave * G::WAVE_LDS;
  lsum = half_sum(lsum);
  __syncthreads();  // every wave is done with the K/V staging memory
  float *ml = reinterpret_cast<float *>(wlds + 32 * G::OPITCH);
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const f32x4 v = {oacc[db][4 * r4], oacc[db][4 * r4 + 1], oacc[db][4 * r4 + 2], oacc[db][4 * r4 + 3]};
      *reinterpret_cast<f32x4 *>(wlds + lq * G::OPITCH + (32 * db + 8 * r4 + 4 * hf) * 4) = v;
    }
  if (hf == 0) {
    ml[lq] = mref;
    ml[32 + lq] = lsum;
  }
  __syncthreads();
  // wave (wm, wk) finishes d-range [wk*D/WK, (wk+1)*D/WK) of its query block: items = (query, 8 d)
  constexpr int DW = D / WK;  // d columns per wave
  constexpr int CH = DW / 8;  // 16-byte output chunks per query
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

// One wave-wide load from global memory straight into LDS: lane l fetches 16
// bytes at its own address g and they land at lds_base + 16 l (lds_base is
// wave-uniform; the counter to wait on is vmcnt, and loads complete in order).
__device__ __forceinline__ void load_to_lds(const char *g, unsigned char *lds_base) {
  __builtin_amdgcn_global_load_lds(g, (__attribute__((address_space(3))) void *)lds_base, 16, 0, 0);
}
constexpr int kWaitVm0 = 0x0F70;      // s_waitcnt vmcnt(0), other counters untouched
constexpr int kWaitVm8 = 0x0F78;      // s_waitcnt vmcnt(8)
constexpr int kWaitLgkm0 = 0xC07F;    // s_waitcnt lgkmcnt(0), other counters untouched

// Body of the wave-private kernel for the WM*32 queries from q0 of (sequence b,
// query head h, KV head g); every thread of a workgroup of 64*WM*WK threads
// calls it with the same arguments (it contains barriers).
template <int D, int WM, int WK, bool GATHER>
__device__ __forceinline__ void key_split_body(const AttnArgs &a, int b, int g, int h, int q0, int N, int P,
                                               unsigned char *smem) {
  using G = Geo<D>;
  constexpr int KK = D / 16;  // d-steps of the first product
  constexpr int DB = D / 32;  // 32-row blocks of O^T
  constexpr int VL = D / 16;  // 16-byte V loads per lane per block (32 rows * D*2 bytes / 64 lanes / 16)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int T = P + N;
  const int wm = wave / WK, wk = wave % WK;
  const int lq = lane & 31, hf = lane >> 5;
  unsigned char *wlds = smem + wave * G::WAVE_LDS;

  const uint16_t *kc = static_cast<const uint16_t *>(a.k_cache) + b * a.cs[0] + g * a.cs[2];
  const uint16_t *vc = static_cast<const uint16_t *>(a.v_cache) + b * a.cs[0] + g * a.cs[2];
  const uint16_t *ks = static_cast<const uint16_t *>(a.k_suf) + b * a.ks[0] + g * a.ks[2];
  const uint16_t *vs = static_cast<const uint16_t *>(a.v_suf) + b * a.ks[0] + g * a.ks[2];

  bf16x8 qf[KK];
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float mref = -INFINITY, lsum = 0.f;
  const float sc = a.scale * kLog2e;

  const int NB = (T + 31) >> 5;  // 32-key blocks; this wave takes wk, wk+WK, ...

  // K and V blocks take the same way: coalesced 16-byte loads (a wave-wide load
  // covers whole rows: lane -> (row, 16-byte column)), a wave-private LDS stage,
  // and fragment reads from there.  (Reading K fragments straight from global
  // memory costs four times the address-unit cycles: every load touches 32 rows
  // for 32 bytes each, and at small sizes those cycles are the critical path.)
  auto row_ptr = [&](const uint16_t *cache, const uint16_t *suf, int t) -> const uint16_t * {
    t = min(t, T - 1);
    return t < P ? cache + int64_t(cache_row<GATHER>(a, b, t)) * a.cs[1] : suf + int64_t(t - P) * a.ks[1];
  };
  constexpr int VCOL = D / 8;          // 16-byte columns per row
  constexpr int RPL = 64 / VCOL;       // rows covered by one wave-wide load
  const int vcol = lane % VCOL, vr0 = lane / VCOL;
  u32x4 kreg[VL], vreg[VL];
  auto load_kv = [&](int jb) {
#pragma unroll
    for (int i = 0; i < VL; ++i) {
      const int t = 32 * jb + RPL * i + vr0;
      kreg[i] = *reinterpret_cast<const u32x4 *>(row_ptr(kc, ks, t) + 8 * vcol);
      vreg[i] = *reinterpret_cast<const u32x4 *>(row_ptr(vc, vs, t) + 8 * vcol);
    }
  };
  auto stage_kv = [&](int jb) {
#pragma unroll
    for (int i = 0; i < VL; ++i) {
      const int r = RPL * i + vr0;
      u32x4 v = vreg[i];
      if (32 * jb + r >= T) v = u32x4{0, 0, 0, 0};  // keys beyond T contribute exact zeros
      *reinterpret_cast<u32x4 *>(wlds + r * G::KPITCH + 16 * vcol) = kreg[i];
      *reinterpret_cast<u32x4 *>(wlds + G::KBYTES + r * G::VPITCH + 16 * vcol) = v;
    }
  };

  auto block = [&](int jb) {
    stage_kv(jb);
    const int jn = jb + WK;
    if (jn < NB) load_kv(jn);  // in flight while this block is worked on
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(wlds + lq * G::KPITCH + (16 * kk + 8 * hf) * 2);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s, 0, 0, 0);
    }
    bf16x8 vf[DB][2];
    load_v_frags<D>(vf, lane, wlds + G::KBYTES);
    softmax_pv<D>(s, oacc, mref, lsum, 32 * jb, T, sc, lane, vf);
  };

  // (machinery of the head_dim-128 path, described where it is used below)
  unsigned char *wl = smem + __builtin_amdgcn_readfirstlane(wave) * G::WAVE_LDS;  // scalar base for the loads
  constexpr int KB = 32 * D * 2;                    // K rows, then V rows
  const int pp = lane & 15, lr = lane >> 4;         // 16-byte position and row (of 4) inside a wave-wide load
  int kcol[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) kcol[q] = 16 * (pp ^ ((4 * q + lr) & 15));
  const int vswz = 64 * ((pp >> 2) ^ (lr & 3)) + 16 * (pp & 3);
  const char *kcb = reinterpret_cast<const char *>(kc), *vcb = reinterpret_cast<const char *>(vc);
  const char *ksb = reinterpret_cast<const char *>(ks), *vsb = reinterpret_cast<const char *>(vs);
  const int64_t cpitch = a.cs[1] * 2, spitch = a.ks[1] * 2;
  const int32_t *crows = GATHER ? a.cache_rows + int64_t(b) * a.C : nullptr;
  const int Cmax = a.C - 1;
  int64_t roff[8];  // byte offset of this lane's row of wave-wide load i, from the cache or the suffix base
  // A block that lies wholly in the cache or wholly in the suffix (all but one or
  // two of a wave's blocks) is a wave-uniform base, stepped by four rows per load
  // on the scalar unit, plus a 32-bit lane offset computed once; the general form
  // costs about ten vector instructions per load.
  uint32_t kofc[4], kofs[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    kofc[q] = uint32_t(lr * cpitch + kcol[q]);
    kofs[q] = uint32_t(lr * spitch + kcol[q]);
  }
  const uint32_t vofc = uint32_t(lr * cpitch + vswz), vofs = uint32_t(lr * spitch + vswz);
  auto issue_k = [=, &roff](int jb) __attribute__((always_inline)) {
    const int t0 = 32 * jb;
    if (!GATHER && t0 + 32 <= P) {
      const char *base = kcb + int64_t(t0) * cpitch;
#pragma unroll
      for (int i = 0; i < 8; ++i) load_to_lds(base + int64_t(4 * i) * cpitch + kofc[i & 3], wl + 1024 * i);
      return;
    }
    if (t0 >= P && t0 + 32 <= T) {
      const char *base = ksb + int64_t(t0 - P) * spitch;
#pragma unroll
      for (int i = 0; i < 8; ++i) load_to_lds(base + int64_t(4 * i) * spitch + kofs[i & 3], wl + 1024 * i);
      return;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int t = min(32 * jb + 4 * i + lr, T - 1);
      int crow = t;
      if (GATHER && t < P) crow = min(max(crows[t], 0), Cmax);  // a bad index must not leave the buffer
      roff[i] = t < P ? int64_t(crow) * cpitch : int64_t(t - P) * spitch;
      load_to_lds((t < P ? kcb : ksb) + roff[i] + kcol[i & 3], wl + 1024 * i);
    }
  };
  auto issue_v = [=, &roff](int jb) __attribute__((always_inline)) {
    const int t0 = 32 * jb;
    if (!GATHER && t0 + 32 <= P) {
      const char *base = vcb + int64_t(t0) * cpitch;
#pragma unroll
      for (int i = 0; i < 8; ++i) load_to_lds(base + int64_t(4 * i) * cpitch + vofc, wl + KB + 1024 * i);
      return;
    }
    if (t0 >= P && t0 + 32 <= T) {
      const char *base = vsb + int64_t(t0 - P) * spitch;
#pragma unroll
      for (int i = 0; i < 8; ++i) load_to_lds(base + int64_t(4 * i) * spitch + vofs, wl + KB + 1024 * i);
      return;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int t = min(32 * jb + 4 * i + lr, T - 1);
      load_to_lds((t < P ? vcb : vsb) + roff[i] + vswz, wl + KB + 1024 * i);
    }
  };
  const int wk_s = __builtin_amdgcn_readfirstlane(wk);  // the same value, known to be wave-uniform
  if constexpr (D == 128) {
    if (wk_s < NB) {
      issue_k(wk_s);
      issue_v(wk_s);
    }
  } else {
    if (wk < NB) load_kv(wk);
  }
  // (the first K/V block is already on its way)
  // Q fragments (B operand of S^T = K.Q^T): query lq of this wave, d = 16*kk + 8*hf + 0..7.
  // The WK waves of a query block need the same 32 rows: the workgroup fetches
  // its WM*32 rows once, coalesced, into LDS (behind the wave regions), and every
  // wave reads its fragments from there.  (Fetched per wave and per fragment,
  // each load touched 32 rows for 32 bytes: four times the cache lines, times
  // WK waves - 40 % of all L1 traffic of a short step.)
  {
    constexpr int QCOL = D / 8;  // 16-byte columns per row
    unsigned char *qlds = smem + WM * WK * G::WAVE_LDS;
    const uint16_t *qb = static_cast<const uint16_t *>(a.q) + b * a.qs[0] + h * a.qs[2];
    for (int i = tid; i < WM * 32 * QCOL; i += 64 * WM * WK) {
      const int r = i / QCOL, c = i % QCOL;
      const u32x4 v = *reinterpret_cast<const u32x4 *>(qb + int64_t(min(q0 + r, N - 1)) * a.qs[1] + 8 * c);
      *reinterpret_cast<u32x4 *>(qlds + r * G::KPITCH + 16 * c) = v;
    }
  }
  __syncthreads();
#pragma unroll
  for (int kk = 0; kk < KK; ++kk)
    qf[kk] = *reinterpret_cast<const bf16x8 *>(smem + WM * WK * G::WAVE_LDS + (wm * 32 + lq) * G::KPITCH + (16 * kk + 8 * hf) * 2);

  if constexpr (D == 128) {
    // head_dim 128: K and V rows go from global memory straight into this wave's
    // LDS region (no staging registers, no LDS store instructions on the critical
    // path: at these sizes the eight waves' staging traffic, 128 KB written per
    // block step, was a good part of a block's time).  A wave-wide load fills 1 KB
    // = 4 unpadded rows of 256 bytes; bank conflicts are avoided by a swizzle that
    // the loading lane applies to its GLOBAL address: K keeps 16-byte chunk c of
    // row r at chunk position c ^ (r & 15), V keeps 64-byte chunk c at c ^ (r & 3).
    // One region per wave: the K rows of the wave's next block are requested as
    // soon as this block's K fragments sit in registers, its V rows as soon as
    // the V^T fragments do.
    const int y16 = 16 * (hf ^ (lq & 15));
    int jb = wk_s;
    // (the first block was requested before the Q rows, see above)
    for (; jb < NB; jb += WK) {
      const bool more = jb + WK < NB;
      __builtin_amdgcn_s_waitcnt(kWaitVm8);  // all but the newest 8 loads (this block's V rows) have landed: K is there
      bf16x8 kf[KK];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kf[kk] = *reinterpret_cast<const bf16x8 *>(wlds + lq * (D * 2) + ((32 * kk) ^ y16));
      __builtin_amdgcn_s_waitcnt(kWaitLgkm0);  // fragments are in registers: the K rows may be overwritten
      if (more) issue_k(jb + WK);
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], s, 0, 0, 0);
      if (more) __builtin_amdgcn_s_waitcnt(kWaitVm8);  // V rows of this block (the next block's 8 K loads are newer)
      else __builtin_amdgcn_s_waitcnt(kWaitVm0);
      if (32 * jb + 32 > T) {  // keys beyond T contribute exact zeros: their owners overwrite the V slots
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (32 * jb + 4 * i + lr >= T) *reinterpret_cast<u32x4 *>(wlds + KB + 1024 * i + 16 * lane) = u32x4{0, 0, 0, 0};
      }
      bf16x8 vf[DB][2];
      load_v_frags<D, true>(vf, lane, wlds + KB);
      __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
      if (more) issue_v(jb + WK);
      softmax_pv<D>(s, oacc, mref, lsum, 32 * jb, T, sc, lane, vf);
    }
    __builtin_amdgcn_s_waitcnt(kWaitVm0);  // nothing of this wave is still on its way into LDS
  } else {
    for (int jb = wk; jb < NB; jb += WK) block(jb);
  }
  merge_store<D, WM, WK>(a, oacc, mref, lsum, smem, b, h, q0, N);
}

template <int D, int WM, int WK, bool GATHER>
__global__ __launch_bounds__(64 * WM * WK, 2) void attn_bf16_kernel(AttnArgs a_in, AttnLayers layers) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const AttnArgs a = for_layer(a_in, layers);
  const Place pl = place(a, 32 * WM);
  if (!pl.valid) return;
  const int N = min(max(a.suffix_len[pl.b], 0), a.S);
  if (pl.q0 >= N) return;
  const int P = min(max(a.prefix_len[pl.b], 0), a.C);
  key_split_body<D, WM, WK, GATHER>(a, pl.b, pl.g, pl.h, pl.q0, N, P, smem);
}

template <int D, int WM, int WK, bool GATHER>
int32_t launch_g(AttnArgs a, const AttnLayers &layers, hipStream_t st) {
  const int64_t nwg = place_grid(a, 32 * WM);
  if (nwg > 0x7fffffff) {
    set_error("lsp_attn_step: launch of %lld workgroups is too large", (long long)nwg);
    return LSP_ERR_UNSUPPORTED;
  }
  const dim3 grid(static_cast<unsigned>(nwg), layers.n > 0 ? layers.n : 1, 1);
  const size_t lds = size_t(WM * WK) * Geo<D>::WAVE_LDS + size_t(WM) * 32 * Geo<D>::KPITCH;  // wave regions + Q rows
  auto kern = attn_bf16_kernel<D, WM, WK, GATHER>;
  static std::atomic<uint64_t> configured{0};  // per instantiation, one bit per device
  if (const int32_t rc = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, configured, "lsp_attn_step: hipFuncSetAttribute")) return rc;
  kern<<<grid, 64 * WM * WK, lds, st>>>(a, layers);
  LSP_CHECK_LAUNCH("lsp_attn_step: bf16 launch");
  return LSP_OK;
}

// ---- long-suffix kernel: K/V blocks shared by the WM waves through LDS -----------
template <int D>
struct TileGeo {
  static constexpr int KPITCH = D * 2 + 16;  // bytes per K row: 16 mod 256 keeps 16-byte column reads conflict-free
  static constexpr int VPITCH = Geo<D>::VPITCH;
  static constexpr int KBYTES = 32 * KPITCH;
  static constexpr int STAGE = KBYTES + 32 * VPITCH;
};

template <int D, int WM, int OCC, int PD, bool GATHER>
__global__ __launch_bounds__(64 * WM, OCC) void attn_bf16_tile_kernel(AttnArgs a_in, AttnLayers layers) {
  const AttnArgs a = for_layer(a_in, layers);
  using TG = TileGeo<D>;
  constexpr int NT = 64 * WM;
  constexpr int KK = D / 16;
  constexpr int DB = D / 32;
  constexpr int CPR = D / 8;               // 16-byte pieces per row
  constexpr int PIECES = 32 * CPR / NT;    // pieces of K (and of V) per thread per block
  static_assert(32 * CPR % NT == 0, "loader mapping");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const Place pl = place(a, 32 * WM);
  if (!pl.valid) return;
  const int b = pl.b, g = pl.g, h = pl.h, q0 = pl.q0;
  const int N = min(max(a.suffix_len[b], 0), a.S);
  const int P = min(max(a.prefix_len[b], 0), a.C);
  if (q0 >= N) return;
  const int T = P + N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, hf = lane >> 5;

  const uint16_t *kc = static_cast<const uint16_t *>(a.k_cache) + b * a.cs[0] + g * a.cs[2];
  const uint16_t *vc = static_cast<const uint16_t *>(a.v_cache) + b * a.cs[0] + g * a.cs[2];
  const uint16_t *ks = static_cast<const uint16_t *>(a.k_suf) + b * a.ks[0] + g * a.ks[2];
  const uint16_t *vs = static_cast<const uint16_t *>(a.v_suf) + b * a.ks[0] + g * a.ks[2];

  // a wave none of whose 32 queries is active only fetches its share of the K/V
  // blocks and keeps the barriers
  const bool live = q0 + 32 * __builtin_amdgcn_readfirstlane(wave) < N;
  const int qi = q0 + wave * 32 + lq;
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
  const int NB = (T + 31) >> 5;

  // loader: piece i of this thread is (row, 16-byte column) = ((tid + NT*i) / CPR, (tid + NT*i) % CPR).
  // PD register sets hold the blocks in flight: the loop is throughput-bound by
  // bytes in flight per compute unit, so the prefetch distance is a tuning knob.
  u32x4 kreg[PD][PIECES], vreg[PD][PIECES];
  // Per-thread byte offsets of piece i inside a block that lies wholly in the
  // cache or wholly in the suffix: (row, column) of the piece times the strides,
  // computed once.  Such a block then costs one 64-bit add per load, on top of a
  // wave-uniform base that the scalar unit computes; only the block that
  // straddles the cache/suffix boundary, the ragged last block and the gather
  // form take the general per-row path.
  int64_t offc[PIECES], offs[PIECES];
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    const int pc = tid + NT * i;
    offc[i] = (int64_t(pc / CPR) * a.cs[1] + 8 * (pc % CPR)) * 2;
    offs[i] = (int64_t(pc / CPR) * a.ks[1] + 8 * (pc % CPR)) * 2;
  }
  auto load_block = [&](int jb, u32x4 (&kr)[PIECES], u32x4 (&vr)[PIECES]) {
    const int t0 = 32 * jb;
    if (!GATHER && t0 + 32 <= P) {
      const int64_t base = int64_t(t0) * a.cs[1] * 2;  // wave-uniform
      const char *kb = reinterpret_cast<const char *>(kc) + base, *vb = reinterpret_cast<const char *>(vc) + base;
#pragma unroll
      for (int i = 0; i < PIECES; ++i) {
        kr[i] = *reinterpret_cast<const u32x4 *>(kb + offc[i]);
        vr[i] = *reinterpret_cast<const u32x4 *>(vb + offc[i]);
      }
      return;
    }
    if (t0 >= P && t0 + 32 <= T) {
      const int64_t base = int64_t(t0 - P) * a.ks[1] * 2;
      const char *kb = reinterpret_cast<const char *>(ks) + base, *vb = reinterpret_cast<const char *>(vs) + base;
#pragma unroll
      for (int i = 0; i < PIECES; ++i) {
        kr[i] = *reinterpret_cast<const u32x4 *>(kb + offs[i]);
        vr[i] = *reinterpret_cast<const u32x4 *>(vb + offs[i]);
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int pc = tid + NT * i;
      const int t = min(t0 + pc / CPR, T - 1);
      const int64_t off = t < P ? int64_t(cache_row<GATHER>(a, b, t)) * a.cs[1] : int64_t(t - P) * a.ks[1];
      const uint16_t *kp = (t < P ? kc : ks) + off + 8 * (pc % CPR);
      const uint16_t *vp = (t < P ? vc : vs) + off + 8 * (pc % CPR);
      kr[i] = *reinterpret_cast<const u32x4 *>(kp);
      vr[i] = *reinterpret_cast<const u32x4 *>(vp);
    }
  };
  auto store_block = [&](int jb, const u32x4 (&kr)[PIECES], const u32x4 (&vr)[PIECES]) {
    unsigned char *st = smem + (jb & 1) * TG::STAGE;
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int pc = tid + NT * i;
      const int r = pc / CPR, c = pc % CPR;
      u32x4 v = vr[i];
      if (32 * jb + r >= T) v = u32x4{0, 0, 0, 0};  // keys beyond T contribute exact zeros
      *reinterpret_cast<u32x4 *>(st + r * TG::KPITCH + 16 * c) = kr[i];
      *reinterpret_cast<u32x4 *>(st + TG::KBYTES + r * TG::VPITCH + 16 * c) = v;
    }
  };

  // prologue: block 0 goes to stage 0; register set u then holds block u+1
  load_block(0, kreg[0], vreg[0]);
  store_block(0, kreg[0], vreg[0]);
#pragma unroll
  for (int u = 0; u < PD; ++u)
    if (u + 1 < NB) load_block(u + 1, kreg[u], vreg[u]);
  __syncthreads();
  for (int jb0 = 0; jb0 < NB; jb0 += PD) {
#pragma unroll
    for (int u = 0; u < PD; ++u) {
      const int jb = jb0 + u;
      if (jb >= NB) break;
      // block jb+1 (register set u) goes into the stage that every wave finished
      // reading before the last barrier; the set is refilled with block jb+1+PD.
      // Issue order of a block: all K fragment reads; the staging traffic of the
      // blocks ahead (which covers the reads' latency); the first product; all
      // V^T fragment reads (they land while the chain of the first product and
      // the exponentials run); soft-max; second product.
      const unsigned char *st = smem + (jb & 1) * TG::STAGE;
      bf16x8 kf[KK];
      if (live) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
          kf[kk] = *reinterpret_cast<const bf16x8 *>(st + lq * TG::KPITCH + (16 * kk + 8 * hf) * 2);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (jb + 1 < NB) store_block(jb + 1, kreg[u], vreg[u]);
      if (jb + 1 + PD < NB) load_block(jb + 1 + PD, kreg[u], vreg[u]);
      if (live) {
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], s, 0, 0, 0);
        bf16x8 vf[DB][2];
        load_v_frags<D>(vf, lane, st + TG::KBYTES);
        __builtin_amdgcn_sched_barrier(0);
        softmax_pv<D>(s, oacc, mref, lsum, 32 * jb, T, sc, lane, vf);
      }
      __syncthreads();
    }
  }
  // No key split here, so a lane already owns whole outputs: normalise and store
  // its 4-element runs directly (8 bytes each; once per workgroup, after a long
  // key loop, so the short stores do not matter and no LDS is needed).
  lsum = half_sum(lsum);
  if (qi < N) {
    const float inv = 1.0f / lsum;
    uint16_t *op = static_cast<uint16_t *>(a.out) + b * a.os[0] + int64_t(qi) * a.os[1] + h * a.os[2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 w;
        w.x = pack_bf16(oacc[db][4 * r4] * inv, oacc[db][4 * r4 + 1] * inv);
        w.y = pack_bf16(oacc[db][4 * r4 + 2] * inv, oacc[db][4 * r4 + 3] * inv);
        *reinterpret_cast<u32x2 *>(op + 32 * db + 8 * r4 + 4 * hf) = w;
      }
  }
}

template <int D, int WM, int OCC, int PD, bool GATHER>
int32_t launch_tile_g(AttnArgs a, const AttnLayers &layers, hipStream_t st) {
  const int64_t nwg = place_grid(a, 32 * WM);
  if (nwg > 0x7fffffff) {
    set_error("lsp_attn_step: launch of %lld workgroups is too large", (long long)nwg);
    return LSP_ERR_UNSUPPORTED;
  }
  const size_t lds = 2 * size_t(TileGeo<D>::STAGE);  // two shared stages
  auto kern = attn_bf16_tile_kernel<D, WM, OCC, PD, GATHER>;
  static std::atomic<uint64_t> configured{0};  // per instantiation, one bit per device
  if (const int32_t rc = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, configured, "lsp_attn_step: hipFuncSetAttribute")) return rc;
  kern<<<dim3(static_cast<unsigned>(nwg), layers.n > 0 ? layers.n : 1, 1), 64 * WM, lds, st>>>(a, layers);
  LSP_CHECK_LAUNCH("lsp_attn_step: bf16 tile launch");
  return LSP_OK;
}

// ---- long-suffix kernel, head_dim 128: K/V blocks go global -> LDS directly --------
// Same arithmetic as attn_bf16_tile_kernel, different plumbing.  Every 32-key
// block is fetched with two wave-wide global_load_lds_dwordx4 per wave (1 KB = 4
// rows of K, 1 KB = 4 rows of V) into a ring of NS stages of 16 KB, NS-BS blocks
// ahead of the products: the prefetch depth costs LDS instead of registers and
// no LDS store instruction is issued.  Rows are unpadded and swizzled as in the
// key-split body.  LDS holds the K tiles of all stages first, then the V tiles,
// so that every fragment read is a per-lane address computed once plus an
// immediate offset (the loop is unrolled NS times).
// The workgroup synchronises once every BS blocks, not every block: before
// that barrier a wave waits until its shares of the next BS blocks have landed;
// between barriers the eight waves run free (up to BS blocks apart), so the two
// waves of a SIMD drift out of phase and use the matrix and the vector pipeline
// at different times.  Iteration j requests block j+NS-BS into the stage that
// block j-BS was read from, which every wave left before the last barrier.
// (Measured on config 4, NS = 8: 704 us for the tile kernel, 702 us with a
// barrier per block, 685 us with one every two, 680 us with one every four.)
struct RingLoad {
  const char *kc, *vc, *ks, *vs;   // this (sequence, KV head)'s cache and suffix rows
  int64_t cpitch, spitch;          // bytes between rows
  uint32_t kc_off, vc_off, ks_off, vs_off;  // row-in-block * pitch + swizzled column (cache / suffix)
  const int32_t *cache_rows;       // indexed cache: this sequence's row table, else null
  int kcol, vcol, lr, P, T, C;
};
template <bool GATHER>
__device__ __forceinline__ void ring_issue(RingLoad L, int jb, unsigned char *kdst, unsigned char *vdst) {
  const int t0 = 32 * jb;
  const char *kp, *vp;
  if (!GATHER && t0 + 32 <= L.P) {            // block wholly in the cache: wave-uniform base + fixed lane offset
    const int64_t base = int64_t(t0) * L.cpitch;
    kp = L.kc + base + L.kc_off;
    vp = L.vc + base + L.vc_off;
  } else if (t0 >= L.P && t0 + 32 <= L.T) {   // wholly in the suffix
    const int64_t base = int64_t(t0 - L.P) * L.spitch;
    kp = L.ks + base + L.ks_off;
    vp = L.vs + base + L.vs_off;
  } else {                                    // straddles the boundary, ragged end, or indexed cache rows
    const int t = min(t0 + L.lr, L.T - 1);
    if (t < L.P) {
      int crow = t;
      if (GATHER) crow = min(max(L.cache_rows[t], 0), L.C - 1);  // a bad index must not leave the buffer
      kp = L.kc + int64_t(crow) * L.cpitch + L.kcol;
      vp = L.vc + int64_t(crow) * L.cpitch + L.vcol;
    } else {
      kp = L.ks + int64_t(t - L.P) * L.spitch + L.kcol;
      vp = L.vs + int64_t(t - L.P) * L.spitch + L.vcol;
    }
  }
  load_to_lds(kp, kdst);
  load_to_lds(vp, vdst);
}
template <int NS, int BS, bool GATHER>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bf16_ring_kernel(AttnArgs a_in, AttnLayers layers) {
  const AttnArgs a = for_layer(a_in, layers);
  constexpr int D = 128, WM = 8, KK = D / 16, DB = D / 32;
  constexpr int TILE = 32 * D * 2, VBASE = NS * TILE;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const Place pl = place(a, 32 * WM);
  if (!pl.valid) return;
  const int b = pl.b, g = pl.g, h = pl.h, q0 = pl.q0;
  const int N = min(max(a.suffix_len[b], 0), a.S);
  const int P = min(max(a.prefix_len[b], 0), a.C);
  // A sequence whose suffix is down to a few rows (the late steps of a decode
  // loop) would keep this wide tile busy for the whole key range with most of
  // its queries masked.  Its first tiles then each take ONE block of 32 queries
  // and split the KEY range between their waves instead.  Lengths live in device
  // memory, so the choice is made here, per workgroup, not by the launcher.
  // (This workgroup owns its compute unit anyway, so the larger LDS footprint of
  // the key-split mode costs no occupancy.)
  {
    const int tile = q0 / (32 * WM), QT = (a.S + 32 * WM - 1) / (32 * WM);
    const int short_rows = 32 * min(QT, kShortSuffix / 32);
    if (N <= short_rows) {
      if (32 * tile < N) key_split_body<D, 1, WM, GATHER>(a, b, g, h, 32 * tile, N, P, smem);
      return;
    }
  }
  if (q0 >= N) return;
  const int T = P + N;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int lq = lane & 31, hf = lane >> 5;

  // A wave none of whose 32 queries is active (the last tile of a sequence) only
  // fetches its share of the K/V blocks and keeps the barriers: the wave that
  // shares its SIMD then has the matrix and vector pipes to itself.
  const bool live = q0 + 32 * wave_s < N;
  const int qi = q0 + wave * 32 + lq;
  const uint16_t *qp = static_cast<const uint16_t *>(a.q) + b * a.qs[0] + int64_t(min(qi, N - 1)) * a.qs[1] + h * a.qs[2];
  bf16x8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8 *>(qp + 16 * kk + 8 * hf);
  asm volatile("" ::: "memory");  // the Q loads stay ahead of the requests below: the first wait then covers them

  // loader: this lane owns row lr of every block and 16-byte position pp of it
  RingLoad L;
  L.kc = reinterpret_cast<const char *>(static_cast<const uint16_t *>(a.k_cache) + b * a.cs[0] + g * a.cs[2]);
  L.vc = reinterpret_cast<const char *>(static_cast<const uint16_t *>(a.v_cache) + b * a.cs[0] + g * a.cs[2]);
  L.ks = reinterpret_cast<const char *>(static_cast<const uint16_t *>(a.k_suf) + b * a.ks[0] + g * a.ks[2]);
  L.vs = reinterpret_cast<const char *>(static_cast<const uint16_t *>(a.v_suf) + b * a.ks[0] + g * a.ks[2]);
  L.cpitch = a.cs[1] * 2;
  L.spitch = a.ks[1] * 2;
  {
    const int pp = lane & 15;
    L.lr = 4 * wave + (lane >> 4);
    L.kcol = 16 * (pp ^ (L.lr & 15));
    L.vcol = 64 * ((pp >> 2) ^ (L.lr & 3)) + 16 * (pp & 3);
    L.kc_off = uint32_t(L.lr * L.cpitch + L.kcol);
    L.vc_off = uint32_t(L.lr * L.cpitch + L.vcol);
    L.ks_off = uint32_t(L.lr * L.spitch + L.kcol);
    L.vs_off = uint32_t(L.lr * L.spitch + L.vcol);
  }
  L.cache_rows = GATHER ? a.cache_rows + int64_t(b) * a.C : nullptr;
  L.P = P;
  L.T = T;
  L.C = a.C;
  const int NB = (T + 31) >> 5;
  static_assert(NS % BS == 0 && NS >= 2 * BS, "ring depth and barrier period");
  constexpr int kWaitRing = 0x0F70 | (2 * (NS - 2 * BS));  // s_waitcnt vmcnt: all but the newest NS-2BS blocks (two loads each) have landed
#define LSP_RING_ISSUE(jb_, slot_) \
  ring_issue<GATHER>(L, (jb_), smem + (slot_) * TILE + 1024 * wave_s, smem + VBASE + (slot_) * TILE + 1024 * wave_s)
  // prologue: blocks 0 .. NS-BS-1 into their stages (block indices beyond the
  // last one fetch the last block again, into a stage nobody reads, so that the
  // number of loads in flight is the same everywhere)
#pragma unroll
  for (int u = 0; u < NS - BS; ++u) LSP_RING_ISSUE(min(u, NB - 1), u);

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float mref = -INFINITY, lsum = 0.f;
  const float sc = a.scale * kLog2e;

  // Fragment addresses, computed once.  K: row lq of a tile, 16-byte chunk
  // 2*kk + hf at its swizzled position.  V^T: as in load_v_frags (SWZ form), one
  // address per 32-wide d block; the k2 steps and fragment halves are offsets.
  const unsigned char *kaddr[KK], *vaddr[DB];
  {
    const int y16 = 16 * (hf ^ (lq & 15));
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kaddr[kk] = smem + lq * (D * 2) + ((32 * kk) ^ y16);
    const int s16 = lane & 15, r3 = (s16 >> 2) & 3;
    const unsigned char *vbase = smem + VBASE + (4 * hf + (s16 >> 2)) * (D * 2) + (16 * ((lane >> 4) & 1) + 4 * (s16 & 3)) * 2;
#pragma unroll
    for (int db = 0; db < DB; ++db) vaddr[db] = vbase + 64 * (db ^ r3);
  }
  // keys beyond T contribute exact zeros: once the block has landed, the lanes
  // that own such rows overwrite their V slots (cold: the ragged last block only)
  auto zero_beyond = [&](int jb, int slot) {
    if (32 * jb + 32 <= T || jb >= NB) return;
    if (32 * jb + L.lr >= T)
      *reinterpret_cast<u32x4 *>(smem + VBASE + slot * TILE + 1024 * wave + 16 * lane) = u32x4{0, 0, 0, 0};
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
  };
  auto sync = [&]() {  // plain barrier: newer loads stay in flight; no LDS access is moved across it
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  __builtin_amdgcn_s_waitcnt(kWaitRing);  // blocks 0 .. BS-1 (and the Q rows) have arrived
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) asm volatile("" : "+v"(qf[kk]));  // (their wait is here, not in the loop)
#pragma unroll
  for (int k = 0; k < BS; ++k) zero_beyond(k, k);
  sync();
  for (int jb0 = 0; jb0 < NB; jb0 += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      const int jb = jb0 + u;
      if (jb >= NB) break;
      // the stage that block jb-BS was read from is free since the last barrier
      LSP_RING_ISSUE(min(jb + NS - BS, NB - 1), (u + NS - BS) % NS);
      if (live) {
        bf16x8 kf[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[kk] = *reinterpret_cast<const bf16x8 *>(kaddr[kk] + u * TILE);
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], s, 0, 0, 0);
        bf16x8 vf[DB][2];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int k2 = 0; k2 < 2; ++k2) vf[db][k2] = vt_read<D * 2>(vaddr[db] + u * TILE + (16 * k2) * (D * 2));
        __builtin_amdgcn_sched_barrier(0);
        softmax_pv<D>(s, oacc, mref, lsum, 32 * jb, T, sc, lane, vf);
      }
      if ((u % BS) == BS - 1) {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(kWaitRing);  // blocks jb+1 .. jb+BS have landed
#pragma unroll
        for (int k = 1; k <= BS; ++k) zero_beyond(jb + k, (u + k) % NS);
        sync();
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(kWaitVm0);  // nothing of this wave is still on its way into LDS
#undef LSP_RING_ISSUE
  lsum = half_sum(lsum);
  if (qi < N) {
    const float inv = 1.0f / lsum;
    uint16_t *op = static_cast<uint16_t *>(a.out) + b * a.os[0] + int64_t(qi) * a.os[1] + h * a.os[2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 w;
        w.x = pack_bf16(oacc[db][4 * r4] * inv, oacc[db][4 * r4 + 1] * inv);
        w.y = pack_bf16(oacc[db][4 * r4 + 2] * inv, oacc[db][4 * r4 + 3] * inv);
        *reinterpret_cast<u32x2 *>(op + 32 * db + 8 * r4 + 4 * hf) = w;
      }
  }
}

template <int NS, int BS, bool GATHER>
int32_t launch_ring_g(AttnArgs a, const AttnLayers &layers, hipStream_t st) {
  const int64_t nwg = place_grid(a, 256);
  if (nwg > 0x7fffffff) {
    set_error("lsp_attn_step: launch of %lld workgroups is too large", (long long)nwg);
    return LSP_ERR_UNSUPPORTED;
  }
  // the ring, or the key-split mode's eight wave regions + 32 Q rows
  const size_t lds_ring = size_t(NS) * 2 * 32 * 256;
  const size_t lds_split = 8 * size_t(Geo<128>::WAVE_LDS) + 32 * size_t(Geo<128>::KPITCH);
  const size_t lds = lds_ring > lds_split ? lds_ring : lds_split;
  auto kern = attn_bf16_ring_kernel<NS, BS, GATHER>;
  static std::atomic<uint64_t> configured{0};  // per instantiation, one bit per device
  if (const int32_t rc = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, configured, "lsp_attn_step: hipFuncSetAttribute")) return rc;
  kern<<<dim3(static_cast<unsigned>(nwg), layers.n > 0 ? layers.n : 1, 1), 512, lds, st>>>(a, layers);
  LSP_CHECK_LAUNCH("lsp_attn_step: bf16 ring launch");
  return LSP_OK;
}

// ---- long-suffix kernel, head_dim 128, contiguous cache: hand-scheduled block loop ----
// Same tile (256 queries, 8 waves of 32, two waves per SIMD), same LDS ring and the
// same arithmetic as attn_bf16_ring_kernel; what differs is who fixes the issue
// order.  The block loop is one generated inline-asm statement (gen_attn_pipe.py
// describes its pipeline, register map and synchronisation): a one-block software
// pipeline per wave in which the soft-max of block j is issued between the matrix
// instructions of S(j+1) = K(j+1).Q^T, every LDS fragment is requested half a block
// before it is used, and no instruction waits on the one before it.
// The loop only handles full 32-row blocks that lie wholly in the cache or wholly in
// the suffix.  The ragged ends (the last P % 32 cache rows, the last N % 32 suffix
// rows: at most two blocks per tile) are done first, by compiler-scheduled code with
// the same fragment layout, on the same running (m, l, O) state.
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bf16_pipe_kernel(AttnArgs a_in,
                                                                                                       AttnLayers layers) {
  const AttnArgs a = for_layer(a_in, layers);
  constexpr int D = 128, WM = 8, KK = D / 16, DB = D / 32, NS = 8;
  constexpr int TILE = 32 * D * 2, VBASE = NS * TILE;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const Place pl = place(a, 32 * WM);
  if (!pl.valid) return;
  const int b = pl.b, g = pl.g, h = pl.h, q0 = pl.q0;
  const int N = min(max(a.suffix_len[b], 0), a.S);
  const int P = min(max(a.prefix_len[b], 0), a.C);
  if (q0 >= N) return;
  // A tile with at most 32 active rows - a sequence down to its last rows, or the tail of a longer
  // suffix that ends just past a multiple of 256 - would keep seven waves idle for the whole key
  // range: its one block of queries goes to the key-split body (as in attn_bf16_ring_kernel), which
  // shares the KEY range between the eight waves instead.
  if (N - q0 <= kShortSuffixPipe) {
    key_split_body<D, 1, WM, false>(a, b, g, h, q0, N, P, smem);
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int lq = lane & 31, hf = lane >> 5;

  const int qi = q0 + wave * 32 + lq;
  const uint16_t *qp = static_cast<const uint16_t *>(a.q) + b * a.qs[0] + int64_t(min(qi, N - 1)) * a.qs[1] + h * a.qs[2];
  bf16x8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8 *>(qp + 16 * kk + 8 * hf);

  const char *kc = reinterpret_cast<const char *>(static_cast<const uint16_t *>(a.k_cache) + b * a.cs[0] + g * a.cs[2]);
  const char *vc = reinterpret_cast<const char *>(static_cast<const uint16_t *>(a.v_cache) + b * a.cs[0] + g * a.cs[2]);
  const char *ks = reinterpret_cast<const char *>(static_cast<const uint16_t *>(a.k_suf) + b * a.ks[0] + g * a.ks[2]);
  const char *vs = reinterpret_cast<const char *>(static_cast<const uint16_t *>(a.v_suf) + b * a.ks[0] + g * a.ks[2]);
  const int64_t cpitch = a.cs[1] * 2, spitch = a.ks[1] * 2;
  // loader: this lane owns row lr of every block and 16-byte position pp of it
  const int pp = lane & 15, lr = 4 * wave + (lane >> 4);
  const int kcol = 16 * (pp ^ (lr & 15)), vcol = 64 * ((pp >> 2) ^ (lr & 3)) + 16 * (pp & 3);

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float mref = -INFINITY, lsum = 0.f;
  const float sc = a.scale * kLog2e;

  // fragment addresses inside stage 0 (as in attn_bf16_ring_kernel)
  const unsigned char *kaddr[KK], *vaddr[DB];
  {
    const int y16 = 16 * (hf ^ (lq & 15));
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kaddr[kk] = smem + lq * (D * 2) + ((32 * kk) ^ y16);
    const int s16 = lane & 15, r3 = (s16 >> 2) & 3;
    const unsigned char *vbase = smem + VBASE + (4 * hf + (s16 >> 2)) * (D * 2) + (16 * ((lane >> 4) & 1) + 4 * (s16 & 3)) * 2;
#pragma unroll
    for (int db = 0; db < DB; ++db) vaddr[db] = vbase + 64 * (db ^ r3);
  }

  // ---- ragged ends: rows [32*nc, P) of the cache and rows [32*ns, N) of the suffix ----
  const int nc = P >> 5, ns = N >> 5;
  auto ragged_block = [&](const char *kbase, const char *vbase, int64_t pitch, int cnt) {
    // this lane's row, clamped into the block; rows >= cnt are masked below and their V slots zeroed
    const int64_t off = int64_t(min(lr, cnt - 1)) * pitch;
    load_to_lds(kbase + off + kcol, smem + 1024 * wave_s);
    load_to_lds(vbase + off + vcol, smem + VBASE + 1024 * wave_s);
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
    if (lr >= cnt) *reinterpret_cast<u32x4 *>(smem + VBASE + 1024 * wave + 16 * lane) = u32x4{0, 0, 0, 0};
    __syncthreads();
    bf16x8 kf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = *reinterpret_cast<const bf16x8 *>(kaddr[kk]);
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], s, 0, 0, 0);
    bf16x8 vf[DB][2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2) vf[db][k2] = vt_read<D * 2>(vaddr[db] + (16 * k2) * (D * 2));
    softmax_pv<D>(s, oacc, mref, lsum, 0, cnt, sc, lane, vf);
    __syncthreads();  // stage 0 is free again
  };
  if (P & 31) ragged_block(kc + int64_t(32 * nc) * cpitch, vc + int64_t(32 * nc) * cpitch, cpitch, P & 31);
  if (N & 31) ragged_block(ks + int64_t(32 * ns) * spitch, vs + int64_t(32 * ns) * spitch, spitch, N & 31);

  // ---- the full blocks ----
  if (nc + ns > 0) {
    u32x16 qf_lo, qf_hi, addr;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const u32x4 lo = __builtin_bit_cast(u32x4, qf[kk]), hi = __builtin_bit_cast(u32x4, qf[kk + 4]);
      qf_lo[4 * kk] = lo.x; qf_lo[4 * kk + 1] = lo.y; qf_lo[4 * kk + 2] = lo.z; qf_lo[4 * kk + 3] = lo.w;
      qf_hi[4 * kk] = hi.x; qf_hi[4 * kk + 1] = hi.y; qf_hi[4 * kk + 2] = hi.z; qf_hi[4 * kk + 3] = hi.w;
    }
    const uint32_t lds0 = uint32_t(uintptr_t((__attribute__((address_space(3))) unsigned char *)smem));
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) addr[kk] = uint32_t(uintptr_t((__attribute__((address_space(3))) const unsigned char *)kaddr[kk]));
#pragma unroll
    for (int db = 0; db < DB; ++db) addr[8 + db] = uint32_t(uintptr_t((__attribute__((address_space(3))) const unsigned char *)vaddr[db]));
    addr[12] = uint32_t(lr * cpitch + kcol);
    addr[13] = uint32_t(lr * cpitch + vcol);
    addr[14] = uint32_t(lr * spitch + kcol);
    addr[15] = uint32_t(lr * spitch + vcol);
    const uint64_t kc_base = reinterpret_cast<uint64_t>(kc), vc_base = reinterpret_cast<uint64_t>(vc);
    const uint64_t ks_base = reinterpret_cast<uint64_t>(ks), vs_base = reinterpret_cast<uint64_t>(vs);
    const uint32_t cstep = uint32_t(32 * cpitch), sstep = uint32_t(32 * spitch);
    const uint32_t nc_u = uint32_t(nc), nb = uint32_t(nc + ns);
    const uint32_t ldsk = lds0 + 1024u * uint32_t(wave_s);
    float nm = -mref;
    if (q0 + 32 * wave_s < N) {
      const uint32_t nc = nc_u;  // (the name the generated statement uses)
#include "lsp_attn_pipe_loop.inc"
    } else {
      // none of this wave's 32 queries is active (last tile of a suffix that is not a multiple of 256
      // rows): it keeps its share of the loads and meets the others at the barriers, nothing else
      const uint32_t nc = nc_u;
#include "lsp_attn_pipe_idle_loop.inc"
    }
    mref = -nm;
  }

  lsum = half_sum(lsum);
  if (qi < N) {
    const float inv = 1.0f / lsum;
    uint16_t *op = static_cast<uint16_t *>(a.out) + b * a.os[0] + int64_t(qi) * a.os[1] + h * a.os[2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        u32x2 w;
        w.x = pack_bf16(oacc[db][4 * r4] * inv, oacc[db][4 * r4 + 1] * inv);
        w.y = pack_bf16(oacc[db][4 * r4 + 2] * inv, oacc[db][4 * r4 + 3] * inv);
        *reinterpret_cast<u32x2 *>(op + 32 * db + 8 * r4 + 4 * hf) = w;
      }
  }
}

int32_t launch_pipe(AttnArgs a, const AttnLayers &layers, hipStream_t st) {
  const int64_t nwg = place_grid(a, 256);
  if (nwg > 0x7fffffff) {
    set_error("lsp_attn_step: launch of %lld workgroups is too large", (long long)nwg);
    return LSP_ERR_UNSUPPORTED;
  }
  const size_t lds_ring = size_t(8) * 2 * 32 * 256;
  const size_t lds_split = 8 * size_t(Geo<128>::WAVE_LDS) + 32 * size_t(Geo<128>::KPITCH);
  const size_t lds = lds_ring > lds_split ? lds_ring : lds_split;
  auto kern = attn_bf16_pipe_kernel;
  static std::atomic<uint64_t> configured{0};
  if (const int32_t rc = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, configured, "lsp_attn_step: hipFuncSetAttribute")) return rc;
  kern<<<dim3(static_cast<unsigned>(nwg), layers.n > 0 ? layers.n : 1, 1), 512, lds, st>>>(a, layers);
  LSP_CHECK_LAUNCH("lsp_attn_step: bf16 pipelined launch");
  return LSP_OK;
}

// contiguous cache, or rows through an index (Scattered-Margin measurement)
template <int D, int WM, int WK>
int32_t launch(const AttnArgs &a, const AttnLayers &layers, hipStream_t st) {
  return a.cache_rows ? launch_g<D, WM, WK, true>(a, layers, st) : launch_g<D, WM, WK, false>(a, layers, st);
}
template <int D, int WM, int OCC, int PD>
int32_t launch_tile(const AttnArgs &a, const AttnLayers &layers, hipStream_t st) {
  return a.cache_rows ? launch_tile_g<D, WM, OCC, PD, true>(a, layers, st) : launch_tile_g<D, WM, OCC, PD, false>(a, layers, st);
}

template <int D>
int32_t dispatch(const AttnArgs &a, const AttnLayers &layers, hipStream_t st) {
  // Enough (sequence, head, row) triples to give every compute unit several
  // query tiles: the shared-tile kernel, with the widest tile the suffix fills.
  // Otherwise the wave-private kernel with the key range split between waves.
  // upper bound on (b,h,row) triples of the launch
  const int64_t rows = int64_t(a.B) * a.Hq * a.S * (layers.n > 0 ? layers.n : 1);
  if (rows / 128 >= 256) {
    if constexpr (D == 128) {
      // suffix buffers of more than 128 rows: the hand-scheduled loop (its loads keep a row's byte offset inside
      // a 32-row block in 32 bits, which the row-stride limit of the entry point guarantees); an indexed cache
      // keeps the compiler-scheduled ring kernel
      if (a.S > 128) return a.cache_rows ? launch_ring_g<8, 4, true>(a, layers, st) : launch_pipe(a, layers, st);
    }
    return launch_tile<D, 4, 2, 4>(a, layers, st);
  }
  if (rows / 64 >= 512) return launch<D, 2, 2>(a, layers, st);
  if (rows / 32 >= 512) return launch<D, 1, 4>(a, layers, st);
  return launch<D, 1, 8>(a, layers, st);
}

}  // namespace

size_t attn_bf16_workspace_bytes(int32_t, int32_t, int32_t, int32_t) { return 0; }

int32_t launch_attn_bf16(const AttnArgs &a, const AttnLayers &layers, hipStream_t st) {
  if (a.D == 128) return dispatch<128>(a, layers, st);
  if (a.D == 64) return dispatch<64>(a, layers, st);
  set_error("lsp_attn_step: bf16 head_dim %d not built (64, 128)", a.D);
  return LSP_ERR_UNSUPPORTED;
}

}  // namespace lsp
