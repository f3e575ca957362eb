// Internal: resolved arguments shared by the attention kernels.
#pragma once
#include "lsp_common.h"

namespace lsp {

struct AttnArgs {
  const void *q, *k_suf, *v_suf, *k_cache, *v_cache;
  void *out;
  const int32_t *prefix_len, *suffix_len;
  int32_t B, S, Hq, Hkv, D, C;
  float scale;
  int64_t qs[3], ks[3], cs[3], os[3];  // element strides: batch, row, head
  void *workspace;
  int32_t unit_group;  // set by the bf16 launcher: units per placement group
  const int32_t *cache_rows;  // gather form only: key t < P_b of sequence b is cache row cache_rows[b*C + t]; else null
};

// Operands of several layers for ONE launch (lsp_attn_step_layers): passed to the
// kernels by value, the layer is the slow grid index.  n = 0: single-layer call,
// the pointers in AttnArgs are used as they are.
constexpr int kMaxAttnLayers = 32;
struct AttnLayers {
  int32_t n;
  const void *q[kMaxAttnLayers], *k_suf[kMaxAttnLayers], *v_suf[kMaxAttnLayers];
  const void *k_cache[kMaxAttnLayers], *v_cache[kMaxAttnLayers];
  void *out[kMaxAttnLayers];
};
// This workgroup's layer (grid index y) replaces the operand pointers.
__device__ __forceinline__ AttnArgs for_layer(const AttnArgs &in, const AttnLayers &L) {
  AttnArgs a = in;
  if (L.n > 0) {
    const int l = blockIdx.y;
    a.q = L.q[l]; a.k_suf = L.k_suf[l]; a.v_suf = L.v_suf[l];
    a.k_cache = L.k_cache[l]; a.v_cache = L.v_cache[l]; a.out = L.out[l];
  }
  return a;
}

// Cache row that holds key t (t < P_b) of sequence b.
template <bool GATHER>
__device__ __forceinline__ int cache_row(const AttnArgs &a, int b, int t) {
  if (!GATHER) return t;
  const int r = a.cache_rows[int64_t(b) * a.C + t];
  return min(max(r, 0), a.C - 1);  // a bad index must not leave the buffer
}

int32_t launch_attn_f32(const AttnArgs &a, hipStream_t st);
int32_t launch_attn_bf16(const AttnArgs &a, const AttnLayers &layers, hipStream_t st);
size_t attn_bf16_workspace_bytes(int32_t B, int32_t S, int32_t Hq, int32_t D);

}  // namespace lsp
