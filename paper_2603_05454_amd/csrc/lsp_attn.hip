// lsp_attn_step: argument checking and dispatch (see include/lsp.h).
#include <math.h>

#include "lsp_attn.h"

namespace lsp {
namespace {

constexpr int64_t kMaxRowStride = int64_t(1) << 24;

bool resolve(const int64_t in[3], int64_t out[3], int64_t rows, int64_t heads, int64_t D) {
  if (in[0] == 0 && in[1] == 0 && in[2] == 0) {
    out[2] = D;
    out[1] = heads * D;
    out[0] = rows * heads * D;
    return true;
  }
  for (int k = 0; k < 3; ++k) out[k] = in[k];
  return in[2] >= D && in[1] > 0 && in[0] >= 0;
}

int32_t check(const lsp_attn_desc *d, AttnArgs &a) {
  LSP_CHECK_ARG(d != nullptr, "lsp_attn: null descriptor");
  LSP_CHECK_ARG(d->dtype == LSP_F32 || d->dtype == LSP_BF16, "lsp_attn: unknown dtype %d", d->dtype);
  LSP_CHECK_ARG(d->B > 0 && d->S > 0 && d->Hq > 0 && d->Hkv > 0 && d->D > 0 && d->C > 0,
                "lsp_attn: non-positive dimension");
  LSP_CHECK_ARG(d->Hq % d->Hkv == 0, "lsp_attn: Hq=%d is not a multiple of Hkv=%d", d->Hq, d->Hkv);
  LSP_CHECK_ARG(d->B <= 65535 && d->Hq <= 65535, "lsp_attn: B and Hq must be <= 65535");
  LSP_CHECK_ARG(d->scale >= 0.f && isfinite(d->scale), "lsp_attn: bad scale");
  a.B = d->B; a.S = d->S; a.Hq = d->Hq; a.Hkv = d->Hkv; a.D = d->D; a.C = d->C;
  a.scale = d->scale > 0.f ? d->scale : 1.0f / sqrtf(float(d->D));
  LSP_CHECK_ARG(resolve(d->q_stride, a.qs, d->S, d->Hq, d->D) &&
                    resolve(d->kv_suf_stride, a.ks, d->S, d->Hkv, d->D) &&
                    resolve(d->cache_stride, a.cs, d->C, d->Hkv, d->D) &&
                    resolve(d->o_stride, a.os, d->S, d->Hq, d->D),
                "lsp_attn: bad strides");
  // the kernels keep byte offsets of up to 32 rows of a K/V block in 32 bits
  LSP_CHECK_ARG(a.ks[1] <= kMaxRowStride && a.cs[1] <= kMaxRowStride,
                "lsp_attn: K/V row strides above %lld elements are not supported", (long long)kMaxRowStride);
  const int64_t per16 = 16 / int64_t(elem_size(d->dtype));
  for (int k = 0; k < 3; ++k)
    LSP_CHECK_ARG(a.qs[k] % per16 == 0 && a.ks[k] % per16 == 0 && a.cs[k] % per16 == 0 && a.os[k] % per16 == 0,
                  "lsp_attn: strides must be multiples of 16 bytes");
  return LSP_OK;
}

}  // namespace
}  // namespace lsp

extern "C" size_t lsp_attn_workspace_bytes(const lsp_attn_desc *d) {
  if (d == nullptr || d->dtype != LSP_BF16) return 0;
  return lsp::attn_bf16_workspace_bytes(d->B, d->S, d->Hq, d->D);
}

namespace lsp {
namespace {
int32_t attn_entry(const lsp_attn_desc *d, const void *q, const void *k_suf, const void *v_suf,
                   const void *k_cache, const void *v_cache, const int32_t *cache_rows,
                   const int32_t *prefix_len, const int32_t *suffix_len, void *out, void *workspace,
                   size_t workspace_bytes, void *stream) {
  AttnArgs a;
  const int32_t rc = check(d, a);
  if (rc != LSP_OK) return rc;
  LSP_CHECK_ARG(q && k_suf && v_suf && k_cache && v_cache && prefix_len && suffix_len && out,
                "lsp_attn_step: null pointer");
  LSP_CHECK_ARG(aligned16(q) && aligned16(k_suf) && aligned16(v_suf) && aligned16(k_cache) &&
                    aligned16(v_cache) && aligned16(out),
                "lsp_attn_step: pointers must be 16-byte aligned");
  const size_t need = lsp_attn_workspace_bytes(d);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need ||
                   (reinterpret_cast<uintptr_t>(workspace) & 255u))) {
    set_error("lsp_attn_step: workspace of %zu bytes (256-byte aligned) required, got %zu", need, workspace_bytes);
    return LSP_ERR_WORKSPACE;
  }
  a.q = q; a.k_suf = k_suf; a.v_suf = v_suf; a.k_cache = k_cache; a.v_cache = v_cache; a.out = out;
  a.prefix_len = prefix_len; a.suffix_len = suffix_len; a.workspace = workspace;
  a.cache_rows = cache_rows;
  a.unit_group = 1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  AttnLayers none;
  none.n = 0;
  return d->dtype == LSP_F32 ? launch_attn_f32(a, st) : launch_attn_bf16(a, none, st);
}
}  // namespace
}  // namespace lsp

extern "C" int32_t lsp_attn_step_layers(const lsp_attn_desc *d, int32_t num_layers, const void *const *q_layers,
                                        const void *const *k_suf_layers, const void *const *v_suf_layers,
                                        const void *const *k_cache_layers, const void *const *v_cache_layers,
                                        const int32_t *prefix_len, const int32_t *suffix_len,
                                        void *const *out_layers, void *workspace, size_t workspace_bytes,
                                        void *stream) {
  using namespace lsp;
  AttnArgs a;
  const int32_t rc = check(d, a);
  if (rc != LSP_OK) return rc;
  LSP_CHECK_ARG(num_layers > 0, "lsp_attn_step_layers: num_layers must be positive");
  LSP_CHECK_ARG(q_layers && k_suf_layers && v_suf_layers && k_cache_layers && v_cache_layers && out_layers &&
                    prefix_len && suffix_len,
                "lsp_attn_step_layers: null pointer");
  for (int l = 0; l < num_layers; ++l) {
    LSP_CHECK_ARG(q_layers[l] && k_suf_layers[l] && v_suf_layers[l] && k_cache_layers[l] && v_cache_layers[l] && out_layers[l],
                  "lsp_attn_step_layers: null operand in layer %d", l);
    LSP_CHECK_ARG(aligned16(q_layers[l]) && aligned16(k_suf_layers[l]) && aligned16(v_suf_layers[l]) &&
                      aligned16(k_cache_layers[l]) && aligned16(v_cache_layers[l]) && aligned16(out_layers[l]),
                  "lsp_attn_step_layers: operands of layer %d must be 16-byte aligned", l);
  }
  const size_t need = lsp_attn_workspace_bytes(d);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))) {
    set_error("lsp_attn_step_layers: workspace of %zu bytes (256-byte aligned) required, got %zu", need, workspace_bytes);
    return LSP_ERR_WORKSPACE;
  }
  a.prefix_len = prefix_len; a.suffix_len = suffix_len; a.workspace = workspace;
  a.cache_rows = nullptr;
  a.unit_group = 1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int l0 = 0; l0 < num_layers; l0 += kMaxAttnLayers) {
    const int nl = num_layers - l0 < kMaxAttnLayers ? num_layers - l0 : kMaxAttnLayers;
    if (d->dtype == LSP_F32) {  // the fp32 kernel is a precision path: one launch per layer
      for (int l = l0; l < l0 + nl; ++l) {
        a.q = q_layers[l]; a.k_suf = k_suf_layers[l]; a.v_suf = v_suf_layers[l];
        a.k_cache = k_cache_layers[l]; a.v_cache = v_cache_layers[l]; a.out = out_layers[l];
        const int32_t r = launch_attn_f32(a, st);
        if (r != LSP_OK) return r;
      }
      continue;
    }
    AttnLayers L;
    L.n = nl;
    for (int l = 0; l < kMaxAttnLayers; ++l) {
      const int s = l < nl ? l0 + l : l0;  // unused slots repeat a valid layer
      L.q[l] = q_layers[s]; L.k_suf[l] = k_suf_layers[s]; L.v_suf[l] = v_suf_layers[s];
      L.k_cache[l] = k_cache_layers[s]; L.v_cache[l] = v_cache_layers[s]; L.out[l] = out_layers[s];
    }
    a.q = L.q[0]; a.k_suf = L.k_suf[0]; a.v_suf = L.v_suf[0];
    a.k_cache = L.k_cache[0]; a.v_cache = L.v_cache[0]; a.out = L.out[0];
    const int32_t r = launch_attn_bf16(a, L, st);
    if (r != LSP_OK) return r;
  }
  return LSP_OK;
}

extern "C" int32_t lsp_attn_step(const lsp_attn_desc *d, const void *q, const void *k_suf,
                                 const void *v_suf, const void *k_cache, const void *v_cache,
                                 const int32_t *prefix_len, const int32_t *suffix_len, void *out,
                                 void *workspace, size_t workspace_bytes, void *stream) {
  return lsp::attn_entry(d, q, k_suf, v_suf, k_cache, v_cache, nullptr, prefix_len, suffix_len, out,
                         workspace, workspace_bytes, stream);
}

extern "C" int32_t lsp_attn_step_gather(const lsp_attn_desc *d, const void *q, const void *k_suf,
                                        const void *v_suf, const void *k_cache, const void *v_cache,
                                        const int32_t *cache_row_index, const int32_t *prefix_len,
                                        const int32_t *suffix_len, void *out, void *workspace,
                                        size_t workspace_bytes, void *stream) {
  LSP_CHECK_ARG(cache_row_index != nullptr, "lsp_attn_step_gather: null row index");
  return lsp::attn_entry(d, q, k_suf, v_suf, k_cache, v_cache, cache_row_index, prefix_len, suffix_len,
                         out, workspace, workspace_bytes, stream);
}
