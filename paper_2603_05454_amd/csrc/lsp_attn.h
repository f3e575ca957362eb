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
};

int32_t launch_attn_f32(const AttnArgs &a, hipStream_t st);
int32_t launch_attn_bf16(const AttnArgs &a, hipStream_t st);
size_t attn_bf16_workspace_bytes(int32_t B, int32_t S, int32_t Hq, int32_t D);

}  // namespace lsp
