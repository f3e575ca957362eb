/*
 * liblsp - per-denoising-step hot path of the Longest Stable Prefix (LSP)
 * scheduler for diffusion language models, for AMD MI355X (gfx950).
 *
 * One scheduler iteration (Algorithm 1, lines 4-10 of the paper) is three
 * calls:
 *   lsp_attn_step   attention of the active-suffix queries over
 *                   [committed-prefix KV cache || suffix K/V]   (line 4)
 *   lsp_confidence  top-1 id, logit margin (Eq. 1) and top-1 probability of
 *                   every active position                       (line 5)
 *   lsp_commit      stability mask, longest stable prefix L'(tau), snap to the
 *                   last delimiter, fallback, commit and contiguous KV append
 *                                                               (lines 7-10)
 *
 * Conventions
 *  - Plain C ABI.  Every pointer documented as "device" is GPU memory owned by
 *    the caller; the library never allocates, frees or keeps it.  Pointers
 *    documented as "host" are read during the call only.
 *  - Every call validates its arguments on the host first; on an error nothing
 *    is launched.  Work is enqueued on `stream` (a hipStream_t passed as
 *    void*, NULL = the default stream) and the call returns without
 *    synchronising: outputs are valid in stream order.
 *  - Sequence state lives on the device: prefix_len[b] (rows of sequence b in
 *    the cache, P_b) and suffix_len[b] (active positions, N_b).  No call reads
 *    them on the host, so a step needs no device-to-host transfer.
 *  - Element types: LSP_F32 (IEEE binary32) and LSP_BF16 (bfloat16).
 *  - Dense layouts, innermost dimension contiguous:
 *      suffix Q / O     [B, S, Hq,  D]
 *      suffix K / V     [B, S, Hkv, D]      row u = u-th active position
 *      cache  K / V     [B, C, Hkv, D]      per layer, token-major, so the rows
 *                                           committed in one step form ONE
 *                                           contiguous block per sequence
 *      logits           [B, S, V]
 *    Strides (in elements) may be given for the outer dimensions.
 *  - Return value: LSP_OK or a negative lsp_status; lsp_last_error() gives a
 *    text for the calling thread's last failure.
 */
#ifndef LSP_H
#define LSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { LSP_F32 = 0, LSP_BF16 = 1 } lsp_dtype;

typedef enum {
  LSP_OK = 0,
  LSP_ERR_INVALID_ARG = -1, /* null pointer, bad dimension, misaligned pointer or stride */
  LSP_ERR_UNSUPPORTED = -2, /* dtype / head_dim combination that is not built */
  LSP_ERR_WORKSPACE = -3,   /* workspace missing or smaller than lsp_*_workspace_bytes */
  LSP_ERR_HIP = -4          /* the HIP runtime refused a launch */
} lsp_status;

/* Bits of status_flags[b] written by lsp_commit. */
#define LSP_FLAG_CACHE_FULL 1  /* commit length was cut to the cache room C - P_b */
#define LSP_FLAG_TOKENS_FULL 2 /* commit length was cut to the token buffer room T - P_b */
#define LSP_FLAG_NO_THRESHOLD 4 /* adaptive sizing: no threshold puts L' in [alpha N, beta N]; the nearer bound was used */

const char *lsp_version(void);
const char *lsp_last_error(void);

/* ------------------------------------------------------------------------- *
 * Suffix attention (Algorithm 1 line 4; Section 3.2 "bidirectional lookahead"
 * and "approximate KV caching for prefix states").
 *
 * For every sequence b, query head h and active row i < N_b:
 *     O[b,i,h,:] = softmax_t( scale * Q[b,i,h,:] . K*[t,g,:] ) . V*[t,g,:]
 * where t runs over the P_b cached rows and then the N_b suffix rows, no mask
 * of any kind, and g = h / (Hq/Hkv).  Rows i >= N_b of O are not written.
 * Sequences with N_b = 0 cost nothing.
 * ------------------------------------------------------------------------- */
typedef struct {
  int32_t dtype;          /* lsp_dtype of Q, K, V and O */
  int32_t B, S, Hq, Hkv;  /* S = rows of the suffix buffers */
  int32_t D;              /* head dim: 64 or 128 */
  int32_t C;              /* cache capacity in rows */
  float scale;            /* soft-max scale; 0 selects 1/sqrt(D) */
  /* element strides of (batch, row, head); all three 0 selects the dense default */
  int64_t q_stride[3];
  int64_t kv_suf_stride[3];
  int64_t cache_stride[3];
  int64_t o_stride[3];
} lsp_attn_desc;

size_t lsp_attn_workspace_bytes(const lsp_attn_desc *desc);

/*
 * q, k_suf, v_suf, k_cache, v_cache, out: device, 16-byte aligned, strides
 * multiples of 16 bytes; the row strides of the K/V buffers (suffix and cache)
 * at most 2^24 elements.  prefix_len, suffix_len: device int32[B], with
 * 0 <= P_b <= C and 0 <= N_b <= S (not checked on the host; values are
 * clamped to those ranges on the device).  workspace: device, at least
 * lsp_attn_workspace_bytes(desc) bytes, 256-byte aligned (may be NULL when
 * that size is 0).
 */
int32_t lsp_attn_step(const lsp_attn_desc *desc, const void *q, const void *k_suf,
                      const void *v_suf, const void *k_cache, const void *v_cache,
                      const int32_t *prefix_len, const int32_t *suffix_len, void *out,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * lsp_attn_step for every layer of the denoiser call in ONE launch (Algorithm 1
 * line 4 runs the attention once per layer inside each iteration of the line-3
 * loop; late in the loop, when few positions are active, a launch per layer
 * costs more than the work).  q_layers, k_suf_layers, v_suf_layers,
 * k_cache_layers, v_cache_layers, out_layers: HOST arrays of num_layers DEVICE
 * pointers (read during the call), each operand as for lsp_attn_step; all
 * layers share the descriptor (shapes, strides) and the length arrays.  Layers
 * are independent: out_layers[l] depends on layer l's operands only.  More than
 * 32 layers are issued as several launches of 32; fp32 operands as one launch
 * per layer.
 */
int32_t lsp_attn_step_layers(const lsp_attn_desc *desc, int32_t num_layers, const void *const *q_layers,
                             const void *const *k_suf_layers, const void *const *v_suf_layers,
                             const void *const *k_cache_layers, const void *const *v_cache_layers,
                             const int32_t *prefix_len, const int32_t *suffix_len,
                             void *const *out_layers, void *workspace, size_t workspace_bytes,
                             void *stream);

/* ------------------------------------------------------------------------- *
 * Per-position confidence (Eq. 1; Algorithm 1 line 5).
 *
 * For every sequence b and active row i < N_b, over the row z = logits[b,i,:]:
 *     top1_id  = the lowest index attaining max_v z[v]
 *     margin   = z_(1) - z_(2), one fp32 subtraction, where z_(2) is the
 *                largest entry other than top1_id (so 0 on a tied maximum)
 *     top1_prob= 1 / sum_v exp(z[v] - z_(1))        (fp32 accumulation)
 * Rows i >= N_b are neither read nor written.  Precondition: the row maximum
 * is finite and the row holds no NaN (-inf entries are fine).
 * ------------------------------------------------------------------------- */
size_t lsp_confidence_workspace_bytes(int32_t B, int32_t S, int32_t V);

/*
 * logits: device, element type `dtype`; row (b,i) starts at element
 * b*batch_stride + i*row_stride (0 selects the dense S*V / V).  Any alignment
 * of at least the element size is accepted; 16-byte aligned rows take the fast
 * path.  suffix_len: device int32[B] or NULL (= all S rows active).
 * top1_id (int32), top1_prob (fp32), margin (fp32): device, [B,S] dense.
 */
int32_t lsp_confidence(int32_t dtype, const void *logits, int32_t B, int32_t S, int32_t V,
                       int64_t row_stride, int64_t batch_stride, const int32_t *suffix_len,
                       int32_t *top1_id, float *top1_prob, float *margin,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * lsp_confidence for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and launches as lsp_confidence,
 * but the per-segment results of split rows (the only scratch that call needs:
 * rows are split when B*S < 128) go to a buffer of
 * lsp_confidence_static_scratch_bytes() = 65536 bytes that is part of the
 * library's device image; each GPU the library runs on holds its own copy until
 * the process ends.  The call allocates and frees nothing (its first use on a
 * GPU looks up the buffer's address).  A shape whose launch plan needs more
 * than the buffer holds returns LSP_ERR_UNSUPPORTED and launches nothing.
 * Every call on one GPU shares that GPU's buffer: calls whose execution may
 * overlap on one GPU (different streams, or several host threads) race; calls
 * in stream order on one stream do not.  Nothing has to be cleared between
 * calls (every value read was written by the same call).
 */
size_t lsp_confidence_static_scratch_bytes(void);
int32_t lsp_confidence_static(int32_t dtype, const void *logits, int32_t B, int32_t S, int32_t V,
                              int64_t row_stride, int64_t batch_stride, const int32_t *suffix_len,
                              int32_t *top1_id, float *top1_prob, float *margin, void *stream);

/* ------------------------------------------------------------------------- *
 * Boundary search, snap, commit and append (Section 3.2: L'(tau), the snap
 * equation and the monotone-progress fallback; Algorithm 1 lines 7-10).
 *
 * Per sequence b, with N = N_b and P = P_b on entry:
 *   stable_mask[b,i] = (i < N and margin[b,i] > tau)           (strict)
 *   raw_boundary[b]  = L' = first i with stable_mask = 0, else N; with
 *                      adaptive = 1 the threshold is chosen per sequence instead
 *                      (Section 3.2 "targeted block sizing", Eq. 2; Algorithm 1
 *                      line 6): with lo = ceil(alpha N), hi = max(lo, floor(beta N))
 *                      (one fp32 multiplication each) and L0 the length tau
 *                      gives, L' = L0 if lo <= L0 <= hi; otherwise the smallest
 *                      (L0 < lo) or largest (L0 > hi) length in [lo, hi] that
 *                      SOME threshold produces - a length a < N is produced by
 *                      a threshold exactly when margin[a] is below the minimum
 *                      of margin[0..a-1], a = N always - and if there is none,
 *                      lo resp. hi with LSP_FLAG_NO_THRESHOLD set.  tau_used[b]
 *                      = tau, margin[a] (-inf for a = N) or NaN in these cases.
 *                      stable_mask stays relative to tau.
 *   snapped_boundary = the largest length j in [1, L'] with L' - j <= window
 *                      whose last token top1_id[b,j-1] is in the delimiter
 *                      set; L' when there is none, when snap_enabled = 0 or
 *                      when L' = 0.  window < 0 = no limit.
 *   commit_len[b]    = L = min(N, max(snapped_boundary, min_commit)), cut to
 *                      max_commit when that is > 0 (the fixed-prefix variant of
 *                      the sizing ablation, Table 2), then to the cache room
 *                      C - P and the token room T - P (a cut to room sets the
 *                      matching LSP_FLAG_* bit in status_flags[b]).
 *   tokens[b, P..P+L) = top1_id[b, 0..L)
 *   for every layer: cache rows [P, P+L) = suffix rows [0, L), K and V - one
 *                      contiguous block of L*Hkv*D elements each
 *   prefix_len[b] = P + L ; suffix_len[b] = N - L
 * ------------------------------------------------------------------------- */
typedef struct {
  int32_t kv_dtype;       /* lsp_dtype of the K/V buffers */
  int32_t B, S, V;
  int32_t Hkv, D, C;      /* K/V row = Hkv*D contiguous elements; its byte size must be a multiple of 16 */
  int32_t num_layers;     /* 0 = boundary search and token commit only */
  int32_t T;              /* length of one sequence's token buffer */
  float tau;              /* margin threshold, logit units; +-inf allowed */
  int32_t window;         /* W */
  int32_t min_commit;     /* L_min >= 0 */
  int32_t snap_enabled;
  int64_t suf_batch_stride;   /* elements between sequences in a suffix K/V buffer; 0 = S*Hkv*D */
  int64_t cache_batch_stride; /* elements between sequences in a cache; 0 = C*Hkv*D */
  int32_t adaptive;       /* 1 = choose the threshold per sequence (Eq. 2) */
  float alpha, beta;      /* acceptance interval, 0 < alpha <= beta <= 1 (read when adaptive) */
  int32_t max_commit;     /* > 0: upper bound of the commit length; 0 = none */
} lsp_commit_desc;

size_t lsp_commit_workspace_bytes(const lsp_commit_desc *desc);

/*
 * margin (fp32), top1_id (int32): device [B,S], as written by lsp_confidence.
 * delimiter_bitmap: device uint32[ceil(V/32)], bit (v%32) of word v/32 set
 * when id v is a delimiter.  Ids outside [0,V) are treated as non-delimiters.
 * k_suf_layers, v_suf_layers, k_cache_layers, v_cache_layers: HOST arrays of
 * num_layers DEVICE pointers (read during the call; may all be NULL when
 * num_layers = 0).  Buffers 16-byte aligned; a cache must not overlap the
 * suffix buffers.
 * tokens: device int32 [B,T] in/out, or NULL.  prefix_len, suffix_len: device
 * int32[B] in/out.  stable_mask: device uint8 [B,S].  raw_boundary,
 * snapped_boundary, commit_len, status_flags: device int32[B] out
 * (status_flags may be NULL).  tau_used: device fp32[B] out, or NULL.
 * Limits: B <= 65535, S <= 65536.
 */
int32_t lsp_commit(const lsp_commit_desc *desc, const float *margin, const int32_t *top1_id,
                   const uint32_t *delimiter_bitmap,
                   const void *const *k_suf_layers, const void *const *v_suf_layers,
                   void *const *k_cache_layers, void *const *v_cache_layers,
                   int32_t *tokens, int32_t *prefix_len, int32_t *suffix_len,
                   uint8_t *stable_mask, int32_t *raw_boundary, int32_t *snapped_boundary,
                   int32_t *commit_len, int32_t *status_flags, float *tau_used,
                   void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------- *
 * Scattered-Margin baseline (Section 4.3.3: LSP's block size, but the most
 * confident positions from anywhere in the active sequence) - the pieces
 * needed to MEASURE what the prefix-first topology saves.
 * ------------------------------------------------------------------------- */

/*
 * Per sequence b: the k = min(count[b], N_b) active positions with the largest
 * margins; equal margins are taken in position order.  sel_index[b, 0..k)
 * lists them ascending, the rest of the row is -1; sel_mask[b, i] = 1 for a
 * selected position (0 elsewhere, inactive positions included).
 * margin: device fp32 [B,S]; suffix_len, count: device int32[B]; sel_index:
 * device int32 [B,S]; sel_mask: device uint8 [B,S].  S <= 8192.
 */
int32_t lsp_select_scattered(const float *margin, int32_t B, int32_t S, const int32_t *suffix_len,
                             const int32_t *count, int32_t *sel_index, uint8_t *sel_mask,
                             void *stream);

/*
 * Gathered append: for every layer, cache rows [P_b, P_b + k_b) receive the
 * suffix rows sel_index[b, 0..k_b) in that order (K and V), with k_b = count[b]
 * cut to the cache room C - P_b and to the length of the list, which ends at
 * its first negative entry (lsp_select_scattered pads with -1 when fewer than
 * count[b] positions are active: no more positions can be committed than
 * exist); then appended[b] = k_b (device int32[B], required) and
 * prefix_len[b] += k_b.  suffix_len is not touched: after a scattered commit
 * the remaining positions are no longer a suffix.  Layouts, alignment and the
 * HOST pointer tables as for lsp_commit; strides in elements, 0 = dense.
 * Indices above S-1 are clamped into the buffer.
 */
int32_t lsp_kv_gather_append(int32_t kv_dtype, int32_t B, int32_t S, int32_t Hkv, int32_t D, int32_t C,
                             int32_t num_layers, int64_t suf_batch_stride, int64_t cache_batch_stride,
                             const int32_t *sel_index, const int32_t *count,
                             const void *const *k_suf_layers, const void *const *v_suf_layers,
                             void *const *k_cache_layers, void *const *v_cache_layers,
                             int32_t *prefix_len, int32_t *appended, void *stream);

/*
 * lsp_attn_step over a cache that is addressed through a row index, as a cache
 * fragmented by scattered commits is: key t < P_b of sequence b is cache row
 * cache_row_index[b*C + t] (device int32 [B,C]; values outside [0,C) are
 * clamped into the buffer).  Everything else as lsp_attn_step.
 */
int32_t lsp_attn_step_gather(const lsp_attn_desc *desc, const void *q, const void *k_suf,
                             const void *v_suf, const void *k_cache, const void *v_cache,
                             const int32_t *cache_row_index, const int32_t *prefix_len,
                             const int32_t *suffix_len, void *out, void *workspace,
                             size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------- *
 * Output head fused with the per-position confidence (Algorithm 1 lines 4-5:
 * the last projection of the denoiser call p_theta, then Eq. 1).
 *
 * For every sequence b and active row i < N_b the logits
 *     z[v] = sum_k hidden[b,i,k] * weight[v,k]       (bf16 operands, fp32 sums)
 * are produced tile by tile on the matrix cores and reduced at once to
 * top1_id / margin / top1_prob, defined exactly as for lsp_confidence on z; z
 * itself is never written to memory and is NOT rounded to bf16, so margins and
 * probabilities differ from "GEMM, store bf16 logits, lsp_confidence" by that
 * rounding.  Summation order is the kernel's: results match an exact
 * evaluation to fp32 accumulation error (about 1e-6 * sum_k |h_k w_k|), and the
 * id is the exact arg-max wherever the exact margin exceeds that error.
 * Rows i >= N_b are not written.
 * ------------------------------------------------------------------------- */
size_t lsp_lm_head_confidence_workspace_bytes(int32_t B, int32_t S, int32_t V);

/*
 * dtype: LSP_BF16 only (LSP_ERR_UNSUPPORTED otherwise).  hidden: device, row
 * (b,i) = K elements at b*hidden_batch_stride + i*hidden_row_stride (0 selects
 * dense S*K / K).  weight: device, vocabulary entry v = K elements at
 * v*weight_row_stride (0 = K) - the usual [V, K] layout of an output
 * embedding.  K a multiple of 8; pointers 16-byte aligned and strides multiples
 * of 8 elements.  suffix_len: device int32[B] or NULL (= all S rows active).
 * top1_id (int32), top1_prob (fp32), margin (fp32): device, [B,S] dense.
 * workspace: device, 16-byte aligned, at least
 * lsp_lm_head_confidence_workspace_bytes(B,S,V) bytes (per row and 256-entry
 * vocabulary tile one 16-byte partial result).
 */
int32_t lsp_lm_head_confidence(int32_t dtype, const void *hidden, const void *weight, int32_t B,
                               int32_t S, int32_t K, int32_t V, int64_t hidden_row_stride,
                               int64_t hidden_batch_stride, int64_t weight_row_stride,
                               const int32_t *suffix_len, int32_t *top1_id, float *top1_prob,
                               float *margin, void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------- *
 * Flip bookkeeping for a decode loop (Section 4.3.4: share of active-suffix
 * positions whose top-1 prediction changes between consecutive steps).
 *
 * Call once per step after lsp_confidence and BEFORE lsp_commit.  last_id
 * [B,G] holds, per generation position (0 = first generated token), the top-1
 * id it had at the previous step, or -1.  With done_b = prefix_len[b] -
 * base_prefix_len[b], for u < N_b: position j = done_b + u; if last_id[b,j] >=
 * 0 the position is compared (it counts as a flip when last_id[b,j] !=
 * top1_id[b,u]); then last_id[b,j] = top1_id[b,u].
 * counters: device int64[4], accumulated: [0] flips, [1] positions compared,
 * [2] and [3] the same restricted to sequences with window_lo <= done_b <=
 * window_hi (the paper quotes the rate for the mid-stage of generation, 25-75 %
 * complete; pass window_lo > window_hi for no window).
 * step_counts: device int32 [B,2] or NULL; when given, this call's flips and
 * compared positions of every sequence are WRITTEN there (a per-step trace).
 * ------------------------------------------------------------------------- */
int32_t lsp_flip_update(const int32_t *top1_id, int32_t B, int32_t S, int32_t G,
                        const int32_t *prefix_len, const int32_t *suffix_len,
                        const int32_t *base_prefix_len, int32_t *last_id,
                        int64_t *counters, int32_t window_lo, int32_t window_hi,
                        int32_t *step_counts, void *stream);

/* ------------------------------------------------------------------------- *
 * Measurement helper (used by the benchmark, not part of the scheduler step):
 * a bare streaming read of `bytes` bytes of device memory by `workgroups`
 * workgroups of 512 threads (16-byte non-temporal loads, each workgroup one
 * contiguous segment; bytes must be a multiple of 16 * workgroups), XOR-folded
 * into out[workgroups] (device uint32, accumulated).  What it takes is the
 * floor under lsp_confidence for logits of that size: the one pass over the
 * logits that Eq. 1 needs, with nothing computed.
 * ------------------------------------------------------------------------- */
int32_t lsp_bench_read(const void *buffer, int64_t bytes, int32_t workgroups, uint32_t *out, void *stream);

/* ------------------------------------------------------------------------- *
 * Measurement helper (used by the benchmark, not part of the scheduler step):
 * a bare loop of v_mfma_f32_32x32x16_bf16 with no memory traffic inside it,
 * `workgroups` workgroups of 512 threads (two waves per SIMD), `iters`
 * iterations of 8 matrix instructions per wave = workgroups * 8 * iters * 8 *
 * 32768 flop per launch.  operands: device buffer of 16 * 512 * 16 bytes (per
 * lane 8 A and 8 B fragments of 8 bf16, fragment s of lane t at 16-byte vector
 * s * 512 + t, B fragments after the A fragments), read once per lane.
 * out: device float [workgroups * 512], overwritten (keeps the loop alive).
 * The rate it sustains depends on the operand VALUES (the chip lowers its
 * clock under the power that random operands draw), which makes it the
 * matrix-pipe ceiling for the attention of Algorithm 1 line 4 on such data.
 * ------------------------------------------------------------------------- */
int32_t lsp_bench_mfma(const void *operands, int32_t iters, int32_t workgroups, float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LSP_H */
