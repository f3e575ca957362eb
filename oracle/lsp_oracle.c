/*
 * CPU oracle for the per-step hot path of the Longest Stable Prefix (LSP)
 * scheduler.  TEST INFRASTRUCTURE ONLY: it is called by the tests, by the
 * smoke check and by the benchmark's cpu_baseline leg, never by the product
 * path, and it shares no code with the HIP library.
 *
 * Every routine is the plain definition written out: straight loops, double
 * precision for floating point (single precision only where one IEEE
 * subtraction is the definition), no blocking, no fusion.  OpenMP only
 * spreads independent output rows over cores.
 *
 *   oracle_attention*  - the attention inside the denoiser call of
 *                        Algorithm 1 line 4: active-suffix queries attend,
 *                        without any mask (Section 3.2, bidirectional
 *                        lookahead), to the cached prefix K/V followed by the
 *                        suffix's own K/V (Section 3.2, approximate KV caching).
 *   oracle_confidence  - top-1 id and logit margin of Eq. 1 (Algorithm 1
 *                        line 5), plus the top-1 soft-max probability.
 *   oracle_lm_head_confidence - the output head (hidden state times the
 *                        vocabulary matrix) feeding those same three results
 *                        without ever storing the logits (Algorithm 1 lines 4-5).
 *   oracle_select_scattered, oracle_gather_append - the Scattered-Margin
 *                        baseline of Section 4.3.3 (same block size, scattered
 *                        positions) and the cache update it implies.
 *   oracle_commit      - L'(tau) of Section 3.2 (longest all-stable run from
 *                        the left), the boundary snap and L_min / fallback of
 *                        the unnumbered snap equation and Algorithm 1 lines
 *                        7-8, the commit and contiguous cache append of
 *                        Algorithm 1 lines 9-10.
 *
 * Element types: dtype 0 = IEEE fp32, dtype 1 = bfloat16 stored as uint16
 * (upper half of an fp32).  All tensors dense, row-major, innermost last.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double ld(const void *p, int dtype, int64_t i)
{
    if (dtype == 0)
        return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* One (b, i, h) output row of D values. */
static void attn_row(int dtype, const void *q, const void *ks, const void *vs,
                     const void *kc, const void *vc, int P, int N,
                     int b, int i, int h, int S, int Hq, int Hkv, int D, int C,
                     double scale, double *s, float *out)
{
    int g = h / (Hq / Hkv);
    int64_t qo = (((int64_t)b * S + i) * Hq + h) * D;
    int T = P + N;
    double m = -INFINITY;
    for (int t = 0; t < T; ++t) {
        const void *K = t < P ? kc : ks;
        int64_t ko = t < P ? (((int64_t)b * C + t) * Hkv + g) * D
                           : (((int64_t)b * S + (t - P)) * Hkv + g) * D;
        double acc = 0.0;
        for (int d = 0; d < D; ++d)
            acc += ld(q, dtype, qo + d) * ld(K, dtype, ko + d);
        s[t] = acc * scale;
        if (s[t] > m) m = s[t];
    }
    double den = 0.0;
    for (int t = 0; t < T; ++t) {
        s[t] = exp(s[t] - m);
        den += s[t];
    }
    for (int d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int t = 0; t < T; ++t) {
            const void *Vp = t < P ? vc : vs;
            int64_t vo = t < P ? (((int64_t)b * C + t) * Hkv + g) * D
                               : (((int64_t)b * S + (t - P)) * Hkv + g) * D;
            acc += s[t] * ld(Vp, dtype, vo + d);
        }
        out[d] = (float)(acc / den);
    }
}

/* out[B,S,Hq,D] fp32; rows i >= suffix_len[b] are left untouched. */
int oracle_attention(int dtype, const void *q, const void *ks, const void *vs,
                     const void *kc, const void *vc,
                     const int32_t *prefix_len, const int32_t *suffix_len,
                     int B, int S, int Hq, int Hkv, int D, int C, double scale, float *out)
{
    if (Hq % Hkv) return -1;
    int64_t rows = (int64_t)B * S * Hq;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(C + S + 1));
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < rows; ++r) {
            int h = (int)(r % Hq);
            int i = (int)((r / Hq) % S);
            int b = (int)(r / ((int64_t)Hq * S));
            if (i >= suffix_len[b]) continue;
            attn_row(dtype, q, ks, vs, kc, vc, prefix_len[b], suffix_len[b], b, i, h,
                     S, Hq, Hkv, D, C, scale, s, out + r * D);
        }
        free(s);
    }
    return 0;
}

/* Sampled form: rows[n][3] = (b, i, h); out[n, D] fp32. */
int oracle_attention_rows(int dtype, const void *q, const void *ks, const void *vs,
                          const void *kc, const void *vc,
                          const int32_t *prefix_len, const int32_t *suffix_len,
                          int B, int S, int Hq, int Hkv, int D, int C, double scale,
                          int n, const int32_t *rows, float *out)
{
    (void)B;
    if (Hq % Hkv) return -1;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(C + S + 1));
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n; ++r) {
            int b = rows[3 * r], i = rows[3 * r + 1], h = rows[3 * r + 2];
            attn_row(dtype, q, ks, vs, kc, vc, prefix_len[b], suffix_len[b], b, i, h,
                     S, Hq, Hkv, D, C, scale, s, out + (int64_t)r * D);
        }
        free(s);
    }
    return 0;
}

/*
 * Eq. 1 per active position: id = lowest index attaining the maximum, z2 = the
 * largest value among all other entries (equal to z1 when the maximum is
 * duplicated, so the margin is 0 on a tie), margin = one fp32 subtraction,
 * p1 = 1 / sum_v exp(z_v - z1) in double.  suffix_len may be NULL (all S rows).
 * Rows i >= suffix_len[b] are left untouched.  Returns -2 if a row's maximum
 * is not finite or the row holds a NaN.
 */
int oracle_confidence(int dtype, const void *logits, int B, int S, int V,
                      const int32_t *suffix_len,
                      int32_t *top1_id, float *top1_prob, float *margin)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (int64_t r = 0; r < (int64_t)B * S; ++r) {
        int b = (int)(r / S), i = (int)(r % S);
        if (suffix_len && i >= suffix_len[b]) continue;
        int64_t base = r * V;
        int id = 0;
        double z1 = ld(logits, dtype, base);
        for (int v = 0; v < V; ++v) {
            double z = ld(logits, dtype, base + v);
            if (z != z) bad = 1;
            if (z > z1) { z1 = z; id = v; }
        }
        double z2 = -INFINITY;
        for (int v = 0; v < V; ++v) {
            if (v == id) continue;
            double z = ld(logits, dtype, base + v);
            if (z > z2) z2 = z;
        }
        if (!(z1 > -INFINITY && z1 < INFINITY)) bad = 1;
        double den = 0.0;
        for (int v = 0; v < V; ++v)
            den += exp(ld(logits, dtype, base + v) - z1);
        top1_id[r] = id;
        margin[r] = (float)z1 - (float)z2;
        top1_prob[r] = (float)(1.0 / den);
    }
    return bad ? -2 : 0;
}

static int is_delim(const uint32_t *bitmap, int32_t id)
{
    return (bitmap[id >> 5] >> (id & 31)) & 1u;
}

/*
 * Adaptive threshold of Section 3.2 ("targeted block sizing", Eq. 2; Algorithm 1
 * line 6): find a threshold tau_k whose run length L'(tau_k) lies in
 * [lo, hi] = [ceil(alpha N), max(lo, floor(beta N))], via the prefix minimum
 * pm[i] = min(margin[0..i]).
 *
 * L'(t) is the first i with margin[i] <= t (N if none), so a length a with
 * 1 <= a < N is reachable by some threshold exactly when margin[a] <
 * pm[a-1] (any t in [margin[a], pm[a-1]) gives it); a = N is reachable by any
 * t < pm[N-1].  L0 is the length the caller's own threshold tau gives.
 *   lo <= L0 <= hi : keep it (tau_k = tau).
 *   L0 <  lo       : the SMALLEST reachable length in [lo, hi] (tau is lowered
 *                    as little as possible); tau_k = margin[a], or -inf for a = N.
 *   L0 >  hi       : the LARGEST reachable length in [lo, hi] (tau is raised as
 *                    little as possible).
 *   no reachable length in [lo, hi]: no threshold satisfies Eq. 2; the nearer
 *                    interval bound is used (lo or hi), tau_k = NaN and
 *                    *no_threshold = 1.
 * lo and hi are computed with one single-precision multiplication each.
 */
static int adaptive_length(const float *mg, int N, int L0, float tau, float alpha, float beta,
                           float *tau_k, int *no_threshold)
{
    int lo = (int)ceilf(alpha * (float)N);
    int hi = (int)floorf(beta * (float)N);
    if (lo < 0) lo = 0;
    if (lo > N) lo = N;
    if (hi > N) hi = N;
    if (hi < lo) hi = lo;
    *tau_k = tau;
    if (L0 >= lo && L0 <= hi) return L0;
    int first = -1, last = -1;          /* reachable lengths inside [lo, hi] */
    float pm = INFINITY;                /* prefix minimum of margin[0..a-1] */
    for (int a = 0; a <= N; ++a) {
        int reachable = a == N ? 1 : (a == 0 ? 1 : mg[a] < pm);
        if (reachable && a >= lo && a <= hi) {
            if (first < 0) first = a;
            last = a;
        }
        if (a < N && mg[a] < pm) pm = mg[a];
    }
    if (first < 0) {
        *no_threshold = 1;
        *tau_k = NAN;
        return L0 < lo ? lo : hi;
    }
    int a = L0 < lo ? first : last;
    *tau_k = a == N ? -INFINITY : mg[a];
    return a;
}

/*
 * Boundary search, snap, commit and append for every sequence.
 *
 * mask_i = margin_i > tau (strict) for i < N;  L' = first i with mask_i = 0,
 * else N.  L_snap = the largest length j in [1, L'] with L' - j <= W whose
 * last token id[j-1] is a delimiter; L' itself if there is none, if snapping
 * is off or if L' = 0.  (window < 0 means no window limit.)
 * When `adaptive` is set, L' is replaced by adaptive_length() above (the mask
 * output stays relative to the caller's tau); tau_used[b] receives tau_k.
 * L = min(N, max(L_snap, L_min)), cut to max_commit when that is > 0 (the
 * fixed-prefix variant of the sizing ablation, Table 2), then clamped to the cache room C - P
 * (status bit 0 set when that clamp bites) and to the token buffer room T - P
 * (status bit 1).
 * Commit: tokens[b, P..P+L) = id[b, 0..L); for every layer the first L suffix
 * K and V rows are copied to cache rows [P, P+L); P += L, N -= L.
 * K/V layer tensors may be NULL pointers arrays (scan only).
 */
int oracle_commit(int kv_dtype, int B, int S, int V, int Hkv, int D, int C, int layers, int T,
                  float tau, int window, int min_commit, int snap_enabled,
                  int adaptive, float alpha, float beta, int max_commit,
                  const float *margin, const int32_t *top1_id, const uint32_t *bitmap,
                  const void *const *k_suf, const void *const *v_suf,
                  void *const *k_cache, void *const *v_cache,
                  int32_t *tokens, int32_t *prefix_len, int32_t *suffix_len,
                  uint8_t *stable_mask, int32_t *raw_boundary, int32_t *snapped_boundary,
                  int32_t *commit_len, int32_t *status_flags, float *tau_used)
{
    (void)V;
    size_t esz = kv_dtype == 0 ? 4 : 2;
    size_t row = (size_t)Hkv * D * esz;
    for (int b = 0; b < B; ++b) {
        int N = suffix_len[b], P = prefix_len[b];
        const float *mg = margin + (int64_t)b * S;
        const int32_t *id = top1_id + (int64_t)b * S;
        uint8_t *mk = stable_mask + (int64_t)b * S;
        for (int i = 0; i < S; ++i)
            mk[i] = (i < N && mg[i] > tau) ? 1 : 0;
        int Lp = N;
        for (int i = 0; i < N; ++i)
            if (!mk[i]) { Lp = i; break; }
        float tk = tau;
        int no_threshold = 0;
        if (adaptive && N > 0)
            Lp = adaptive_length(mg, N, Lp, tau, alpha, beta, &tk, &no_threshold);
        if (tau_used) tau_used[b] = tk;
        int Ls = Lp;
        if (snap_enabled && Lp > 0) {
            for (int j = Lp; j >= 1; --j) {
                if (window >= 0 && Lp - j > window) break;
                if (is_delim(bitmap, id[j - 1])) { Ls = j; break; }
            }
        }
        int L = Ls > min_commit ? Ls : min_commit;
        if (L > N) L = N;
        if (max_commit > 0 && L > max_commit) L = max_commit;
        int flag = no_threshold ? 4 : 0;
        if (L > C - P) { L = C - P > 0 ? C - P : 0; flag |= 1; }
        if (tokens && L > T - P) { L = T - P > 0 ? T - P : 0; flag |= 2; }
        raw_boundary[b] = Lp;
        snapped_boundary[b] = Ls;
        commit_len[b] = L;
        if (status_flags) status_flags[b] = flag;
        if (tokens)
            for (int i = 0; i < L; ++i)
                tokens[(int64_t)b * T + P + i] = id[i];
        if (k_suf)
            for (int l = 0; l < layers; ++l) {
                memcpy((char *)k_cache[l] + ((size_t)b * C + P) * row,
                       (const char *)k_suf[l] + (size_t)b * S * row, (size_t)L * row);
                memcpy((char *)v_cache[l] + ((size_t)b * C + P) * row,
                       (const char *)v_suf[l] + (size_t)b * S * row, (size_t)L * row);
            }
        prefix_len[b] = P + L;
        suffix_len[b] = N - L;
    }
    return 0;
}

/*
 * Scattered-Margin selection (Section 4.3.3, the baseline that keeps LSP's block
 * size but drops its topology): of the N_b active positions of sequence b, the
 * count[b] positions with the largest margins, wherever they are; among equal
 * margins the lower position wins.  sel_index[b, 0..k) lists them in ascending
 * position order (entries beyond k are -1), sel_mask[b, i] = 1 for a selected
 * position.  k = min(count[b], N_b), not below 0.
 */
int oracle_select_scattered(int B, int S, const float *margin, const int32_t *suffix_len,
                            const int32_t *count, int32_t *sel_index, uint8_t *sel_mask)
{
    for (int b = 0; b < B; ++b) {
        int N = suffix_len[b];
        int k = count[b] < N ? count[b] : N;
        if (k < 0) k = 0;
        const float *mg = margin + (int64_t)b * S;
        uint8_t *mk = sel_mask + (int64_t)b * S;
        int32_t *ix = sel_index + (int64_t)b * S;
        for (int i = 0; i < S; ++i) { mk[i] = 0; ix[i] = -1; }
        for (int r = 0; r < k; ++r) {          /* pick the best remaining position k times */
            int best = -1;
            for (int i = 0; i < N; ++i)
                if (!mk[i] && (best < 0 || mg[i] > mg[best])) best = i;
            mk[best] = 1;
        }
        int n = 0;
        for (int i = 0; i < N; ++i)
            if (mk[i]) ix[n++] = i;
    }
    return 0;
}

/*
 * Gathered append: what the cache update becomes when the committed positions
 * are scattered.  For every layer, cache rows [P_b, P_b + k_b) receive the suffix
 * rows sel_index[b, 0..k_b) in that order (K and V), k_b = count[b] cut to the
 * cache room C - P_b; prefix_len[b] += k_b.  (suffix_len is left alone: with
 * scattered commits the remaining active positions are no longer a suffix.)
 */
int oracle_gather_append(int kv_dtype, int B, int S, int Hkv, int D, int C, int layers,
                         const int32_t *sel_index, const int32_t *count,
                         const void *const *k_suf, const void *const *v_suf,
                         void *const *k_cache, void *const *v_cache, int32_t *prefix_len)
{
    size_t esz = kv_dtype == 0 ? 4 : 2;
    size_t row = (size_t)Hkv * D * esz;
    for (int b = 0; b < B; ++b) {
        int P = prefix_len[b];
        int k = count[b];
        if (k > C - P) k = C - P > 0 ? C - P : 0;
        if (k < 0) k = 0;
        for (int j = 0; j < k; ++j) {
            int src = sel_index[(int64_t)b * S + j];
            if (src < 0) { /* the list ends here: fewer positions were active than count[b] */
                k = j;
                break;
            }
            for (int l = 0; l < layers; ++l) {
                memcpy((char *)k_cache[l] + ((size_t)b * C + P + j) * row,
                       (const char *)k_suf[l] + ((size_t)b * S + src) * row, row);
                memcpy((char *)v_cache[l] + ((size_t)b * C + P + j) * row,
                       (const char *)v_suf[l] + ((size_t)b * S + src) * row, row);
            }
        }
        prefix_len[b] = P + k;
    }
    return 0;
}

/*
 * The output head of the denoiser call followed by Eq. 1 (Algorithm 1 lines
 * 4-5), with the logits kept in double and never rounded to a storage type:
 *   z[r][v] = sum_k hidden[r][k] * weight[v][k]        (hidden [B*S, K], weight [V, K])
 * then, per active row, the same three results as oracle_confidence: the lowest
 * index attaining the maximum, the gap to the largest other entry, and
 * 1 / sum_v exp(z_v - z1).  The margin is the double difference rounded once
 * to fp32.  Optionally returns the full logits (z_out [B*S, V] doubles, may be
 * NULL).  Rows i >= suffix_len[b] are left untouched.
 */
int oracle_lm_head_confidence(int dtype, const void *hidden, const void *weight,
                              int B, int S, int K, int V, const int32_t *suffix_len,
                              int32_t *top1_id, float *top1_prob, float *margin, double *z_out)
{
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (int64_t r = 0; r < (int64_t)B * S; ++r) {
        int b = (int)(r / S), i = (int)(r % S);
        if (suffix_len && i >= suffix_len[b]) continue;
        double *z = (double *)malloc(sizeof(double) * (size_t)V);
        if (!z) { bad = 1; continue; }
        for (int v = 0; v < V; ++v) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += ld(hidden, dtype, r * K + k) * ld(weight, dtype, (int64_t)v * K + k);
            z[v] = acc;
            if (acc != acc) bad = 1;
        }
        int id = 0;
        for (int v = 1; v < V; ++v)
            if (z[v] > z[id]) id = v;
        double z2 = -INFINITY;
        for (int v = 0; v < V; ++v)
            if (v != id && z[v] > z2) z2 = z[v];
        if (!(z[id] > -INFINITY && z[id] < INFINITY)) bad = 1;
        double den = 0.0;
        for (int v = 0; v < V; ++v)
            den += exp(z[v] - z[id]);
        top1_id[r] = id;
        margin[r] = (float)(z[id] - z2);
        top1_prob[r] = (float)(1.0 / den);
        if (z_out) memcpy(z_out + r * V, z, sizeof(double) * (size_t)V);
        free(z);
    }
    return bad ? -2 : 0;
}

/* Threads the OpenMP loops above will use (reported next to oracle timings). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
