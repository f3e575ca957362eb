/*
 * TEST INFRASTRUCTURE ONLY: runs every routine of the CPU oracle (lsp_oracle.c,
 * included below as the same translation unit) over small ragged shapes whose
 * buffers are allocated at their exact size, so that a build under
 * -fsanitize=address,undefined reports any access outside them, any signed
 * overflow or misaligned access.  Inputs come from a fixed linear congruential
 * sequence; a checksum of all outputs is printed so that the sanitized and the
 * plain build can be compared.  No arithmetic of the method lives here.
 */
#include <stdio.h>

#include "lsp_oracle.c"

static uint64_t lcg_state = 0x2545F4914F6CDD1DULL;
static uint32_t lcg(void)
{
    lcg_state = lcg_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (uint32_t)(lcg_state >> 33);
}
static float unif(void) { return (float)(lcg() % 20001) / 10000.0f - 1.0f; } /* [-1, 1] */

static void *fill(int dtype, int64_t n, float scale)
{
    size_t esz = dtype == 0 ? 4 : 2;
    void *p = malloc((size_t)n * esz + (n == 0));
    for (int64_t i = 0; i < n; ++i) {
        float f = unif() * scale;
        if (dtype == 0)
            ((float *)p)[i] = f;
        else {
            uint32_t u;
            memcpy(&u, &f, 4);
            ((uint16_t *)p)[i] = (uint16_t)(u >> 16);
        }
    }
    return p;
}

static uint64_t sum = 1469598103934665603ULL;
static void mix(const void *p, size_t bytes)
{
    const unsigned char *c = (const unsigned char *)p;
    for (size_t i = 0; i < bytes; ++i) sum = (sum ^ c[i]) * 1099511628211ULL;
}

static int run_case(int dtype, int B, int S, int Hq, int Hkv, int D, int C, int V, int layers, int K)
{
    int rc = 0;
    size_t esz = dtype == 0 ? 4 : 2;
    int32_t *pl = malloc(sizeof(int32_t) * B), *sl = malloc(sizeof(int32_t) * B);
    for (int b = 0; b < B; ++b) {
        pl[b] = (int32_t)(lcg() % (uint32_t)(C + 1));
        sl[b] = (int32_t)(lcg() % (uint32_t)(S + 1));
    }
    pl[0] = C;          /* a full cache */
    if (B > 1) sl[1] = 0; /* an empty suffix */
    if (B > 2) { pl[2] = 0; sl[2] = S; }

    /* attention, whole and by rows */
    void *q = fill(dtype, (int64_t)B * S * Hq * D, 1.0f), *ks = fill(dtype, (int64_t)B * S * Hkv * D, 1.0f);
    void *vs = fill(dtype, (int64_t)B * S * Hkv * D, 1.0f);
    float *out = malloc(sizeof(float) * (size_t)B * S * Hq * D);
    for (int64_t i = 0; i < (int64_t)B * S * Hq * D; ++i) out[i] = -7.0f;
    void **kcl = malloc(sizeof(void *) * layers), **vcl = malloc(sizeof(void *) * layers);
    void **ksl = malloc(sizeof(void *) * layers), **vsl = malloc(sizeof(void *) * layers);
    for (int l = 0; l < layers; ++l) {
        kcl[l] = fill(dtype, (int64_t)B * C * Hkv * D, 1.0f);
        vcl[l] = fill(dtype, (int64_t)B * C * Hkv * D, 1.0f);
        ksl[l] = l == 0 ? ks : fill(dtype, (int64_t)B * S * Hkv * D, 1.0f);
        vsl[l] = l == 0 ? vs : fill(dtype, (int64_t)B * S * Hkv * D, 1.0f);
    }
    rc |= oracle_attention(dtype, q, ks, vs, kcl[0], vcl[0], pl, sl, B, S, Hq, Hkv, D, C, 0.125, out);
    mix(out, sizeof(float) * (size_t)B * S * Hq * D);
    int nrows = 0;
    int32_t *rows = malloc(sizeof(int32_t) * 3 * (size_t)B * 2 + 4);
    for (int b = 0; b < B; ++b)
        if (sl[b] > 0) {
            rows[3 * nrows] = b; rows[3 * nrows + 1] = 0; rows[3 * nrows + 2] = Hq - 1; ++nrows;
            rows[3 * nrows] = b; rows[3 * nrows + 1] = sl[b] - 1; rows[3 * nrows + 2] = 0; ++nrows;
        }
    float *orow = malloc(sizeof(float) * (size_t)(nrows + 1) * D);
    rc |= oracle_attention_rows(dtype, q, ks, vs, kcl[0], vcl[0], pl, sl, B, S, Hq, Hkv, D, C, 0.125, nrows, rows, orow);
    mix(orow, sizeof(float) * (size_t)nrows * D);

    /* confidence */
    void *z = fill(dtype, (int64_t)B * S * V, 4.0f);
    int32_t *ids = malloc(sizeof(int32_t) * (size_t)B * S);
    float *prob = malloc(sizeof(float) * (size_t)B * S), *mar = malloc(sizeof(float) * (size_t)B * S);
    for (int i = 0; i < B * S; ++i) { ids[i] = -1; prob[i] = 0.f; mar[i] = 0.f; }
    rc |= oracle_confidence(dtype, z, B, S, V, sl, ids, prob, mar);
    rc |= oracle_confidence(dtype, z, B, S, V, NULL, ids, prob, mar);
    mix(ids, sizeof(int32_t) * (size_t)B * S); mix(mar, sizeof(float) * (size_t)B * S);

    /* output head + confidence */
    void *hid = fill(dtype, (int64_t)B * S * K, 1.0f), *wt = fill(dtype, (int64_t)V * K, 0.5f);
    int32_t *ids2 = malloc(sizeof(int32_t) * (size_t)B * S);
    float *prob2 = malloc(sizeof(float) * (size_t)B * S), *mar2 = malloc(sizeof(float) * (size_t)B * S);
    double *zz = malloc(sizeof(double) * (size_t)B * S * V);
    for (int i = 0; i < B * S; ++i) { ids2[i] = -1; prob2[i] = 0.f; mar2[i] = 0.f; }
    for (int64_t i = 0; i < (int64_t)B * S * V; ++i) zz[i] = 0.0;
    rc |= oracle_lm_head_confidence(dtype, hid, wt, B, S, K, V, sl, ids2, prob2, mar2, zz);
    rc |= oracle_lm_head_confidence(dtype, hid, wt, B, S, K, V, NULL, ids2, prob2, mar2, NULL);
    mix(ids2, sizeof(int32_t) * (size_t)B * S);

    /* selection and gathered append (counts above the active positions and above the cache room) */
    int32_t *cnt = malloc(sizeof(int32_t) * B), *sel = malloc(sizeof(int32_t) * (size_t)B * S);
    uint8_t *selm = malloc((size_t)B * S);
    for (int b = 0; b < B; ++b) cnt[b] = (int32_t)(lcg() % (uint32_t)(S + 3));
    rc |= oracle_select_scattered(B, S, mar, sl, cnt, sel, selm);
    mix(sel, sizeof(int32_t) * (size_t)B * S);
    int32_t *pl2 = malloc(sizeof(int32_t) * B);
    memcpy(pl2, pl, sizeof(int32_t) * B);
    rc |= oracle_gather_append((int)dtype, B, S, Hkv, D, C, layers, sel, cnt, (const void *const *)ksl,
                               (const void *const *)vsl, kcl, vcl, pl2);
    mix(pl2, sizeof(int32_t) * B);

    /* commit: every sizing mode, snap on and off, token buffer shorter than the cache */
    uint32_t *bitmap = calloc((size_t)(V + 31) / 32, 4);
    for (int v = 0; v < V; v += 3) bitmap[v / 32] |= 1u << (v % 32);
    int T = C - 1;
    int32_t *tokens = malloc(sizeof(int32_t) * (size_t)B * T);
    uint8_t *mask = malloc((size_t)B * S);
    int32_t *raw = malloc(sizeof(int32_t) * B), *snap = malloc(sizeof(int32_t) * B);
    int32_t *clen = malloc(sizeof(int32_t) * B), *flags = malloc(sizeof(int32_t) * B);
    float *tauu = malloc(sizeof(float) * B);
    for (int mode = 0; mode < 6; ++mode) {
        int32_t *p3 = malloc(sizeof(int32_t) * B), *s3 = malloc(sizeof(int32_t) * B);
        memcpy(p3, pl, sizeof(int32_t) * B);
        memcpy(s3, sl, sizeof(int32_t) * B);
        for (int i = 0; i < B * T; ++i) tokens[i] = -1;
        int window = mode == 0 ? 0 : mode == 1 ? -1 : 3;
        rc |= oracle_commit((int)dtype, B, S, V, Hkv, D, C, mode == 5 ? 0 : layers, T, mode == 2 ? INFINITY : 0.3f, window,
                            mode % 3, mode != 3, mode == 4, 0.25f, 0.5f, mode == 1 ? 2 : 0, mar, ids, bitmap,
                            (const void *const *)ksl, (const void *const *)vsl, kcl, vcl, tokens, p3, s3, mask, raw, snap, clen,
                            flags, tauu);
        mix(p3, sizeof(int32_t) * B); mix(s3, sizeof(int32_t) * B); mix(clen, sizeof(int32_t) * B);
        mix(snap, sizeof(int32_t) * B); mix(raw, sizeof(int32_t) * B); mix(mask, (size_t)B * S);
        mix(tokens, sizeof(int32_t) * (size_t)B * T);
        free(p3); free(s3);
    }
    for (int l = 0; l < layers; ++l) { mix(kcl[l], (size_t)B * C * Hkv * D * esz); mix(vcl[l], (size_t)B * C * Hkv * D * esz); }

    for (int l = 0; l < layers; ++l) {
        free(kcl[l]); free(vcl[l]);
        if (l) { free(ksl[l]); free(vsl[l]); }
    }
    free(kcl); free(vcl); free(ksl); free(vsl);
    free(q); free(ks); free(vs); free(out); free(rows); free(orow); free(z); free(ids); free(prob); free(mar);
    free(hid); free(wt); free(ids2); free(prob2); free(mar2); free(zz); free(cnt); free(sel); free(selm); free(pl2);
    free(bitmap); free(tokens); free(mask); free(raw); free(snap); free(clen); free(flags); free(tauu); free(pl); free(sl);
    return rc;
}

int main(void)
{
    int rc = 0;
    /*            dtype B  S   Hq Hkv D   C   V    layers K */
    rc |= run_case(0, 1, 1, 1, 1, 8, 2, 2, 1, 8);
    rc |= run_case(0, 3, 17, 4, 2, 16, 23, 37, 2, 8);
    rc |= run_case(1, 4, 33, 6, 2, 8, 40, 131, 3, 16);
    rc |= run_case(1, 5, 9, 3, 3, 32, 9, 1000, 1, 24);
    printf("rc=%d checksum=%016llx threads=%d\n", rc, (unsigned long long)sum, oracle_num_threads());
    return rc != 0;
}
