/* Driver for the sanitizer build of the CPU oracle (test infrastructure): calls every oracle entry point on
 * small seeded inputs, edge cases included (one-token vocabularies, empty contexts, -inf logits, ids outside
 * the vocabulary, the largest candidate and tree shapes), and prints one checksum per call.  Built with
 * -fsanitize=address,undefined, any out-of-bounds access, leak or undefined operation ends it with an error;
 * the checksums must equal those of the same driver built without sanitizers. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "aasd_oracle.h"

static uint32_t g_state = 12345u;
static uint32_t rnd(void) { g_state = g_state * 1664525u + 1013904223u; return g_state >> 8; }
static double unit(void) { return (double)rnd() / 16777216.0; }

static uint64_t sum_bytes(uint64_t h, const void *p, size_t n)
{
    const unsigned char *b = (const unsigned char *)p;
    for (size_t i = 0; i < n; ++i) h = (h ^ b[i]) * 1099511628211ull;
    return h;
}

static int check(int rc, const char *what)
{
    if (rc != 0) { fprintf(stderr, "%s returned %d\n", what, rc); exit(2); }
    return rc;
}

static void fill_logits_f32(float *z, size_t n, int with_inf)
{
    for (size_t i = 0; i < n; ++i) {
        z[i] = (float)((unit() - 0.5) * 12.0);
        if (with_inf && rnd() % 11 == 0) z[i] = -INFINITY;
    }
}

static void fill_logits_bf16(uint16_t *z, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        float f = (float)((unit() - 0.5) * 12.0);
        uint32_t u;
        memcpy(&u, &f, 4);
        z[i] = (uint16_t)(u >> 16);
    }
}

static void run_align(int dtype, int64_t rows, int32_t V, int32_t m_x, int32_t c, int mode, int with_inf)
{
    const int64_t stride = V + 3;
    void *z = malloc((size_t)rows * stride * (dtype == ORC_F32 ? 4 : 2));
    if (dtype == ORC_F32) fill_logits_f32((float *)z, (size_t)(rows * stride), with_inf);
    else fill_logits_bf16((uint16_t *)z, (size_t)(rows * stride));
    if (with_inf)   /* at least one finite logit per row */
        for (int64_t r = 0; r < rows; ++r) ((float *)z)[r * stride] = 0.5f;
    int32_t *nt = (int32_t *)malloc(sizeof(int32_t) * rows);
    for (int64_t r = 0; r < rows; ++r) nt[r] = (int32_t)(rnd() % (uint32_t)(V + 2)) - 1;   /* -1 .. V: none, valid, one past */
    int32_t *am = malloc(4 * rows), *rank = malloc(4 * rows), *ex = malloc(4 * rows * (m_x ? m_x : 1));
    uint8_t *mis = malloc(rows), *nx = malloc(rows);
    double *H = malloc(8 * rows), *pn = malloc(8 * rows), *pm = malloc(8 * rows), *dm = malloc(8 * rows * (m_x ? m_x : 1));
    check(orc_align_sample(z, dtype, rows, V, stride, nt, m_x, c, mode, 77u, ((uint64_t)3 << 32) + 5, am, mis, H, pn, pm, rank, ex, nx, dm),
          "orc_align_sample");
    uint64_t h = 1469598103934665603ull;
    h = sum_bytes(h, am, 4 * rows); h = sum_bytes(h, mis, rows); h = sum_bytes(h, rank, 4 * rows);
    h = sum_bytes(h, ex, 4 * rows * m_x); h = sum_bytes(h, nx, rows); h = sum_bytes(h, H, 8 * rows);
    printf("align dtype=%d rows=%lld V=%d m=%d c=%d mode=%d inf=%d: %016llx\n", dtype, (long long)rows, V, m_x, c, mode, with_inf,
           (unsigned long long)h);
    check(orc_align_sample(z, dtype, rows, V, stride, NULL, m_x, c, mode, 1u, 0u, am, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL),
          "orc_align_sample (optional outputs absent)");
    free(z); free(nt); free(am); free(rank); free(ex); free(mis); free(nx); free(H); free(pn); free(pm); free(dm);
}

static void run_retrieve(int32_t B, int64_t cap, int32_t n_min, int32_t n_max, int32_t k, int32_t C, int32_t m_x, uint32_t alphabet)
{
    int32_t *tok = malloc(4 * B * cap), *len = malloc(4 * B), *plen = malloc(4 * B);
    for (int64_t i = 0; i < B * cap; ++i) tok[i] = (int32_t)(rnd() % alphabet);
    for (int32_t b = 0; b < B; ++b) { len[b] = (int32_t)(rnd() % (uint32_t)(cap + 1)); plen[b] = (int32_t)(rnd() % (uint32_t)(cap + 1)); }
    len[0] = (int32_t)cap; if (B > 1) len[1] = 0;
    int32_t *ex = NULL; uint8_t *nx = NULL;
    if (m_x) {
        ex = malloc(4 * B * cap * m_x); nx = malloc(B * cap);
        for (int64_t i = 0; i < B * cap * m_x; ++i) ex[i] = (int32_t)(rnd() % 50);
        for (int64_t i = 0; i < B * cap; ++i) nx[i] = (uint8_t)(rnd() % (uint32_t)(m_x + 1));
    }
    int32_t *dr = malloc(4 * B * C * k), *dl = malloc(4 * B * C), *sp = malloc(4 * B * C), *nc = malloc(4 * B), *kl = malloc(4 * B);
    int32_t *dx = m_x ? malloc(4 * B * C * k * m_x) : NULL;
    uint8_t *st = malloc(B * C * k);
    check(orc_retrieve_drafts(tok, cap, len, plen, B, n_min, n_max, k, C, ex, nx, m_x, cap, dr, dl, sp, nc, kl, dx, st), "orc_retrieve_drafts");
    uint64_t h = 1469598103934665603ull;
    h = sum_bytes(h, dr, 4 * B * C * k); h = sum_bytes(h, dl, 4 * B * C); h = sum_bytes(h, sp, 4 * B * C);
    h = sum_bytes(h, nc, 4 * B); h = sum_bytes(h, kl, 4 * B); h = sum_bytes(h, st, B * C * k);
    if (dx) h = sum_bytes(h, dx, 4 * B * C * k * m_x);
    printf("retrieve B=%d cap=%lld n=%d..%d k=%d C=%d m=%d: %016llx\n", B, (long long)cap, n_min, n_max, k, C, m_x, (unsigned long long)h);
    free(tok); free(len); free(plen); free(ex); free(nx); free(dr); free(dl); free(sp); free(nc); free(kl); free(dx); free(st);
}

static void run_verify(int dtype, int32_t B, int32_t C, int32_t k, int32_t V, uint32_t flags, int with_strict)
{
    const int32_t R = 1 + C * k;
    const int64_t rs = V + 1, ss = (int64_t)(R + 1) * rs;
    void *z = malloc((size_t)B * ss * (dtype == ORC_F32 ? 4 : 2));
    if (dtype == ORC_F32) fill_logits_f32((float *)z, (size_t)(B * ss), 0);
    else fill_logits_bf16((uint16_t *)z, (size_t)(B * ss));
    int32_t *dr = malloc(4 * B * C * k), *dl = malloc(4 * B * C);
    uint8_t *st = malloc(B * C * k);
    for (int i = 0; i < B * C * k; ++i) { dr[i] = (int32_t)(rnd() % (uint32_t)(V + 2)) - 1; st[i] = (uint8_t)(rnd() & 1); }
    for (int i = 0; i < B * C; ++i) dl[i] = (int32_t)(rnd() % (uint32_t)(k + 3)) - 1;   /* -1 .. k+1: clamped by the oracle */
    int32_t *al = malloc(4 * B), *bc = malloc(4 * B), *nt = malloc(4 * B), *ra = malloc(4 * B * R), *tr = malloc(4 * B * C * k);
    double *re = malloc(8 * B * R), *rp = malloc(8 * B * R), *tp = malloc(8 * B * C * k), *td = malloc(8 * B * C * k), *tm = malloc(8 * B * C * k);
    uint32_t *near = malloc(4 * B);
    check(orc_verify(z, dtype, B, C, k, V, rs, ss, dr, dl, with_strict ? st : NULL, 0.1, 0.1, flags, al, bc, nt, re, rp, ra, tp, td, tm, near),
          "orc_verify");
    uint64_t h = 1469598103934665603ull;
    h = sum_bytes(h, al, 4 * B); h = sum_bytes(h, bc, 4 * B); h = sum_bytes(h, nt, 4 * B); h = sum_bytes(h, ra, 4 * B * R);
    h = sum_bytes(h, re, 8 * B * R); h = sum_bytes(h, tp, 8 * B * C * k); h = sum_bytes(h, near, 4 * B);
    check(orc_verify_topk(z, dtype, B, C, k, V, rs, ss, dr, dl, 3, al, bc, nt, ra, tr), "orc_verify_topk");
    h = sum_bytes(h, al, 4 * B); h = sum_bytes(h, tr, 4 * B * C * k);
    printf("verify dtype=%d B=%d C=%d k=%d V=%d flags=%u strict=%d: %016llx\n", dtype, B, C, k, V, flags, with_strict, (unsigned long long)h);
    free(z); free(dr); free(dl); free(st); free(al); free(bc); free(nt); free(ra); free(tr); free(re); free(rp); free(tp); free(td); free(tm); free(near);
}

static void run_tree(int32_t B, int32_t C, int32_t k, int32_t m_x, int32_t N, int32_t V, uint32_t alphabet)
{
    int32_t *dr = malloc(4 * B * C * k), *dl = malloc(4 * B * C), *dx = m_x ? malloc(4 * B * C * k * m_x) : NULL, *root = malloc(4 * B);
    uint8_t *st = malloc(B * C * k);
    for (int i = 0; i < B * C * k; ++i) { dr[i] = (int32_t)(rnd() % alphabet) - (rnd() % 29 == 0); st[i] = (uint8_t)(rnd() & 1); }
    for (int i = 0; i < B * C; ++i) dl[i] = (int32_t)(rnd() % (uint32_t)(k + 1));
    for (int i = 0; i < B * C * k * m_x; ++i) dx[i] = (rnd() & 1) ? (int32_t)(rnd() % alphabet) : -1;
    for (int i = 0; i < B; ++i) root[i] = i;
    const int32_t W = (N + 31) / 32;
    int32_t *tok = malloc(4 * B * N), *par = malloc(4 * B * N), *dep = malloc(4 * B * N), *nn = malloc(4 * B), *cn = malloc(4 * B * C * k);
    uint8_t *ns = malloc(B * N);
    uint32_t *mask = malloc(4 * (size_t)B * N * W);
    check(orc_build_tree(dr, dl, st, dx, m_x, root, B, C, k, N, tok, par, dep, ns, nn, mask, cn), "orc_build_tree");
    uint64_t h = 1469598103934665603ull;
    h = sum_bytes(h, tok, 4 * B * N); h = sum_bytes(h, par, 4 * B * N); h = sum_bytes(h, dep, 4 * B * N); h = sum_bytes(h, ns, B * N);
    h = sum_bytes(h, nn, 4 * B); h = sum_bytes(h, mask, 4 * (size_t)B * N * W); h = sum_bytes(h, cn, 4 * B * C * k);
    float *z = malloc(4 * (size_t)B * N * V);
    fill_logits_f32(z, (size_t)B * N * V, 0);
    int32_t *al = malloc(4 * B), *bn = malloc(4 * B), *path = malloc(4 * B * 16), *nt = malloc(4 * B), *ra = malloc(4 * B * N);
    double *re = malloc(8 * B * N), *rp = malloc(8 * B * N), *np_ = malloc(8 * B * N), *nd = malloc(8 * B * N), *nm = malloc(8 * B * N);
    uint32_t *near = malloc(4 * B);
    check(orc_verify_tree(z, ORC_F32, B, N, V, V, (int64_t)N * V, tok, par, ns, nn, 0.1, 0.1, 0u, al, bn, path, nt, re, rp, ra, np_, nd, nm, near),
          "orc_verify_tree");
    h = sum_bytes(h, al, 4 * B); h = sum_bytes(h, bn, 4 * B); h = sum_bytes(h, path, 4 * B * 16); h = sum_bytes(h, nt, 4 * B);
    h = sum_bytes(h, ra, 4 * B * N); h = sum_bytes(h, re, 8 * B * N);
    printf("tree B=%d C=%d k=%d m=%d N=%d V=%d: %016llx\n", B, C, k, m_x, N, V, (unsigned long long)h);
    free(dr); free(dl); free(dx); free(root); free(st); free(tok); free(par); free(dep); free(nn); free(cn); free(ns); free(mask); free(z);
    free(al); free(bn); free(path); free(nt); free(ra); free(re); free(rp); free(np_); free(nd); free(nm); free(near);
}

int main(void)
{
    uint32_t out[4];
    const uint32_t ctr[4] = {0, 0, 0, 0}, key[2] = {0, 0};
    orc_philox4x32_10(ctr, key, out);
    printf("philox %08x %08x %08x %08x\n", out[0], out[1], out[2], out[3]);
    for (int mode = 0; mode < 3; ++mode) {
        run_align(ORC_F32, 23, 1, 1, 1, mode, 0);
        run_align(ORC_BF16, 40, 2, 1, 2, mode, 0);
        run_align(ORC_F32, 31, 9, 4, 8, mode, 1);
        run_align(ORC_BF16, 57, 777, 2, 4, mode, 0);
        run_align(ORC_BF16, 9, 4099, 0, 1, mode, 0);
    }
    run_retrieve(1, 1, 1, 1, 1, 1, 0, 2);
    run_retrieve(7, 90, 1, 8, 16, 32, 4, 3);
    run_retrieve(5, 1500, 2, 4, 8, 16, 2, 5);
    run_retrieve(3, 40, 3, 3, 4, 1, 0, 2);
    run_verify(ORC_F32, 1, 1, 1, 1, 0u, 0);
    run_verify(ORC_BF16, 4, 32, 16, 37, 0u, 1);
    run_verify(ORC_F32, 6, 3, 5, 500, ORC_VERIFY_NO_CLAMP, 1);
    run_verify(ORC_BF16, 3, 16, 8, 1000, 0u, 0);
    run_tree(3, 1, 1, 0, 1, 5, 3);
    run_tree(4, 16, 8, 2, 385, 50, 40);
    run_tree(2, 32, 16, 4, 512, 20, 7);
    run_tree(5, 8, 8, 2, 7, 30, 3);
    return 0;
}
