/*
 * CPU oracle for the AASD hot path.  TEST INFRASTRUCTURE ONLY: see aasd_oracle.h.
 *
 * Everything real-valued is fp64.  There is no blocking, fusion or reordering
 * beyond what the definitions state: softmax is "subtract the max, exponentiate,
 * divide by the sum"; entropy is -sum p ln p; the top-c list is found by c
 * linear scans; retrieval compares every window with the suffix token by token.
 */
#include "aasd_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as   */
/* easy as 1, 2, 3", SC'11).                                                  */
/* ------------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(prod1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prod1;
        uint32_t n2 = (uint32_t)(prod0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prod0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; /* key schedule: Weyl sequence, golden ratio   */
        k1 += 0xBB67AE85u; /*                              and sqrt(3)-1 */
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------------- */
/* exact widening of the stored logits                                        */
/* ------------------------------------------------------------------------- */
static double widen_one(const void *row, int dtype, int64_t v)
{
    if (dtype == ORC_F32) {
        float f;
        memcpy(&f, (const char *)row + 4 * v, 4);
        return (double)f;
    } else { /* bf16 = the upper 16 bits of an IEEE binary32 */
        uint16_t h;
        memcpy(&h, (const char *)row + 2 * v, 2);
        uint32_t bits = (uint32_t)h << 16;
        float f;
        memcpy(&f, &bits, 4);
        return (double)f;
    }
}

static size_t elt_bytes(int dtype) { return dtype == ORC_F32 ? 4 : 2; }

int orc_widen_row(const void *row, int dtype, int32_t V, double *z)
{
    if (!row || !z || V <= 0 || (dtype != ORC_F32 && dtype != ORC_BF16)) return -1;
    for (int32_t v = 0; v < V; ++v) z[v] = widen_one(row, dtype, v);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* softmax, entropy, greedy pick of one row                                   */
/* ------------------------------------------------------------------------- */
int orc_row_softmax(const void *row, int dtype, int32_t V, double *p)
{
    if (orc_widen_row(row, dtype, V, p) != 0) return -1;
    double m = p[0];
    for (int32_t v = 1; v < V; ++v)
        if (p[v] > m) m = p[v];
    double S = 0.0;
    for (int32_t v = 0; v < V; ++v) {
        p[v] = exp(p[v] - m);
        S += p[v];
    }
    for (int32_t v = 0; v < V; ++v) p[v] /= S;
    return 0;
}

/* z already widened; e is scratch for V doubles (the unnormalised softmax) */
static void stats_of(const double *z, int32_t V, double *e, double *m_out, double *S_out,
                     double *H_out, int32_t *argmax_out)
{
    double m = z[0];
    int32_t am = 0;
    for (int32_t v = 1; v < V; ++v)
        if (z[v] > m) { m = z[v]; am = v; } /* strict >: the smallest index wins ties */
    double S = 0.0;
    for (int32_t v = 0; v < V; ++v) {
        e[v] = exp(z[v] - m);
        S += e[v];
    }
    double H = 0.0;
    for (int32_t v = 0; v < V; ++v) {
        double p = e[v] / S;
        if (p > 0.0) H -= p * log(p);
    }
    *m_out = m; *S_out = S; *H_out = H; *argmax_out = am;
}

int orc_row_stats(const void *row, int dtype, int32_t V, double *m, double *S, double *H,
                  int32_t *argmax)
{
    if (!row || V <= 0 || (dtype != ORC_F32 && dtype != ORC_BF16)) return -1;
    double *z = (double *)malloc(sizeof(double) * 2 * (size_t)V);
    if (!z) return -2;
    orc_widen_row(row, dtype, V, z);
    double mm, SS, HH;
    int32_t am;
    stats_of(z, V, z + V, &mm, &SS, &HH, &am);
    if (m) *m = mm;
    if (S) *S = SS;
    if (H) *H = HH;
    if (argmax) *argmax = am;
    free(z);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* alignment sampling                                                         */
/* ------------------------------------------------------------------------- */

/* order of preference among tokens: larger logit first, then smaller id */
static int better(double za, int32_t a, double zb, int32_t b)
{
    return za > zb || (za == zb && a < b);
}

int orc_align_sample(const void *logits, int dtype, int64_t rows, int32_t V, int64_t row_stride,
                     const int32_t *next_tok, int32_t m_x, int32_t c, int mode, uint64_t seed,
                     uint64_t row_id_base, int32_t *argmax, uint8_t *misaligned, double *entropy,
                     double *p_next, double *p_max, int32_t *rank, int32_t *extras,
                     uint8_t *n_extras, double *draw_margin)
{
    if (!logits || rows < 0 || V <= 0 || row_stride < V) return -1;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return -1;
    if (m_x < 0 || m_x > 4 || c < m_x || c > 8 || c < 1) return -1;
    if (mode != ORC_EXTRAS_TOP && mode != ORC_EXTRAS_SAMPLE && mode != ORC_EXTRAS_GUMBEL) return -1;

    double *z = (double *)malloc(sizeof(double) * 2 * (size_t)V);
    if (!z) return -2;

    for (int64_t r = 0; r < rows; ++r) {
        const char *row = (const char *)logits + (size_t)r * (size_t)row_stride * elt_bytes(dtype);
        orc_widen_row(row, dtype, V, z);

        /* greedy pick, softmax normaliser, entropy of the prefill distribution */
        double m, S, H;
        int32_t am;
        stats_of(z, V, z + V, &m, &S, &H, &am);
        if (argmax) argmax[r] = am;
        if (entropy) entropy[r] = H;
        if (p_max) p_max[r] = 1.0 / S;

        for (int32_t j = 0; j < m_x; ++j) {
            if (extras) extras[r * m_x + j] = -1;
            if (draw_margin) draw_margin[r * m_x + j] = -1.0;
        }
        if (n_extras) n_extras[r] = 0;

        int32_t nt = next_tok ? next_tok[r] : -1;
        if (nt < 0 || nt >= V) { /* no next prompt token for this row */
            if (misaligned) misaligned[r] = 0;
            if (p_next) p_next[r] = 0.0;
            if (rank) rank[r] = -1;
            continue;
        }

        /* Sec. 2.3: the position is aligned iff the prompt's next token is a
         * greedy pick, i.e. no token has a strictly larger logit. */
        double zstar = z[nt];
        int32_t rk = 0;
        for (int32_t v = 0; v < V; ++v)
            if (z[v] > zstar) ++rk;
        int mis = rk > 0;
        if (misaligned) misaligned[r] = (uint8_t)mis;
        if (rank) rank[r] = rk;
        if (p_next) p_next[r] = exp(zstar - m) / S;
        if (!mis || m_x == 0) continue;

        if (mode == ORC_EXTRAS_GUMBEL) {
            /* Sec. 3.2 read literally: the extras are SAMPLED from the whole output distribution of
             * the prefill row.  m_x draws without replacement, proportional to the softmax
             * probability, over every token except the prompt token itself (it is the draft token
             * already).  Drawing without replacement in proportion to p is the same as ranking the
             * tokens by z_v + G_v with independent standard Gumbel G_v (Gumbel-top-k), which needs
             * one uniform per token: token v uses word (v mod 4) of the Philox block with counter
             * (row id, v div 4, tag).  x in (0,1) -> E = -ln(1-x) is Exp(1) -> G = -ln E. */
            uint64_t row_id = row_id_base + (uint64_t)r;
            uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
            double *kap = z + V; /* the keys z_v + G_v (the softmax scratch is free again) */
            for (int32_t v0 = 0; v0 < V; v0 += 4) {
                uint32_t ctr[4] = {(uint32_t)row_id, (uint32_t)(row_id >> 32), (uint32_t)(v0 >> 2),
                                   0x47554D42u};
                uint32_t rnd[4];
                orc_philox4x32_10(ctr, key, rnd);
                for (int32_t j = 0; j < 4 && v0 + j < V; ++j) {
                    double x = ((double)(rnd[j] >> 9) + 0.5) * (1.0 / 8388608.0);
                    double E = -log1p(-x);
                    kap[v0 + j] = z[v0 + j] - log(E);
                }
            }
            int32_t picked[5];
            int n_picked = 0;
            for (int pick = 0; pick <= m_x; ++pick) { /* one more than needed: it gives the last margin */
                int32_t best = -1;
                for (int32_t v = 0; v < V; ++v) {
                    int taken = (v == nt) || kap[v] == -INFINITY; /* p_v = 0 cannot be drawn */
                    for (int q = 0; q < n_picked; ++q)
                        if (picked[q] == v) taken = 1;
                    if (taken) continue;
                    if (best < 0 || better(kap[v], v, kap[best], best)) best = v;
                }
                if (best < 0) break;
                picked[n_picked++] = best;
            }
            int n_out = n_picked < m_x ? n_picked : m_x;
            for (int i = 0; i < n_out; ++i) {
                if (extras) extras[r * m_x + i] = picked[i];
                if (draw_margin)
                    draw_margin[r * m_x + i] =
                        i + 1 < n_picked ? kap[picked[i]] - kap[picked[i + 1]] : INFINITY;
            }
            if (n_extras) n_extras[r] = (uint8_t)n_out;
            continue;
        }

        /* Fig. 2: the tokens ranked above the prompt token are the extras.
         * Candidate list K = the top-c tokens of the row (logit descending,
         * id ascending) that are strictly more likely than the prompt token. */
        int32_t K[8];
        int nK = 0;
        for (int pick = 0; pick < c; ++pick) {
            int32_t best = -1;
            for (int32_t v = 0; v < V; ++v) {
                int taken = 0;
                for (int q = 0; q < nK; ++q)
                    if (K[q] == v) taken = 1;
                if (taken) continue;
                if (best < 0 || better(z[v], v, z[best], best)) best = v;
            }
            if (best < 0 || !(z[best] > zstar)) break; /* the rest rank at or below it */
            K[nK++] = best;
        }

        int32_t chosen[4];
        int n_chosen = 0;
        if (mode == ORC_EXTRAS_TOP || nK <= m_x) {
            /* deterministic: best first, capped at m_x; consumes no random numbers */
            for (int i = 0; i < nK && i < m_x; ++i) chosen[n_chosen++] = K[i];
        } else {
            /* seeded draws without replacement, proportional to the softmax
             * probability restricted to K */
            uint64_t row_id = row_id_base + (uint64_t)r;
            int32_t remaining[8];
            int n_rem = nK;
            for (int i = 0; i < nK; ++i) remaining[i] = K[i];
            for (int j = 0; j < m_x; ++j) {
                uint32_t ctr[4] = {(uint32_t)row_id, (uint32_t)(row_id >> 32), (uint32_t)j,
                                   0x41415344u};
                uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
                uint32_t rnd[4];
                orc_philox4x32_10(ctr, key, rnd);
                double u = (double)(rnd[0] >> 8) * (1.0 / 16777216.0);

                double W = 0.0;
                for (int i = 0; i < n_rem; ++i) W += exp(z[remaining[i]] - m);
                double target = u * W;
                double cum = 0.0;
                int pick = n_rem - 1;
                double margin = INFINITY;
                int decided = 0;
                for (int i = 0; i < n_rem; ++i) {
                    cum += exp(z[remaining[i]] - m);
                    if (i < n_rem - 1) { /* the last edge cannot change the pick */
                        double d = fabs(target - cum) / W;
                        if (d < margin) margin = d;
                    }
                    if (!decided && cum > target) { pick = i; decided = 1; }
                }
                if (draw_margin) draw_margin[r * m_x + j] = margin;
                chosen[n_chosen++] = remaining[pick];
                for (int i = pick; i + 1 < n_rem; ++i) remaining[i] = remaining[i + 1];
                --n_rem;
            }
        }
        for (int i = 0; i < n_chosen; ++i)
            if (extras) extras[r * m_x + i] = chosen[i];
        if (n_extras) n_extras[r] = (uint8_t)n_chosen;
    }
    free(z);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* n-gram draft retrieval                                                     */
/* ------------------------------------------------------------------------- */
int orc_retrieve_drafts(const int32_t *tokens, int64_t tok_stride, const int32_t *len,
                        const int32_t *prompt_len, int32_t B, int32_t n_min, int32_t n_max,
                        int32_t k, int32_t C, const int32_t *extras, const uint8_t *n_extras,
                        int32_t m_x, int64_t extras_stride, int32_t *drafts, int32_t *draft_len,
                        int32_t *src_pos, int32_t *n_cand, int32_t *key_len,
                        int32_t *draft_extras, uint8_t *strict)
{
    if (!tokens || !len || !prompt_len || B < 0) return -1;
    if (n_min < 1 || n_min > n_max || n_max > 8) return -1;
    if (k < 1 || k > 16 || C < 1 || C > 32) return -1;
    if (m_x < 0 || m_x > 4) return -1;
    if (draft_extras && m_x > 0 && (!extras || !n_extras)) return -1;

    for (int32_t b = 0; b < B; ++b) {
        const int32_t *tok = tokens + (size_t)b * (size_t)tok_stride;
        int32_t L = len[b];
        int32_t PL = prompt_len[b];
        if (L < 0 || L > tok_stride) L = 0; /* invalid length: nothing to retrieve */

        /* Algorithm 1: try the longest key first and stop at the first key
         * length that occurs earlier in the context.  A "hit" p is a position
         * whose preceding n tokens equal the last n tokens of the context and
         * that still has at least one continuation token (p <= L-1). */
        int32_t hits[32];
        int32_t n_hits = 0, used_n = 0;
        for (int32_t n = n_max; n >= n_min && n_hits == 0; --n) {
            if (n >= L) continue;
            /* scan from the end so that the latest occurrences come first */
            for (int32_t p = L - 1; p >= n && n_hits < C; --p) {
                int same = 1;
                for (int32_t i = 0; i < n; ++i)
                    if (tok[p - n + i] != tok[L - n + i]) { same = 0; break; }
                if (same) hits[n_hits++] = p;
            }
            if (n_hits > 0) used_n = n;
        }
        if (n_cand) n_cand[b] = n_hits;
        if (key_len) key_len[b] = used_n;

        for (int32_t c = 0; c < C; ++c) {
            size_t bc = (size_t)b * (size_t)C + (size_t)c;
            int32_t p = c < n_hits ? hits[c] : -1;
            int32_t dl = 0;
            if (p >= 0) dl = (L - p) < k ? (L - p) : k;
            if (src_pos) src_pos[bc] = p;
            if (draft_len) draft_len[bc] = dl;
            for (int32_t j = 0; j < k; ++j) {
                int in = j < dl;
                if (drafts) drafts[bc * k + j] = in ? tok[p + j] : -1;
                /* tokens copied from generated context are verified strictly (Sec. 3.3) */
                if (strict) strict[bc * k + j] = (uint8_t)(in && (p + j >= PL));
                if (draft_extras) {
                    for (int32_t e = 0; e < m_x; ++e) {
                        int32_t val = -1;
                        /* prefill row p+j-1 predicted the token at p+j; it has a
                         * next prompt token iff p+j <= PL-1 */
                        if (in && p + j <= PL - 1) {
                            size_t row = (size_t)b * (size_t)extras_stride + (size_t)(p + j - 1);
                            if (e < n_extras[row]) val = extras[row * m_x + e];
                        }
                        draft_extras[(bc * k + j) * m_x + e] = val;
                    }
                }
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* conditional verification                                                   */
/* ------------------------------------------------------------------------- */
int orc_verify(const void *logits, int dtype, int32_t B, int32_t C, int32_t k, int32_t V,
               int64_t row_stride, int64_t seq_stride, const int32_t *drafts,
               const int32_t *draft_len, const uint8_t *strict, double alpha, double beta,
               uint32_t flags, int32_t *accept_len, int32_t *best_cand, int32_t *next_token,
               double *row_entropy, double *row_pmax, int32_t *row_argmax, double *tok_p,
               double *tok_delta, double *tok_margin, uint32_t *near_count)
{
    if (!logits || !drafts || !draft_len || B < 0 || V <= 0) return -1;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return -1;
    if (k < 1 || k > 16 || C < 1 || C > 32) return -1;
    const int32_t R = 1 + C * k;
    if (row_stride < V || seq_stride < (int64_t)R * row_stride) return -1;

    double *z = (double *)malloc(sizeof(double) * 2 * (size_t)V);
    double *m = (double *)malloc(sizeof(double) * (size_t)R);
    double *S = (double *)malloc(sizeof(double) * (size_t)R);
    double *H = (double *)malloc(sizeof(double) * (size_t)R);
    int32_t *am = (int32_t *)malloc(sizeof(int32_t) * (size_t)R);
    if (!z || !m || !S || !H || !am) { free(z); free(m); free(S); free(H); free(am); return -2; }

    for (int32_t b = 0; b < B; ++b) {
        const char *seq = (const char *)logits + (size_t)b * (size_t)seq_stride * elt_bytes(dtype);
        /* the verification distribution of every node (Sec. 3.2: P_M(x | F(node))) */
        for (int32_t r = 0; r < R; ++r) {
            const char *row = seq + (size_t)r * (size_t)row_stride * elt_bytes(dtype);
            orc_widen_row(row, dtype, V, z);
            stats_of(z, V, z + V, &m[r], &S[r], &H[r], &am[r]);
            if (row_entropy) row_entropy[(size_t)b * R + r] = H[r];
            if (row_pmax) row_pmax[(size_t)b * R + r] = 1.0 / S[r];
            if (row_argmax) row_argmax[(size_t)b * R + r] = am[r];
        }

        int32_t best_c = 0, best_a = 0;
        uint32_t near = 0;
        for (int32_t c = 0; c < C; ++c) {
            size_t bc = (size_t)b * (size_t)C + (size_t)c;
            int32_t dl = draft_len[bc];
            if (dl < 0) dl = 0;
            if (dl > k) dl = k;
            int32_t a = 0;      /* leading tokens accepted so far */
            int rejected = 0;   /* Sec. 2.1: a rejection rejects everything after it */
            for (int32_t j = 1; j <= k; ++j) {
                size_t idx = bc * k + (size_t)(j - 1);
                double p = 0.0, delta = 0.0, margin = -1.0;
                if (j <= dl) {
                    int32_t rho = (j == 1) ? 0 : 1 + c * k + (j - 2);
                    const char *row = seq + (size_t)rho * (size_t)row_stride * elt_bytes(dtype);
                    int32_t t = drafts[idx];
                    int valid = t >= 0 && t < V;
                    double zt = valid ? widen_one(row, dtype, t) : 0.0;
                    p = valid ? exp(zt - m[rho]) / S[rho] : 0.0;
                    double Delta = 1.0 / S[rho];              /* Eq. 6 */
                    double thr = alpha * H[rho] + beta;       /* Eq. 5, natural log */
                    int is_strict = strict ? strict[idx] != 0 : 0;
                    int pass;
                    if (flags & ORC_VERIFY_NO_CLAMP) {        /* Eq. 3 / Eq. 4 without Delta */
                        delta = thr;
                        pass = valid && p >= delta;
                    } else {
                        delta = is_strict ? Delta : (thr < Delta ? thr : Delta);
                        /* equal logits are equal probabilities: a token that
                         * attains the row maximum always passes (Sec. 3.3) */
                        pass = valid && (p >= delta || zt == m[rho]);
                    }
                    if (!rejected) {
                        margin = fabs(p - delta);
                        if (margin < 1e-6) ++near;
                        if (pass) ++a; else rejected = 1;
                    }
                }
                if (tok_p) tok_p[idx] = p;
                if (tok_delta) tok_delta[idx] = delta;
                if (tok_margin) tok_margin[idx] = margin;
            }
            if (a > best_a) { best_a = a; best_c = c; } /* lowest c on ties */
        }
        if (accept_len) accept_len[b] = best_a;
        if (best_cand) best_cand[b] = best_c;
        if (next_token) {
            int32_t rho = best_a == 0 ? 0 : 1 + best_c * k + (best_a - 1);
            next_token[b] = am[rho];
        }
        if (near_count) near_count[b] = near;
    }
    free(z); free(m); free(S); free(H); free(am);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* top-k verification (the ablation of Sec. 4.4)                              */
/* ------------------------------------------------------------------------- */
int orc_verify_topk(const void *logits, int dtype, int32_t B, int32_t C, int32_t k, int32_t V,
                    int64_t row_stride, int64_t seq_stride, const int32_t *drafts,
                    const int32_t *draft_len, int32_t topk, int32_t *accept_len,
                    int32_t *best_cand, int32_t *next_token, int32_t *row_argmax,
                    int32_t *tok_rank)
{
    if (!logits || !drafts || !draft_len || B < 0 || V <= 0 || topk < 1) return -1;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return -1;
    if (k < 1 || k > 16 || C < 1 || C > 32) return -1;
    const int32_t R = 1 + C * k;
    if (row_stride < V || seq_stride < (int64_t)R * row_stride) return -1;

    double *z = (double *)malloc(sizeof(double) * (size_t)V);
    if (!z) return -2;
    for (int32_t b = 0; b < B; ++b) {
        const char *seq = (const char *)logits + (size_t)b * (size_t)seq_stride * elt_bytes(dtype);
        int32_t best_c = 0, best_a = 0;
        for (int32_t c = 0; c < C; ++c) {
            size_t bc = (size_t)b * (size_t)C + (size_t)c;
            int32_t dl = draft_len[bc];
            if (dl < 0) dl = 0;
            if (dl > k) dl = k;
            int32_t a = 0;
            int rejected = 0;
            for (int32_t j = 1; j <= k; ++j) {
                size_t idx = bc * k + (size_t)(j - 1);
                int32_t rk = -1;
                if (j <= dl) {
                    /* the draft token is accepted iff it is among the topk most likely tokens of
                     * the row that verifies it: fewer than topk tokens are strictly more likely */
                    int32_t rho = (j == 1) ? 0 : 1 + c * k + (j - 2);
                    const char *row = seq + (size_t)rho * (size_t)row_stride * elt_bytes(dtype);
                    int32_t t = drafts[idx];
                    int pass = 0;
                    if (t >= 0 && t < V) {
                        orc_widen_row(row, dtype, V, z);
                        rk = 0;
                        for (int32_t v = 0; v < V; ++v)
                            if (z[v] > z[t]) ++rk;
                        pass = rk < topk;
                    }
                    if (!rejected) { if (pass) ++a; else rejected = 1; }
                }
                if (tok_rank) tok_rank[idx] = rk;
            }
            if (a > best_a) { best_a = a; best_c = c; } /* lowest c on ties */
        }
        if (accept_len) accept_len[b] = best_a;
        if (best_cand) best_cand[b] = best_c;
        for (int32_t r = 0; r < R; ++r) {
            int need = row_argmax != NULL || (next_token && r == (best_a == 0 ? 0 : 1 + best_c * k + (best_a - 1)));
            if (!need) continue;
            const char *row = seq + (size_t)r * (size_t)row_stride * elt_bytes(dtype);
            orc_widen_row(row, dtype, V, z);
            int32_t am = 0;
            for (int32_t v = 1; v < V; ++v)
                if (z[v] > z[am]) am = v;
            if (row_argmax) row_argmax[(size_t)b * R + r] = am;
            if (next_token && r == (best_a == 0 ? 0 : 1 + best_c * k + (best_a - 1))) next_token[b] = am;
        }
    }
    free(z);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* draft tree and tree attention mask                                         */
/* ------------------------------------------------------------------------- */
int orc_build_tree(const int32_t *drafts, const int32_t *draft_len, const uint8_t *strict,
                   const int32_t *draft_extras, int32_t m_x, const int32_t *root_tok, int32_t B,
                   int32_t C, int32_t k, int32_t max_nodes, int32_t *node_token,
                   int32_t *node_parent, int32_t *node_depth, uint8_t *node_strict,
                   int32_t *n_nodes, uint32_t *mask, int32_t *cand_node)
{
    if (!drafts || !draft_len || B < 0) return -1;
    if (k < 1 || k > 16 || C < 1 || C > 32 || m_x < 0 || m_x > 4) return -1;
    if (max_nodes < 1 || max_nodes > 512) return -1;   /* 16 candidates x 8 tokens x (1 + 2 extras) + root = 385 (Sec. 3.2, Sec. 4.1) */
    const int32_t N = max_nodes, W = (N + 31) / 32;
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    int32_t *par = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    int32_t *dep = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    uint8_t *str = (uint8_t *)malloc((size_t)N);
    if (!tok || !par || !dep || !str) { free(tok); free(par); free(dep); free(str); return -2; }

    for (int32_t b = 0; b < B; ++b) {
        int32_t n = 1;
        tok[0] = root_tok ? root_tok[b] : -1; par[0] = -1; dep[0] = 0; str[0] = 0;
        int32_t cur[32];                       /* node at the end of each candidate's path so far */
        for (int32_t c = 0; c < C; ++c) cur[c] = 0;
        if (cand_node)
            for (int32_t i = 0; i < C * k; ++i) cand_node[(size_t)b * C * k + i] = -1;

        for (int32_t j = 1; j <= k; ++j) {                 /* layer by layer */
            int32_t next_cur[32];
            for (int32_t c = 0; c < C; ++c) next_cur[c] = -1;
            for (int32_t c = 0; c < C; ++c) {
                size_t bc = (size_t)b * C + c;
                int32_t dl = draft_len[bc] < 0 ? 0 : (draft_len[bc] > k ? k : draft_len[bc]);
                if (cur[c] < 0 || j > dl) continue;
                for (int32_t slot = 0; slot <= m_x; ++slot) {
                    int32_t t;
                    int is_strict;
                    if (slot == 0) {
                        t = drafts[bc * k + (j - 1)];
                        is_strict = strict ? strict[bc * k + (j - 1)] != 0 : 0;
                    } else {
                        if (!draft_extras) break;
                        t = draft_extras[(bc * k + (j - 1)) * m_x + (slot - 1)];
                        is_strict = 0;             /* extras are verified conditionally */
                    }
                    if (t < 0) { if (slot == 0) break; else continue; }  /* no token: the path ends here */
                    int32_t found = -1;
                    for (int32_t i = 1; i < n; ++i)
                        if (par[i] == cur[c] && tok[i] == t) { found = i; break; }
                    if (found < 0 && n < N) {
                        found = n++;
                        tok[found] = t; par[found] = cur[c]; dep[found] = j; str[found] = (uint8_t)is_strict;
                    } else if (found >= 0 && !is_strict) {
                        str[found] = 0;            /* one conditional source is enough */
                    }
                    if (slot == 0) {
                        next_cur[c] = found;       /* -1 if the node budget is exhausted */
                        if (cand_node) cand_node[bc * k + (j - 1)] = found;
                    }
                }
            }
            for (int32_t c = 0; c < C; ++c) cur[c] = next_cur[c];
        }

        if (n_nodes) n_nodes[b] = n;
        for (int32_t i = 0; i < N; ++i) {
            size_t bi = (size_t)b * N + i;
            int used = i < n;
            if (node_token) node_token[bi] = used ? tok[i] : -1;
            if (node_parent) node_parent[bi] = used ? par[i] : -1;
            if (node_depth) node_depth[bi] = used ? dep[i] : 0;
            if (node_strict) node_strict[bi] = used ? str[i] : 0;
            if (mask) {
                for (int32_t w = 0; w < W; ++w) mask[bi * W + w] = 0;
                if (used)
                    for (int32_t a = i; a >= 0; a = par[a]) mask[bi * W + a / 32] |= 1u << (a % 32);
            }
        }
    }
    free(tok); free(par); free(dep); free(str);
    return 0;
}

int orc_verify_tree(const void *logits, int dtype, int32_t B, int32_t N, int32_t V,
                    int64_t row_stride, int64_t seq_stride, const int32_t *node_token,
                    const int32_t *node_parent, const uint8_t *node_strict,
                    const int32_t *n_nodes, double alpha, double beta, uint32_t flags,
                    int32_t *accept_len, int32_t *best_node, int32_t *accept_path,
                    int32_t *next_token, double *row_entropy, double *row_pmax,
                    int32_t *row_argmax, double *node_p, double *node_delta, double *node_margin,
                    uint32_t *near_count)
{
    if (!logits || !node_token || !node_parent || !n_nodes || B < 0 || V <= 0) return -1;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return -1;
    if (N < 1 || N > 512 || row_stride < V || seq_stride < (int64_t)N * row_stride) return -1;

    double *z = (double *)malloc(sizeof(double) * 2 * (size_t)V);
    double *m = (double *)malloc(sizeof(double) * (size_t)N);
    double *S = (double *)malloc(sizeof(double) * (size_t)N);
    double *H = (double *)malloc(sizeof(double) * (size_t)N);
    int32_t *am = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    int *ok = (int *)malloc(sizeof(int) * (size_t)N);      /* node and all its ancestors pass */
    int32_t *depth = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    if (!z || !m || !S || !H || !am || !ok || !depth) {
        free(z); free(m); free(S); free(H); free(am); free(ok); free(depth);
        return -2;
    }
    for (int32_t b = 0; b < B; ++b) {
        const char *seq = (const char *)logits + (size_t)b * (size_t)seq_stride * elt_bytes(dtype);
        int32_t n = n_nodes[b] < 1 ? 1 : (n_nodes[b] > N ? N : n_nodes[b]);
        for (int32_t i = 0; i < N; ++i) {
            size_t bi = (size_t)b * N + i;
            if (i < n) {
                const char *row = seq + (size_t)i * (size_t)row_stride * elt_bytes(dtype);
                orc_widen_row(row, dtype, V, z);
                stats_of(z, V, z + V, &m[i], &S[i], &H[i], &am[i]);
            }
            if (row_entropy) row_entropy[bi] = i < n ? H[i] : 0.0;
            if (row_pmax) row_pmax[bi] = i < n ? 1.0 / S[i] : 0.0;
            if (row_argmax) row_argmax[bi] = i < n ? am[i] : -1;
        }
        ok[0] = 1; depth[0] = 0;
        int32_t best = 0;
        uint32_t near = 0;
        for (int32_t i = 1; i < N; ++i) {
            size_t bi = (size_t)b * N + i;
            double p = 0.0, delta = 0.0, margin = -1.0;
            if (i < n) {
                int32_t par = node_parent[bi];
                int valid_par = par >= 0 && par < i;       /* parents precede their children */
                int32_t t = node_token[bi];
                int valid = valid_par && t >= 0 && t < V;
                int pass = 0;
                if (valid_par) {
                    const char *row = seq + (size_t)par * (size_t)row_stride * elt_bytes(dtype);
                    double zt = valid ? widen_one(row, dtype, t) : 0.0;
                    p = valid ? exp(zt - m[par]) / S[par] : 0.0;
                    double Delta = 1.0 / S[par];
                    double thr = alpha * H[par] + beta;
                    int is_strict = node_strict ? node_strict[bi] != 0 : 0;
                    if (flags & ORC_VERIFY_NO_CLAMP) {
                        delta = thr;
                        pass = valid && p >= delta;
                    } else {
                        delta = is_strict ? Delta : (thr < Delta ? thr : Delta);
                        pass = valid && (p >= delta || zt == m[par]);
                    }
                    depth[i] = depth[par] + 1;
                    if (ok[par]) {                         /* the node is reached: it is evaluated */
                        margin = fabs(p - delta);
                        if (margin < 1e-6) ++near;
                    }
                    ok[i] = ok[par] && pass;
                } else {
                    ok[i] = 0; depth[i] = 0;
                }
                if (ok[i] && depth[i] > depth[best]) best = i;   /* deepest; lowest index on ties */
            }
            if (node_p) node_p[bi] = p;
            if (node_delta) node_delta[bi] = delta;
            if (node_margin) node_margin[bi] = margin;
        }
        if (node_p) node_p[(size_t)b * N] = 0.0;
        if (node_delta) node_delta[(size_t)b * N] = 0.0;
        if (node_margin) node_margin[(size_t)b * N] = -1.0;
        if (accept_len) accept_len[b] = depth[best];
        if (best_node) best_node[b] = best;
        if (next_token) next_token[b] = am[best];
        if (near_count) near_count[b] = near;
        if (accept_path) {
            for (int32_t d = 0; d < 16; ++d) accept_path[(size_t)b * 16 + d] = -1;
            for (int32_t a = best; a > 0; a = node_parent[(size_t)b * N + a])
                if (depth[a] >= 1 && depth[a] <= 16) accept_path[(size_t)b * 16 + depth[a] - 1] = a;
        }
    }
    free(z); free(m); free(S); free(H); free(am); free(ok); free(depth);
    return 0;
}
