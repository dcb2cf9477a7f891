// Per-token decision and accept-prefix scan of conditional verification (Sec. 3.3, Eq. 4-6).
//
// One workgroup per sequence.  First the wave partials that the sweep left in the workspace
// are merged per row (maximum, sum of exponentials, entropy, greedy pick), a group of lanes per
// row, into LDS.  Then, with 16 lanes per candidate (k <= 16 draft tokens), four
// candidates per wave and up to 32 candidates per workgroup, each lane decides its token; a wave
// ballot turns the decisions of a candidate into a bit field whose trailing ones are the
// accepted prefix (the cascade rule of Sec. 2.1); one thread then takes the longest candidate.
#pragma once

#include "row_finish.hip.h"

namespace aasd {

constexpr int kTailBlock = 16 * AASD_MAX_CANDIDATES;  // 512

struct VerifyTailParams {
    const void* logits;
    int32_t B, C, k, V;
    int64_t row_stride, seq_stride;
    const int32_t* drafts;
    const int32_t* draft_len;
    const uint8_t* strict;
    float alpha, beta;
    uint32_t flags;
    int32_t* accept_len;
    int32_t* best_cand;
    int32_t* next_token;
    float* tok_p;
    float* tok_delta;
    uint32_t* near_count;
    float* row_entropy;   // optional [B, R]
    float* row_pmax;      // optional [B, R]
    int32_t* row_argmax;  // optional [B, R]
    const WavePartial* partials;  // [B * R][npart]
    int32_t npart;
};

constexpr int kMaxVerifyRows = 1 + AASD_MAX_CANDIDATES * AASD_MAX_DRAFT;  // 513

template <int DT>
__global__ __launch_bounds__(kTailBlock) void verify_tail_kernel(VerifyTailParams p)
{
    __shared__ int lead[AASD_MAX_CANDIDATES];
    __shared__ unsigned near_c[AASD_MAX_CANDIDATES];
    __shared__ float4 stats[kMaxVerifyRows];  // per row {max logit, S, H, bits of argmax}

    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int cand = tid >> 4, j = tid & 15;  // j: 0-based position in the draft
    const int C = p.C, k = p.k, R = 1 + C * k;

    // ---- statistics of the sequence's rows from the sweep's partials ----
    // G lanes per row (G = npart rounded up to a power of two), 64/G rows per wave at a time
    {
        int G = 1;
        while (G < p.npart) G <<= 1;
        const int rows_per_pass = kTailBlock / G;
        const int sub = tid / G, s = tid - sub * G;  // row slot of this lane, partial index within the row
        for (int r0 = 0; r0 < R; r0 += rows_per_pass) {
            const int r = r0 + sub;
            const bool have_row = r < R;
            const int64_t row = (int64_t)b * R + (have_row ? r : 0);
            WavePartial wp;
            wp.m = -INFINITY; wp.S = 0.f; wp.T = 0.f; wp.code = 0x7fffffff;
            if (have_row && s < p.npart) wp = p.partials[row * p.npart + s];
            float m = wp.m;
            for (int o = 1; o < G; o <<= 1) m = fmaxf(m, __shfl_xor(m, o));
            const bool live = wp.S > 0.f;
            float dl2 = 0.f, f = 0.f;
            if (live) partial_scale(wp.m, m, dl2, f);
            float S = live ? wp.S * f : 0.f;
            float T2 = live ? (wp.T + dl2 * wp.S) * f : 0.f;
            int code = live && wp.m == m ? wp.code : 0x7fffffff;
            for (int o = 1; o < G; o <<= 1) {
                S += __shfl_xor(S, o);
                T2 += __shfl_xor(T2, o);
                code = min(code, __shfl_xor(code, o));
            }
            if (have_row && s == 0) {
                const RowShape rs = row_shape<DT>(p.logits, (int64_t)b * p.seq_stride + (int64_t)r * p.row_stride, p.V);
                int am = 0;
                if ((unsigned)code < (unsigned)p.V) {
                    am = code;
                    const int len = (code >= rs.head && code < rs.tail0) ? Elt<DT>::kPerVec : 1;
                    for (int e = 0; e < len; ++e)
                        if (load_elt<DT>(rs.base, code + e) == m) { am = code + e; break; }
                }
                const float H = entropy_from_sums(S, T2);
                stats[r] = make_float4(m, S, H, __int_as_float(am));
                if (p.row_entropy) p.row_entropy[row] = H;
                if (p.row_pmax) p.row_pmax[row] = 1.0f / S;
                if (p.row_argmax) p.row_argmax[row] = am;
            }
        }
    }
    __syncthreads();

    int dl = 0;
    if (cand < C) {
        dl = p.draft_len[(size_t)b * C + cand];
        dl = dl < 0 ? 0 : (dl > k ? k : dl);
    }
    const bool slot = cand < C && j < k;
    const bool in = slot && j < dl;
    const size_t idx = ((size_t)b * C + (cand < C ? cand : 0)) * k + (j < k ? j : 0);

    bool pass = false, near = false;
    float pf = 0.f, df = 0.f;
    if (in) {
        const int rho = (j == 0) ? 0 : 1 + cand * k + (j - 1);  // the row that follows the previous token
        const int t = p.drafts[idx];
        const float4 st = stats[rho];
        const double m = (double)st.x, S = (double)st.y, H = (double)st.z;
        const bool valid = t >= 0 && t < p.V;
        float zt = 0.f;
        if (valid) zt = load_elt<DT>(p.logits, (int64_t)b * p.seq_stride + (int64_t)rho * p.row_stride + t);
        const double pr = valid ? exp((double)zt - m) / S : 0.0;
        const double Delta = 1.0 / S;                                // Eq. 6
        const double thr = (double)p.alpha * H + (double)p.beta;     // Eq. 5
        double delta;
        if (p.flags & AASD_VERIFY_NO_CLAMP) {
            delta = thr;
            pass = valid && pr >= delta;
        } else {
            const bool is_strict = p.strict != nullptr && p.strict[idx] != 0;
            delta = is_strict ? Delta : fmin(thr, Delta);
            pass = valid && (pr >= delta || zt == st.x);             // Eq. 4; ties with the maximum pass
        }
        near = fabs(pr - delta) < 1e-6;
        pf = (float)pr;
        df = (float)delta;
    }
    if (slot) {
        if (p.tok_p) p.tok_p[idx] = pf;
        if (p.tok_delta) p.tok_delta[idx] = df;
    }

    // accept-prefix: trailing ones of the candidate's 16-bit field
    const unsigned shift = (unsigned)(lane >> 4) * 16u;
    const unsigned field = (unsigned)((__ballot(pass) >> shift) & 0xffffull);
    const unsigned nfield = (unsigned)((__ballot(near && in) >> shift) & 0xffffull);
    const int a = __ffs(~field) - 1;  // bit 16 of ~field is always set, so a <= 16; a <= dl because bit dl is clear
    if (j == 0 && cand < C) {
        lead[cand] = a;
        // evaluated tokens: the accepted ones and the first failure
        const unsigned ev = (a + 1 >= 32) ? 0xffffffffu : ((1u << (a + 1)) - 1u);
        near_c[cand] = (unsigned)__popc(nfield & ev);
    }
    __syncthreads();
    if (tid == 0) {
        int best_a = 0, best_c = 0;
        unsigned near_total = 0;
        for (int c = 0; c < C; ++c) {
            if (lead[c] > best_a) { best_a = lead[c]; best_c = c; }  // lowest index on ties
            near_total += near_c[c];
        }
        const int rho = best_a == 0 ? 0 : 1 + best_c * k + (best_a - 1);
        p.accept_len[b] = best_a;
        p.best_cand[b] = best_c;
        p.next_token[b] = __float_as_int(stats[rho].w);
        if (p.near_count) p.near_count[b] = near_total;
    }
}

}  // namespace aasd
