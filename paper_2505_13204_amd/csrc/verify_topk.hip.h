// Top-k verification, the ablation of Sec. 4.4: a draft token is accepted iff fewer than K tokens of the row
// that verifies it have a strictly larger logit, i.e. iff its logit is at least the K-th largest of the row.
// The K-th largest logit of every row comes from the alignment sweep's candidate lists (with the "next token"
// at -inf every row lists the chunks that can hold its top-K).
#pragma once

#include "row_finish.hip.h"

namespace aasd {

struct RowKthParams {
    AlignFinishParams f;   // logits, V, row/seq strides via (rows_per_seq, seq_stride), partials, lists, npart, c = K
    int32_t rows_per_seq;
    int64_t seq_stride;
    float* kth;            // [rows] K-th largest logit (-inf if the row has fewer than K finite logits)
    int32_t* argmax;       // [rows]
};

// One wave per row: merge the partials, find the greedy pick, select the exact top-K from the listed chunks.
template <int DT>
__global__ __launch_bounds__(kFinishBlock) void row_kth_kernel(RowKthParams q)
{
    __shared__ float cand_z[kFinishBlock / kWave][kFinishCandCap];
    __shared__ int cand_i[kFinishBlock / kWave][kFinishCandCap];
    __shared__ unsigned cand_n[kFinishBlock / kWave];

    const AlignFinishParams& p = q.f;
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * (kFinishBlock / kWave) + wid;
    if (row >= p.rows) return;  // whole wave; the kernel has no barrier
    const int V = p.V, np = p.npart;

    WavePartial wp;
    wp.m = -INFINITY; wp.S = 0.f; wp.T = 0.f; wp.code = 0x7fffffff; wp.cnt = 0; wp.nlist = 0; wp.thr2 = -INFINITY;
    if (lane < np) wp = p.partials[row * np + lane];
    const float m = wave_max(wp.m);
    float thr2 = wave_max(wp.thr2);
    const int code = wave_min(wp.S > 0.f && wp.m == m ? wp.code : 0x7fffffff);
    const int64_t off = (row / q.rows_per_seq) * q.seq_stride + (row % q.rows_per_seq) * p.row_stride;
    const RowShape rs = row_shape<DT>(p.logits, off, V);
    const int am = wave_first_max<DT>(rs, V, code, m, lane);

    float kz[AASD_MAX_CANDSET];
    int ki[AASD_MAX_CANDSET];
    int nK = 0;
#pragma unroll
    for (int i = 0; i < AASD_MAX_CANDSET; ++i) { kz[i] = 0.f; ki[i] = -1; }
    if (m > -INFINITY)
        row_topc_from_lists<DT>(p, rs, row, wp, -INFINITY, thr2, lane, cand_z[wid], cand_i[wid], &cand_n[wid], kz, ki, nK);
    if (lane == 0) {
        float kth = -INFINITY;
#pragma unroll
        for (int i = 0; i < AASD_MAX_CANDSET; ++i)
            if (i == p.c - 1 && nK >= p.c) kth = kz[i];
        q.kth[row] = kth;
        q.argmax[row] = am;
    }
}

struct VerifyTopkTailParams {
    const void* logits;
    int32_t B, C, k, V;
    int64_t row_stride, seq_stride;
    const int32_t* drafts;
    const int32_t* draft_len;
    const float* kth;        // [B * R]
    const int32_t* argmax;   // [B * R]
    int32_t* accept_len;
    int32_t* best_cand;
    int32_t* next_token;
    int32_t* row_argmax;     // [B, R] or null
    uint8_t* tok_pass;       // [B, C, k] or null: 1 = within the top K, 0 = not (or beyond draft_len)
};

// One wave per sequence, a lane per candidate: cascade over its tokens, then the longest candidate.
template <int DT>
__global__ __launch_bounds__(kWave) void verify_topk_tail_kernel(VerifyTopkTailParams p)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int R = 1 + p.C * p.k;
    const char* seq = (const char*)p.logits + (size_t)b * (size_t)p.seq_stride * Elt<DT>::kBytes;
    int a = 0;
    if (lane < p.C) {
        const size_t bc = (size_t)b * p.C + lane;
        int dl = p.draft_len[bc];
        dl = dl < 0 ? 0 : (dl > p.k ? p.k : dl);
        bool alive = true;
        for (int j = 1; j <= p.k; ++j) {
            bool pass = false;
            if (j <= dl) {
                const int rho = j == 1 ? 0 : 1 + lane * p.k + (j - 2);
                const int t = p.drafts[bc * p.k + (j - 1)];
                if (t >= 0 && t < p.V) {
                    const float zt = load_elt<DT>(seq + (size_t)rho * (size_t)p.row_stride * Elt<DT>::kBytes, t);
                    pass = zt >= p.kth[(size_t)b * R + rho];
                }
                if (alive && pass) ++a; else alive = false;
            }
            if (p.tok_pass) p.tok_pass[bc * p.k + (j - 1)] = pass ? 1 : 0;
        }
    }
    // longest candidate, lowest index on ties
    int key = lane < p.C ? (a << 8) | (255 - lane) : -1;
    key = wave_max(key);
    const int best_a = key >> 8, best_c = 255 - (key & 255);
    if (lane == 0) {
        p.accept_len[b] = best_a;
        p.best_cand[b] = best_c;
        const int rho = best_a == 0 ? 0 : 1 + best_c * p.k + (best_a - 1);
        p.next_token[b] = p.argmax[(size_t)b * R + rho];
    }
    if (p.row_argmax)
        for (int r = lane; r < R; r += kWave) p.row_argmax[(size_t)b * R + r] = p.argmax[(size_t)b * R + r];
}

}  // namespace aasd
