// Fused single-pass row sweep: softmax normaliser, entropy, greedy pick and (for prefill
// rows) rank of the next prompt token and the candidate tokens ranked above it.
//
// One workgroup owns one logits row and reads it from HBM exactly once with 16-byte loads.
// Per element the sweep does: unpack, one FMA into the log2 domain, one hardware exp2, one add
// (sum of exponentials) and one FMA (sum of exponent * exponential, which gives the entropy as
// ln S - T/S, Eq. 5 of Sec. 3.3 rewritten so that both terms are non-negative).  Everything
// that would cost more per element is done per 16-byte chunk instead:
//   - the running maximum and the position of the chunk that set it (the greedy pick is then
//     found by re-reading that one chunk),
//   - the reference exponent of the running sums, which is only moved when a chunk exceeds it
//     by more than 44 nats (floating point does not care about a common scale),
//   - one chunk maximum per chunk parked in LDS, from which the few chunks that can hold a
//     top-c token are found after the sweep and re-read (Sec. 3.2 / Fig. 2 need the tokens
//     ranked above the prompt token, not a full sort).
#pragma once

#include "common.hip.h"

namespace aasd {

constexpr int kNumAcc = 4;      // independent partial sums per lane (shorter rounding chains, more ILP)
constexpr int kCandCap = 256;   // LDS candidate buffer entries per row
constexpr float kRefSlack = 44.0f;  // nats a chunk may exceed the reference exponent before it is moved

struct SweepParams {
    const void* logits;
    int32_t V;
    int64_t row_stride;    // elements
    int64_t seq_stride;    // elements, verification only (rows_per_seq rows per sequence)
    int32_t rows_per_seq;  // 1 for prefill rows
    // alignment sampling
    const int32_t* next_tok;
    int32_t m_x, c, mode;
    uint64_t seed, row_id_base;
    int32_t* argmax;
    uint8_t* misaligned;
    float* entropy;
    float* p_next;
    float* p_max;
    int32_t* rank;
    int32_t* extras;
    uint8_t* n_extras;
    uint32_t* near_count;
    int32_t cm_enabled;  // chunk maxima fit in LDS
    // verification
    float4* stats;  // [rows] {max logit, S, H, bits of argmax}
    float* row_entropy;
    float* row_pmax;
    int32_t* row_argmax;
};

// Running state of one lane.
struct LaneAcc {
    float vmax;   // largest logit seen
    int code;     // index of the first element of the chunk that set vmax
    float r2;     // reference exponent (log2 units) of s and t
    float rlim;   // chunk maximum above which the reference must move
    float s[kNumAcc];  // sum of 2^(z*log2e - r2)
    float t[kNumAcc];  // sum of (z*log2e - r2) * 2^(z*log2e - r2)
    unsigned cnt_u;    // elements with z > z_next, counted wave-wide (same value in every lane)
    unsigned cnt_l;    // the same for elements handled under divergence (per lane)
};

__device__ __forceinline__ void lane_acc_init(LaneAcc& a)
{
    a.vmax = -INFINITY; a.code = 0x7fffffff;
    a.r2 = kNegHuge; a.rlim = -INFINITY;
#pragma unroll
    for (int i = 0; i < kNumAcc; ++i) { a.s[i] = 0.f; a.t[i] = 0.f; }
    a.cnt_u = 0; a.cnt_l = 0;
}

// Fold N consecutive elements (first index idx0) into the lane state.
// CLAMP: exponents are floored at a finite value so that -inf logits contribute exactly zero.
// COUNT: count elements above zcmp.  UNIFORM: all 64 lanes are active (ballot counting).
template <int N, bool CLAMP, bool COUNT, bool UNIFORM>
__device__ __forceinline__ float accumulate(LaneAcc& a, const float (&z)[N], int idx0, float zcmp)
{
    float cmax = z[0];
#pragma unroll
    for (int e = 1; e < N; ++e) cmax = fmaxf(cmax, z[e]);
    a.code = cmax > a.vmax ? idx0 : a.code;
    a.vmax = fmaxf(a.vmax, cmax);
    if (cmax > a.rlim) {  // rare: first chunk of the lane, or a jump of more than kRefSlack nats
        float nr2 = cmax * kLog2e;
        if (CLAMP) nr2 = fmaxf(nr2, kNegHuge);
        const float d = a.r2 - nr2;
        const float f = __builtin_amdgcn_exp2f(d);
#pragma unroll
        for (int i = 0; i < kNumAcc; ++i) {
            a.t[i] = (a.t[i] + d * a.s[i]) * f;
            a.s[i] *= f;
        }
        a.r2 = nr2;
        a.rlim = cmax + kRefSlack;
    }
    const float nr = -a.r2;
#pragma unroll
    for (int e = 0; e < N; ++e) {
        float d2 = fmaf(z[e], kLog2e, nr);
        if (CLAMP) d2 = fmaxf(d2, kNegHuge);
        const float ex = __builtin_amdgcn_exp2f(d2);
        a.s[e % kNumAcc] += ex;
        a.t[e % kNumAcc] = fmaf(d2, ex, a.t[e % kNumAcc]);
        if (COUNT) {
            if (UNIFORM) a.cnt_u += (unsigned)__popcll(__ballot(z[e] > zcmp));
            else a.cnt_l += (z[e] > zcmp) ? 1u : 0u;
        }
    }
    return cmax;
}

// Where a row's bytes sit relative to 16-byte boundaries.
struct RowShape {
    const char* base;   // first element
    const u32x4* vbase; // first aligned 16-byte vector
    int head;           // elements before vbase
    int nvec;           // full vectors
    int tail0;          // index of the first element after the vectors
};

template <int DT>
__device__ __forceinline__ RowShape row_shape(const void* logits, int64_t elt_offset, int V)
{
    RowShape s;
    s.base = (const char*)logits + elt_offset * Elt<DT>::kBytes;
    const uintptr_t addr = (uintptr_t)s.base;
    int head = (int)(((16u - (unsigned)(addr & 15u)) & 15u) / Elt<DT>::kBytes);
    s.head = head < V ? head : V;
    s.nvec = (V - s.head) / Elt<DT>::kPerVec;
    s.tail0 = s.head + s.nvec * Elt<DT>::kPerVec;
    s.vbase = (const u32x4*)(s.base + (size_t)s.head * Elt<DT>::kBytes);
    return s;
}

template <int DT>
__device__ __forceinline__ void cm_store(unsigned char* cm, int vec, float cmax)
{
    if constexpr (DT == AASD_BF16) ((uint16_t*)cm)[vec] = (uint16_t)(__float_as_uint(cmax) >> 16);
    else ((float*)cm)[vec] = cmax;
}
template <int DT>
__device__ __forceinline__ float cm_load(const unsigned char* cm, int vec)
{
    if constexpr (DT == AASD_BF16) return bits_to_float((uint32_t)((const uint16_t*)cm)[vec] << 16);
    else return ((const float*)cm)[vec];
}

// The single HBM pass of one lane over its share of the row: vectors tid, tid+BLOCK, ...
// loaded U at a time with the next batch in flight while the current one is folded in.
template <int DT, bool CLAMP, bool COUNT, int BLOCK, int U>
__device__ __forceinline__ void sweep_lane(LaneAcc& a, const RowShape& rs, int V, int tid, float zcmp,
                                           bool store_cm, unsigned char* cm)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    lane_acc_init(a);

    if (tid < rs.head) {
        const float z1[1] = {load_elt<DT>(rs.base, tid)};
        accumulate<1, CLAMP, COUNT, false>(a, z1, tid, zcmp);
    }

    // Full batches of BLOCK*U vectors.  Two register buffers alternate: while one batch is folded
    // in, the loads of the next are in flight, and no buffer is ever copied.  The batch base is
    // uniform (scalar registers), the lane offset a 32-bit byte offset.
    constexpr int kPerSuper = BLOCK * U;
    constexpr unsigned kBatchBytes = (unsigned)kPerSuper * 16u;
    const int nsuper = rs.nvec / kPerSuper;
    const char* const sbase = (const char*)rs.vbase;
    const unsigned voff = (unsigned)tid * 16u;
    auto load_batch = [&](u32x4 (&buf)[U], int it) {
        const char* b = sbase + (size_t)it * kBatchBytes;
#pragma unroll
        for (int u = 0; u < U; ++u) buf[u] = *(const u32x4*)(b + (voff + (unsigned)u * (BLOCK * 16u)));
    };
    auto fold_batch = [&](const u32x4 (&buf)[U], int it) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float z[EPV];
            unpack<DT>(buf[u], z);
            const int vec = (it * U + u) * BLOCK + tid;
            const float cmax = accumulate<EPV, CLAMP, COUNT, true>(a, z, rs.head + vec * EPV, zcmp);
            if (store_cm) cm_store<DT>(cm, vec, cmax);
        }
    };
    u32x4 bufA[U], bufB[U];
    int it = 0;
    if (nsuper > 0) load_batch(bufA, 0);
    while (it + 1 < nsuper) {
        load_batch(bufB, it + 1);
        fold_batch(bufA, it);
        if (it + 2 < nsuper) load_batch(bufA, it + 2);
        fold_batch(bufB, it + 1);
        it += 2;
    }
    if (it < nsuper) fold_batch(bufA, it);
    {   // fewer than BLOCK*U vectors remain
        const int vec0 = nsuper * kPerSuper + tid;
        u32x4 rem[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (vec0 + u * BLOCK < rs.nvec) rem[u] = rs.vbase[vec0 + u * BLOCK];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int vec = vec0 + u * BLOCK;
            if (vec < rs.nvec) {
                float z[EPV];
                unpack<DT>(rem[u], z);
                const float cmax = accumulate<EPV, CLAMP, COUNT, false>(a, z, rs.head + vec * EPV, zcmp);
                if (store_cm) cm_store<DT>(cm, vec, cmax);
            }
        }
    }
    if (tid < V - rs.tail0) {
        const int idx = rs.tail0 + tid;
        const float z1[1] = {load_elt<DT>(rs.base, idx)};
        accumulate<1, CLAMP, COUNT, false>(a, z1, idx, zcmp);
    }
}

// LDS used by the row reductions of one workgroup.
template <int NW>
struct SweepShared {
    float gmax[NW][8];   // maxima of the 8-lane groups of every wave
    float S[NW];
    float T[NW];
    int code[NW];
    unsigned cnt[NW];
    unsigned ncand;
    float cand_z[kCandCap];
    int cand_i[kCandCap];
    float fb_z[2][NW];   // exact fallback selection, double-buffered by round
    int fb_i[2][NW];
};

// Exact top-c by c full re-reads of the row; only used when the candidate buffer overflowed
// (hundreds of tokens tied near the top).  All threads of the block must call it.
template <int DT, int BLOCK>
__device__ void topc_by_rescan(const RowShape& rs, int V, int tid, float znext, int c,
                               SweepShared<BLOCK / kWave>& sh, float (&kz)[AASD_MAX_CANDSET],
                               int (&ki)[AASD_MAX_CANDSET], int& nK)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    constexpr int NW = BLOCK / kWave;
    const int lane = tid & 63, wid = tid >> 6;
    float pz = INFINITY;
    int pi = -1;
    nK = 0;
    for (int r = 0; r < c; ++r) {
        float bz = -INFINITY;
        int bi = 0x7fffffff;
        auto consider = [&](float z, int idx) {
            const bool after_prev = (r == 0) || z < pz || (z == pz && idx > pi);
            if (z > znext && after_prev && better(z, idx, bz, bi)) { bz = z; bi = idx; }
        };
        if (tid < rs.head) consider(load_elt<DT>(rs.base, tid), tid);
        for (int vec = tid; vec < rs.nvec; vec += BLOCK) {
            float z[EPV];
            unpack<DT>(rs.vbase[vec], z);
#pragma unroll
            for (int e = 0; e < EPV; ++e) consider(z[e], rs.head + vec * EPV + e);
        }
        if (tid < V - rs.tail0) consider(load_elt<DT>(rs.base, rs.tail0 + tid), rs.tail0 + tid);
        wave_best(bz, bi);
        if (lane == 0) { sh.fb_z[r & 1][wid] = bz; sh.fb_i[r & 1][wid] = bi; }
        __syncthreads();
        bz = sh.fb_z[r & 1][0]; bi = sh.fb_i[r & 1][0];
#pragma unroll
        for (int w = 1; w < NW; ++w)
            if (better(sh.fb_z[r & 1][w], sh.fb_i[r & 1][w], bz, bi)) { bz = sh.fb_z[r & 1][w]; bi = sh.fb_i[r & 1][w]; }
        if (bi == 0x7fffffff) break;  // same decision in every thread
        pz = bz; pi = bi;
#pragma unroll
        for (int q = 0; q < AASD_MAX_CANDSET; ++q)
            if (q == r) { kz[q] = bz; ki[q] = bi; }
        nK = r + 1;
    }
}

// Top-c of the buffered candidates by wave 0 (c rounds of "best remaining").
__device__ __forceinline__ void topc_from_buffer(const float* cand_z, const int* cand_i, int n, int lane, int c,
                                                 float (&kz)[AASD_MAX_CANDSET], int (&ki)[AASD_MAX_CANDSET], int& nK)
{
    constexpr int kPerLane = kCandCap / kWave;
    float lz[kPerLane];
    int li[kPerLane];
#pragma unroll
    for (int q = 0; q < kPerLane; ++q) {
        const int e = lane + q * kWave;
        lz[q] = e < n ? cand_z[e] : -INFINITY;
        li[q] = e < n ? cand_i[e] : 0x7fffffff;
    }
    nK = 0;
    for (int r = 0; r < c; ++r) {
        float bz = lz[0];
        int bi = li[0];
#pragma unroll
        for (int q = 1; q < kPerLane; ++q)
            if (better(lz[q], li[q], bz, bi)) { bz = lz[q]; bi = li[q]; }
        wave_best(bz, bi);
        if (bi == 0x7fffffff) break;
#pragma unroll
        for (int q = 0; q < kPerLane; ++q)
            if (li[q] == bi) { lz[q] = -INFINITY; li[q] = 0x7fffffff; }
#pragma unroll
        for (int q = 0; q < AASD_MAX_CANDSET; ++q)
            if (q == r) { kz[q] = bz; ki[q] = bi; }
        nK = r + 1;
    }
}

// Choose the extra draft tokens of a misaligned row from its ranked candidate list K
// (Sec. 3.2; reading: TOP takes the best-ranked, SAMPLE draws without replacement).
__device__ __forceinline__ void choose_extras(const SweepParams& p, int64_t row, float m,
                                              const float (&kz)[AASD_MAX_CANDSET],
                                              const int (&ki)[AASD_MAX_CANDSET], int nK)
{
    int chosen[AASD_MAX_EXTRAS];
    int n_chosen = 0;
    if (p.mode == AASD_EXTRAS_TOP || nK <= p.m_x) {
        for (int i = 0; i < nK && i < p.m_x; ++i) chosen[n_chosen++] = ki[i];
    } else {
        float w[AASD_MAX_CANDSET];
        int id[AASD_MAX_CANDSET];
        int n_rem = nK;
        for (int i = 0; i < nK; ++i) { w[i] = expf(kz[i] - m); id[i] = ki[i]; }
        const uint64_t row_id = p.row_id_base + (uint64_t)row;
        unsigned near = 0;
        for (int j = 0; j < p.m_x; ++j) {
            uint32_t rnd[4];
            philox4x32_10((uint32_t)row_id, (uint32_t)(row_id >> 32), (uint32_t)j, 0x41415344u,
                          (uint32_t)p.seed, (uint32_t)(p.seed >> 32), rnd);
            const float u = (float)(rnd[0] >> 8) * (1.0f / 16777216.0f);  // 24 bits: exact in fp32
            float W = 0.f;
            for (int i = 0; i < n_rem; ++i) W += w[i];
            const float target = u * W;
            float cum = 0.f, margin = INFINITY;
            int pick = n_rem - 1;
            bool decided = false;
            for (int i = 0; i < n_rem; ++i) {
                cum += w[i];
                if (i < n_rem - 1) margin = fminf(margin, fabsf(target - cum));
                if (!decided && cum > target) { pick = i; decided = true; }
            }
            if (margin < 1e-6f * W) ++near;
            chosen[n_chosen++] = id[pick];
            for (int i = pick; i + 1 < n_rem; ++i) { w[i] = w[i + 1]; id[i] = id[i + 1]; }
            --n_rem;
        }
        if (near && p.near_count) atomicAdd(p.near_count, near);
    }
    for (int j = 0; j < p.m_x; ++j) p.extras[row * p.m_x + j] = j < n_chosen ? chosen[j] : -1;
    p.n_extras[row] = (uint8_t)n_chosen;
}

// One attempt at a row.  Returns false (in every thread) if the sums came out non-finite,
// which happens when the row holds -inf logits; the caller then repeats with CLAMP.
template <int DT, bool ALIGN, bool COUNT, bool CLAMP, int BLOCK, int U>
__device__ __forceinline__ bool process_row(const SweepParams& p, int64_t row, const RowShape& rs,
                                            SweepShared<BLOCK / kWave>& sh, unsigned char* cm)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    constexpr int NW = BLOCK / kWave;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int V = p.V;

    int nt = -1;
    float znext = 0.f;
    if (ALIGN) {
        nt = p.next_tok ? p.next_tok[row] : -1;
        if (nt >= V) nt = -1;
        if (nt >= 0) znext = load_elt<DT>(rs.base, nt);
    }
    const bool has_next = ALIGN && nt >= 0;
    const bool want_cand = has_next && p.m_x > 0;
    const float zcmp = has_next ? znext : INFINITY;

    LaneAcc a;
    sweep_lane<DT, CLAMP, ALIGN && COUNT, BLOCK, U>(a, rs, V, tid, zcmp, want_cand && p.cm_enabled, cm);

    // ---- round 1: row maximum, and a lower bound on the c-th largest logit ----
    float g = a.vmax;
    g = fmaxf(g, __shfl_xor(g, 1));
    g = fmaxf(g, __shfl_xor(g, 2));
    g = fmaxf(g, __shfl_xor(g, 4));
    if ((lane & 7) == 0) sh.gmax[wid][lane >> 3] = g;
    if (tid == 0) sh.ncand = 0;
    __syncthreads();
    float G = sh.gmax[0][lane & 7];
#pragma unroll
    for (int w = 1; w < NW; ++w) G = fmaxf(G, sh.gmax[w][lane & 7]);
    // G: maximum over class j = lane & 7, the j-th 8-lane group of every wave (a partition of the row)
    float m = G;
    m = fmaxf(m, __shfl_xor(m, 1));
    m = fmaxf(m, __shfl_xor(m, 2));
    m = fmaxf(m, __shfl_xor(m, 4));
    float thr2 = -INFINITY;
    if (ALIGN) {
        // Merge the 8 classes into c' >= c classes (c' a power of two).  Each class maximum is a
        // distinct element, so the smallest of them is a lower bound on the c-th largest logit.
        const int merge = p.c > 4 ? 1 : (p.c > 2 ? 2 : (p.c > 1 ? 4 : 8));
        thr2 = G;
        for (int o = 1; o < merge; o <<= 1) thr2 = fmaxf(thr2, __shfl_xor(thr2, o));
        for (int o = merge; o < 8; o <<= 1) thr2 = fminf(thr2, __shfl_xor(thr2, o));
    }

    // ---- lane sums brought to the common reference m ----
    const float M2 = m * kLog2e;
    const float res = fmaf(m, kLog2e, -M2);  // rounding error of M2, so that the maximum weighs exactly 1
    float ssum = (a.s[0] + a.s[1]) + (a.s[2] + a.s[3]);
    float tsum = (a.t[0] + a.t[1]) + (a.t[2] + a.t[3]);
    const float dlt = (a.r2 - M2) - res;
    const float f = __builtin_amdgcn_exp2f(dlt);
    float Sp = ssum * f;
    float Tp = (tsum + dlt * ssum) * f;

    // ---- candidates ranked above the prompt token (misaligned rows only) ----
    const bool mis = has_next && (znext < m);
    if (ALIGN && want_cand && mis) {
        auto consider = [&](float z, int idx) {
            if (z > znext && z >= thr2) {
                const unsigned pos = atomicAdd(&sh.ncand, 1u);
                if (pos < (unsigned)kCandCap) { sh.cand_z[pos] = z; sh.cand_i[pos] = idx; }
            }
        };
        if (a.vmax > znext && a.vmax >= thr2) {  // only lanes that saw a qualifying element look again
            if (tid < rs.head) consider(load_elt<DT>(rs.base, tid), tid);
            for (int vec = tid; vec < rs.nvec; vec += BLOCK) {
                const float cmx = p.cm_enabled ? cm_load<DT>(cm, vec) : INFINITY;  // own entries: no barrier needed
                if (cmx > znext && cmx >= thr2) {
                    float z[EPV];
                    unpack<DT>(rs.vbase[vec], z);
#pragma unroll
                    for (int e = 0; e < EPV; ++e) consider(z[e], rs.head + vec * EPV + e);
                }
            }
            if (tid < V - rs.tail0) consider(load_elt<DT>(rs.base, rs.tail0 + tid), rs.tail0 + tid);
        }
    }

    // ---- round 2: sums, position of the maximum, rank ----
    Sp = wave_sum(Sp);
    Tp = wave_sum(Tp);
    const int code = wave_min(a.vmax == m ? a.code : 0x7fffffff);
    unsigned cnt = 0;
    if (ALIGN && COUNT) cnt = a.cnt_u + wave_sum(a.cnt_l);
    if (lane == 0) { sh.S[wid] = Sp; sh.T[wid] = Tp; sh.code[wid] = code; sh.cnt[wid] = cnt; }
    __syncthreads();
    float S = 0.f, T2 = 0.f;
    int bcode = 0x7fffffff;
    unsigned rank = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        S += sh.S[w]; T2 += sh.T[w];
        bcode = min(bcode, sh.code[w]);
        rank += sh.cnt[w];
    }
    if (!CLAMP) {
        if (!(S > 0.f) || !(S < INFINITY) || T2 != T2) return false;
    }

    float kz[AASD_MAX_CANDSET];
    int ki[AASD_MAX_CANDSET];
    int nK = 0;
#pragma unroll
    for (int q = 0; q < AASD_MAX_CANDSET; ++q) { kz[q] = 0.f; ki[q] = -1; }
    if (ALIGN && want_cand && mis) {
        const unsigned nc = sh.ncand;
        if (nc > (unsigned)kCandCap) topc_by_rescan<DT, BLOCK>(rs, V, tid, znext, p.c, sh, kz, ki, nK);
        else if (wid == 0) topc_from_buffer(sh.cand_z, sh.cand_i, (int)nc, lane, p.c, kz, ki, nK);
    }

    if (tid == 0) {
        // greedy pick: first element of chunk `bcode` that attains the maximum
        int am = 0;
        if ((unsigned)bcode < (unsigned)V) {  // always, unless the row holds no comparable value at all
            am = bcode;
            const int len = (bcode >= rs.head && bcode < rs.tail0) ? EPV : 1;
            for (int e = 0; e < len; ++e)
                if (load_elt<DT>(rs.base, bcode + e) == m) { am = bcode + e; break; }
        }
        // fp32 is enough for the per-row scalars: logf/expf are good to an ulp, far inside the tolerance
        float H = logf(S) - (float)kLn2 * T2 / S;
        if (H < 0.f) H = 0.f;
        const float pmax = 1.0f / S;
        if (ALIGN) {
            p.argmax[row] = am;
            p.entropy[row] = H;
            p.p_max[row] = pmax;
            p.misaligned[row] = mis ? 1 : 0;
            p.p_next[row] = has_next ? expf(znext - m) / S : 0.f;
            if (COUNT) p.rank[row] = has_next ? (int32_t)rank : -1;
            if (p.m_x > 0) {
                if (want_cand && mis) choose_extras(p, row, m, kz, ki, nK);
                else {
                    for (int j = 0; j < p.m_x; ++j) p.extras[row * p.m_x + j] = -1;
                    p.n_extras[row] = 0;
                }
            }
        } else {
            p.stats[row] = make_float4(m, S, H, __int_as_float(am));
            if (p.row_entropy) p.row_entropy[row] = H;
            if (p.row_pmax) p.row_pmax[row] = pmax;
            if (p.row_argmax) p.row_argmax[row] = am;
        }
    }
    return true;
}

template <int DT, bool ALIGN, bool COUNT, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void row_sweep_kernel(SweepParams p, int64_t row0)
{
    extern __shared__ __align__(16) unsigned char cm[];  // chunk maxima of this row (alignment sampling only)
    __shared__ SweepShared<BLOCK / kWave> sh;
    const int64_t row = row0 + blockIdx.x;
    const int64_t off = (row / p.rows_per_seq) * p.seq_stride + (row % p.rows_per_seq) * p.row_stride;
    const RowShape rs = row_shape<DT>(p.logits, off, p.V);
    if (!process_row<DT, ALIGN, COUNT, false, BLOCK, U>(p, row, rs, sh, cm)) {
        __syncthreads();  // everyone has read the failed attempt's partials
        process_row<DT, ALIGN, COUNT, true, BLOCK, U>(p, row, rs, sh, cm);
    }
}

}  // namespace aasd
