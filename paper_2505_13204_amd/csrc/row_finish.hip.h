// Merging the wave partials of a row, and the per-row scalar work of alignment sampling
// (Sec. 2.3, Sec. 3.2): greedy pick, entropy, probability and rank of the prompt's next token,
// the misalignment flag, and the choice of the extra draft tokens.
//
// One wave per row: lane s holds partial s (at most 64 per row).  The chunks that the sweep
// listed for the row are re-read here (a lane per chunk, all loads in flight together) and the
// top-c tokens above the prompt token are selected from them.
#pragma once

#include "row_sweep.hip.h"

namespace aasd {

// Statistics of a whole row, merged from its partials.
struct RowStats {
    float m;     // largest logit
    float S;     // sum of e^(z - m); max probability = 1/S
    float H;     // entropy in nats: ln S - (sum of (z - m) e^(z - m)) / S
    int code;    // first element of the chunk that holds the first maximum
    unsigned cnt;
};

__device__ __forceinline__ float entropy_from_sums(float S, float T2)
{
    const float H = logf(S) - (float)kLn2 * T2 / S;
    return H < 0.f ? 0.f : H;
}

// Index of the first element equal to m in the chunk that starts at `code` (wave-cooperative).
template <int DT>
__device__ __forceinline__ int wave_first_max(const RowShape& rs, int V, int code, float m, int lane)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    if ((unsigned)code >= (unsigned)V) return 0;  // only if the row held no comparable value at all
    const int len = (code >= rs.head && code < rs.tail0) ? EPV : 1;
    const bool hit = lane < len && load_elt<DT>(rs.base, code + lane) == m;
    const unsigned long long b = __ballot(hit);
    return b ? code + (__ffsll((long long)b) - 1) : code;
}

struct AlignFinishParams {
    const void* logits;
    int32_t V;
    int64_t row_stride;
    int64_t rows;
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
    const WavePartial* partials;
    const int32_t* lists;
    int32_t npart;  // partials per row
};

constexpr int kFinishCandCap = 128;  // candidate tokens buffered per row

// Choose the extra draft tokens of a misaligned row from its ranked candidate list K
// (Sec. 3.2; reading: TOP takes the best-ranked, SAMPLE draws without replacement).
__device__ __forceinline__ void choose_extras(const AlignFinishParams& p, int64_t row, float m,
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

constexpr int kFinishBlock = 256;  // four rows per workgroup

// Visit the elements of the r-th listed chunk of the row (lists are concatenated partial by partial).
template <int DT, typename F>
__device__ __forceinline__ void visit_listed_chunk(const AlignFinishParams& p, const RowShape& rs, int64_t row, int part,
                                                   int entry, F&& f)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    const int first = p.lists[(row * p.npart + part) * kListCap + entry];
    if ((unsigned)first >= (unsigned)p.V) return;
    if (first >= rs.head && first < rs.tail0) {
        float z[EPV];
        unpack<DT>(*(const u32x4*)(rs.base + (size_t)first * Elt<DT>::kBytes), z);
#pragma unroll
        for (int e = 0; e < EPV; ++e) f(z[e], first + e);
    } else {
        f(load_elt<DT>(rs.base, first), first);
    }
}

// Exact top-c (logit descending, id ascending) of one row among the tokens above `znext`, from the chunk
// positions that the sweep listed; called by all 64 lanes of the wave that owns the row.  `wp` is the lane's
// partial (lane s holds partial s), thr2 the row's lower bound on its c-th largest logit.  cand_z / cand_i /
// cand_n: kFinishCandCap LDS slots and a counter owned by this wave.
template <int DT>
__device__ __forceinline__ void row_topc_from_lists(const AlignFinishParams& p, const RowShape& rs, int64_t row,
                                                    const WavePartial& wp, float znext, float thr2, int lane,
                                                    float* cand_z, int* cand_i, unsigned* cand_n,
                                                    float (&kz)[AASD_MAX_CANDSET], int (&ki)[AASD_MAX_CANDSET], int& nK)
{
    const int np = p.npart;
    // The waves' maxima are np different tokens, so the c-th largest of them is another lower bound on the row's
    // c-th largest logit, and a much tighter one than any single wave's when the row was cut into many short
    // pieces (64 waves of 2000 tokens each would otherwise let through more candidates than the buffer holds).
    if (np >= p.c) {
        float v = lane < np ? wp.m : -INFINITY, kth = -INFINITY;
        for (int r = 0; r < p.c; ++r) {
            const float mx = wave_max(v);
            kth = mx;
            const unsigned long long owners = __ballot(v == mx);
            if (lane == __ffsll((long long)owners) - 1) v = -INFINITY;   // one wave gives up its maximum per round
        }
        thr2 = fmaxf(thr2, kth);
    }
    // inclusive prefix of the list lengths: entry e of the row belongs to the first partial whose prefix exceeds e.
    // A partial whose maximum is below the row's bound (or not above znext) cannot hold a candidate: its list is
    // skipped, which matters when a row was cut into many segments (up to 64 lists).
    const int incl = wave_inclusive_scan((lane < np && wp.m >= thr2 && wp.m > znext) ? wp.nlist : 0);
    const int total = __shfl(incl, 63);
    auto locate = [&](int e, int& part, int& entry) {  // all lanes call it together
        // binary search for the number of partials whose inclusive prefix is <= e
        int pos = 0;
#pragma unroll
        for (int step = 32; step > 0; step >>= 1) {
            const int probe = pos + step;
            const int v = __shfl(incl, probe - 1 < 63 ? probe - 1 : 63);
            if (probe <= np && v <= e) pos = probe;
        }
        part = pos < np ? pos : np - 1;
        const int before = __shfl(incl, pos > 0 ? pos - 1 : 0);
        entry = e - (pos > 0 ? before : 0);
    };
    if (lane == 0) *cand_n = 0;
    for (int e0 = 0; e0 < total; e0 += kWave) {
        const int e = e0 + lane;
        int part, entry;
        locate(e, part, entry);
        if (e < total) {
            visit_listed_chunk<DT>(p, rs, row, part, entry, [&](float z, int idx) {
                if (z > znext && z >= thr2) {
                    const unsigned pos = atomicAdd(&*cand_n, 1u);
                    if (pos < (unsigned)kFinishCandCap) { cand_z[pos] = z; cand_i[pos] = idx; }
                }
            });
        }
    }
    __threadfence_block();
    const unsigned n = *cand_n;
    if (n <= (unsigned)kFinishCandCap) {
        constexpr int kPerLane = kFinishCandCap / kWave;
        float lz[kPerLane];
        int li[kPerLane];
#pragma unroll
        for (int q = 0; q < kPerLane; ++q) {
            const int e = lane + q * kWave;
            lz[q] = e < (int)n ? cand_z[e] : -INFINITY;
            li[q] = e < (int)n ? cand_i[e] : 0x7fffffff;
        }
        wave_topc<kPerLane>(lz, li, p.c, kz, ki, nK);
    } else {
        // very many ties near the top: c exact rounds of "best token after the previous pick"
        float pz = INFINITY;
        int pi = -1;
        for (int r = 0; r < p.c; ++r) {
            float bz = -INFINITY;
            int bi = 0x7fffffff;
            for (int e0 = 0; e0 < total; e0 += kWave) {
                const int e = e0 + lane;
                int part, entry;
                locate(e, part, entry);
                if (e < total) {
                    visit_listed_chunk<DT>(p, rs, row, part, entry, [&](float z, int idx) {
                        const bool after_prev = (r == 0) || z < pz || (z == pz && idx > pi);
                        if (z > znext && after_prev && better(z, idx, bz, bi)) { bz = z; bi = idx; }
                    });
                }
            }
            wave_best(bz, bi);
            if (bi == 0x7fffffff) break;
            pz = bz; pi = bi;
            set_pick(kz, ki, r, bz, bi);
            nK = r + 1;
        }
    }
}

template <int DT>
__global__ __launch_bounds__(kFinishBlock) void align_finish_kernel(AlignFinishParams p)
{
    __shared__ float cand_z[kFinishBlock / kWave][kFinishCandCap];
    __shared__ int cand_i[kFinishBlock / kWave][kFinishCandCap];
    __shared__ unsigned cand_n[kFinishBlock / kWave];

    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * (kFinishBlock / kWave) + wid;
    if (row >= p.rows) return;  // whole wave; the kernel has no barrier
    const int V = p.V, np = p.npart;

    // The kernel is a chain of dependent loads; the logit of the prompt's next token depends on nothing computed
    // here, so its two loads go first and overlap with those of the partials and of the argmax chunk.
    const RowShape rs = row_shape<DT>(p.logits, row * p.row_stride, V);
    int nt = p.next_tok ? p.next_tok[row] : -1;
    if (nt >= V) nt = -1;
    const bool has_next = nt >= 0;
    const float znext = has_next ? load_elt<DT>(rs.base, nt) : 0.f;

    // ---- merge the partials: lane s holds partial s ----
    WavePartial wp;
    wp.m = -INFINITY; wp.S = 0.f; wp.T = 0.f; wp.code = 0x7fffffff; wp.cnt = 0; wp.nlist = 0; wp.thr2 = -INFINITY;
    if (lane < np) wp = p.partials[row * np + lane];
    const float m = wave_max(wp.m);
    float thr2 = wave_max(wp.thr2);  // each wave's bound holds for the row: take the tightest
    const bool live = wp.S > 0.f;
    float dl = 0.f, f = 0.f;
    if (live) partial_scale(wp.m, m, dl, f);
    const float S = wave_sum(live ? wp.S * f : 0.f);
    const float T2 = wave_sum(live ? (wp.T + dl * wp.S) * f : 0.f);
    const int code = wave_min(live && wp.m == m ? wp.code : 0x7fffffff);
    const unsigned rank = wave_sum(wp.cnt);

    const int am = wave_first_max<DT>(rs, V, code, m, lane);
    const float H = entropy_from_sums(S, T2);
    const bool mis = has_next && znext < m;

    // ---- top-c of the row among the tokens of the listed chunks ----
    float kz[AASD_MAX_CANDSET];
    int ki[AASD_MAX_CANDSET];
    int nK = 0;
#pragma unroll
    for (int q = 0; q < AASD_MAX_CANDSET; ++q) { kz[q] = 0.f; ki[q] = -1; }
    if (mis && p.m_x > 0)
        row_topc_from_lists<DT>(p, rs, row, wp, znext, thr2, lane, cand_z[wid], cand_i[wid], &cand_n[wid], kz, ki, nK);

    if (lane == 0) {
        p.argmax[row] = am;
        p.entropy[row] = H;
        p.p_max[row] = 1.0f / S;
        p.misaligned[row] = mis ? 1 : 0;
        p.p_next[row] = has_next ? expf(znext - m) / S : 0.f;
        if (p.rank) p.rank[row] = has_next ? (int32_t)rank : -1;
        if (p.m_x > 0) {
            if (mis) choose_extras(p, row, m, kz, ki, nK);
            else {
                for (int j = 0; j < p.m_x; ++j) p.extras[row * p.m_x + j] = -1;
                p.n_extras[row] = 0;
            }
        } else if (p.n_extras) {
            p.n_extras[row] = 0;   // m = 0: no extras; a count array that was passed anyway is still defined
        }
    }
}

}  // namespace aasd
