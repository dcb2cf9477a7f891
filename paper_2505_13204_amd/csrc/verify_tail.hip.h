// Per-token decision and accept-prefix scan of conditional verification (Sec. 3.3, Eq. 4-6).
//
// One workgroup per sequence.  First the wave partials that the sweep left in the workspace
// are merged per row (maximum, sum of exponentials, entropy, greedy pick), a group of lanes per
// row, into LDS.  Then, with 16 lanes per candidate (k <= 16 draft tokens) and four
// candidates per wave, each lane decides its token; a wave
// ballot turns the decisions of a candidate into a bit field whose trailing ones are the
// accepted prefix (the cascade rule of Sec. 2.1); one thread then takes the longest candidate.
//
// The same work exists in two launch forms: as a kernel of its own after the sweep
// (verify_tail_kernel), and inside the sweep kernel (verify_fused_kernel), where the workgroup
// that is the last to finish a row segment of a sequence does that sequence's tail.
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

struct TailShared {
    int lead[AASD_MAX_CANDIDATES];
    unsigned near_c[AASD_MAX_CANDIDATES];
    float4 stats[kMaxVerifyRows];  // per row {max logit, S, H, bits of argmax}
};

// What a thread needs of the drafts before it can decide its tokens: none of it depends on the row statistics.
template <int NT>
struct TailInputs {
    static constexpr int kCandPerPass = NT / 16;   // 16 lanes per candidate
    static constexpr int kPasses = (AASD_MAX_CANDIDATES + kCandPerPass - 1) / kCandPerPass;
    int dl[kPasses], tok[kPasses];
    float zt[kPasses];     // logit of the draft token in the row that verifies it
    bool strict[kPasses];
};

// Loads the draft lengths, tokens and flags of sequence b.
template <int NT>
__device__ __forceinline__ void tail_load_drafts(const VerifyTailParams& p, int b, TailInputs<NT>& in)
{
    const int tid = threadIdx.x, j = tid & 15;  // j: 0-based position in the draft
    const int C = p.C, k = p.k;
#pragma unroll
    for (int ps = 0; ps < TailInputs<NT>::kPasses; ++ps) {
        const int cand = ps * TailInputs<NT>::kCandPerPass + (tid >> 4);
        int dl = 0;
        if (cand < C) {
            dl = p.draft_len[(size_t)b * C + cand];
            dl = dl < 0 ? 0 : (dl > k ? k : dl);
        }
        in.dl[ps] = dl;
        in.tok[ps] = -1; in.zt[ps] = 0.f; in.strict[ps] = false;
        if (cand < C && j < k) {   // every slot of the candidate, whatever its length: the loads need not wait for draft_len
            const size_t idx = ((size_t)b * C + cand) * k + j;
            in.tok[ps] = p.drafts[idx];
            in.strict[ps] = p.strict != nullptr && p.strict[idx] != 0;
        }
    }
}

// Loads the logit of every draft token in the row that verifies it (needs the tokens).
template <int DT, int NT>
__device__ __forceinline__ void tail_load_logits(const VerifyTailParams& p, int b, TailInputs<NT>& in)
{
    const int tid = threadIdx.x, j = tid & 15;
#pragma unroll
    for (int ps = 0; ps < TailInputs<NT>::kPasses; ++ps) {
        const int cand = ps * TailInputs<NT>::kCandPerPass + (tid >> 4);
        const int t = in.tok[ps];
        if (cand < p.C && j < p.k && t >= 0 && t < p.V) {
            const int rho = (j == 0) ? 0 : 1 + cand * p.k + (j - 1);  // the row that follows the previous token
            in.zt[ps] = load_elt<DT>(p.logits, (int64_t)b * p.seq_stride + (int64_t)rho * p.row_stride + t);
        }
    }
}

// The tail of sequence b, run by all NT threads of a workgroup (NT a multiple of 64).
// COHERENT: the partials were written by other workgroups of this same launch (see store_partial_coherent).
// EXACT: the partials name the first maximum of their share itself, so the greedy pick needs no second look at the row.
template <int DT, int NT, bool COHERENT, bool EXACT>
__device__ __forceinline__ void verify_tail_block(const VerifyTailParams& p, int b, const TailInputs<NT>& in, TailShared& sh)
{
    constexpr int kCandPerPass = TailInputs<NT>::kCandPerPass;
    constexpr int kPasses = TailInputs<NT>::kPasses;
    const int tid = threadIdx.x, lane = tid & 63;
    const int j = tid & 15;
    const int C = p.C, k = p.k, R = 1 + C * k;

    // ---- statistics of the sequence's rows from the sweep's partials ----
    // G lanes per row (G = npart rounded up to a power of two), NT/G rows at a time
    {
        int G = 1;
        while (G < p.npart) G <<= 1;
        const int rows_per_pass = NT / G;
        const int sub = tid / G, s = tid - sub * G;  // row slot of this lane, partial index within the row
        for (int r0 = 0; r0 < R; r0 += rows_per_pass) {
            const int r = r0 + sub;
            const bool have_row = r < R;
            const int64_t row = (int64_t)b * R + (have_row ? r : 0);
            WavePartial wp;
            wp.m = -INFINITY; wp.S = 0.f; wp.T = 0.f; wp.code = 0x7fffffff;
            if (have_row && s < p.npart) {
                if (COHERENT) wp = load_partial_coherent(p.partials + row * p.npart + s);
                else wp = p.partials[row * p.npart + s];
            }
            const float m = group_reduce(wp.m, G, [](float x, float y) { return fmaxf(x, y); });
            const bool live = wp.S > 0.f;
            float dl2 = 0.f, f = 0.f;
            if (live) partial_scale(wp.m, m, dl2, f);
            const float S = group_reduce(live ? wp.S * f : 0.f, G, [](float x, float y) { return x + y; });
            const float T2 = group_reduce(live ? (wp.T + dl2 * wp.S) * f : 0.f, G, [](float x, float y) { return x + y; });
            const int code = group_reduce(live && wp.m == m ? wp.code : 0x7fffffff, G, [](int x, int y) { return min(x, y); });
            if (have_row && s == 0) {
                // EXACT: the code is the greedy pick itself.  Otherwise it names the chunk that holds it, and the pick is
                // found below, by a load that is in flight while the tokens are decided (they do not need it).
                const int am = (unsigned)code < (unsigned)p.V ? code : (EXACT ? 0 : -1);
                const float H = entropy_from_sums(S, T2);
                sh.stats[r] = make_float4(m, S, H, __int_as_float(am));
                if (p.row_entropy) p.row_entropy[row] = H;
                if (p.row_pmax) p.row_pmax[row] = 1.0f / S;
                if (EXACT && p.row_argmax) p.row_argmax[row] = am;
            }
        }
    }
    __syncthreads();

    // the chunks that hold the rows' maxima (a thread per row): asked for here, used after the decisions
    constexpr int kRowsPerThread = EXACT ? 0 : (kMaxVerifyRows + NT - 1) / NT;
    u32x4 am_chunk[kRowsPerThread > 0 ? kRowsPerThread : 1];
    if (!EXACT) {
#pragma unroll
        for (int q = 0; q < kRowsPerThread; ++q) {
            const int r = tid + q * NT;
            am_chunk[q] = u32x4{0u, 0u, 0u, 0u};
            if (r < R) {
                const int code = __float_as_int(sh.stats[r].w);
                const RowShape rs = row_shape<DT>(p.logits, (int64_t)b * p.seq_stride + (int64_t)r * p.row_stride, p.V);
                if (code >= rs.head && code < rs.tail0) am_chunk[q] = rs.vbase[(code - rs.head) / Elt<DT>::kPerVec];
            }
        }
    }

#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) {
        const int cand = ps * kCandPerPass + (tid >> 4);
        if (ps * kCandPerPass >= C) break;   // the same in every thread
        const int dl = in.dl[ps];
        const bool slot = cand < C && j < k;
        const bool inside = slot && j < dl;
        const size_t idx = ((size_t)b * C + (cand < C ? cand : 0)) * k + (j < k ? j : 0);

        bool pass = false, near = false;
        float pf = 0.f, df = 0.f;
        if (inside) {
            const int rho = (j == 0) ? 0 : 1 + cand * k + (j - 1);
            const int t = in.tok[ps];
            const float4 st = sh.stats[rho];
            const double m = (double)st.x, S = (double)st.y, H = (double)st.z;
            const bool valid = t >= 0 && t < p.V;
            const float zt = in.zt[ps];
            const double pr = valid ? exp((double)zt - m) / S : 0.0;
            const double Delta = 1.0 / S;                                // Eq. 6
            const double thr = (double)p.alpha * H + (double)p.beta;     // Eq. 5
            double delta;
            if (p.flags & AASD_VERIFY_NO_CLAMP) {
                delta = thr;
                pass = valid && pr >= delta;
            } else {
                delta = in.strict[ps] ? Delta : fmin(thr, Delta);
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
        const unsigned nfield = (unsigned)((__ballot(near && inside) >> shift) & 0xffffull);
        const int a = __ffs(~field) - 1;  // bit 16 of ~field is always set, so a <= 16; a <= dl because bit dl is clear
        if (j == 0 && cand < C) {
            sh.lead[cand] = a;
            // evaluated tokens: the accepted ones and the first failure
            const unsigned ev = (a + 1 >= 32) ? 0xffffffffu : ((1u << (a + 1)) - 1u);
            sh.near_c[cand] = (unsigned)__popc(nfield & ev);
        }
    }
    if (!EXACT) {
#pragma unroll
        for (int q = 0; q < kRowsPerThread; ++q) {
            const int r = tid + q * NT;
            if (r < R) {
                const int code = __float_as_int(sh.stats[r].w);
                int am = code < 0 ? 0 : code;   // a chunk of the aligned body: its first element equal to the maximum
                const RowShape rs = row_shape<DT>(p.logits, (int64_t)b * p.seq_stride + (int64_t)r * p.row_stride, p.V);
                if (code >= rs.head && code < rs.tail0) {
                    float z[Elt<DT>::kPerVec];
                    unpack<DT>(am_chunk[q], z);
                    const float m = sh.stats[r].x;
#pragma unroll
                    for (int e = Elt<DT>::kPerVec - 1; e >= 0; --e)
                        if (z[e] == m) am = code + e;
                }
                sh.stats[r].w = __int_as_float(am);
                if (p.row_argmax) p.row_argmax[(int64_t)b * R + r] = am;
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        int best_a = 0, best_c = 0;
        unsigned near_total = 0;
        for (int c = 0; c < C; ++c) {
            if (sh.lead[c] > best_a) { best_a = sh.lead[c]; best_c = c; }  // lowest index on ties
            near_total += sh.near_c[c];
        }
        const int rho = best_a == 0 ? 0 : 1 + best_c * k + (best_a - 1);
        p.accept_len[b] = best_a;
        p.best_cand[b] = best_c;
        p.next_token[b] = __float_as_int(sh.stats[rho].w);
        if (p.near_count) p.near_count[b] = near_total;
    }
}

template <int DT>
__global__ __launch_bounds__(kTailBlock) void verify_tail_kernel(VerifyTailParams p)
{
    __shared__ TailShared sh;
    TailInputs<kTailBlock> in;
    tail_load_drafts<kTailBlock>(p, blockIdx.x, in);
    tail_load_logits<DT, kTailBlock>(p, blockIdx.x, in);
    verify_tail_block<DT, kTailBlock, false, false>(p, blockIdx.x, in, sh);
}

// Sweep and tail in one launch.  Grid = rows x segments as for row_sweep_kernel.
//
// Every sequence has a counter, zero before the launch.  A workgroup whose waves have written their
// partials (with stores that go to memory, and waited until memory has them) adds one to its sequence's
// counter; the workgroup that brings it to rows_per_seq * nseg knows that every partial of the sequence
// is in memory, puts the counter back to zero and does the sequence's tail.  No workgroup waits for
// another, so the launch cannot stall however its workgroups are scheduled.
// Additions to ONE address are served one after the other (some tens of nanoseconds each), and the
// workgroups of a short launch all finish at about the same time; so when a sequence has many workgroups
// they first count in `ngroups` group counters (workgroup u of the sequence in group u mod ngroups), and
// only the last of each group adds to the sequence's counter.  Every counter has a 128-byte line of its
// own: counters that share a line are served one after the other like a single one.
constexpr int kCounterWords = 32;   // 128 bytes

struct VerifyFusedParams {
    SweepParams s;
    VerifyTailParams t;
    unsigned* counters;   // [B][1 + (ngroups > 1 ? ngroups : 0)][kCounterWords]
    int32_t ngroups;      // 1: the sequence's counter alone
    uint32_t rps_magic;   // floor(2^32 / rows_per_seq) + 1: row / rows_per_seq = (row * magic) >> 32, exact for row < 2^22
};

__device__ __forceinline__ bool arrive_is_last(unsigned* counter, unsigned expected)
{
    const unsigned before = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (before != expected - 1u) return false;
    __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // nobody else touches it again in this launch
    return true;
}

template <int DT, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void verify_fused_kernel(VerifyFusedParams p, int64_t row0)
{
    constexpr int NW = BLOCK / kWave;
    __shared__ SweepShared<1> sh_store;
    SweepShared<NW>& sh = *reinterpret_cast<SweepShared<NW>*>(&sh_store);  // never touched: no alignment sampling here
    __shared__ TailShared tail_sh;
    __shared__ WavePartial wave_part[NW];
    __shared__ int s_last;

    const uint32_t q = div_by_segments(blockIdx.x, p.s.nseg, p.s.nseg_magic);
    const int64_t row = row0 + q;
    const int seg = (int)(blockIdx.x - q * (uint32_t)p.s.nseg);
    const int b = (int)__umulhi((uint32_t)row, p.rps_magic);   // row / rows_per_seq: this form's launches have few rows
    const int tid = threadIdx.x;

    sweep_unit<DT, false, false, BLOCK, U, false, true, 4 * U>(p.s, row, seg, sh, nullptr, wave_part);   // 4, 8 or 16 loads per lane in flight
    // the drafts of the sequence: only the workgroup that turns out to be the sequence's last needs them, but asked
    // for here they arrive while the partial travels to memory and the workgroup is counted in
    TailInputs<BLOCK> in;
    tail_load_drafts<BLOCK>(p.t, b, in);
    __syncthreads();

    // the first wave merges the workgroup's wave partials into ONE partial per (row, segment), sends it to
    // memory, waits until memory has it, and counts the workgroup in
    if (tid < kWave) {
        const WavePartial out = merge_wave_partials<NW>(wave_part, tid);
        if (tid == 0) {
            store_partial_coherent(p.s.partials + (row * p.s.nseg + seg), out);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

            const int lines = p.ngroups > 1 ? 1 + p.ngroups : 1;
            unsigned* base = p.counters + (size_t)b * lines * kCounterWords;
            const unsigned per_seq = (unsigned)p.s.rows_per_seq * (unsigned)p.s.nseg;
            bool last;
            if (p.ngroups > 1) {
                const unsigned u = (unsigned)(row - (int64_t)b * p.s.rows_per_seq) * (unsigned)p.s.nseg + (unsigned)seg;
                const unsigned g = u % (unsigned)p.ngroups;
                const unsigned in_group = (per_seq - g + (unsigned)p.ngroups - 1u) / (unsigned)p.ngroups;
                last = arrive_is_last(base + (size_t)(1 + g) * kCounterWords, in_group) && arrive_is_last(base, (unsigned)p.ngroups);
            } else {
                last = arrive_is_last(base, per_seq);
            }
            s_last = last ? 1 : 0;
        }
    }
    __syncthreads();
    if (!s_last) return;   // the same in every thread of the workgroup
    tail_load_logits<DT, BLOCK>(p.t, b, in);                         // in flight together with the partials
    verify_tail_block<DT, BLOCK, true, true>(p.t, b, in, tail_sh);   // p.t.npart = nseg: one partial per workgroup
}

}  // namespace aasd
