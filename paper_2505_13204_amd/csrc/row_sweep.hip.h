// Fused single-pass row sweep: softmax normaliser, entropy, greedy pick and (for prefill
// rows) rank of the next prompt token and the candidate tokens ranked above it.
//
// A row is read from HBM exactly once with 16-byte non-temporal loads.  A workgroup owns one row, or one of
// several contiguous segments of a row when there are too few rows to fill the GPU.  Every
// wave works on its own: it folds its share into a partial result (maximum, sum of
// exponentials, entropy sum, position of the maximum, rank count, the chunks that may hold its
// best candidates) with wave shuffles only and writes that partial to the workspace.  A second, small kernel merges
// the partials of a row and does the per-row scalar work (see row_finish.hip.h), so the
// streaming kernel has no barrier and no serial tail.
// Per element the sweep does: unpack, one FMA into the log2 domain, one hardware exp2, one add
// (sum of exponentials) and one FMA (sum of exponent * exponential, which gives the entropy as
// ln S - T/S, Eq. 5 of Sec. 3.3 rewritten so that both terms are non-negative).  Everything
// that would cost more per element is done per 16-byte chunk instead:
//   - the running maximum and the position of the chunk that set it (the greedy pick is then
//     found by re-reading that one chunk),
//   - the reference exponent of the running sums, which is only moved when a chunk exceeds it
//     by more than a few nats (floating point does not care about a common scale, but the
//     entropy sum loses accuracy if its largest term is far from the reference),
//   - the second largest chunk maximum of the lane, and one chunk maximum per chunk parked in LDS:
//     after the sweep a lane with one qualifying chunk names it directly, a lane with several finds
//     them in LDS; only the positions of those chunks are written out, and the
//     finish kernel re-reads those chunks (Sec. 3.2 / Fig. 2 need the tokens ranked above the
//     prompt token, not a full sort).
#pragma once

#include "common.hip.h"

namespace aasd {

constexpr int kNumAcc = 4;      // independent partial sums per lane (shorter rounding chains, more ILP)
// Nats a chunk may exceed the lane's reference exponent before the reference is moved.  The sum t carries
// the term d*2^d of the largest element, which cancels when the sums are brought to the row maximum; its
// rounding error is eps*d, so d is kept small: 4 nats bound the entropy error of a peaked row by ~2e-7 nats.
constexpr float kRefSlack = 4.0f;  // nats a chunk may exceed the reference exponent before it is moved

// What one wave leaves behind for the finish kernel.
struct WavePartial {
    float m;       // largest logit of the wave's share (-inf: the share was empty)
    float S;       // sum of e^(z - m) over the share
    float T;       // sum of log2(e^(z - m)) * e^(z - m)  (log2 units, <= 0)
    int code;      // index of the first element of the chunk that holds the first maximum (EXACT sweeps: of that maximum itself)
    unsigned cnt;  // elements with z > z_next
    int nlist;     // chunks listed for this wave (they hold every token of its share that can be in the row's top-c)
    float thr2;    // a lower bound on the c-th largest logit of the wave's share
    int pad;
};

// A partial that another workgroup of the SAME launch will read (one-launch verification) goes to memory and
// comes from memory word by word with device-scope atomic accesses: these pass through the caches that are
// private to a compute unit or to one of the GPU's dies, where a plain store could linger and a plain load
// could hit a stale line.  (A device-scope fence would do as well, but it writes back and invalidates the
// whole die-level cache each time, which costs microseconds per workgroup.)
__device__ __forceinline__ void store_partial_coherent(WavePartial* out, const WavePartial& wp)
{
    static_assert(sizeof(WavePartial) == 32, "WavePartial is four 64-bit words");
    const uint64_t* src = reinterpret_cast<const uint64_t*>(&wp);
    uint64_t* dst = reinterpret_cast<uint64_t*>(out);
#pragma unroll
    for (int i = 0; i < 4; ++i) __hip_atomic_store(dst + i, src[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ WavePartial load_partial_coherent(const WavePartial* in)
{
    WavePartial wp;
    uint64_t* dst = reinterpret_cast<uint64_t*>(&wp);
    const uint64_t* src = reinterpret_cast<const uint64_t*>(in);
#pragma unroll
    for (int i = 0; i < 4; ++i) dst[i] = __hip_atomic_load(src + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return wp;
}

constexpr int kMaxPartials = 64;   // partials per row (segments x waves): one lane each in the finish kernel
constexpr int kListCap = 48;       // chunk positions a wave may list

struct SweepParams {
    const void* logits;
    int32_t V;
    int64_t row_stride;    // elements
    int64_t seq_stride;    // elements, verification only (rows_per_seq rows per sequence)
    int32_t rows_per_seq;  // 1 for prefill rows
    int32_t cand_all;      // alignment sweep: list the top-c candidates of EVERY row (as if the next token had logit -inf)
    const int32_t* rows_used;  // optional [sequences]: rows of a sequence at or beyond max(this count, 1) are skipped
    const int32_t* next_tok;  // alignment sampling only
    int32_t want_cand;     // candidates are wanted (m > 0)
    int32_t c;
    int32_t cm_enabled;    // chunk maxima fit in LDS
    int32_t cm_stride;     // bytes between the chunk-maximum rows of neighbouring lanes
    int32_t nseg;          // segments per row
    uint32_t nseg_magic;   // floor(2^32 / nseg) + 1 (0 for nseg = 1): u / nseg = (u * magic) >> 32, exact for u < 2^28
    int32_t merge_waves;   // verification sweep: the workgroup merges its waves' partials and writes ONE per (row, segment)
    int32_t seg_vecs;      // 16-byte vectors per segment (a multiple of the block size)
    WavePartial* partials; // [rows][nseg * waves per block]
    int32_t* lists;        // [rows][nseg * waves per block][kListCap] first-element indices of listed chunks
};

// Running state of one lane.
struct LaneAcc {
    float vmax;   // largest logit seen
    float v2;     // second largest chunk maximum (alignment sweep only): tells whether one chunk can hold all the lane's candidates
    int code;     // index of the first element of the chunk that set vmax
    float r2;     // reference exponent (log2 units) of s and t
    float rlim;   // chunk maximum above which the reference must move
    float s[kNumAcc];  // sum of 2^(z*log2e - r2)
    float t[kNumAcc];  // sum of (z*log2e - r2) * 2^(z*log2e - r2)
    unsigned cnt_u;    // elements with z > z_next, counted wave-wide (same value in every lane)
    unsigned cnt_l;    // the same for elements handled under divergence (per lane)
    u32x4 best;        // EXACT sweeps: the 16 bytes of the chunk that set vmax, so that the maximum's own index needs no second read
};

__device__ __forceinline__ void lane_acc_init(LaneAcc& a)
{
    a.vmax = -INFINITY; a.v2 = -INFINITY; a.code = 0x7fffffff;
    a.r2 = kNegHuge; a.rlim = -INFINITY;
#pragma unroll
    for (int i = 0; i < kNumAcc; ++i) { a.s[i] = 0.f; a.t[i] = 0.f; }
    a.cnt_u = 0; a.cnt_l = 0;
    a.best = u32x4{0u, 0u, 0u, 0u};
}

// Fold N consecutive elements (first index idx0) into the lane state.
// CLAMP: exponents are floored at a finite value so that -inf logits contribute exactly zero.
// COUNT: count elements above zcmp.  UNIFORM: all 64 lanes are active (ballot counting).
// EXACT: the chunk that sets the lane's maximum is kept (a.best, four selects per chunk), so that the index of
// the maximum itself can be told after the sweep without reading the row again; `raw` is the chunk as loaded.
template <int N, bool CLAMP, bool COUNT, bool UNIFORM, bool SECOND, bool EXACT = false>
__device__ __forceinline__ float accumulate(LaneAcc& a, const float (&z)[N], int idx0, float zcmp, const u32x4* raw = nullptr)
{
    float cmax = z[0];
#pragma unroll
    for (int e = 1; e < N; ++e) cmax = fmaxf(cmax, z[e]);
    if (SECOND) a.v2 = fmaxf(a.v2, fminf(cmax, a.vmax));   // the smaller of the new maximum and the old one
    const bool higher = cmax > a.vmax;
    a.code = higher ? idx0 : a.code;
    if (EXACT && N > 1) {
        a.best.x = higher ? raw->x : a.best.x; a.best.y = higher ? raw->y : a.best.y;
        a.best.z = higher ? raw->z : a.best.z; a.best.w = higher ? raw->w : a.best.w;
    }
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
        if (COUNT && !UNIFORM) a.cnt_l += (z[e] > zcmp) ? 1u : 0u;
    }
    if (COUNT && UNIFORM) {
        // Rank of the prompt's next token: elements above it, counted wave-wide.  Where that token is the row's
        // greedy pick or close to it (most prompt positions), almost no chunk holds such an element: one test of
        // the chunk maxima skips the per-element count for the whole wave.
        if (__ballot(cmax > zcmp) != 0ull) {
#pragma unroll
            for (int e = 0; e < N; ++e) a.cnt_u += (unsigned)__popcll(__ballot(z[e] > zcmp));
        }
    }
    return cmax;
}

// Where a row's bytes sit relative to 16-byte boundaries.
struct RowShape {
    const char* base;   // first element of the row
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

// Index of the first element equal to m in the chunk that starts at `code` (the sweep names the chunk that holds a
// row's maximum, not the element): one 16-byte load for a chunk of the aligned body, the element itself otherwise.
template <int DT>
__device__ __forceinline__ int first_equal_in_chunk(const RowShape& rs, int code, float m)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    if (code < rs.head || code >= rs.tail0) return code;
    const u32x4 v = rs.vbase[(code - rs.head) / EPV];
    float z[EPV];
    unpack<DT>(v, z);
    int at = code;
#pragma unroll
    for (int e = EPV - 1; e >= 0; --e)
        if (z[e] == m) at = code + e;
    return at;
}

// The part of a row one workgroup sweeps: a run of vectors, plus the unaligned head elements
// (first segment) and tail elements (last segment) of the row.
struct SegShape {
    const char* base;    // first element of the row (scalar loads index from here)
    const u32x4* vbase;  // first vector of the segment
    int first_idx;       // element index of vbase[0]
    int nvec;            // vectors in the segment
    int head_n;          // head elements [0, head_n) handled here
    int tail0, tail_n;   // tail elements [tail0, tail0 + tail_n) handled here
};

template <int DT>
__device__ __forceinline__ SegShape seg_shape(const RowShape& r, int V, int seg, int nseg, int seg_vecs)
{
    SegShape s;
    const int v_lo = min(seg * seg_vecs, r.nvec);
    const int v_hi = min(v_lo + seg_vecs, r.nvec);
    s.base = r.base;
    s.vbase = r.vbase + v_lo;
    s.first_idx = r.head + v_lo * Elt<DT>::kPerVec;
    s.nvec = v_hi - v_lo;
    s.head_n = seg == 0 ? r.head : 0;
    s.tail0 = r.tail0;
    s.tail_n = seg == nseg - 1 ? V - r.tail0 : 0;
    return s;
}

// Chunk maxima in LDS, lane-contiguous: entry j of a lane is the maximum of its j-th chunk (vector
// j*BLOCK + tid of the segment), stored in the logits' own type.  The rows of neighbouring lanes are
// cm_stride bytes apart, an odd number of 16-byte slots, so that 16-byte reads of eight neighbouring
// lanes fall into distinct banks.  A lane only ever reads what it wrote itself: no barrier is needed.
template <int DT>
__device__ __forceinline__ void cm_store(unsigned char* cm_lane, int j, float cmax)
{
    if constexpr (DT == AASD_BF16) ((uint16_t*)cm_lane)[j] = (uint16_t)(__float_as_uint(cmax) >> 16);
    else ((float*)cm_lane)[j] = cmax;
}
// U consecutive entries starting at entry j0 (j0 a multiple of U): one wide LDS store.
template <int DT, int U>
__device__ __forceinline__ void cm_store_batch(unsigned char* cm_lane, int j0, const float (&cmax)[U])
{
    if constexpr (DT == AASD_BF16 && (U == 2 || U == 4)) {
        uint32_t w[U / 2];
#pragma unroll
        for (int q = 0; q < U / 2; ++q)
            w[q] = (__float_as_uint(cmax[2 * q + 1]) & 0xffff0000u) | (__float_as_uint(cmax[2 * q]) >> 16);
        if constexpr (U == 4) *(uint2*)(cm_lane + j0 * 2) = make_uint2(w[0], w[1]);
        else *(uint32_t*)(cm_lane + j0 * 2) = w[0];
    } else if constexpr (DT == AASD_F32 && U == 4) {
        *(float4*)(cm_lane + j0 * 4) = make_float4(cmax[0], cmax[1], cmax[2], cmax[3]);
    } else if constexpr (DT == AASD_F32 && U == 2) {
        *(float2*)(cm_lane + j0 * 4) = make_float2(cmax[0], cmax[1]);
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) cm_store<DT>(cm_lane, j0 + u, cmax[u]);
    }
}

// The single HBM pass of one lane over its share of the row: vectors tid, tid+BLOCK, ...
// loaded U at a time with the next batch in flight while the current one is folded in.
template <int DT, bool CLAMP, bool COUNT, bool SECOND, int BLOCK, int U, bool EXACT = false>
__device__ __forceinline__ void sweep_lane(LaneAcc& a, const SegShape& rs, int tid, float zcmp,
                                           bool store_cm, unsigned char* cm_lane)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    lane_acc_init(a);

    if (tid < rs.head_n) {
        const float z1[1] = {load_elt<DT>(rs.base, tid)};
        accumulate<1, CLAMP, COUNT, false, SECOND, EXACT>(a, z1, tid, zcmp);
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
        for (int u = 0; u < U; ++u)  // read once: non-temporal loads keep the stream out of the caches' way (+8 % bandwidth, measured)
            buf[u] = __builtin_nontemporal_load((const u32x4*)(b + (voff + (unsigned)u * (BLOCK * 16u))));
    };
    auto fold_batch = [&](const u32x4 (&buf)[U], int it) {
        float cmax[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float z[EPV];
            unpack<DT>(buf[u], z);
            const int vec = (it * U + u) * BLOCK + tid;
            cmax[u] = accumulate<EPV, CLAMP, COUNT, true, SECOND, EXACT>(a, z, rs.first_idx + vec * EPV, zcmp, &buf[u]);
        }
        if (store_cm) cm_store_batch<DT, U>(cm_lane, it * U, cmax);
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
            if (vec0 + u * BLOCK < rs.nvec) rem[u] = __builtin_nontemporal_load(rs.vbase + (vec0 + u * BLOCK));
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int vec = vec0 + u * BLOCK;
            if (vec < rs.nvec) {
                float z[EPV];
                unpack<DT>(rem[u], z);
                const float cmax = accumulate<EPV, CLAMP, COUNT, false, SECOND, EXACT>(a, z, rs.first_idx + vec * EPV, zcmp, &rem[u]);
                if (store_cm) cm_store<DT>(cm_lane, nsuper * U + u, cmax);
            }
        }
    }
    if (tid < rs.tail_n) {
        const int idx = rs.tail0 + tid;
        const float z1[1] = {load_elt<DT>(rs.base, idx)};
        accumulate<1, CLAMP, COUNT, false, SECOND, EXACT>(a, z1, idx, zcmp);
    }
}

// The same pass for a SHORT launch (verification of one decode step), where every workgroup of the launch is on
// the GPU from the start and nothing but the lane's own loads can hide memory latency: a ring of D vectors per
// lane is requested at once, and each vector's slot is refilled as soon as it has been folded in, so D loads per
// lane stay in flight from the first instruction to the last vector.  (With two alternating buffers a lane waits a
// full memory round trip for every other batch; a long launch hides that behind its other workgroups, a short one
// does not: measured 18 us for 74 MB against 12 us for a plain read of the same bytes.)
// Elements are folded in the same order as in sweep_lane, so the lane's sums are the same bit for bit.
template <int DT, bool CLAMP, int BLOCK, int D, bool EXACT>
__device__ __forceinline__ void sweep_lane_ring(LaneAcc& a, const SegShape& rs, int tid)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    lane_acc_init(a);
    const int nfull = rs.nvec / BLOCK;                      // vectors that every lane owns
    const bool extra = tid < rs.nvec - nfull * BLOCK;       // the first lanes own one more
    const u32x4* const lane_base = rs.vbase + tid;

    float zh = 0.f, zt = 0.f;
    if (tid < rs.head_n) zh = load_elt<DT>(rs.base, tid);
    u32x4 ring[D];
#pragma unroll
    for (int j = 0; j < D; ++j)
        if (j < nfull) ring[j] = __builtin_nontemporal_load(lane_base + (size_t)j * BLOCK);
    u32x4 xv = {0u, 0u, 0u, 0u};
    if (extra) xv = __builtin_nontemporal_load(lane_base + (size_t)nfull * BLOCK);
    if (tid < rs.tail_n) zt = load_elt<DT>(rs.base, rs.tail0 + tid);

    if (tid < rs.head_n) {
        const float z1[1] = {zh};
        accumulate<1, CLAMP, false, false, false, EXACT>(a, z1, tid, 0.f);
    }
    for (int base = 0; base < nfull; base += D) {
#pragma unroll
        for (int j = 0; j < D; ++j) {
            const int i = base + j;
            if (i < nfull) {   // the same in every lane
                float z[EPV];
                const u32x4 raw = ring[j];
                unpack<DT>(raw, z);
                if (i + D < nfull) ring[j] = __builtin_nontemporal_load(lane_base + (size_t)(i + D) * BLOCK);
                accumulate<EPV, CLAMP, false, true, false, EXACT>(a, z, rs.first_idx + (i * BLOCK + tid) * EPV, 0.f, &raw);
            }
        }
    }
    if (extra) {
        float z[EPV];
        unpack<DT>(xv, z);
        accumulate<EPV, CLAMP, false, false, false, EXACT>(a, z, rs.first_idx + (nfull * BLOCK + tid) * EPV, 0.f, &xv);
    }
    if (tid < rs.tail_n) {
        const float z1[1] = {zt};
        accumulate<1, CLAMP, false, false, false, EXACT>(a, z1, rs.tail0 + tid, 0.f);
    }
}

// Visit every element of this lane's share once more (used by the rare exact fallback).
template <int DT, int BLOCK, typename F>
__device__ __forceinline__ void for_each_own_element(const SegShape& rs, int tid, F&& f)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    if (tid < rs.head_n) f(load_elt<DT>(rs.base, tid), tid);
    for (int vec = tid; vec < rs.nvec; vec += BLOCK) {
        float z[EPV];
        unpack<DT>(rs.vbase[vec], z);
#pragma unroll
        for (int e = 0; e < EPV; ++e) f(z[e], rs.first_idx + vec * EPV + e);
    }
    if (tid < rs.tail_n) f(load_elt<DT>(rs.base, rs.tail0 + tid), rs.tail0 + tid);
}

// Record the r-th pick in the (register-resident) ranked list.
__device__ __forceinline__ void set_pick(float (&kz)[AASD_MAX_CANDSET], int (&ki)[AASD_MAX_CANDSET], int r, float z, int i)
{
#pragma unroll
    for (int q = 0; q < AASD_MAX_CANDSET; ++q)
        if (q == r) { kz[q] = z; ki[q] = i; }
}

// Exact top-c of the wave's share above z_next by c re-reads of the share; only used when the
// candidate buffer overflowed (more than 64 tokens of one wave tied near the top).
template <int DT, int BLOCK>
__device__ void wave_topc_by_rescan(const SegShape& rs, int tid, float znext, int c, float (&kz)[AASD_MAX_CANDSET],
                                    int (&ki)[AASD_MAX_CANDSET], int& nK)
{
    float pz = INFINITY;
    int pi = -1;
    nK = 0;
    for (int r = 0; r < c; ++r) {
        float bz = -INFINITY;
        int bi = 0x7fffffff;
        for_each_own_element<DT, BLOCK>(rs, tid, [&](float z, int idx) {
            const bool after_prev = (r == 0) || z < pz || (z == pz && idx > pi);
            if (z > znext && after_prev && better(z, idx, bz, bi)) { bz = z; bi = idx; }
        });
        wave_best(bz, bi);
        if (bi == 0x7fffffff) break;  // the same in every lane
        pz = bz; pi = bi;
        set_pick(kz, ki, r, bz, bi);
        nK = r + 1;
    }
}

// Top-c of per-lane entries (PER_LANE each, invalid ones at -inf / INT_MAX): c rounds of "best remaining".
template <int PER_LANE>
__device__ __forceinline__ void wave_topc(float (&lz)[PER_LANE], int (&li)[PER_LANE], int c, float (&kz)[AASD_MAX_CANDSET],
                                          int (&ki)[AASD_MAX_CANDSET], int& nK)
{
    nK = 0;
    for (int r = 0; r < c; ++r) {
        float bz = lz[0];
        int bi = li[0];
#pragma unroll
        for (int q = 1; q < PER_LANE; ++q)
            if (better(lz[q], li[q], bz, bi)) { bz = lz[q]; bi = li[q]; }
        wave_best(bz, bi);
        if (bi == 0x7fffffff) break;
#pragma unroll
        for (int q = 0; q < PER_LANE; ++q)
            if (li[q] == bi) { lz[q] = -INFINITY; li[q] = 0x7fffffff; }
        set_pick(kz, ki, r, bz, bi);
        nK = r + 1;
    }
}

// LDS of the sweep kernel besides the chunk maxima: one short list of chunk positions per wave.
template <int NW>
struct SweepShared {
    int list[NW][kListCap];
    unsigned count[NW];
};

// One attempt of a wave at its share.  Returns false (in every lane) if the sums came out
// non-finite, which happens when the share holds -inf logits; the caller repeats with CLAMP.
template <int DT, bool ALIGN, bool COUNT, bool CLAMP, int BLOCK, int U, bool COHERENT, bool EXACT, int RING>
__device__ __forceinline__ bool process_wave(const SweepParams& p, const SegShape& rs, bool has_next, float znext,
                                             SweepShared<BLOCK / kWave>& sh, unsigned char* cm_lane, const RowShape& row_s,
                                             WavePartial* out, int32_t* out_list)
{
    constexpr int EPV = Elt<DT>::kPerVec;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const bool want_cand = ALIGN && has_next && p.want_cand;
    const float zcmp = has_next ? znext : INFINITY;

    LaneAcc a;
    if constexpr (RING > 0) sweep_lane_ring<DT, CLAMP, BLOCK, RING, EXACT>(a, rs, tid);
    else sweep_lane<DT, CLAMP, ALIGN && COUNT, ALIGN, BLOCK, U, EXACT>(a, rs, tid, zcmp, want_cand && p.cm_enabled, cm_lane);

    // ---- wave maximum, and a lower bound on the c-th largest logit of the wave's share ----
    const float G = quad_max(a.vmax);  // the maximum of this lane's 4-lane group
    const float m = wave_max(a.vmax);
    float thr2 = -INFINITY;
    if (ALIGN && want_cand && znext < m) {   // the same in every lane
        // The 16 group maxima are 16 distinct elements, so the c-th largest of them (c <= 8) bounds the
        // c-th largest logit from below; the number of elements above this bound has a light tail, unlike a
        // minimum over c classes.  Every lane ranks its group's maximum among the 16 (ties by group index;
        // the values arrive by constant-lane reads, no chain of dependent shuffles), and the group whose rank
        // is c - 1 names the bound.
        const int g = lane >> 2;
        int rank = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const float x = __shfl(G, q << 2);
            rank += (x > G || (x == G && q < g)) ? 1 : 0;
        }
        const unsigned long long owners = __ballot(rank == p.c - 1);
        thr2 = __shfl(G, __ffsll((long long)owners) - 1);
    }

    // ---- lane sums brought to the common reference m ----
    const float M2 = m * kLog2e;
    const float res = fmaf(m, kLog2e, -M2);  // rounding error of M2, so that the maximum weighs exactly 1
    const float ssum = (a.s[0] + a.s[1]) + (a.s[2] + a.s[3]);
    const float tsum = (a.t[0] + a.t[1]) + (a.t[2] + a.t[3]);
    const float dlt = (a.r2 - M2) - res;
    const float f = __builtin_amdgcn_exp2f(dlt);
    const float S = wave_sum(ssum * f);
    const float T = wave_sum((tsum + dlt * ssum) * f);
    if (!CLAMP) {
        if (!(S > 0.f) || !(S < INFINITY) || T != T) return false;
    }
    int own = a.vmax == m ? a.code : 0x7fffffff;
    if (EXACT && a.vmax == m && a.code >= row_s.head && a.code < row_s.tail0) {
        // the lane's maximum lies in a 16-byte chunk that it kept: the first element of the chunk that attains it
        float zb[EPV];
        unpack<DT>(a.best, zb);
        int off = 0;
#pragma unroll
        for (int e = EPV - 1; e >= 0; --e) off = zb[e] == m ? e : off;
        own = a.code + off;
    }
    const int code = wave_min(own);
    unsigned cnt = 0;
    if (ALIGN && COUNT) cnt = a.cnt_u + wave_sum(a.cnt_l);

    // ---- chunks of this wave's share that can hold a token of the row's top-c above the prompt token ----
    int nlist = 0;
    if (want_cand && znext < m) {
        if (lane == 0) sh.count[wid] = 0;
        auto note = [&](int first_elem) {
            const unsigned pos = atomicAdd(&sh.count[wid], 1u);
            if (pos < (unsigned)kListCap) sh.list[wid][pos] = first_elem;
        };
        const bool qualifies = a.vmax > znext && a.vmax >= thr2;
        // Almost every qualifying lane has exactly one chunk at or above the bound, the one that set its maximum,
        // and knows where it is; only a lane whose second largest chunk maximum qualifies too looks again.
        const bool several = qualifies && a.v2 > znext && a.v2 >= thr2;
        if (qualifies && !several) note(a.code);
        if (several) {
            if (tid < rs.head_n) {
                const float z = load_elt<DT>(rs.base, tid);
                if (z > znext && z >= thr2) note(tid);
            }
            if (p.cm_enabled) {
                // this lane's chunk maxima, 16 bytes at a time (LDS only; entries past the lane's last chunk are ignored)
                const int nown = tid < rs.nvec ? (rs.nvec - tid + BLOCK - 1) / BLOCK : 0;
                for (int j0 = 0; j0 < nown; j0 += EPV) {
                    float cmx[EPV];
                    unpack<DT>(*(const u32x4*)(cm_lane + (size_t)j0 * Elt<DT>::kBytes), cmx);
                    unsigned hits = 0;   // straight-line test of the EPV maxima; the rare hits are handled after it
#pragma unroll
                    for (int e = 0; e < EPV; ++e)
                        hits |= (j0 + e < nown && cmx[e] > znext && cmx[e] >= thr2) ? 1u << e : 0u;
                    while (hits) {
                        const int e = __ffs((int)hits) - 1;
                        hits &= hits - 1;
                        note(rs.first_idx + ((j0 + e) * BLOCK + tid) * EPV);
                    }
                }
            } else {
                // vocabulary too large for LDS: look at every chunk again
                for (int vec = tid; vec < rs.nvec; vec += BLOCK) {
                    float z[EPV];
                    unpack<DT>(rs.vbase[vec], z);
                    float cmx = z[0];
#pragma unroll
                    for (int e = 1; e < EPV; ++e) cmx = fmaxf(cmx, z[e]);
                    if (cmx > znext && cmx >= thr2) note(rs.first_idx + vec * EPV);
                }
            }
            if (tid < rs.tail_n) {
                const float z = load_elt<DT>(rs.base, rs.tail0 + tid);
                if (z > znext && z >= thr2) note(rs.tail0 + tid);
            }
        }
        __threadfence_block();  // the wave's LDS appends are complete before they are read back
        const unsigned n = sh.count[wid];
        if (n <= (unsigned)kListCap) {
            nlist = (int)n;
            if (lane < nlist) out_list[lane] = sh.list[wid][lane];
        } else {
            // more than kListCap chunks tie near the top: find the share's exact top-c and list their chunks
            float kz[AASD_MAX_CANDSET];
            int ki[AASD_MAX_CANDSET];
#pragma unroll
            for (int q = 0; q < AASD_MAX_CANDSET; ++q) { kz[q] = 0.f; ki[q] = -1; }
            wave_topc_by_rescan<DT, BLOCK>(rs, tid, znext, p.c, kz, ki, nlist);
            if (lane < nlist) {
                int idx = -1;
#pragma unroll
                for (int q = 0; q < AASD_MAX_CANDSET; ++q)
                    if (q == lane) idx = ki[q];
                const bool in_body = idx >= row_s.head && idx < row_s.tail0;
                out_list[lane] = in_body ? row_s.head + (idx - row_s.head) / EPV * EPV : idx;
            }
        }
    }

    if (lane == 0) {
        WavePartial wp;
        wp.m = m; wp.S = S; wp.T = T; wp.code = code; wp.cnt = cnt; wp.nlist = nlist; wp.thr2 = thr2; wp.pad = 0;
        if (COHERENT) store_partial_coherent(out, wp);
        else *out = wp;
    }
    return true;
}

// One unit of work: segment `seg` of row `row`; every wave writes one WavePartial.
// COHERENT: the partial is written for a reader in another workgroup of the same launch.
// EXACT: the partial's `code` is the index of the share's first maximum itself (verification only).
// local_out: if given (an array of one WavePartial per wave, in LDS), the waves leave their partials there and
// nothing goes to the workspace: the caller merges them.
// RING > 0: the short-launch form of the pass with that many loads per lane in flight (verification only).
template <int DT, bool ALIGN, bool COUNT, int BLOCK, int U, bool COHERENT = false, bool EXACT = false, int RING = 0>
__device__ __forceinline__ void sweep_unit(const SweepParams& p, int64_t row, int seg, SweepShared<BLOCK / kWave>& sh,
                                           unsigned char* cm, WavePartial* local_out = nullptr)
{
    constexpr int NW = BLOCK / kWave;
    // rows of consecutive sequences that follow one another in memory (the usual case) need no division
    const int64_t off = p.seq_stride == (int64_t)p.rows_per_seq * p.row_stride
                            ? row * p.row_stride
                            : (row / p.rows_per_seq) * p.seq_stride + (row % p.rows_per_seq) * p.row_stride;
    const RowShape row_s = row_shape<DT>(p.logits, off, p.V);
    const SegShape rs = seg_shape<DT>(row_s, p.V, seg, p.nseg, p.seg_vecs);
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;

    const int64_t slot = (row * p.nseg + seg) * NW + wid;
    WavePartial* out = local_out ? local_out + wid : p.partials + slot;
    int32_t* out_list = ALIGN ? p.lists + slot * kListCap : nullptr;

    // a wave whose lanes own no element at all leaves the neutral partial
    const bool owns = tid < rs.head_n || tid < rs.nvec || tid < rs.tail_n;
    if (__ballot(owns) == 0ull) {
        if (lane == 0) {
            WavePartial wp;
            wp.m = -INFINITY; wp.S = 0.f; wp.T = 0.f; wp.code = 0x7fffffff; wp.cnt = 0; wp.nlist = 0; wp.thr2 = -INFINITY; wp.pad = 0;
            if (COHERENT) store_partial_coherent(out, wp);
            else *out = wp;
        }
        return;
    }

    int nt = -1;
    float znext = 0.f;
    if (ALIGN) {
        nt = p.next_tok ? p.next_tok[row] : -1;
        if (nt >= p.V) nt = -1;
        if (nt >= 0) znext = load_elt<DT>(row_s.base, nt);
        if (p.cand_all) znext = -INFINITY;
    }
    const bool has_next = ALIGN && (nt >= 0 || p.cand_all);
    unsigned char* cm_lane = cm + (size_t)tid * (size_t)p.cm_stride;
    static_assert(!(EXACT && ALIGN) && !(RING > 0 && ALIGN), "the alignment sweep lists chunks by their first element");
    if (!process_wave<DT, ALIGN, COUNT, false, BLOCK, U, COHERENT, EXACT, RING>(p, rs, has_next, znext, sh, cm_lane, row_s, out, out_list))
        process_wave<DT, ALIGN, COUNT, true, BLOCK, U, COHERENT, EXACT, RING>(p, rs, has_next, znext, sh, cm_lane, row_s, out, out_list);
}

// Scale factor and exponent shift that bring a partial with maximum pm to the row maximum m.
__device__ __forceinline__ void partial_scale(float pm, float m, float& dl, float& f)
{
    dl = (pm - m) * kLog2e;  // <= 0, log2 units
    f = __builtin_amdgcn_exp2f(dl);
}

// The partials of a workgroup's NW waves (in LDS) merged into one; called by the lanes of the first wave, the
// result is complete in every lane.
template <int NW>
__device__ __forceinline__ WavePartial merge_wave_partials(const WavePartial* wave_part, int lane)
{
    WavePartial wp;
    wp.m = -INFINITY; wp.S = 0.f; wp.T = 0.f; wp.code = 0x7fffffff;
    if (lane < NW) wp = wave_part[lane];
    const float m = group_reduce(wp.m, NW, [](float x, float y) { return fmaxf(x, y); });
    const bool live = wp.S > 0.f;
    float dl2 = 0.f, f = 0.f;
    if (live) partial_scale(wp.m, m, dl2, f);
    const float S = group_reduce(live ? wp.S * f : 0.f, NW, [](float x, float y) { return x + y; });
    const float T2 = group_reduce(live ? (wp.T + dl2 * wp.S) * f : 0.f, NW, [](float x, float y) { return x + y; });
    const int code = group_reduce(live && wp.m == m ? wp.code : 0x7fffffff, NW, [](int x, int y) { return min(x, y); });
    WavePartial out;
    out.m = m; out.S = S; out.T = T2; out.code = code; out.cnt = 0; out.nlist = 0; out.thr2 = -INFINITY; out.pad = 0;
    return out;
}

// u / nseg for a unit index below 2^28 (a launch has at most 2^22) without an integer division: one multiply.
__device__ __forceinline__ uint32_t div_by_segments(uint32_t u, int nseg, uint32_t magic)
{
    return div_small(u, nseg, magic);
}

// Streaming kernel: grid = rows x segments; the launch starts at row row0.
template <int DT, bool ALIGN, bool COUNT, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void row_sweep_kernel(SweepParams p, int64_t row0)
{
    constexpr int NW = BLOCK / kWave;
    extern __shared__ __align__(16) unsigned char cm[];  // chunk maxima of this segment (alignment sampling only)
    __shared__ SweepShared<ALIGN ? NW : 1> sh_store;
    SweepShared<NW>& sh = *reinterpret_cast<SweepShared<NW>*>(&sh_store);  // not touched unless ALIGN

    const uint32_t q = div_by_segments(blockIdx.x, p.nseg, p.nseg_magic);
    const int64_t row = row0 + q;
    const int seg = (int)(blockIdx.x - q * (uint32_t)p.nseg);
    if constexpr (!ALIGN) {
        if (p.merge_waves) {   // one partial per workgroup: a short launch with many segments per row, whose tail is then shorter
            __shared__ WavePartial wave_part[NW];
            sweep_unit<DT, ALIGN, COUNT, BLOCK, U>(p, row, seg, sh, cm, wave_part);
            __syncthreads();
            if (threadIdx.x < kWave) {
                const WavePartial out = merge_wave_partials<NW>(wave_part, threadIdx.x);
                if (threadIdx.x == 0) p.partials[row * p.nseg + seg] = out;
            }
            return;
        }
    }
    sweep_unit<DT, ALIGN, COUNT, BLOCK, U>(p, row, seg, sh, cm);
}

// The same sweep for sequences that use only their first max(rows_used[seq], 1) rows (tree verification).
// The launch covers at most BLOCK sequences.  Every workgroup first scans their row counts into LDS, which
// numbers the used rows consecutively; the workgroups then share those rows x segments round robin, so the
// work is spread evenly however uneven the sequences are.  Rows that are not in use are neither read nor
// given partials.  The grid is sized to the machine, not to the input: a workgroup whose first unit lies
// beyond the total ends at once.
template <int DT, int BLOCK, int U>
__global__ __launch_bounds__(BLOCK) void row_sweep_used_kernel(SweepParams p, int64_t seq0, int nseq)
{
    constexpr int NW = BLOCK / kWave;
    __shared__ SweepShared<1> sh_store;
    SweepShared<NW>& sh = *reinterpret_cast<SweepShared<NW>*>(&sh_store);  // never touched: no alignment sampling here
    __shared__ int offs[BLOCK + 1];   // offs[s] = used rows of the sequences before s
    __shared__ int wave_total[NW];

    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    int v = 0;
    if (tid < nseq) {
        v = p.rows_used[seq0 + tid];
        v = v < 1 ? 1 : (v > p.rows_per_seq ? p.rows_per_seq : v);
    }
    const int incl = wave_inclusive_scan(v);
    if (lane == 63) wave_total[wid] = incl;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w2 = 0; w2 < NW; ++w2) before += (w2 < wid) ? wave_total[w2] : 0;
    offs[tid + 1] = before + incl;
    if (tid == 0) offs[0] = 0;
    __syncthreads();

    const int units = __builtin_amdgcn_readfirstlane(offs[nseq]) * p.nseg;
    for (int unit = blockIdx.x; unit < units; unit += gridDim.x) {
        const int crow = (int)div_by_segments((uint32_t)unit, p.nseg, p.nseg_magic);
        int lo = 0, hi = nseq;   // the sequence s with offs[s] <= crow < offs[s + 1]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (offs[mid] <= crow) lo = mid; else hi = mid;
        }
        // the unit is the same in every lane: keep it in scalar registers (values read from LDS arrive in vector ones)
        const int r_in_seq = __builtin_amdgcn_readfirstlane(crow - offs[lo]);
        const int seq_local = __builtin_amdgcn_readfirstlane(lo);
        const int64_t row = (seq0 + seq_local) * p.rows_per_seq + r_in_seq;
        sweep_unit<DT, false, false, BLOCK, U>(p, row, unit - crow * p.nseg, sh, nullptr);
    }
}

}  // namespace aasd
