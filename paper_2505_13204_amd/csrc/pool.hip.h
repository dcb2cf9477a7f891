// Persistent draft pool (Sec. 3.1; Algorithm 1: the dictionary from n-grams to the positions that follow
// them, built once over the prompt and extended by the windows that end in the newly generated tokens).
//
// Per sequence and key length n the pool is a chained hash table in HBM: head[bucket] is the latest position
// whose n preceding tokens hash to the bucket, prev[p] the one before it.  Positions are inserted in
// ascending order, so a chain lists them latest first, which is the order retrieval wants.  Chains mix
// n-grams that collide: every visited position is compared token by token, so results never depend on the
// hash.  A lookup follows one chain per key length instead of scanning the context.
#pragma once

#include "retrieve.hip.h"

namespace aasd {

struct PoolLayout {
    int32_t B, capacity, n_min, n_max;
    int32_t log2_table;   // buckets per table = 1 << log2_table
    // byte offsets from the pool's base
    size_t counters;      // int32 [B][NL]: next position to insert
    size_t tables;        // per (b, nl): head[1 << log2_table] then prev[capacity + 1], int32
    size_t table_stride;  // bytes per (b, nl)
};

__device__ __forceinline__ uint32_t pool_bucket(const int32_t* tok, int p, int n, int log2_table)
{
    uint32_t h = 0;
    for (int i = 0; i < n; ++i) h = h * kHashBase + (uint32_t)tok[p - n + i];
    return (h * 0x85EBCA6Bu) >> (32 - log2_table);
}

struct PoolUpdateParams {
    char* pool;
    PoolLayout lay;
    const int32_t* tokens;
    int64_t tok_stride;
    const int32_t* len;
    int32_t reset;
};

// One wave per (sequence, key length), for the few new positions of a decode step (and as the general case
// of any range).  Positions are taken 64 at a time in ascending order: a lane links its
// position to the nearest lower lane of the batch with the same bucket, else to the table's head as it was
// before the batch; the highest lane of each bucket becomes the new head.  The batch's stores are fenced
// before the next batch reads the heads (the reads bypass the vector cache).
__device__ __forceinline__ void pool_update_wave(const PoolUpdateParams& q, int b, int nl, int lane)
{
    const PoolLayout& L = q.lay;
    const int NL = L.n_max - L.n_min + 1;
    const int n = L.n_min + nl;
    int32_t* counter = (int32_t*)(q.pool + L.counters) + (size_t)b * NL + nl;
    int32_t* head = (int32_t*)(q.pool + L.tables + ((size_t)b * NL + nl) * L.table_stride);
    int32_t* prev = head + ((size_t)1 << L.log2_table);
    const int32_t* tok = q.tokens + (int64_t)b * q.tok_stride;
    int len = q.len[b];
    if (len < 0 || (int64_t)len > q.tok_stride) len = 0;
    if (len > L.capacity) len = L.capacity;

    int start;
    if (q.reset) {
        const int T = 1 << L.log2_table;
        for (int i = lane; i < T; i += kWave) head[i] = -1;
        __threadfence();
        start = n;
    } else {
        start = *counter;
        if (start < n) start = n;
    }
    for (int p0 = start; p0 <= len; p0 += kWave) {
        const int p = p0 + lane;
        const bool have = p <= len;
        const int bucket = have ? (int)pool_bucket(tok, p, n, L.log2_table) : -1;
        int h = -1;
        if (have) h = __hip_atomic_load(&head[bucket], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int last = -1;
        bool later = false;
        const int cnt = min(kWave, len + 1 - p0);   // the batch's positions sit in lanes 0 .. cnt-1 (a decode step: a few)
        for (int j = 0; j < cnt; ++j) {
            const int bj = __builtin_amdgcn_readlane(bucket, j);
            if (bj == bucket && j < lane) last = j;
            if (bj == bucket && j > lane) later = true;
        }
        if (have) {
            prev[p] = last >= 0 ? p0 + last : h;
            if (!later) __hip_atomic_store(&head[bucket], p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __threadfence();
    }
    if (lane == 0) *counter = (len + 1 > start) ? len + 1 : start;
}

constexpr int kPoolBuildWaves = 16;                         // waves per workgroup of the build kernel
constexpr int kPoolBuildBlock = kPoolBuildWaves * kWave;
constexpr int kPoolBuildTile = 8192;                        // positions staged in LDS at a time
constexpr int kPoolBuildDepth = 32;                         // batches whose head exchanges are in flight together
constexpr uint32_t kPoolBucketMask = (1u << 25) - 1u;       // a bucket has at most 25 bits (capacity <= 2^24)

// Many positions at once (the build over a prompt): a workgroup per (sequence, key length), a tile of positions
// at a time, in two phases.  Phase 1, all waves, a batch of 64 consecutive positions each: the bucket of every
// position; a lane links its position to the nearest lower lane of the batch with the same bucket; the lowest
// and the highest lane of every bucket are noted in LDS (with the bucket: flag and lane in the 7 spare bits).
// Phase 2, the first wave, batch by batch in ascending order: the highest lane of a bucket exchanges the head for
// its position, and what the exchange returns (the head before the batch) becomes the link of the bucket's
// lowest lane.  All exchanges come from one wave in program order, so the chains descend without a fence between
// batches, and the exchanges of 32 batches are in flight together.  A decode step's few new positions take the
// one-wave path above.
__global__ __launch_bounds__(kPoolBuildBlock) void pool_build_kernel(PoolUpdateParams q)
{
    __shared__ uint32_t linfo[kPoolBuildTile];
    __shared__ int32_t ltok[kPoolBuildTile + AASD_MAX_KEY];   // ltok[i] = tok[t0 - AASD_MAX_KEY + i]
    const PoolLayout& L = q.lay;
    const int NL = L.n_max - L.n_min + 1;
    const int b = blockIdx.x / NL, nl = blockIdx.x - b * NL;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int n = L.n_min + nl;
    int32_t* counter = (int32_t*)(q.pool + L.counters) + (size_t)b * NL + nl;
    int32_t* head = (int32_t*)(q.pool + L.tables + ((size_t)b * NL + nl) * L.table_stride);
    int32_t* prev = head + ((size_t)1 << L.log2_table);
    const int32_t* tok = q.tokens + (int64_t)b * q.tok_stride;
    int len = q.len[b];
    if (len < 0 || (int64_t)len > q.tok_stride) len = 0;
    if (len > L.capacity) len = L.capacity;

    int start = n;
    if (!q.reset) {
        start = *counter;
        if (start < n) start = n;
        if (len + 1 - start <= kWave) {
            if (wid == 0) pool_update_wave(q, b, nl, lane);
            return;
        }
    } else {
        const int T = 1 << L.log2_table;
        for (int i = tid; i < T; i += kPoolBuildBlock) head[i] = -1;
        __threadfence();
    }
    __syncthreads();    // the table is empty; every wave has read the counter before it is written below

    for (int t0 = start; t0 <= len; t0 += kPoolBuildTile) {
        const int tile_n = min(kPoolBuildTile, len + 1 - t0);
        // the tile's tokens and the AASD_MAX_KEY before them, all loads in flight together (start >= n, so every
        // window of the tile lies at or after position 0)
        for (int i = tid; i < tile_n + AASD_MAX_KEY; i += kPoolBuildBlock) {
            const int src = t0 - AASD_MAX_KEY + i;
            ltok[i] = (src >= 0 && src < len) ? tok[src] : 0;
        }
        __syncthreads();
        // phase 1
        for (int g0 = wid * kWave; g0 < tile_n; g0 += kPoolBuildBlock) {
            const int i = g0 + lane;
            const bool have = i < tile_n;
            const uint32_t bucket = have ? pool_bucket(ltok, AASD_MAX_KEY + i, n, L.log2_table) : 0xFFFFFFFFu;
            unsigned long long same = 0;
#pragma unroll
            for (int j = 0; j < kWave; ++j) {
                const uint32_t bj = (uint32_t)__builtin_amdgcn_readlane((int)bucket, j);
                if (bj == bucket) same |= 1ull << j;
            }
            if (have) {
                const unsigned long long lower = same & ((1ull << lane) - 1ull);
                const bool top = (same >> lane) == 1ull;
                const int low = __ffsll((long long)same) - 1;
                if (lower) prev[t0 + i] = t0 + g0 + (63 - __clzll((long long)lower));
                linfo[i] = bucket | ((uint32_t)low << 25) | (top ? 0x80000000u : 0u);
            }
        }
        __syncthreads();
        // phase 2
        if (wid == 0) {
            for (int g0 = 0; g0 < tile_n; g0 += kWave * kPoolBuildDepth) {
                int old[kPoolBuildDepth];
#pragma unroll
                for (int d = 0; d < kPoolBuildDepth; ++d) {
                    const int i = g0 + d * kWave + lane;
                    const uint32_t v = i < tile_n ? linfo[i] : 0u;
                    old[d] = -1;
                    if (v & 0x80000000u)
                        old[d] = __hip_atomic_exchange(&head[v & kPoolBucketMask], t0 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int d = 0; d < kPoolBuildDepth; ++d) {
                    const int i = g0 + d * kWave + lane;
                    const uint32_t v = i < tile_n ? linfo[i] : 0u;
                    if (v & 0x80000000u) prev[t0 + g0 + d * kWave + (int)((v >> 25) & 63u)] = old[d];
                }
            }
        }
        __syncthreads();   // the tile's notes are no longer read
    }
    if (tid == 0) *counter = (len + 1 > start) ? len + 1 : start;
}

struct PoolRetrieveParams {
    const char* pool;
    PoolLayout lay;
    RetrieveParams r;   // tokens, lengths, k, C, extras table and all outputs as for the stateless kernel
};

// One wave per sequence.  Longest key first: the chain of the key's bucket is followed from the head; a
// visited position p counts if it has a continuation (p <= len - 1) and its n preceding tokens equal the
// key (lane i compares token i).  The first key length with a hit wins; at most C hits, latest first.
__device__ __forceinline__ void pool_retrieve_wave(const PoolRetrieveParams& q, int b, int lane, int32_t* pos)
{
    const PoolLayout& L = q.lay;
    const RetrieveParams& p = q.r;
    const int NL = L.n_max - L.n_min + 1;
    const int32_t* tok = p.tokens + (int64_t)b * p.tok_stride;
    int len = p.len[b];
    if (len < 0 || (int64_t)len > p.tok_stride) len = 0;
    const int plen = p.prompt_len[b];
    const int n_cap = min(L.n_max, len - 1);  // a key must be shorter than the context

    int found = 0, n_star = 0;
    for (int n = n_cap; n >= L.n_min && found == 0; --n) {
        const int nl = n - L.n_min;
        const int32_t* head = (const int32_t*)(q.pool + L.tables + ((size_t)b * NL + nl) * L.table_stride);
        const int32_t* prev = head + ((size_t)1 << L.log2_table);
        const int key_tok = lane < n ? tok[len - n + lane] : 0;
        int cur = head[pool_bucket(tok, len, n, L.log2_table)];
        for (int hops = 0; hops <= L.capacity && cur >= n && cur <= L.capacity && found < p.C; ++hops) {
            const int nxt = prev[cur];
            if (cur <= len - 1) {
                const bool same = lane < n ? tok[cur - n + lane] == key_tok : true;
                if (__all(same)) {
                    if (lane == 0) pos[found] = cur;
                    ++found;
                }
            }
            if (nxt >= cur) break;  // chains strictly descend: anything else is not a chain of this pool
            cur = nxt;
        }
        if (found > 0) n_star = n;
    }
    __threadfence_block();   // the wave's own LDS writes of pos[] before its lanes read them
    write_candidates<kWave>(p, b, tok, len, plen, pos, found, n_star, lane);
}

__global__ __launch_bounds__(kWave) void pool_retrieve_kernel(PoolRetrieveParams q)
{
    __shared__ int32_t pos[AASD_MAX_CANDIDATES];
    pool_retrieve_wave(q, blockIdx.x, threadIdx.x, pos);
}

// One decode step in one launch: a workgroup per sequence with one wave per key length.  Every wave first
// indexes the new positions of its table; after a barrier the first wave looks the key up.
__global__ __launch_bounds__(AASD_MAX_KEY * kWave) void pool_step_kernel(PoolRetrieveParams q)
{
    __shared__ int32_t pos[AASD_MAX_CANDIDATES];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    PoolUpdateParams u;
    u.pool = const_cast<char*>(q.pool); u.lay = q.lay; u.tokens = q.r.tokens; u.tok_stride = q.r.tok_stride;
    u.len = q.r.len; u.reset = 0;
    pool_update_wave(u, b, wid, lane);
    __threadfence();
    __syncthreads();
    if (wid == 0) pool_retrieve_wave(q, b, lane, pos);
}

}  // namespace aasd
