// n-gram draft retrieval over the token buffer (Sec. 3.1; Algorithm 1, longest key first).
//
// One workgroup per sequence.  The context is staged through LDS in tiles.  Each lane owns a
// run of consecutive positions of the tile and slides a polynomial hash of the n_min tokens
// before the position along its run (one multiply-add in, one out per step); positions whose
// hash equals the hash of the context's last n_min tokens are confirmed token by token and
// extended backwards to the longest matching key (at most n_max).  The hash is only a filter:
// every reported hit has been compared exactly.  The longest key length found anywhere wins;
// a second, descending pass over the per-position match lengths compacts the hits of that
// length in order (wave ballot + popcount prefix), latest occurrence first, at most C.
#pragma once

#include "common.hip.h"

namespace aasd {

constexpr int kRetrieveBlock = 1024;       // threads per sequence when there are few sequences (latency)
constexpr int kRetrieveBlockSmall = 256;   // and when there are many (more sequences in flight per compute unit)
constexpr int kRetrieveTileSlots = 64;  // tiles whose longest match is remembered (later ones are always looked at again)
constexpr uint32_t kHashBase = 0x9E3779B1u;  // odd multiplier of the window hash (mod 2^32)

struct RetrieveParams {
    const int32_t* tokens;
    int64_t tok_stride;
    const int32_t* len;
    const int32_t* prompt_len;
    int32_t B, n_min, n_max, k, C;
    const int32_t* extras;
    const uint8_t* n_extras;
    int32_t m_x;
    int64_t extras_stride;
    int32_t* drafts;
    int32_t* draft_len;
    int32_t* src_pos;
    int32_t* n_cand;
    int32_t* key_len;
    int32_t* draft_extras;
    uint8_t* strict;
    int32_t run;   // positions per lane per tile (odd: LDS accesses of a wave then hit distinct banks)
    int32_t tile;  // positions per tile = threads per workgroup * run
};

// Write the outputs of one sequence from the candidate positions pos[0 .. ncand) (latest first): the
// continuations, their lengths and source flags, and the alignment extras of the copied prompt positions.
template <int BLOCK>
__device__ __forceinline__ void write_candidates(const RetrieveParams& p, int b, const int32_t* tok, int len, int plen,
                                                 const int32_t* pos, int ncand, int n_star, int tid)
{
    const int C = p.C, k = p.k;
    for (int i = tid; i < C * k; i += BLOCK) {
        const int c = i / k, j = i - c * k;
        const size_t bc = (size_t)b * C + c;
        const int pp = c < ncand ? pos[c] : -1;
        const int dl = pp >= 0 ? min(k, len - pp) : 0;
        const bool in = j < dl;
        p.drafts[bc * k + j] = in ? tok[pp + j] : -1;
        p.strict[bc * k + j] = (in && pp + j >= plen) ? 1 : 0;  // copied from generated context
        if (p.draft_extras) {
            for (int e = 0; e < p.m_x; ++e) {
                int32_t val = -1;
                // prefill row pp+j-1 predicted the token at pp+j; it has a next prompt token iff pp+j <= plen-1
                if (in && pp + j <= plen - 1 && (int64_t)(pp + j - 1) < p.extras_stride) {
                    const size_t row = (size_t)b * p.extras_stride + (size_t)(pp + j - 1);
                    const int32_t x = p.extras[row * p.m_x + e];   // asked for beside the count, not after it
                    if (e < (int)p.n_extras[row]) val = x;
                }
                p.draft_extras[(bc * k + j) * p.m_x + e] = val;
            }
        }
        if (j == 0) {
            p.draft_len[bc] = dl;
            p.src_pos[bc] = pp;
        }
    }
    if (tid == 0) {
        p.n_cand[b] = ncand;
        p.key_len[b] = ncand > 0 ? n_star : 0;
    }
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void retrieve_kernel(RetrieveParams p)
{
    constexpr int NW = BLOCK / kWave;
    extern __shared__ __align__(16) unsigned char smem[];
    int32_t* ltok = (int32_t*)smem;                           // ltok[i] = tok[tlo - AASD_MAX_KEY + i]
    uint8_t* ell = (uint8_t*)(ltok + AASD_MAX_KEY + p.tile);  // match length of every position of the tile
    __shared__ int32_t suffix[AASD_MAX_KEY];                  // suffix[i] = tok[len - 1 - i]
    __shared__ int s_best;
    __shared__ int tile_best[kRetrieveTileSlots];             // longest match inside each of the first tiles
    __shared__ int wave_cnt[NW];
    __shared__ int32_t pos[AASD_MAX_CANDIDATES];

    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int32_t* tok = p.tokens + (int64_t)b * p.tok_stride;
    int len = p.len[b];
    if (len < 0 || (int64_t)len > p.tok_stride) len = 0;
    const int plen = p.prompt_len[b];
    const int n_min = p.n_min, C = p.C, k = p.k;
    const int n_cap = min(p.n_max, len - 1);  // a key must be shorter than the context

    // A context that fits one tile is staged at once, and the continuations are then read from LDS instead of
    // through further dependent loads from memory.  The last tokens (the keys) are asked for beside the tile's,
    // so the chain of dependent loads is: length, tokens.
    const bool one_tile = len <= p.tile;
    int32_t last_tok = 0;
    if (tid < AASD_MAX_KEY && len - 1 - tid >= 0) last_tok = tok[len - 1 - tid];
    if (one_tile)
        for (int i = tid; i < len + AASD_MAX_KEY; i += BLOCK) ltok[i] = i >= AASD_MAX_KEY ? tok[i - AASD_MAX_KEY] : 0;
    if (tid < AASD_MAX_KEY) suffix[tid] = last_tok;
    if (tid == 0) s_best = 0;
    for (int i = tid; i < kRetrieveTileSlots; i += BLOCK) tile_best[i] = 0;
    __syncthreads();

    int n_star = 0, count = 0;
    if (n_cap >= n_min) {
        // hash of the last n_min tokens, and B^n_min for sliding
        uint32_t hs = 0, bpow = 1;
        for (int i = 0; i < n_min; ++i) {
            hs = hs * kHashBase + (uint32_t)suffix[n_min - 1 - i];
            bpow *= kHashBase;
        }
        // A short context is spread over all threads: a thread's run of positions is a serial loop, so it is made
        // as short as the context allows (odd, like the host's choice for a full tile).
        const int tile = p.tile;
        const int run = one_tile ? min(p.run, ((len + BLOCK - 1) / BLOCK) | 1) : p.run;
        const int ntiles = (len + tile - 1) / tile;

        // Stage tile t and compute the match length of each of its positions.
        auto stage_and_match = [&](int t) -> int {
            const int tlo = t * tile;
            const int thi = min(tlo + tile, len);
            const int first = tlo - AASD_MAX_KEY;
            if (!one_tile) {
                for (int i = tid; i < thi - first; i += BLOCK) ltok[i] = (first + i >= 0) ? tok[first + i] : 0;
                __syncthreads();
            }
            int best = 0;
            const int pstart = tlo + tid * run;
            uint32_t h = 0;
            bool have = false;
            for (int q = 0; q < run; ++q) {
                const int pp = pstart + q;
                if (pp >= thi) break;
                int l = 0;
                if (pp >= n_min) {
                    if (!have) {  // first position of the run: hash the window tok[pp-n_min .. pp-1] directly
                        h = 0;
                        for (int i = 0; i < n_min; ++i) h = h * kHashBase + (uint32_t)ltok[pp - n_min + i - first];
                        have = true;
                    } else {      // slide by one: drop tok[pp-1-n_min], take tok[pp-1]
                        h = h * kHashBase - (uint32_t)ltok[pp - 1 - n_min - first] * bpow + (uint32_t)ltok[pp - 1 - first];
                    }
                    if (h == hs) {
                        const int cap = min(n_cap, pp);
                        int ll = 0;
                        while (ll < cap && ltok[pp - 1 - ll - first] == suffix[ll]) ++ll;
                        if (ll >= n_min) l = ll;  // otherwise a hash collision
                    }
                }
                ell[pp - tlo] = (uint8_t)l;
                best = max(best, l);
            }
            return best;
        };

        // pass A: longest key that occurs anywhere, and in which tiles
        int best = 0;
        for (int t = 0; t < ntiles; ++t) {
            if (t > 0) __syncthreads();  // the previous tile is no longer read
            int tb = stage_and_match(t);
            best = max(best, tb);
            if (ntiles > 1 && t < kRetrieveTileSlots) {   // which tiles hold the longest key matters only if there are several
                tb = wave_max(tb);
                if (lane == 0 && tb > 0) atomicMax(&tile_best[t], tb);
            }
        }
        best = wave_max(best);
        if (lane == 0 && best > 0) atomicMax(&s_best, best);
        __syncthreads();
        n_star = s_best;

        // pass B: hits of that key length, latest first.  Tiles without such a hit are skipped; in the others a
        // thread counts the hits of its run, one scan over the threads (in descending position order) gives every
        // thread the number of later hits, and it writes its own, latest first, while there is room.
        if (n_star > 0) {
            int resident = ntiles - 1;   // the tile whose match lengths are in LDS
            for (int t = ntiles - 1; t >= 0 && count < C; --t) {
                if (ntiles > 1 && t < kRetrieveTileSlots && tile_best[t] < n_star) continue;   // the same in every thread
                if (t != resident) {   // every thread is past the barrier that ended its reads of the tile before
                    stage_and_match(t);
                    resident = t;
                }
                // a thread reads the match lengths of its own run only: no barrier between writing and counting them
                const int tlo = t * tile;
                const int thi = min(tlo + tile, len);
                const int pstart = tlo + tid * run;
                int mine = 0;
                for (int q = 0; q < run; ++q) {
                    const int pp = pstart + q;
                    if (pp < thi && ell[pp - tlo] >= n_star) ++mine;
                }
                // hits in threads with a higher index: over the lanes bit by bit of the count (a count is below 64:
                // ballots and population counts, no trips through LDS), then over the waves
                const unsigned long long above = lane == 63 ? 0ull : (~0ull << (lane + 1));
                int later = 0, wave_total = 0;
#pragma unroll
                for (int bit = 0; bit < 6; ++bit) {
                    const unsigned long long has = __ballot((mine >> bit) & 1);
                    later += __popcll(has & above) << bit;
                    wave_total += __popcll(has) << bit;
                }
                if (lane == 0) wave_cnt[wid] = wave_total;
                __syncthreads();
                int total = 0;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const int cw = wave_cnt[w];
                    if (w > wid) later += cw;
                    total += cw;
                }
                int slot = count + later;
                for (int q = run - 1; q >= 0 && mine > 0 && slot < C; --q) {
                    const int pp = pstart + q;
                    if (pp < thi && ell[pp - tlo] >= n_star) pos[slot++] = pp;
                }
                count += total;
                __syncthreads();   // wave_cnt and ell are reused by the next tile
            }
        }
    }
    __syncthreads();

    write_candidates<BLOCK>(p, b, one_tile ? ltok + AASD_MAX_KEY : tok, len, plen, pos, min(count, C), n_star, tid);
}

}  // namespace aasd
