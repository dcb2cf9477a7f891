// Full-vocabulary seeded sampling of the extra draft tokens (Sec. 3.2 read literally: the extras of a
// misaligned position are sampled from the whole output distribution of its prefill row).
// m draws without replacement in proportion to the softmax probability are the m largest keys
// z_v + G_v with independent standard Gumbel G_v (Gumbel-top-k); every token needs one uniform, taken
// from a counter-based generator so that the draws depend on (seed, row id, token) only.
#pragma once

#include "common.hip.h"

namespace aasd {

constexpr int kGumbelBlock = 256;
constexpr float kGumbelNear = 5.0e-5f;            // key gaps below this are reported as near decisions (fp32 keys err by < 1e-5)

struct GumbelParams {
    const void* logits;
    int32_t V;
    int64_t row_stride;
    const int32_t* next_tok;     // [rows]
    const uint8_t* misaligned;   // [rows]: rows with 0 get no extras
    int32_t m_x;
    uint64_t seed, row_id_base;
    int32_t* extras;             // [rows, m_x]
    uint8_t* n_extras;           // [rows]
    float* extra_keys;           // [rows, m_x] or null: the keys of the picks
    uint32_t* near_count;        // or null
    int32_t nseg;                // workgroups per row: each takes a contiguous share of the row's groups of four tokens
    float* part_z;               // [rows, nseg, K] best keys of every share, descending (scratch)
    int32_t* part_i;             // [rows, nseg, K] their tokens (INT_MAX = empty)
};

// Standard Gumbel variate from 23 random bits: x = (bits + 1/2) / 2^23 in (0, 1), E = -ln(1 - x) is a
// unit exponential, G = -ln E = -ln2 (log2(-log2(1 - x)) + log2(ln 2)).  1 - x is exact in fp32, and the
// hardware log2 is accurate to 1e-7 relative also for arguments next to 1 (measured over all 2^22 values of
// x below 1/2), so no series is needed for small x.
__device__ __forceinline__ float gumbel_from_bits(uint32_t word)
{
    const float x = ((float)(word >> 9) + 0.5f) * (1.0f / 8388608.0f);  // exact in fp32
    const float t = -__builtin_amdgcn_logf(1.0f - x);                   // E / ln 2
    return fmaf(-0.69314718f, __builtin_amdgcn_logf(t), 0.36651292f);   // 0.36651292 = -ln(ln 2)
}

// Keep the K largest keys a lane has seen, in descending order.  Elements arrive in ascending token id, so a
// strict comparison keeps equal keys in id order.  Branch-free inside: the caller skips it for a whole wave.
template <int K>
__device__ __forceinline__ void keep_insert(float (&kz)[K], int (&ki)[K], float z, int i)
{
    bool gt[K];
#pragma unroll
    for (int q = 0; q < K; ++q) gt[q] = z > kz[q];
#pragma unroll
    for (int q = K - 1; q > 0; --q) {
        kz[q] = gt[q - 1] ? kz[q - 1] : (gt[q] ? z : kz[q]);
        ki[q] = gt[q - 1] ? ki[q - 1] : (gt[q] ? i : ki[q]);
    }
    kz[0] = gt[0] ? z : kz[0];
    ki[0] = gt[0] ? i : ki[0];
}

// Merge (z, i) into a list sorted by `better` (key descending, id ascending), dropping the last entry.
template <int K>
__device__ __forceinline__ void keep_merge(float (&kz)[K], int (&ki)[K], float z, int i)
{
    if (!better(z, i, kz[K - 1], ki[K - 1])) return;
    kz[K - 1] = z; ki[K - 1] = i;
#pragma unroll
    for (int q = K - 1; q > 0; --q) {
        if (better(kz[q], ki[q], kz[q - 1], ki[q - 1])) {
            const float tz = kz[q]; kz[q] = kz[q - 1]; kz[q - 1] = tz;
            const int ti = ki[q]; ki[q] = ki[q - 1]; ki[q - 1] = ti;
        }
    }
}

// nseg workgroups per row, each over a contiguous share of the row (few misaligned rows would otherwise leave
// most of the GPU idle); workgroups of rows that are not misaligned end at once.  Tokens are handled four at
// a time (one Philox block); a lane keeps its K = m + 1 best keys in registers (the extra one gives the last
// pick's margin); waves merge by "best head" rounds, the workgroup through LDS, and the K best of the share go
// to scratch for gumbel_merge_kernel.  Tokens with a logit of -inf have probability zero and are never drawn.
template <int DT, int K>
__global__ __launch_bounds__(kGumbelBlock) void gumbel_extras_kernel(GumbelParams p, int64_t row0)
{
    constexpr int NW = kGumbelBlock / kWave;
    __shared__ float s_z[NW][K];
    __shared__ int s_i[NW][K];

    const int64_t unit = row0 + blockIdx.x;
    const int64_t row = unit / p.nseg;
    const int seg = (int)(unit - row * p.nseg);
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    if (!p.misaligned[row]) return;   // aligned (or no next token): the merge kernel writes the empty outputs
    const int V = p.V;
    const int nt = p.next_tok ? p.next_tok[row] : -1;
    const char* base = (const char*)p.logits + (size_t)row * (size_t)p.row_stride * Elt<DT>::kBytes;
    const uint64_t row_id = p.row_id_base + (uint64_t)row;
    const uint32_t c0 = (uint32_t)row_id, c1 = (uint32_t)(row_id >> 32);
    const uint32_t k0 = (uint32_t)p.seed, k1 = (uint32_t)(p.seed >> 32);
    // four elements at once when the row starts on a multiple of their size
    const bool wide = ((uintptr_t)base % (4 * Elt<DT>::kBytes)) == 0;

    float kz[K];
    int ki[K];
#pragma unroll
    for (int q = 0; q < K; ++q) { kz[q] = -INFINITY; ki[q] = 0x7fffffff; }

    // Most tokens cannot be among the K best of the row and need not be inserted anywhere: the K-th largest of the
    // wave's 64 lane maxima (tau) is a key that K tokens seen so far reach, so a token below it is out for good.
    // tau is brought up to date after 1, 2, 4, 8, ... steps (it only rises, and a stale one only lets more tokens
    // through); a token at or above it is inserted into its lane's list as before, and the insertion code is
    // skipped whenever no lane of the wave has such a token, which is soon the usual case.  Every lane takes
    // every step (a lane beyond the end of the share holds keys of -inf), so the wave-wide operations see all lanes.
    float tau = -INFINITY;
    const int nquad = (V + 3) >> 2;
    const int per_seg = (nquad + p.nseg - 1) / p.nseg;
    const int q_end = min(nquad, (seg + 1) * per_seg);
    int step = 0, next_update = 1;
    for (int q0 = seg * per_seg; q0 < q_end; q0 += kGumbelBlock, ++step) {
        const int q = q0 + tid;
        const bool have = q < q_end;
        const int v0 = q << 2;
        float z[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (have) {
            if (wide && v0 + 3 < V) {
                if constexpr (DT == AASD_BF16) {
                    const uint2 w = *(const uint2*)(base + (size_t)v0 * 2);
                    z[0] = bits_to_float(w.x << 16); z[1] = bits_to_float(w.x & 0xffff0000u);
                    z[2] = bits_to_float(w.y << 16); z[3] = bits_to_float(w.y & 0xffff0000u);
                } else {
                    const float4 w = *(const float4*)(base + (size_t)v0 * 4);
                    z[0] = w.x; z[1] = w.y; z[2] = w.z; z[3] = w.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) z[j] = v0 + j < V ? load_elt<DT>(base, v0 + j) : -INFINITY;
            }
        }
        uint32_t rnd[4];
        philox4x32_10(c0, c1, (uint32_t)q, 0x47554D42u, k0, k1, rnd);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int v = v0 + j;
            float key = z[j] + gumbel_from_bits(rnd[j]);
            key = (have && v < V && v != nt && key >= tau) ? key : -INFINITY;   // -inf is never kept
            if (__ballot(key > -INFINITY) != 0ull) keep_insert<K>(kz, ki, key, v);
        }
        if (step == next_update - 1) {
            next_update <<= 1;
            float x = kz[0], t = -INFINITY;
#pragma unroll
            for (int r = 0; r < K; ++r) {   // the K-th largest lane maximum, equal values counted as often as they occur
                t = wave_max(x);
                const unsigned long long holders = __ballot(x == t);
                if (lane == __ffsll((long long)holders) - 1) x = -INFINITY;
            }
            tau = t;
        }
    }

    // ---- the wave's K best: a lane whose head wins a round pops it ----
    float wz[K];
    int wi[K];
#pragma unroll
    for (int r = 0; r < K; ++r) {
        float bz = kz[0];
        int bi = ki[0];
        wave_best(bz, bi);
        wz[r] = bz; wi[r] = bi;
        if (bi == ki[0] && bi != 0x7fffffff) {
#pragma unroll
            for (int q = 0; q + 1 < K; ++q) { kz[q] = kz[q + 1]; ki[q] = ki[q + 1]; }
            kz[K - 1] = -INFINITY; ki[K - 1] = 0x7fffffff;
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < K; ++r) { s_z[wid][r] = wz[r]; s_i[wid][r] = wi[r]; }
    }
    __syncthreads();
    if (tid == 0) {
        float fz[K];
        int fi[K];
#pragma unroll
        for (int q = 0; q < K; ++q) { fz[q] = -INFINITY; fi[q] = 0x7fffffff; }
        for (int w = 0; w < NW; ++w)
            for (int r = 0; r < K; ++r)
                if (s_i[w][r] != 0x7fffffff) keep_merge<K>(fz, fi, s_z[w][r], s_i[w][r]);
        const size_t slot = ((size_t)row * p.nseg + seg) * K;
#pragma unroll
        for (int j = 0; j < K; ++j) { p.part_z[slot + j] = fz[j]; p.part_i[slot + j] = fi[j]; }
    }
}

// A thread per row merges the shares' best keys and writes the picks, best first.
template <int K>
__global__ __launch_bounds__(kGumbelBlock) void gumbel_merge_kernel(GumbelParams p, int64_t rows)
{
    const int64_t row = (int64_t)blockIdx.x * kGumbelBlock + threadIdx.x;
    if (row >= rows) return;
    float fz[K];
    int fi[K];
#pragma unroll
    for (int q = 0; q < K; ++q) { fz[q] = -INFINITY; fi[q] = 0x7fffffff; }
    if (p.misaligned[row]) {
        for (int s = 0; s < p.nseg; ++s) {
            const size_t slot = ((size_t)row * p.nseg + s) * K;
            for (int j = 0; j < K; ++j) {
                const int i = p.part_i[slot + j];
                if (i != 0x7fffffff) keep_merge<K>(fz, fi, p.part_z[slot + j], i);
            }
        }
    }
    int n_out = 0;
    bool near = false;
#pragma unroll
    for (int j = 0; j < K - 1; ++j) {
        const bool have = fi[j] != 0x7fffffff;
        p.extras[row * p.m_x + j] = have ? fi[j] : -1;
        if (p.extra_keys) p.extra_keys[row * p.m_x + j] = have ? fz[j] : 0.f;
        if (have) {
            ++n_out;
            if (fi[j + 1] != 0x7fffffff && fz[j] - fz[j + 1] < kGumbelNear) near = true;
        }
    }
    p.n_extras[row] = (uint8_t)n_out;
    if (near && p.near_count) atomicAdd(p.near_count, 1u);
}

}  // namespace aasd
