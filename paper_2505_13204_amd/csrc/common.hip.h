// Device helpers shared by the AASD kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "aasd.h"

namespace aasd {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;   // fp32(log2 e); every exponent below uses this one value
constexpr double kLn2 = 0.69314718055994530942;
constexpr float kNegHuge = -1.0e30f;             // finite stand-in for -inf in the clamped sweep

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT> struct Elt;
template <> struct Elt<AASD_BF16> {
    static constexpr int kBytes = 2;
    static constexpr int kPerVec = 8;  // elements in one 16-byte load
};
template <> struct Elt<AASD_F32> {
    static constexpr int kBytes = 4;
    static constexpr int kPerVec = 4;
};

__device__ __forceinline__ float bits_to_float(uint32_t b) { return __uint_as_float(b); }

// One element of a row, widened exactly to fp32.
template <int DT>
__device__ __forceinline__ float load_elt(const void* row, int64_t idx)
{
    if constexpr (DT == AASD_BF16) {
        return bits_to_float((uint32_t)((const uint16_t*)row)[idx] << 16);
    } else {
        return ((const float*)row)[idx];
    }
}

// The elements of one 16-byte vector in memory order.
template <int DT>
__device__ __forceinline__ void unpack(const u32x4& v, float (&z)[Elt<DT>::kPerVec])
{
    if constexpr (DT == AASD_BF16) {
        // bf16 is the upper half of an fp32: the low element of each dword moves up, the high one is masked
        z[0] = bits_to_float(v.x << 16); z[1] = bits_to_float(v.x & 0xffff0000u);
        z[2] = bits_to_float(v.y << 16); z[3] = bits_to_float(v.y & 0xffff0000u);
        z[4] = bits_to_float(v.z << 16); z[5] = bits_to_float(v.z & 0xffff0000u);
        z[6] = bits_to_float(v.w << 16); z[7] = bits_to_float(v.w & 0xffff0000u);
    } else {
        z[0] = bits_to_float(v.x); z[1] = bits_to_float(v.y);
        z[2] = bits_to_float(v.z); z[3] = bits_to_float(v.w);
    }
}

// Reductions over the 64 lanes of a wave; every lane ends with the result and the combination order is fixed,
// so sums are reproducible.  They go through the cross-lane data path of the vector ALU, not through LDS
// permutes: four steps inside each row of 16 lanes (swap neighbours, swap pairs, mirror the half row, mirror the
// row), after which every lane holds its row's result, then the four rows' results through scalar registers.
// (A butterfly of six LDS permutes has ten times the latency, and a wave's epilogue is a chain of such
// reductions.)
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
constexpr int kDppSwap1 = 0xB1, kDppSwap2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;
__device__ __forceinline__ float lane_value(float v, int lane) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane)); }
__device__ __forceinline__ int lane_value(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }

// maximum of the lane's group of four lanes (lanes 4g .. 4g+3)
__device__ __forceinline__ float quad_max(float v)
{
    v = fmaxf(v, dpp_move<kDppSwap1>(v));
    return fmaxf(v, dpp_move<kDppSwap2>(v));
}
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<kDppSwap1>(v);
    v += dpp_move<kDppSwap2>(v);
    v += dpp_move<kDppHalfMirror>(v);
    v += dpp_move<kDppMirror>(v);
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
__device__ __forceinline__ unsigned wave_sum(unsigned u)
{
    int v = (int)u;
    v += dpp_move<kDppSwap1>(v);
    v += dpp_move<kDppSwap2>(v);
    v += dpp_move<kDppHalfMirror>(v);
    v += dpp_move<kDppMirror>(v);
    return (unsigned)(lane_value(v, 0) + lane_value(v, 16) + lane_value(v, 32) + lane_value(v, 48));
}
__device__ __forceinline__ float wave_max(float v)
{
    v = quad_max(v);
    v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_move<kDppMirror>(v));
    return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
__device__ __forceinline__ int wave_max(int v)
{
    v = max(v, dpp_move<kDppSwap1>(v));
    v = max(v, dpp_move<kDppSwap2>(v));
    v = max(v, dpp_move<kDppHalfMirror>(v));
    v = max(v, dpp_move<kDppMirror>(v));
    return max(max(lane_value(v, 0), lane_value(v, 16)), max(lane_value(v, 32), lane_value(v, 48)));
}
__device__ __forceinline__ int wave_min(int v)
{
    v = min(v, dpp_move<kDppSwap1>(v));
    v = min(v, dpp_move<kDppSwap2>(v));
    v = min(v, dpp_move<kDppHalfMirror>(v));
    v = min(v, dpp_move<kDppMirror>(v));
    return min(min(lane_value(v, 0), lane_value(v, 16)), min(lane_value(v, 32), lane_value(v, 48)));
}

// Inclusive prefix sum over the 64 lanes of a wave (every lane takes part), through the vector ALU's cross-lane
// moves: shifts by 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source add zero), then the last lane of
// row 0 (and of row 2) is added to the next row, and the last lane of row 1 to rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118, kRowBcast15 = 0x142, kRowBcast31 = 0x143;
    v += __builtin_amdgcn_update_dpp(0, v, kRowShr1, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, kRowShr2, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, kRowShr4, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, kRowShr8, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, kRowBcast15, 0xa, 0xf, false);   // into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, kRowBcast31, 0xc, 0xf, false);   // into rows 2 and 3
    return v;
}

// All-reduce over the lane's aligned group of G <= 64 lanes (G a power of two, the same in every lane; every lane of
// the wave takes part): inside a row of 16 lanes through the vector ALU's cross-lane moves, beyond it through scalar
// registers.  The order of combination is fixed.
template <class T, class OP>
__device__ __forceinline__ T group_reduce(T v, int G, OP op)
{
    if (G > 1) v = op(v, dpp_move<kDppSwap1>(v));
    if (G > 2) v = op(v, dpp_move<kDppSwap2>(v));
    if (G > 4) v = op(v, dpp_move<kDppHalfMirror>(v));
    if (G > 8) v = op(v, dpp_move<kDppMirror>(v));
    if (G > 16) {   // 32 or 64 lanes: every row of 16 holds its result by now; the rows' results through scalar registers
        const T r0 = lane_value(v, 0), r1 = lane_value(v, 16), r2 = lane_value(v, 32), r3 = lane_value(v, 48);
        if (G >= 64) v = op(op(r0, r1), op(r2, r3));
        else v = (threadIdx.x & 32) ? op(r2, r3) : op(r0, r1);
    }
    return v;
}

// Total order used for "best token": larger logit first, then smaller id.
__device__ __forceinline__ bool better(float za, int ia, float zb, int ib)
{
    return za > zb || (za == zb && ia < ib);
}
__device__ __forceinline__ void wave_best(float& z, int& i)
{
    const float bz = wave_max(z);
    i = wave_min(z == bz ? i : 0x7fffffff);
    z = bz;
}

// Plain fill of n 32-bit words (used where a memset node must not enter a captured graph).
__global__ __launch_bounds__(256) void fill_u32_kernel(unsigned* dst, unsigned value, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = value;
}

// Philox4x32 with 10 rounds (Salmon et al., SC'11): counter-based, integer only.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    constexpr uint32_t kMul0 = 0xD2511F53u, kMul1 = 0xCD9E8D57u;
    constexpr uint32_t kWeyl0 = 0x9E3779B9u, kWeyl1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kMul0 * c0, p1 = (uint64_t)kMul1 * c2;  // one 32x32->64 multiply each
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += kWeyl0; k1 += kWeyl1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// u / d by one multiply, for u < 2^32 / d: magic = floor(2^32 / d) + 1, computed by the host (0 for d = 1).
__device__ __forceinline__ uint32_t div_small(uint32_t u, int d, uint32_t magic)
{
    return d == 1 ? u : __umulhi(u, magic);
}

}  // namespace aasd
