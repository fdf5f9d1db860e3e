// Pieces shared by the matrix-core kernels: rebuilding fp16 weights from bit-plane words.
#pragma once

#include "hlq_internal.h"

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

// In a plane word, bits p and p+16 are the adjacent weights k0 = 2p, 2p+1 of the word's 32-k block.
// (w << t) & 0x20002000 isolates pair p at bit 13 of both 16-bit halves: as packed fp16 that is
// (2^-7 b[2p], 2^-7 b[2p+1]); with 0x40004000 (bit 14) it is (2 b, 2 b).  Position (13 or 14) and
// left shift that bring pair p there; pair 15 is reached with a right shift by one (shift = -1).
__host__ __device__ constexpr int hlq_pair_pos(int p) { return p == 15 ? 14 : (p == 0 ? 14 : (p % 2 == 1 ? 13 : 14)); }
__host__ __device__ constexpr int hlq_pair_shift(int p) { return p == 15 ? -1 : hlq_pair_pos(p) - p; }

// Pre-scaled scales of one quant segment as packed pairs: s * 2^7 for pairs read at bit 13,
// s / 2 for pairs read at bit 14, and (z, z).  Requires |s| < 512.
template <int Q>
struct HlqSegScales {
    half2v z2, s13[Q], s14[Q];
    // mt: fp16 bit patterns of s_0 .. s_{Q-1}, z (16- or 32-bit containers)
    template <typename T>
    __device__ __forceinline__ void set(const T (&mt)[Q + 1])
    {
        const _Float16 z = __builtin_bit_cast(_Float16, (uint16_t)mt[Q]);
        z2 = (half2v){z, z};
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const _Float16 s = __builtin_bit_cast(_Float16, (uint16_t)mt[j]);
            const _Float16 a = s * (_Float16)128.0f, b = s * (_Float16)0.5f;
            s13[j] = (half2v){a, a};
            s14[j] = (half2v){b, b};
        }
    }
};

// W^ of weights 2p, 2p+1 of one plane-word set (Eq. 3) as packed fp16: (W^[2p], W^[2p + 1]).
template <int Q>
__device__ __forceinline__ uint32_t hlq_rebuild_pair(const uint32_t (&w)[Q], const HlqSegScales<Q> &sc, int p)
{
    half2v o = sc.z2;
#pragma unroll
    for (int j = 0; j < Q; ++j) {
        const uint32_t sh = hlq_pair_shift(p) < 0 ? (w[j] >> 1) : (w[j] << (hlq_pair_shift(p) < 0 ? 0 : hlq_pair_shift(p)));
        const uint32_t m = sh & (hlq_pair_pos(p) == 13 ? 0x20002000u : 0x40004000u);
        o = __builtin_bit_cast(half2v, m) * (hlq_pair_pos(p) == 13 ? sc.s13[j] : sc.s14[j]) + o;
    }
    return __builtin_bit_cast(uint32_t, o);
}

// W^ of the 32 weights of word d of one column: wp[p] = (W^[32d + 2p], W^[32d + 2p + 1]).
// 8 shifts + 16 ANDs per plane and 16 packed FMAs per plane.
template <int Q>
__device__ __forceinline__ void hlq_rebuild_word(const uint32_t (&w)[Q], const HlqSegScales<Q> &sc, uint32_t (&wp)[16])
{
#pragma unroll
    for (int p = 0; p < 16; ++p) wp[p] = hlq_rebuild_pair<Q>(w, sc, p);
}
