// philox.h -- Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11) and the
// draws built on it, device side.  Written from the published definition of the generator:
// ten rounds of two 32x32->64 multiplications by fixed odd constants, with the high halves
// xor-ed into the neighbouring words and the round key, and the key advanced by the Weyl
// constants between rounds.
//
// Keying used by every synthetic draw of the library:
//   key     = (seed low word, seed high word)
//   counter = (group, stream, worker k, iteration t), group = element index / 4
// The four output words give the four elements 4*group .. 4*group+3.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qsr {

struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}

__device__ __forceinline__ U4 draw4(uint64_t seed, uint32_t stream, uint32_t k, uint32_t t,
                                    uint32_t group)
{
    return philox4x32_10(group, stream, k, t, (uint32_t)seed, (uint32_t)(seed >> 32));
}

// Box-Muller on one pair of words.  u1 = ((a>>9)+1/2) 2^-23 lies in (0,1) and u2 = (b>>8) 2^-24
// in [0,1); both are exact in single precision, and the angle is taken through sincospi so that
// no rounding of 2*pi*u2 enters.
__device__ __forceinline__ void box_muller(uint32_t a, uint32_t b, float &za, float &zb)
{
    float u1 = ((float)(a >> 9) + 0.5f) * 1.1920928955078125e-7f;   // 2^-23
    float u2x2 = (float)(b >> 8) * 1.1920928955078125e-7f;          // 2*u2
    float rad = sqrtf(-2.0f * logf(u1));
    float sn, cs;
    sincospif(u2x2, &sn, &cs);
    za = rad * cs;
    zb = rad * sn;
}

// the four standard normals of a group
__device__ __forceinline__ float4 normal4(uint64_t seed, uint32_t stream, uint32_t k, uint32_t t,
                                          uint32_t group)
{
    U4 r = draw4(seed, stream, k, t, group);
    float4 z;
    box_muller(r.x, r.y, z.x, z.y);
    box_muller(r.z, r.w, z.z, z.w);
    return z;
}

// integer in [0, n): high word of r * n
__device__ __forceinline__ uint32_t index_from_word(uint32_t r, uint32_t n)
{
    return (uint32_t)(((uint64_t)r * n) >> 32);
}

}  // namespace qsr
