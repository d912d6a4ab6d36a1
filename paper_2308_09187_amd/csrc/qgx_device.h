// Device-side helpers for the gfx950 kernels: the counter-based generator, wavefront scans and
// reductions, and small bit utilities.  64-wide wavefronts throughout.
#pragma once

#include "qgx_internal.h"

namespace qgx {

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x >> 6); }

// Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  The key schedule is uniform
// across the wave, so the compiler keeps it in scalar registers; the two 32x32->64 products per
// round are the cost.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Two standard normal draws from two words of a Philox block (Box-Muller): u1 = (2 (w >> 9) + 1) 2^-24 in
// (0, 1), u2 = (w' >> 8) 2^-24 in [0, 1), r = sqrt(-2 ln u1), (r cos 2 pi u2, r sin 2 pi u2).  Both
// uniforms are exact in binary32; logarithm, root, sine and cosine are the hardware's (v_log_f32 in base
// 2, v_sin_f32 and v_cos_f32 take their argument in turns), good to about 1e-6, which is ample for noise.
__device__ __forceinline__ float2 box_muller(uint32_t w_radius, uint32_t w_angle)
{
    const float u1 = (float)(2u * (w_radius >> 9) + 1u) * 0x1p-24f;
    const float u2 = (float)(w_angle >> 8) * 0x1p-24f;
    const float r = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(u1));   // -2 ln 2 * log2 u1
    return make_float2(r * __builtin_amdgcn_cosf(u2), r * __builtin_amdgcn_sinf(u2));
}

// Coordinates i0 .. i0 + 3 (i0 a multiple of 4) of F(z) = M z + b.
__device__ __forceinline__ float4 game_operator_row(const GameArgs& G, uint32_t i0)
{
    const float4 z = *reinterpret_cast<const float4*>(G.z + i0);
    const float4 b = *reinterpret_cast<const float4*>(G.b + i0);
    const float2 a = *reinterpret_cast<const float2*>(G.a + (i0 >> 1));
    float4 f;
    f.x = (G.mu * z.x + a.x * z.y) + b.x;
    f.y = (G.mu * z.y - a.x * z.x) + b.y;
    f.z = (G.mu * z.z + a.y * z.w) + b.z;
    f.w = (G.mu * z.w - a.y * z.z) + b.w;
    return f;
}

// The same four coordinates of worker k's dual vector in call `call_id`: F(z) + sigma N, the noise from the
// Philox block with key (seed_lo, seed_hi) and counter (i0 / 4, 1, k, call_id).
__device__ __forceinline__ float4 game_dual_row(const GameArgs& G, uint32_t i0, uint32_t k, uint32_t call_id)
{
    uint32_t w[4];
    philox4x32_10(i0 >> 2, 1u, k, call_id, G.seed_lo, G.seed_hi, w);
    const float2 n01 = box_muller(w[0], w[1]), n23 = box_muller(w[2], w[3]);
    float4 v = game_operator_row(G, i0);
    v.x += G.sigma * n01.x;
    v.y += G.sigma * n01.y;
    v.z += G.sigma * n23.x;
    v.w += G.sigma * n23.y;
    return v;
}

// Between two phases in which the lanes of a wave exchange data through LDS without a workgroup barrier.
// The hardware runs a wave's LDS instructions in the order they were issued; this keeps the compiler from
// moving them across the boundary, or from making one side of the exchange part of a branch that only
// some lanes take.  No instruction is emitted.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Inclusive prefix sum over the 64 lanes of a wave with DPP row shifts and row broadcasts: four
// shifted adds inside each row of 16 lanes, then lane 15 of a row into the next row, then lane 31
// into the upper half.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x)
{
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);   // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);   // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);   // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);   // row_shr:8
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1,3
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2,3
    return x;
}

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
    return x;
}

__device__ __forceinline__ uint32_t wave_or(uint32_t x)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) x |= (uint32_t)__shfl_xor((int)x, off, kWave);
    return x;
}

__device__ __forceinline__ uint32_t bcast_lane(uint32_t x, int src)
{
    return (uint32_t)__shfl((int)x, src, kWave);
}

// A 16-byte load of data that is read once: marked non-temporal, so that it does not push what is
// reused (the coded streams a later kernel reads back) out of the caches.
typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 nt_load4(const float* p)
{
    const nt_f32x4 r = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4*>(p));
    return make_float4(r.x, r.y, r.z, r.w);
}

typedef uint32_t nt_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 nt_load4u(const uint4* p)
{
    const nt_u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4*>(p));
    return make_uint4(r.x, r.y, r.z, r.w);
}

// t^q for a small positive integer q (the same q in every lane).
__device__ __forceinline__ double pow_int(double t, uint32_t q)
{
    double r = 1.0;
    for (; q; q >>= 1) {
        if (q & 1u) r *= t;
        t *= t;
    }
    return r;
}

// s^(1/q) for s >= 1 in binary64: a single-precision guess, then Newton steps on x^q = s (each one
// squares the error, so three reach the last bits from a guess good to 1e-6).
__device__ __forceinline__ double root_int(double s, uint32_t q)
{
    double x = (double)__builtin_amdgcn_exp2f(__builtin_amdgcn_logf((float)s) / (float)q);   // v_exp_f32, v_log_f32: base 2
    for (int it = 0; it < 3; ++it) {
        const double xq1 = pow_int(x, q - 1u);
        x -= (xq1 * x - s) / ((double)q * xq1);
    }
    return x;
}

// LDS accesses by byte address.  A pointer derived from the dynamic LDS array carries the array's
// base as a late-bound addend that the compiler adds again on every access; an address computed once
// as an integer does not.
__device__ __forceinline__ uint32_t lds_address(const void* p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

typedef uint32_t lds_u32x2 __attribute__((ext_vector_type(2)));
typedef float lds_f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint2 lds_load_u2(uint32_t addr)
{
    const lds_u32x2 r = *(const __attribute__((address_space(3))) lds_u32x2*)(uintptr_t)addr;
    return make_uint2(r.x, r.y);
}

__device__ __forceinline__ float4 lds_load_f4(uint32_t addr)
{
    const lds_f32x4 r = *(const __attribute__((address_space(3))) lds_f32x4*)(uintptr_t)addr;
    return make_float4(r.x, r.y, r.z, r.w);
}

__device__ __forceinline__ void raise_error(Scalars* sc, unsigned int bit)
{
    atomicOr(&sc->err, bit);
}

}  // namespace qgx
