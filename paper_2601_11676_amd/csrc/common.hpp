// Device-side helpers shared by the HIP kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace halo {

typedef uint16_t bf16_t;   // storage only: upper half of an IEEE float
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte load

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// float -> bf16, round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// Eight consecutive elements -> eight floats.  p must be 16-byte aligned.
__device__ __forceinline__ void load8(const float *__restrict__ p, float (&o)[8])
{
    float4 a = *reinterpret_cast<const float4 *>(p);
    float4 b = *reinterpret_cast<const float4 *>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}

__device__ __forceinline__ void unpack8(const u32x4 &v, float (&o)[8])
{
    o[0] = bf16_lo(v.x); o[1] = bf16_hi(v.x);
    o[2] = bf16_lo(v.y); o[3] = bf16_hi(v.y);
    o[4] = bf16_lo(v.z); o[5] = bf16_hi(v.z);
    o[6] = bf16_lo(v.w); o[7] = bf16_hi(v.w);
}

__device__ __forceinline__ void load8(const bf16_t *__restrict__ p, float (&o)[8])
{
    u32x4 v = *reinterpret_cast<const u32x4 *>(p);
    unpack8(v, o);
}

// Eight consecutive elements kept as loaded (bf16 stays packed: half the registers) until used.
template <typename WT> struct Piece8;
template <> struct Piece8<float> {
    float4 a, b;
    __device__ __forceinline__ void zero() { a = make_float4(0, 0, 0, 0); b = a; }
    __device__ __forceinline__ void load(const float *__restrict__ p)
    {
        a = *reinterpret_cast<const float4 *>(p);
        b = *reinterpret_cast<const float4 *>(p + 4);
    }
    __device__ __forceinline__ void get(float (&o)[8]) const
    {
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
        o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
};
template <> struct Piece8<bf16_t> {
    u32x4 v;
    __device__ __forceinline__ void zero() { v = u32x4{0u, 0u, 0u, 0u}; }
    __device__ __forceinline__ void load(const bf16_t *__restrict__ p) { v = *reinterpret_cast<const u32x4 *>(p); }
    __device__ __forceinline__ void get(float (&o)[8]) const { unpack8(v, o); }
};

__device__ __forceinline__ void store_out(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_out(bf16_t *p, float v) { *p = f32_to_bf16(v); }

__device__ __forceinline__ void store8(float *p, const float (&v)[8])
{
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}

__device__ __forceinline__ void store8(bf16_t *p, const float (&v)[8])
{
    u32x4 o;
    o.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
    o.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
    o.z = (uint32_t)f32_to_bf16(v[4]) | ((uint32_t)f32_to_bf16(v[5]) << 16);
    o.w = (uint32_t)f32_to_bf16(v[6]) | ((uint32_t)f32_to_bf16(v[7]) << 16);
    *reinterpret_cast<u32x4 *>(p) = o;
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    const int o = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true);
    return v + __builtin_bit_cast(float, o);
}

// v + (v of lane ^ OFF) for every lane, OFF in {32, 16, 8, 4, 2, 1}: one step of the butterfly the
// predictor's summation order is made of.  Each distance uses the cheapest exchange gfx950 has for
// exactly that pairing: the half-wave and row swaps (the sum of the two swapped copies is the sum
// of the pair in both lanes), then the DPP path only (a rotation by 8 within a row, a half-row mirror
// followed by a reversed quad, the quad permutations): nothing goes through the LDS crossbar, whose
// round trip a chain of dependent steps would pay every time.
template <int OFF>
__device__ __forceinline__ float xor_add(float v)
{
    static_assert(OFF == 32 || OFF == 16 || OFF == 8 || OFF == 4 || OFF == 2 || OFF == 1, "butterfly distance");
    if constexpr (OFF == 32) {
        const unsigned u = __builtin_bit_cast(unsigned, v);
        const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
    } else if constexpr (OFF == 16) {
        const unsigned u = __builtin_bit_cast(unsigned, v);
        const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
        return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
    } else if constexpr (OFF == 8) {
        return dpp_add<0x128>(v);           // row_ror:8 -- in a row of 16 lanes, lane i reads lane i ^ 8
    } else if constexpr (OFF == 4) {
        // lane i ^ 4 = (lane i ^ 7) ^ 3: row_half_mirror, then quad_perm [3,2,1,0] folded into the add
        const int m = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xf, 0xf, true);
        const int o = __builtin_amdgcn_update_dpp(0, m, 0x1B, 0xf, 0xf, true);
        return v + __builtin_bit_cast(float, o);
    } else if constexpr (OFF == 2) {
        return dpp_add<0x4E>(v);            // quad_perm [2,3,0,1]
    } else {
        return dpp_add<0xB1>(v);            // quad_perm [1,0,3,2]
    }
}

// Butterfly sum over the 64 lanes of a wave, partner distance 32,16,8,4,2,1.
// Every lane ends with the same value (float addition is commutative).
__device__ __forceinline__ float wave_sum(float v)
{
    v = xor_add<32>(v);
    v = xor_add<16>(v);
    v = xor_add<8>(v);
    v = xor_add<4>(v);
    v = xor_add<2>(v);
    v = xor_add<1>(v);
    return v;
}

// Dot product of length n (multiple of 8) in the fixed order the predictor's ranking
// depends on: lane l takes elements i with (i/8) mod 64 == l by fused multiply-add in
// increasing i starting from +0, then the butterfly above.  Call with a full wave.
template <typename XT, typename WT>
__device__ __forceinline__ float dot_order64(const XT *__restrict__ xp, const WT *__restrict__ wp,
                                             int n, int lane)
{
    float p = 0.0f;
    for (int c = lane; c * 8 < n; c += kWave) {
        float a[8], b[8];
        load8(xp + c * 8, a);
        load8(wp + c * 8, b);
#pragma unroll
        for (int e = 0; e < 8; ++e) p = __builtin_fmaf(a[e], b[e], p);
    }
    return wave_sum(p);
}

// The same dot product (same element-to-lane map, same order, same result bits) for bf16
// operands of a length known at compile time: every piece of both operands is requested before
// the first multiply, so the wave pays one memory latency instead of one per 512 elements.
template <int N>
__device__ __forceinline__ float dot_order64_fixed(const bf16_t *__restrict__ xp, const bf16_t *__restrict__ wp,
                                                   int lane)
{
    static_assert(N % 512 == 0, "whole 16-byte pieces for all 64 lanes");
    constexpr int NC = N / 512;
    u32x4 xv[NC], wv[NC];
#pragma unroll
    for (int k = 0; k < NC; ++k) {
        xv[k] = *reinterpret_cast<const u32x4 *>(xp + (k * kWave + lane) * 8);
        wv[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (k * kWave + lane) * 8));
    }
    float p = 0.0f;
#pragma unroll
    for (int k = 0; k < NC; ++k) {
        float a[8], b[8];
        unpack8(xv[k], a);
        unpack8(wv[k], b);
#pragma unroll
        for (int e = 0; e < 8; ++e) p = __builtin_fmaf(a[e], b[e], p);
    }
    return wave_sum(p);
}

// One row of the predictor's first layer for T tokens (paper Sec. III-B.2), in the fixed order:
// h[t][j] = ReLU(x[t] . At[j]), this wave's row j.  D = row length when it is one of the tuned ones
// (every piece requested before the first multiply), 0 = any length d.
template <int D>
__device__ __forceinline__ void predictor_row_tokens(const bf16_t *__restrict__ x, const bf16_t *__restrict__ At,
                                                     float *__restrict__ h, int T, int d, int r, int j, int lane)
{
    if (j >= r) return;
    for (int t = 0; t < T; ++t) {
        float p;
        if constexpr (D > 0)
            p = dot_order64_fixed<(D > 0 ? D : 512)>(x + (size_t)t * D, At + (size_t)j * D, lane);
        else
            p = dot_order64(x + (size_t)t * d, At + (size_t)j * d, d, lane);
        if (lane == 0) h[(size_t)t * r + j] = p > 0.0f ? p : 0.0f;
    }
}

// The same rows (same order, same bits) with the row of At held in registers and the pieces of x for TB
// tokens requested together: one memory round trip per TB tokens, where the loop above pays one per token.
// (3 * TB * D / 512 + D / 128 registers: for rows of up to 5120 elements and four tokens.)
template <int D, int TB>
__device__ __forceinline__ void predictor_row_tokens_batched(const bf16_t *__restrict__ x, const bf16_t *__restrict__ At,
                                                             float *__restrict__ h, int T, int r, int j, int lane)
{
    static_assert(D % 512 == 0, "whole 16-byte pieces for all 64 lanes");
    if (j >= r) return;
    constexpr int NC = D / 512;
    u32x4 wv[NC];
#pragma unroll
    for (int k = 0; k < NC; ++k)
        wv[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(At + (size_t)j * D + (k * kWave + lane) * 8));
    for (int t0 = 0; t0 < T; t0 += TB) {
        u32x4 xv[TB][NC];
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            const int t = t0 + b < T ? t0 + b : T - 1;
#pragma unroll
            for (int k = 0; k < NC; ++k)
                xv[b][k] = *reinterpret_cast<const u32x4 *>(x + (size_t)t * D + (k * kWave + lane) * 8);
        }
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            float p = 0.0f;
#pragma unroll
            for (int k = 0; k < NC; ++k) {
                float xa[8], wa[8];
                unpack8(xv[b][k], xa);
                unpack8(wv[k], wa);
#pragma unroll
                for (int e = 0; e < 8; ++e) p = __builtin_fmaf(xa[e], wa[e], p);
            }
            p = wave_sum(p);
            if (t0 + b < T && lane == 0) h[(size_t)(t0 + b) * r + j] = p > 0.0f ? p : 0.0f;
        }
    }
}

// 16 bytes per lane from base + offset[lane] straight into LDS, at lds_addr + 16 * lane (no registers in
// between; counted by vmcnt like any load).  All 64 lanes; lds_addr is the same for the whole wave.
// The compiler does not see this load: wait for it with wait_all_loads() before reading the bytes.
__device__ __forceinline__ void load_to_lds16_all(const void *base, uint32_t offset, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(offset), "s"(base),
                 "s"(__builtin_amdgcn_readfirstlane(lds_addr))
                 : "memory");               // m0 is reserved: the compiler sets it anew before each use of its own
}
__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Wave-wide sum through the DPP cross-lane paths (no LDS traffic); result is uniform.
// Used where the summation order is free (FFN dot products), not by the predictor.
__device__ __forceinline__ float wave_sum_fast(float v)
{
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror
    v = dpp_add<0x140>(v);   // row_mirror: every lane of a 16-lane row holds the row sum
    const int iv = __builtin_bit_cast(int, v);
    const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
    const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
    const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
    return (a + b) + (c + d);
}

// acc + a.lo*b.lo + a.hi*b.hi on packed bf16 pairs (v_dot2c_f32_bf16), float accumulate.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), acc, false);
}

__device__ __forceinline__ float silu_mul(float gate, float up)
{
    return gate / (1.0f + expf(-gate)) * up;
}

// The same with the hardware exponential and reciprocal (each within about one unit in the
// last place of float): for results that are rounded to bf16 right afterwards.
__device__ __forceinline__ float silu_mul_fast(float gate, float up)
{
    const float e = __builtin_amdgcn_exp2f(gate * -1.44269504088896341f);
    return gate * __builtin_amdgcn_rcpf(1.0f + e) * up;
}

}  // namespace halo
