// 4-bit codes -> bf16 operands, shared by the kernels over block-quantised weights.
// Storage format: an element is s * (c - 8) with a 4-bit code c and one bf16 scale s per block of
// 128 elements; eight codes per 32-bit word, element 2i of the eight in bits [4i, 4i+3], element
// 2i+1 in bits [16+4i, 16+4i+3], so that (word >> 4i) & 0x000F000F holds the pair (2i, 2i+1) in
// the two halves of a register -- the shape of a packed bf16 pair.
#pragma once
#include "common.hpp"

namespace halo {

constexpr int kQ4Block = 128;

// codes 2i and 2i+1 of a word as the packed bf16 pair (128 + c, 128 + c): or-ing 0x4300 over a code
// gives the bf16 value 128 + c exactly.  A shift and one and-or; the three-operand form is written
// out because the compiler otherwise emits the "and" and the "or" separately (its two constants
// cannot both be literals of one instruction; here they sit in registers).
__device__ __forceinline__ uint32_t q4_pair(uint32_t w, int i)
{
    uint32_t r;
    const uint32_t sh = i ? w >> (4 * i) : w;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(sh), "v"(0x000F000Fu), "v"(0x43004300u));
    return r;
}

// The two constants of the and-or, parked in registers the compiler cannot see through: with them as
// literals it emits an "and" and an "or" per pair (a three-operand instruction takes no two
// literals), with them in registers one v_and_or_b32.
struct Q4Consts {
    uint32_t mask, one28;
};
__device__ __forceinline__ Q4Consts q4_consts()
{
    Q4Consts c;
    asm volatile("v_mov_b32 %0, 0x000F000F\n\tv_mov_b32 %1, 0x43004300" : "=v"(c.mask), "=v"(c.one28));
    return c;
}

// the eight elements of a word as eight bf16 values 128 + c in element order (one 16-byte piece).
// Plain C on purpose: these registers feed matrix instructions, and the compiler only keeps the
// required distance between a vector instruction and a matrix instruction that shares a register
// with it for instructions it can see -- an asm statement is opaque to that bookkeeping (with the
// and-or written as asm, the operand registers of a matrix instruction in flight were overwritten
// and the products came out wrong).
__device__ __forceinline__ u32x4 q4_word_bf16(uint32_t w, const Q4Consts &k)
{
    return u32x4{(w & k.mask) | k.one28, ((w >> 4) & k.mask) | k.one28, ((w >> 8) & k.mask) | k.one28,
                 ((w >> 12) & k.mask) | k.one28};
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

}  // namespace halo
