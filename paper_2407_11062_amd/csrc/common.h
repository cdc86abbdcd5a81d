// Shared device helpers of the eqat HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/eqat.h"

namespace eqat {

typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx3 __attribute__((ext_vector_type(3)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

// Offset that is out of range for every buffer this library binds (tensors are < 2 GiB):
// a buffer load from it returns zeros.
constexpr uint32_t kOobOffset = 0x80000000u;

// A raw buffer resource over [p, p + bytes): loads past the end return 0, stores are dropped.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ intx4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
}
__device__ __forceinline__ intx3 buf_load12(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b96(r, (int)off, 0, 0);
}
__device__ __forceinline__ intx2 buf_load8(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 0);
}
__device__ __forceinline__ int buf_load4(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0);
}

// N words (N = BITS) hold 32 codes of BITS bits, little-endian bit stream.
template <int BITS> struct CodeWords { uint32_t w[BITS]; };

template <int BITS>
__device__ __forceinline__ CodeWords<BITS> load_code_words(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    CodeWords<BITS> c;
    if constexpr (BITS == 2) { intx2 v = buf_load8(r, off); c.w[0] = v[0]; c.w[1] = v[1]; }
    else if constexpr (BITS == 3) { intx3 v = buf_load12(r, off); c.w[0] = v[0]; c.w[1] = v[1]; c.w[2] = v[2]; }
    else { intx4 v = buf_load16(r, off); c.w[0] = v[0]; c.w[1] = v[1]; c.w[2] = v[2]; c.w[3] = v[3]; }
    return c;
}

// Code number IDX (compile time) of a 32-code segment.
template <int BITS, int IDX>
__device__ __forceinline__ uint32_t code_at(const CodeWords<BITS> &c)
{
    constexpr int bit = IDX * BITS, wi = bit >> 5, sh = bit & 31;
    constexpr uint32_t mask = (1u << BITS) - 1u;
    if constexpr (sh + BITS <= 32) return (c.w[wi] >> sh) & mask;
    else return ((c.w[wi] >> sh) | (c.w[wi + 1] << (32 - sh))) & mask;
}

// Runtime-indexed variant (slow paths only).
template <int BITS>
__device__ __forceinline__ uint32_t code_at_rt(const uint32_t *words, int idx)
{
    const int bit = idx * BITS, wi = bit >> 5, sh = bit & 31;
    const uint32_t mask = (1u << BITS) - 1u;
    uint64_t two = words[wi];
    if (sh + BITS > 32) two |= (uint64_t)words[wi + 1] << 32;
    return (uint32_t)(two >> sh) & mask;
}

// ---- working layout of the codes inside the library's workspace ------------------------------------------
// The packed stream the C ABI exposes (CodeWords above) is dense, which makes 3-bit codes straddle words and every
// code cost a shift, a mask and a convert to reach.  Kernels that consume codes in bulk read this layout instead:
//   2 bit : 16 codes per word, code e of the word in bits [8*(e % 4) + 2*(e / 4), +2)
//   3, 4 bit : 8 codes per word, code e of the word in bits [8*(e % 4) + 4*(e / 4), +4)   (3-bit codes zero-extended)
// so that (word >> shift) & 0x0F0F0F0F-style masks leave FOUR CONSECUTIVE codes in the four bytes of a register.
template <int BITS> struct WorkCodes {
    static constexpr int kWords = BITS == 2 ? 2 : 4;              // words per 32-code segment
    static constexpr int kField = BITS == 2 ? 2 : 4;              // bits per field
    static constexpr int kPerWord = 32 / kWords;                  // codes per word
    static constexpr uint32_t kByteMask = BITS == 2 ? 0x03030303u : BITS == 3 ? 0x07070707u : 0x0F0F0F0Fu;
    uint32_t w[kWords];
    // bit position of code e (0..31) of a segment inside its word
    static constexpr int bit_of(int e) { return 8 * ((e % kPerWord) % 4) + kField * ((e % kPerWord) / 4); }
    static constexpr int word_of(int e) { return e / kPerWord; }
    // bytes of the result = codes e0 .. e0+3 (e0 a multiple of 4) after an extra right shift by `pre` bits
    __device__ __forceinline__ uint32_t four(int e0, uint32_t pre = 0) const
    {
        return (w[word_of(e0)] >> (bit_of(e0) + pre)) & kByteMask;
    }
};

template <int BITS>
__device__ __forceinline__ WorkCodes<BITS> load_work_codes(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    WorkCodes<BITS> c;
    if constexpr (BITS == 2) { intx2 v = buf_load8(r, off); c.w[0] = v[0]; c.w[1] = v[1]; }
    else { intx4 v = buf_load16(r, off); c.w[0] = v[0]; c.w[1] = v[1]; c.w[2] = v[2]; c.w[3] = v[3]; }
    return c;
}

__device__ __forceinline__ float byte_to_float(uint32_t v, int b)      // b compile-time after unrolling
{
    return (float)((v >> (8 * b)) & 0xFFu);                            // selected as v_cvt_f32_ubyte<b>
}

// The zero point Eqs.(1),(2) use: round(z), held inside what N bits can store (it is stored at N bits once Block-AP
// ends, and E2E-QP must start from the very model Block-AP trained); the gradient passes straight through both.
__device__ __forceinline__ float zbar_of(float z, float qmax)
{
    return __builtin_amdgcn_fmed3f(__builtin_rintf(z), 0.0f, qmax);
}

// ---- codes -> bf16 What ----------------------------------------------------------------------------------
// A group has only 2^N distinct What values, (q - zbar) * s.  For 2 and 3 bits they are computed once per 32-code
// segment and kept as two byte tables (low and high bytes of the bf16 values); four codes sitting in the four bytes
// of a register then become four bf16 with four byte permutes, instead of four converts, four FMAs and two packs.
// 4 bits (16 values) exceed what one permute can index and keep the arithmetic form.
template <int BITS> struct WhatTable {
    uint32_t lo[2], hi[2];      // byte q of lo / hi = low / high byte of bf16(What(q)); [1] only for 3 bits
    float s, b;                 // What(q) = q * s + b
    __device__ __forceinline__ void build(float s_, float zbar)
    {
        s = s_; b = -zbar * s_;
        if constexpr (BITS <= 3) {
#pragma unroll
            for (int half = 0; half < (BITS == 3 ? 2 : 1); ++half) {
                bf16x2 p01, p23;
                p01[0] = (bf16_t)__builtin_fmaf((float)(4 * half + 0), s, b); p01[1] = (bf16_t)__builtin_fmaf((float)(4 * half + 1), s, b);
                p23[0] = (bf16_t)__builtin_fmaf((float)(4 * half + 2), s, b); p23[1] = (bf16_t)__builtin_fmaf((float)(4 * half + 3), s, b);
                const uint32_t v0 = __builtin_bit_cast(uint32_t, p01), v1 = __builtin_bit_cast(uint32_t, p23);
                lo[half] = __builtin_amdgcn_perm(v1, v0, 0x06040200u);      // bytes 0 and 2 of v0, then of v1
                hi[half] = __builtin_amdgcn_perm(v1, v0, 0x07050301u);      // bytes 1 and 3
            }
            if constexpr (BITS == 2) { lo[1] = lo[0]; hi[1] = hi[0]; }
        }
    }
    // t: four codes in the four bytes -> two registers holding four bf16
    __device__ __forceinline__ void four(uint32_t t, uint32_t &d0, uint32_t &d1) const
    {
        if constexpr (BITS <= 3) {
            const uint32_t x = __builtin_amdgcn_perm(lo[1], lo[0], t), y = __builtin_amdgcn_perm(hi[1], hi[0], t);
            d0 = __builtin_amdgcn_perm(y, x, 0x05010400u);     // x0 y0 x1 y1
            d1 = __builtin_amdgcn_perm(y, x, 0x07030602u);     // x2 y2 x3 y3
        } else {
            bf16x2 p01, p23;
            p01[0] = (bf16_t)__builtin_fmaf(byte_to_float(t, 0), s, b); p01[1] = (bf16_t)__builtin_fmaf(byte_to_float(t, 1), s, b);
            p23[0] = (bf16_t)__builtin_fmaf(byte_to_float(t, 2), s, b); p23[1] = (bf16_t)__builtin_fmaf(byte_to_float(t, 3), s, b);
            d0 = __builtin_bit_cast(uint32_t, p01); d1 = __builtin_bit_cast(uint32_t, p23);
        }
    }
    // codes [8*q8, 8*q8 + 8) of a segment -> eight bf16
    template <int Q8> __device__ __forceinline__ bf16x8 eight(const WorkCodes<BITS> &c) const
    {
        uintx4 u;
        uint32_t d0, d1;
        four(c.four(8 * Q8), d0, d1); u[0] = d0; u[1] = d1;
        four(c.four(8 * Q8 + 4), d0, d1); u[2] = d0; u[3] = d1;
        return __builtin_bit_cast(bf16x8, u);
    }
};

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return (float)v; }

}  // namespace eqat
