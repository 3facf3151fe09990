// Two-level dequantization of the bit-serial layout in registers (Sec. 4.1 "Fused LUT-based dequantization"):
// level 1 turns the bit-plane words of 32 weights into 4-bit codes, level 2 turns a code into the fp16 weight
// with its quantization block's scale and zero baked in.  Shared by the prefill kernel and the small-batch
// matrix-core kernel; both feed the result to MFMA instructions.
#pragma once
#include <hip/hip_fp16.h>

#include "tman_internal.h"

namespace tman {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// (a & mask) | (b & ~mask) and (a & mask) | k as single instructions; the masks live in scalar registers
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) {
    uint32_t d;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(d) : "s"(mask), "v"(a), "v"(b));
    return d;
}
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t k) {
    uint32_t d;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(mask), "v"(k));
    return d;
}

// Level 1: bit planes of 32 weights -> four words of eight 4-bit fields; word o, field f = weight 4f + o.
// For fewer than four planes the upper bits of a field hold bits of other weights; level 2 masks them.
template <int B>
__device__ __forceinline__ void planes_to_codes(const uint32_t (&p)[B], uint32_t (&out)[4]) {
    if constexpr (B == 4) {
        // pair planes (0,1) and (2,3) into 2-bit fields of even / odd weights, then pair those into nibbles
        const uint32_t a = bfi(0x55555555u, p[0], p[1] << 1);  // field e: low two code bits of weight 2e
        const uint32_t b = bfi(0xAAAAAAAAu, p[1], p[0] >> 1);  // same for weight 2e + 1
        const uint32_t c = bfi(0x55555555u, p[2], p[3] << 1);  // high two code bits of weight 2e
        const uint32_t d = bfi(0xAAAAAAAAu, p[3], p[2] >> 1);
        out[0] = bfi(0x33333333u, a, c << 2);  // weights 4f
        out[2] = bfi(0xCCCCCCCCu, c, a >> 2);  // weights 4f + 2
        out[1] = bfi(0x33333333u, b, d << 2);  // weights 4f + 1
        out[3] = bfi(0xCCCCCCCCu, d, b >> 2);  // weights 4f + 3
    } else if constexpr (B == 2) {
        const uint32_t a = bfi(0x55555555u, p[0], p[1] << 1);
        const uint32_t b = bfi(0xAAAAAAAAu, p[1], p[0] >> 1);
        out[0] = a;
        out[2] = a >> 2;
        out[1] = b;
        out[3] = b >> 2;
    } else {
#pragma unroll
        for (int o = 0; o < 4; ++o) out[o] = p[0] >> o;
    }
}

// raw data of one 32-weight block of a stage for one lane (= one row)
template <int B>
struct WRegs {
    uint32_t plane[B];
    uint32_t meta;  // scale (low 16 bits) and zero (high 16 bits) of the block's quantization group
};

// Level 2 for one lane's 32 weights; writes them as fp16, in column order, into its row of the LDS
// weight tile (`wrow` already points at the block's 64 bytes).
//
// Field f of code word o (weight 4f + o) is turned into an fp16 number without moving it to bit 0:
// a nibble at mantissa bits 0..3 of 0x6400 reads 1024 + c, one at bits 4..7 reads 1024 + 16c.  Fields
// f and f + 4 sit 16 bits apart, so one AND-OR makes two such numbers; a single shift by 8 brings
// fields 2, 3, 6, 7 into reach.  The affine map (c - zero) * scale is then one fp32 FMA per weight, rounded to
// fp16 once:  (1024 + c) * s - (1024 + z) * s   or   (1024 + 16c) * s/16 - (64 + z) * s   (the second, constant
// term is itself rounded to fp32 when the block's constants are prepared).
// The FMA writes either half of its destination, which puts weights 4f + o and 4f + o + 1 (from the
// same field of two code words) side by side at no cost.
template <int B, bool HZ>
struct Dequant {
    uint32_t codes[4];
    float mul[2], bias[2];  // [0]: nibble at mantissa bits 0..3, [1]: at bits 4..7
    half2_t P[4][4];        // [o][d]: halves = fields d and d + 4 of code word o, as 1024 + c or 1024 + 16c

    // part 1: level 1 and the block's constants
    __device__ __forceinline__ void start(const WRegs<B>& r) {
        planes_to_codes<B>(r.plane, codes);
        const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)(r.meta & 0xffffu));
        if constexpr (HZ) {
            const float z = (float)__builtin_bit_cast(_Float16, (uint16_t)(r.meta >> 16));
            mul[0] = s;
            bias[0] = -(1024.f + z) * s;
            mul[1] = s * 0.0625f;
            bias[1] = -(64.f + z) * s;
        } else {
            mul[0] = 2.f * s;  // (2c - 1) * s
            bias[0] = -2049.f * s;
            mul[1] = s * 0.125f;
            bias[1] = -129.f * s;
        }
    }
    // part 2: codes -> fp16 integers
    __device__ __forceinline__ void insert() {
        constexpr uint32_t kCodeMask = (1u << B) - 1u;
        constexpr uint32_t kMaskLo = kCodeMask | (kCodeMask << 16), kMaskHi = kMaskLo << 4;
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            const uint32_t c = codes[o], c8 = codes[o] >> 8;
            P[o][0] = __builtin_bit_cast(half2_t, and_or(c, kMaskLo, 0x64006400u));
            P[o][1] = __builtin_bit_cast(half2_t, and_or(c, kMaskHi, 0x64006400u));
            P[o][2] = __builtin_bit_cast(half2_t, and_or(c8, kMaskLo, 0x64006400u));
            P[o][3] = __builtin_bit_cast(half2_t, and_or(c8, kMaskHi, 0x64006400u));
        }
    }
    // part 3: 16-byte piece q (weights 8q .. 8q + 7 = fields 2q, 2q + 1) as four pairs of fp16
    __device__ __forceinline__ u32x4 piece(int q) const {
        u32x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int f = 2 * q + (i >> 1), o = (i & 1) * 2, d = f & 3, t = d & 1;
            const _Float16 va = (f >> 2) ? P[o][d].y : P[o][d].x;
            const _Float16 vb = (f >> 2) ? P[o + 1][d].y : P[o + 1][d].x;
            half2_t w;
            w.x = (_Float16)fmaf((float)va, mul[t], bias[t]);
            w.y = (_Float16)fmaf((float)vb, mul[t], bias[t]);
            out[i] = __builtin_bit_cast(uint32_t, w);
        }
        return out;
    }
    // ... written to its place in an LDS row
    __device__ __forceinline__ void emit(int q, uint8_t* wrow) const { *reinterpret_cast<u32x4*>(wrow + q * 16) = piece(q); }
};

template <int B, bool HZ>
__device__ __forceinline__ void dequant_to_lds(const WRegs<B>& r, uint8_t* wrow) {
    Dequant<B, HZ> dq;
    dq.start(r);
    dq.insert();
#pragma unroll
    for (int q = 0; q < 4; ++q) dq.emit(q, wrow);
}

}  // namespace tman
