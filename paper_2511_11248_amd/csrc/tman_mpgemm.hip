// Prefill mpGEMM: two-level dequantization fused in front of the matrix cores
// (Sec. 4.1 "Unified Layout through Fused LUT-based Dequantization", Sec. 4.2 three-stage pipeline).
//
// The weights stay in the bit-serial layout decoding uses (lane = row, 64 rows x 128 columns per tile
// block).  Per 64-column stage a wave turns the bit-plane words of its 64 rows into fp16 weights:
//   level 1  bit-serial -> bit-parallel (Sec. 4.1 "Bit repacking"): two rounds of bit-field inserts
//            transpose a 4 x 32 bit matrix in 16 ALU ops, giving for each 32-weight block four words
//            of eight 4-bit codes, word o holding the codes of weights 4f + o;
//   level 2  code -> fp16 weight with the block's scale and zero baked in (Sec. 4.1 "Integer-to-float
//            conversion", "Applying scales and zero-points").  The 16-entry conversion table of the
//            paper collapses on this hardware to inserting the code into the mantissa of 1024.0
//            (fp16 0x6400 | c == 1024 + c exactly), and the baked affine table entry
//            D[c] = fp16((c - zero) * scale) is produced by ONE mixed-precision FMA
//            fp16( (1024 + c) * scale - (1024 + zero) * scale ) evaluated in fp32 with a single rounding,
//            with the per-block constants (scale, -(1024 + zero) * scale) computed once per block.
//            A lookup per weight in LDS would compete with the MFMA operand reads for LDS bandwidth.
// The fp16 weight tile goes to LDS and is shared by the four waves of the workgroup (each weight is
// dequantized once per 256 tokens); activations are staged next to it in the k order level 1
// produces.  Pipeline (the GPU form of DMA -> vector -> matrix): global loads of stage s+2 are in
// flight while stage s+1 is dequantized into the other LDS buffer and stage s feeds
// v_mfma_f32_32x32x16_f16 (fp32 accumulation); one barrier per stage.
#include <hip/hip_fp16.h>

#include "tman_internal.h"

namespace tman {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTM = 256;      // rows of W (output features) per workgroup
constexpr int kTN = 256;      // tokens per workgroup
constexpr int kStageK = 64;   // columns per pipeline stage (half a tile block)
constexpr int kRowBytes = kStageK * 2 + 16;  // padded LDS row: 36 dwords, conflict-free 16-byte accesses
constexpr int kWTile = kTM * kRowBytes;
constexpr int kXTile = kTN * kRowBytes;
constexpr int kStageBytes = kWTile + kXTile;
constexpr int kGemmLdsBytes = 2 * kStageBytes;  // double buffered: 147,456 of the CU's 160 KB

struct GemmArgs {
    const uint8_t* tiles;
    const _Float16* x;
    _Float16* y;
    int M, N, K, n_row_blocks, n_ktiles;
};

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }

// Level 1: bit planes of 32 weights -> four words of eight 4-bit codes; word o, field f = weight 4f + o.
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
        out[0] = a & 0x33333333u;
        out[2] = (a >> 2) & 0x33333333u;
        out[1] = b & 0x33333333u;
        out[3] = (b >> 2) & 0x33333333u;
    } else {
#pragma unroll
        for (int o = 0; o < 4; ++o) out[o] = (p[0] >> o) & 0x11111111u;
    }
}

// raw data of one 32-weight block of a stage for one lane (= one row)
template <int B>
struct WRegs {
    uint32_t plane[B];
    uint32_t meta;  // scale (low 16 bits) and zero (high 16 bits) of the block's quantization group
};

template <int B, int GQ, bool HZ>
__device__ __forceinline__ void load_w(WRegs<B>& r, const uint8_t* tile, int kb32, int lane, bool valid) {
    constexpr int CH = kKTile / B;
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int MPL = (kKTile / GQ) * MSZ;
    // kb32: 32-weight block inside the 128-column tile block
    const int v = (kb32 * 32) / CH, ksub = ((kb32 * 32) % CH) / 32;
    const uint8_t* p = tile + v * 1024 + lane * 16 + ksub * B * 4;
    if (!valid) {
#pragma unroll
        for (int i = 0; i < B; ++i) r.plane[i] = 0u;
        r.meta = 0u;
        return;
    }
    if constexpr (B == 4) {
        const u32x4 w = *reinterpret_cast<const u32x4*>(p);
        r.plane[0] = w.x; r.plane[1] = w.y; r.plane[2] = w.z; r.plane[3] = w.w;
    } else if constexpr (B == 2) {
        const u32x2 w = *reinterpret_cast<const u32x2*>(p);
        r.plane[0] = w.x; r.plane[1] = w.y;
    } else {
        r.plane[0] = *reinterpret_cast<const uint32_t*>(p);
    }
    const int gi = (kb32 * 32) / GQ;
    const uint8_t* mp = tile + B * 1024 + lane * MPL + gi * MSZ;
    if constexpr (HZ) r.meta = *reinterpret_cast<const uint32_t*>(mp);
    else r.meta = *reinterpret_cast<const uint16_t*>(mp);
}

// Level 2 for one lane's 32 weights; writes them as fp16 into its row of the LDS weight tile
// (`wrow` already points at the block's 64 bytes).
template <int B, bool HZ>
__device__ __forceinline__ void dequant_to_lds(const WRegs<B>& r, uint8_t* wrow) {
    uint32_t codes[4];
    planes_to_codes<B>(r.plane, codes);
    const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)(r.meta & 0xffffu));
    float mul, bias;  // weight = (1024 + c) * mul + bias, one rounding to fp16
    if constexpr (HZ) {
        const float z = (float)__builtin_bit_cast(_Float16, (uint16_t)(r.meta >> 16));
        mul = s;
        bias = -(1024.f + z) * s;
    } else {
        mul = 2.f * s;  // (2c - 1) * s
        bias = -2049.f * s;
    }
#pragma unroll
    for (int o = 0; o < 4; ++o) {
        u32x4 out;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            // codes of weights 4d + o and 4(d+4) + o, each inserted into the mantissa of 1024.0
            const uint32_t pair = ((codes[o] >> (4 * d)) & 0x000F000Fu) | 0x64006400u;
            const half2_t v = __builtin_bit_cast(half2_t, pair);
            half2_t w;
            w.x = (_Float16)fmaf((float)v.x, mul, bias);
            w.y = (_Float16)fmaf((float)v.y, mul, bias);
            out[d] = __builtin_bit_cast(uint32_t, w);
        }
        *reinterpret_cast<u32x4*>(wrow + o * 16) = out;
    }
}

// activation staging: a unit = one token row, one 32-column block, one pair of 8-column pieces
// (columns 8pp..8pp+7 and 16+8pp..16+8pp+7); two units per thread and stage
struct XRegs {
    u32x4 p[2], q[2];
};
struct XPlan {
    const _Float16* src[2];  // first piece of each unit at stage 0 (nullptr: token beyond N)
    int col[2];              // its column
    int dst[2];              // byte offset of the unit inside the LDS activation tile
};

__device__ __forceinline__ void plan_x(XPlan& pl, const GemmArgs& a, int n0, int tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int u = i * 512 + tid;
        const int n = u >> 2, blk = (u >> 1) & 1, pp = u & 1;
        pl.col[i] = blk * 32 + pp * 8;
        pl.src[i] = (n0 + n < a.N) ? a.x + (size_t)(n0 + n) * a.K + pl.col[i] : nullptr;
        pl.dst[i] = n * kRowBytes + (blk * 32 + 4 * pp) * 2;
    }
}

__device__ __forceinline__ void load_x(XRegs& r, const XPlan& pl, int K, int k0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        u32x4 P = {0u, 0u, 0u, 0u}, Q = {0u, 0u, 0u, 0u};
        if (pl.src[i]) {
            const int gk = k0 + pl.col[i];  // K is a multiple of 32, so pieces are all-or-nothing
            if (gk + 8 <= K) P = *reinterpret_cast<const u32x4*>(pl.src[i] + k0);
            if (gk + 24 <= K) Q = *reinterpret_cast<const u32x4*>(pl.src[i] + k0 + 16);
        }
        r.p[i] = P;
        r.q[i] = Q;
    }
}

// Writes the units in the k order of the weight tile: column 4f + o of a 32-block sits at position
// 8o + slot(f), slot(f) = 2f for f < 4, 2(f - 4) + 1 otherwise (the order dequant_to_lds emits).
__device__ __forceinline__ void store_x(const XRegs& r, const XPlan& pl, uint8_t* xtile) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        uint8_t* dst = xtile + pl.dst[i];
        const u32x4 P = r.p[i], Q = r.q[i];
        // piece P holds f = 2pp (elements 0..3) and 2pp + 1 (elements 4..7); piece Q holds f + 4
        const uint32_t pw[4] = {P.x, P.y, P.z, P.w}, qw[4] = {Q.x, Q.y, Q.z, Q.w};
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            const uint32_t pa = pw[o >> 1], qa = qw[o >> 1], pb = pw[2 + (o >> 1)], qb = qw[2 + (o >> 1)];
            u32x2 w;
            if (o & 1) {
                w.x = (pa >> 16) | (qa & 0xffff0000u);
                w.y = (pb >> 16) | (qb & 0xffff0000u);
            } else {
                w.x = (pa & 0xffffu) | (qa << 16);
                w.y = (pb & 0xffffu) | (qb << 16);
            }
            *reinterpret_cast<u32x2*>(dst + o * 16) = w;
        }
    }
}

template <int B, int GQ, bool HZ>
__global__ void __launch_bounds__(512, 1) mpgemm_kernel(GemmArgs a) {
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int TB = B * 1024 + 64 * (kKTile / GQ) * MSZ;

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, r = lane & 31, h = lane >> 5;
    // eight waves: two per SIMD, so one wave's dequantization overlaps the other's MFMAs.
    // MFMA part: wave (wm, wn) owns 128 rows x 64 tokens of the 256 x 256 tile.
    const int wm = wave >> 2, wn = wave & 3;
    // dequantization part: wave owns row block (wave & 3) and 32-column block (wave >> 2) of each stage
    const int drb = wave & 3, dblk = wave >> 2;
    const int n0 = blockIdx.y * kTN;
    const int rbw = blockIdx.x * 4 + drb;
    const bool wvalid = rbw < a.n_row_blocks;
    const uint8_t* wtiles = a.tiles + (size_t)(wvalid ? rbw : 0) * a.n_ktiles * TB;
    const int n_stages = a.n_ktiles * 2;
    const int wdst = (drb * 64 + lane) * kRowBytes + dblk * 64;  // this lane's 64 bytes in the weight tile

    float16_t acc[4][2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;

    WRegs<B> wr;
    XRegs xr;
    XPlan xp;
    plan_x(xp, a, n0, tid);
    // prologue: stage 0 straight into buffer 0, stage 1 into registers
    load_w<B, GQ, HZ>(wr, wtiles, dblk, lane, wvalid);
    load_x(xr, xp, a.K, 0);
    dequant_to_lds<B, HZ>(wr, smem + wdst);
    store_x(xr, xp, smem + kWTile);
    if (n_stages > 1) {
        load_w<B, GQ, HZ>(wr, wtiles, 2 + dblk, lane, wvalid);
        load_x(xr, xp, a.K, kStageK);
    }
    __syncthreads();

    for (int s = 0; s < n_stages; ++s) {
        uint8_t* cur = smem + (s & 1) * kStageBytes;
        uint8_t* nxt = smem + ((s + 1) & 1) * kStageBytes;
        // stage s+1: registers -> LDS (the other buffer); stage s+2: global -> registers
        if (s + 1 < n_stages) {
            dequant_to_lds<B, HZ>(wr, nxt + wdst);
            store_x(xr, xp, nxt + kWTile);
        }
        if (s + 2 < n_stages) {
            const int s2 = s + 2;
            load_w<B, GQ, HZ>(wr, wtiles + (size_t)(s2 >> 1) * TB, 2 * (s2 & 1) + dblk, lane, wvalid);
            load_x(xr, xp, a.K, s2 * kStageK);
        }
        // stage s: four k16 steps; lanes with h = 0 / 1 take the two 8-column groups of a step
        const uint8_t* wbase = cur + (wm * 128 + r) * kRowBytes + h * 16;
        const uint8_t* xbase = cur + kWTile + (wn * 64 + r) * kRowBytes + h * 16;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            half8_t wf[4], xf[2];
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) wf[mb] = *reinterpret_cast<const half8_t*>(wbase + mb * 32 * kRowBytes + j * 32);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) xf[nb] = *reinterpret_cast<const half8_t*>(xbase + nb * 32 * kRowBytes + j * 32);
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[mb], xf[nb], acc[mb][nb], 0, 0, 0);
        }
        __syncthreads();
    }

    // epilogue: accumulators -> fp16 -> LDS as [token][row] -> coalesced 16-byte stores
    // C[i][j] of a 32x32 block: i = row (8 * (v / 4) + 4 * h + v % 4), j = token (lane % 32)
    constexpr int kOutRow = kTM * 2 + 16;  // bytes per token row of the output tile in LDS
    uint8_t* otile = smem;                 // 256 * 528 = 135,168 bytes, the stage buffers are free now
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            uint8_t* col = otile + (wn * 64 + nb * 32 + r) * kOutRow + (wm * 128 + mb * 32 + 4 * h) * 2;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                half2_t lo, hi;
                lo.x = (_Float16)acc[mb][nb][4 * g + 0];
                lo.y = (_Float16)acc[mb][nb][4 * g + 1];
                hi.x = (_Float16)acc[mb][nb][4 * g + 2];
                hi.y = (_Float16)acc[mb][nb][4 * g + 3];
                u32x2 w = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                *reinterpret_cast<u32x2*>(col + g * 16) = w;  // rows 8g + 4h + 0..3
            }
        }
    __syncthreads();
    const int m0 = blockIdx.x * kTM;
    const bool fast = (a.M % 8 == 0);  // 16-byte aligned rows of y
    for (int piece = tid; piece < kTN * (kTM / 8); piece += 512) {
        const int n = piece / (kTM / 8), c8 = piece % (kTM / 8);
        const int gn = n0 + n, gm = m0 + c8 * 8;
        if (gn >= a.N || gm >= a.M) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(otile + n * kOutRow + c8 * 16);
        _Float16* dst = a.y + (size_t)gn * a.M + gm;
        if (fast && gm + 8 <= a.M) {
            *reinterpret_cast<u32x4*>(dst) = v;
        } else {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            for (int t = 0; t < 8 && gm + t < a.M; ++t)
                dst[t] = __builtin_bit_cast(_Float16, (uint16_t)(w[t >> 1] >> (16 * (t & 1))));
        }
    }
}

template <int B, int GQ, bool HZ>
static int launch_cfg(const GemmArgs& a, hipStream_t st) {
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&mpgemm_kernel<B, GQ, HZ>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLdsBytes) != hipSuccess)
            return TMAN_ERR_LAUNCH;
        attr_set = true;
    }
    dim3 grid((unsigned)((a.M + kTM - 1) / kTM), (unsigned)((a.N + kTN - 1) / kTN));
    hipLaunchKernelGGL((mpgemm_kernel<B, GQ, HZ>), grid, dim3(512), kGemmLdsBytes, st, a);
    return launch_status();
}

template <int B, bool HZ>
static int launch_group(int group, const GemmArgs& a, hipStream_t st) {
    switch (group) {
        case 32: return launch_cfg<B, 32, HZ>(a, st);
        case 64: return launch_cfg<B, 64, HZ>(a, st);
        default: return launch_cfg<B, 128, HZ>(a, st);
    }
}

int launch_mpgemm(const Layout& L, const void* packed, const void* x, int N, void* y, void* workspace,
                  hipStream_t st) {
    (void)workspace;
    GemmArgs a;
    a.tiles = static_cast<const uint8_t*>(packed) + kHeaderBytes;
    a.x = static_cast<const _Float16*>(x);
    a.y = static_cast<_Float16*>(y);
    a.M = L.M;
    a.N = N;
    a.K = L.K;
    a.n_row_blocks = L.n_row_blocks;
    a.n_ktiles = L.n_ktiles;
    if (L.bits == 1) return L.has_zero ? launch_group<1, true>(L.group, a, st) : launch_group<1, false>(L.group, a, st);
    if (L.bits == 2) return launch_group<2, true>(L.group, a, st);
    return launch_group<4, true>(L.group, a, st);
}

}  // namespace tman
