// Prefill mpGEMM: two-level table dequantization fused in front of the matrix cores
// (Sec. 4.1 "Unified Layout through Fused LUT-based Dequantization", Sec. 4.2 pipeline).
//
// The weights stay in the bit-serial layout decoding uses (lane = row, 64 rows x 128 columns per tile
// block).  Per tile block a wave
//   level 1  turns the bit-plane words of its 64 rows back into codes (Sec. 4.1 "Bit repacking";
//            on CDNA4 two rounds of bit-field inserts transpose a 4 x 32 bit matrix in 16 ALU ops,
//            giving for each 32-weight block four words of eight 4-bit fields, word o holding the
//            codes of weights 4f + o),
//   level 2  looks every code up in its quantization block's table D[c] = fp16((c - zero) * scale)
//            (Sec. 4.1 "Integer-to-float conversion", "Applying scales and zero-points"): 2^bits
//            entries per (row, block), built with one fp32 multiply and one rounding each, kept in
//            LDS as dwords [code][row % 32] whose halves belong to rows r and r + 32,
// and feeds the fp16 weights as one operand of v_mfma_f32_32x32x16_f16 (fp32 accumulation).  The
// MFMA wants lanes l and l + 32 to hold the same row with different k; the layout has them hold rows
// l and l + 32, so two code words are exchanged between the wave halves with v_permlane32_swap before
// the lookup: one word then serves rows 0..31, the other rows 32..63.  The activations are the other
// operand, staged per K tile in LDS in the k order level 1 produces.
#include <hip/hip_fp16.h>

#include "tman_internal.h"

namespace tman {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kGemmNTile = 128;                 // tokens per workgroup
constexpr int kXRowHalfs = kKTile + 8;          // padded LDS row of the activation tile (fp16 units)
constexpr int kXTileBytes = kGemmNTile * kXRowHalfs * 2;
constexpr int kTabBytesPerWave = 16 * 32 * 4;   // [code][row % 32] dwords
constexpr int kGemmLdsBytes = kXTileBytes + 4 * kTabBytesPerWave;

struct GemmArgs {
    const uint8_t* tiles;
    const _Float16* x;
    _Float16* y;
    int M, N, K, n_row_blocks, n_ktiles;
};

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }

// Lanes of one wave exchange data through the wave's private LDS table.  The hardware executes the
// LDS operations of a wave in order; this keeps the compiler from moving them across the exchange.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
}

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

template <int B, int GQ, bool HZ>
__global__ void __launch_bounds__(256) mpgemm_kernel(GemmArgs a) {
    constexpr int GPT = kKTile / GQ;
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int MPL = GPT * MSZ;
    constexpr int TB = B * 1024 + 64 * MPL;
    constexpr int CH = kKTile / B;
    constexpr int NCODE = 1 << B;

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    _Float16* xs = reinterpret_cast<_Float16*>(smem);

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 31, h = lane >> 5;
    const int rb = blockIdx.x * 4 + wave;
    const bool valid = rb < a.n_row_blocks;
    const int n0 = blockIdx.y * kGemmNTile;
    uint8_t* tab = smem + kXTileBytes + wave * kTabBytesPerWave;  // this wave's level-2 table
    uint8_t* tab_own = tab + r * 4 + h * 2;   // where this lane's row (r + 32 h) keeps its entries
    const uint8_t* tab_lo = tab + r * 4;      // entries of row r       (rows 0..31 of the block)
    const uint8_t* tab_hi = tab + r * 4 + 2;  // entries of row r + 32  (rows 32..63)

    float16_t acc[2][4];
#pragma unroll
    for (int rh = 0; rh < 2; ++rh)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rh][nb][v] = 0.f;

    for (int kt = 0; kt < a.n_ktiles; ++kt) {
        __syncthreads();  // previous activation tile fully consumed
        // stage activations x[n0 .. n0+127][kt*128 .. +127], each 32-column block reordered so that
        // column 4f + o lands at position o*8 + f (the order level 1 delivers the weights in)
        for (int piece = threadIdx.x; piece < kGemmNTile * (kKTile / 8); piece += 256) {
            const int n = piece / (kKTile / 8), q = piece % (kKTile / 8);
            const int gn = n0 + n, gk = kt * kKTile + q * 8;
            uint4 d = make_uint4(0u, 0u, 0u, 0u);
            if (gn < a.N) {
                if (gk + 8 <= a.K) {
                    d = *reinterpret_cast<const uint4*>(a.x + (size_t)gn * a.K + gk);
                } else {
                    uint32_t e[8];
                    for (int t = 0; t < 8; ++t)
                        e[t] = gk + t < a.K ? (uint32_t)__builtin_bit_cast(uint16_t, a.x[(size_t)gn * a.K + gk + t]) : 0u;
                    d = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
                }
            }
            // elements e0..e7 = columns 8(q%4) + e inside the 32-block; e and e+4 share o = e % 4
            const uint32_t p0 = (d.x & 0xffffu) | (d.z << 16);         // (e0, e4)  o = 0
            const uint32_t p1 = (d.x >> 16) | (d.z & 0xffff0000u);     // (e1, e5)  o = 1
            const uint32_t p2 = (d.y & 0xffffu) | (d.w << 16);         // (e2, e6)  o = 2
            const uint32_t p3 = (d.y >> 16) | (d.w & 0xffff0000u);     // (e3, e7)  o = 3
            uint32_t* row = reinterpret_cast<uint32_t*>(xs + n * kXRowHalfs + (q / 4) * 32 + 2 * (q % 4));
            row[0] = p0;
            row[4] = p1;   // +8 halfs
            row[8] = p2;
            row[12] = p3;
        }
        __syncthreads();
        if (!valid) continue;

        // this wave's tile block: 64 rows x 128 columns, lane = row
        const uint8_t* tile = a.tiles + ((size_t)rb * a.n_ktiles + kt) * TB;
        uint4 c[B];
#pragma unroll
        for (int v = 0; v < B; ++v) c[v] = *reinterpret_cast<const uint4*>(tile + v * 1024 + lane * 16);
        uint32_t meta[(MPL + 3) / 4];
        {
            const uint8_t* mp = tile + B * 1024 + lane * MPL;
            if constexpr (MPL == 2) meta[0] = *reinterpret_cast<const uint16_t*>(mp);
            else if constexpr (MPL == 4) meta[0] = *reinterpret_cast<const uint32_t*>(mp);
            else if constexpr (MPL == 8) { uint2 v = *reinterpret_cast<const uint2*>(mp); meta[0] = v.x; meta[1] = v.y; }
            else { uint4 v = *reinterpret_cast<const uint4*>(mp); meta[0] = v.x; meta[1] = v.y; meta[2] = v.z; meta[3] = v.w; }
        }

#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            // level 2 table of (this lane's row, quantization block gi): one fp32 product, one rounding
            {
                const int mo = gi * MSZ;
                const uint32_t mw = meta[mo / 4];
                const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)((mo % 4) ? (mw >> 16) : (mw & 0xffffu)));
                const float z = HZ ? (float)__builtin_bit_cast(_Float16, (uint16_t)(mw >> 16)) : 0.f;
                wave_lds_sync();  // every lane is done with the previous block's table
#pragma unroll
                for (int cde = 0; cde < NCODE; ++cde) {
                    const float wv = HZ ? ((float)cde - z) * s : (2.f * (float)cde - 1.f) * s;
                    *reinterpret_cast<_Float16*>(tab_own + cde * 128) = (_Float16)wv;
                }
                wave_lds_sync();  // entries are read by other lanes of the wave (after the half swap)
            }
#pragma unroll
            for (int kb = 0; kb < GQ / 32; ++kb) {
                const int kb32 = gi * (GQ / 32) + kb;
                const int v = (kb32 * 32) / CH;
                const int ksub = ((kb32 * 32) % CH) / 32;
                uint32_t planes[B];
#pragma unroll
                for (int i = 0; i < B; ++i) {
                    const int w = ksub * B + i;
                    planes[i] = w == 0 ? c[v].x : w == 1 ? c[v].y : w == 2 ? c[v].z : c[v].w;
                }
                uint32_t codes[4];
                planes_to_codes<B>(planes, codes);
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                    // after the swap: lo = [rows 0..31: word 2pr | word 2pr+1], hi = the same for rows 32..63
                    auto sw = __builtin_amdgcn_permlane32_swap(codes[2 * pr], codes[2 * pr + 1], false, false);
                    const uint32_t lo = sw[0], hi = sw[1];
                    half8_t wlo, whi;
#pragma unroll
                    for (int f = 0; f < 8; ++f) {
                        wlo[f] = *reinterpret_cast<const _Float16*>(tab_lo + ((lo >> (4 * f)) & 15u) * 128);
                        whi[f] = *reinterpret_cast<const _Float16*>(tab_hi + ((hi >> (4 * f)) & 15u) * 128);
                    }
                    // lanes with h = 0 carry word 2pr (columns 4f + 2pr), h = 1 word 2pr+1
                    const _Float16* xrow = xs + r * kXRowHalfs + kb32 * 32 + (2 * pr + h) * 8;
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) {
                        const half8_t xf = *reinterpret_cast<const half8_t*>(xrow + nb * 32 * kXRowHalfs);
                        acc[0][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xf, wlo, acc[0][nb], 0, 0, 0);
                        acc[1][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xf, whi, acc[1][nb], 0, 0, 0);
                    }
                }
            }
        }
    }

    if (!valid) return;
    // C[i][j]: i = token inside the 32-block (8 * (v / 4) + 4 * (lane / 32) + v % 4), j = row % 32
#pragma unroll
    for (int rh = 0; rh < 2; ++rh) {
        const int m = rb * kRows + rh * 32 + r;
        if (m < a.M) {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int n = n0 + nb * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                    if (n < a.N) a.y[(size_t)n * a.M + m] = (_Float16)acc[rh][nb][v];
                }
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
    dim3 grid((unsigned)((a.n_row_blocks + 3) / 4), (unsigned)((a.N + kGemmNTile - 1) / kGemmNTile));
    hipLaunchKernelGGL((mpgemm_kernel<B, GQ, HZ>), grid, dim3(256), kGemmLdsBytes, st, a);
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
