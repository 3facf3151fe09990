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
// The fp16 weight tile goes to LDS and is shared by the waves of the workgroup (each weight is
// dequantized once per 256 tokens); activations are staged next to it unchanged.  Pipeline (the GPU form of DMA -> vector -> matrix): global loads of stage s+2 are in
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

typedef __amdgpu_buffer_rsrc_t rsrc_t;
// raw buffer resource: loads at or beyond `bytes` return zero
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

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

// Loads 32-weight block `kb32` of tile block `tile` of this wave's row block.  `rw` covers the row
// block's tiles or nothing (rows beyond M, stages beyond K), in which case everything reads as zero.
template <int B, int GQ, bool HZ>
__device__ __forceinline__ void load_w(WRegs<B>& r, rsrc_t rw, int tile, int kb32, int lane) {
    constexpr int CH = kKTile / B;
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int MPL = (kKTile / GQ) * MSZ;
    constexpr int TB = B * 1024 + 64 * MPL;
    const int v = (kb32 * 32) / CH, ksub = ((kb32 * 32) % CH) / 32;
    const int so = tile * TB + v * 1024 + ksub * B * 4;
    if constexpr (B == 4) {
        const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(rw, lane * 16, so, 0);
        r.plane[0] = w.x; r.plane[1] = w.y; r.plane[2] = w.z; r.plane[3] = w.w;
    } else if constexpr (B == 2) {
        const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rw, lane * 16, so, 0);
        r.plane[0] = w.x; r.plane[1] = w.y;
    } else {
        r.plane[0] = __builtin_amdgcn_raw_buffer_load_b32(rw, lane * 16, so, 0);
    }
    const int mo = tile * TB + B * 1024 + ((kb32 * 32) / GQ) * MSZ;
    if constexpr (HZ) r.meta = __builtin_amdgcn_raw_buffer_load_b32(rw, lane * MPL, mo, 0);
    else r.meta = __builtin_amdgcn_raw_buffer_load_b16(rw, lane * MPL, mo, 0);
}

// Level 2 for one lane's 32 weights; writes them as fp16, in column order, into its row of the LDS
// weight tile (`wrow` already points at the block's 64 bytes).
//
// Field f of code word o (weight 4f + o) is turned into an fp16 number without moving it to bit 0:
// a nibble at mantissa bits 0..3 of 0x6400 reads 1024 + c, one at bits 4..7 reads 1024 + 16c.  Fields
// f and f + 4 sit 16 bits apart, so one AND-OR makes two such numbers; a single shift by 8 brings
// fields 2, 3, 6, 7 into reach.  The affine map (c - zero) * scale is then one fp32 FMA per weight
// with a single rounding to fp16:  (1024 + c) * s - (1024 + z) * s   or   (1024 + 16c) * s/16 - (64 + z) * s.
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
    // part 3: 16-byte piece q (weights 8q .. 8q + 7 = fields 2q, 2q + 1) -> LDS
    __device__ __forceinline__ void emit(int q, uint8_t* wrow) const {
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
        *reinterpret_cast<u32x4*>(wrow + q * 16) = out;
    }
};

template <int B, bool HZ>
__device__ __forceinline__ void dequant_to_lds(const WRegs<B>& r, uint8_t* wrow) {
    Dequant<B, HZ> dq;
    dq.start(r);
    dq.insert();
#pragma unroll
    for (int q = 0; q < 4; ++q) dq.emit(q, wrow);
}

// activation staging: plain 16-byte pieces (8 columns of one token), eight per producer thread and
// stage; eight consecutive lanes cover the 128 bytes of one token row
constexpr int kXPieces = 8;
struct XRegs {
    u32x4 p[kXPieces];
};
constexpr int kXPieceStride = 32 * kRowBytes;  // pieces i and i + 1 of a thread are 32 tokens apart
constexpr uint32_t kOutOfRange = 0x80000000u;

// `rx` covers the workgroup's token rows from their first column (or nothing); rows beyond N lie
// past its end.  k0: first column of the stage, col: first column of the thread's piece in the stage.
__device__ __forceinline__ void load_x(XRegs& r, rsrc_t rx, const uint32_t (&voff)[kXPieces], int col, int K, int k0) {
    const bool inside = col + 8 <= K - k0;  // K is a multiple of 32, so pieces are all-or-nothing
#pragma unroll
    for (int i = 0; i < kXPieces; ++i)
        r.p[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, inside ? voff[i] : kOutOfRange, k0 * 2, 0);
}

__device__ __forceinline__ void store_x(const XRegs& r, uint8_t* dst) {
#pragma unroll
    for (int i = 0; i < kXPieces; ++i) *reinterpret_cast<u32x4*>(dst + i * kXPieceStride) = r.p[i];
}

// Workgroup = 12 waves, three per SIMD.  Waves 0..7 are consumers: wave (wm, wn) owns 128 rows x 64
// tokens of the 256 x 256 tile and does nothing but read MFMA operands from LDS and issue MFMAs.
// Waves 8..11 are producers: wave p turns row block p of each stage into fp16 in LDS and stages a
// quarter of the activations.  Vector work of the producers and matrix work of the consumers come
// from different waves of a SIMD, so the hardware overlaps them without any help from the schedule.
constexpr int kConsumerWaves = 8;
constexpr int kThreads = 768;

template <int B, int GQ, bool HZ>
__global__ void __launch_bounds__(kThreads, 1) mpgemm_kernel(GemmArgs a) {
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int TB = B * 1024 + 64 * (kKTile / GQ) * MSZ;

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int n0 = blockIdx.y * kTN;
    const int n_stages = (a.K + kStageK - 1) / kStageK;

    float16_t acc[4][2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;
    const int wm = (wave >> 2) & 1, wn = wave & 3, r = lane & 31, h = lane >> 5;

    if (wave >= kConsumerWaves) {
        // ---------------------------------------------------------------- producer
        const int p = wave - kConsumerWaves, ptid = tid - kConsumerWaves * 64;
        const int rbw = blockIdx.x * 4 + p;
        const bool wvalid = rbw < a.n_row_blocks;
        const uint8_t* wsrc = a.tiles + (size_t)(wvalid ? rbw : 0) * a.n_ktiles * TB;
        const int xrows = a.N - n0 < kTN ? a.N - n0 : kTN;
        const _Float16* xsrc = a.x + (size_t)n0 * a.K;
        const uint32_t xbytes = (uint32_t)xrows * (uint32_t)a.K * 2u;
        const int xcol = (ptid & 7) * 8;
        uint32_t xvoff[kXPieces];
#pragma unroll
        for (int i = 0; i < kXPieces; ++i)
            xvoff[i] = ((uint32_t)((ptid >> 3) + 32 * i) * (uint32_t)a.K + (uint32_t)xcol) * 2u;
        const int xdst = kWTile + (ptid >> 3) * kRowBytes + (ptid & 7) * 16;
        const int wdst = (p * 64 + lane) * kRowBytes;  // this lane's 128 bytes in the weight tile

        WRegs<B> wr[2];
        XRegs xr;
        // stage t: global -> registers; a stage beyond K reads zeros
        auto load_stage = [&](int t) {
            const rsrc_t rw = make_rsrc(wsrc, t < n_stages && wvalid ? 0x7fffffffu : 0u);
            load_w<B, GQ, HZ>(wr[0], rw, t >> 1, 2 * (t & 1), lane);
            load_w<B, GQ, HZ>(wr[1], rw, t >> 1, 2 * (t & 1) + 1, lane);
            load_x(xr, make_rsrc(xsrc, t < n_stages ? xbytes : 0u), xvoff, xcol, a.K, t * kStageK);
        };
        auto to_lds = [&](uint8_t* stage) {
            store_x(xr, stage + xdst);
            dequant_to_lds<B, HZ>(wr[0], stage + wdst);
            dequant_to_lds<B, HZ>(wr[1], stage + wdst + 64);
        };
        load_stage(0);
        to_lds(smem);
        load_stage(1);
        __syncthreads();
        for (int s = 0; s < n_stages; ++s) {
            // stage s+1: registers -> LDS (the buffer the consumers are not reading); stage s+2: global -> registers
            to_lds(smem + (kStageBytes - (s & 1) * kStageBytes));
            load_stage(s + 2);
            __syncthreads();
        }
    } else {
        // ---------------------------------------------------------------- consumer
        // MFMA operand addresses: lanes with h = 0 / 1 take the two 8-column groups of a 16-column step
        const int wfrag = (wm * 128 + r) * kRowBytes + h * 16;
        const int xfrag = kWTile + (wn * 64 + r) * kRowBytes + h * 16;
        __syncthreads();
        for (int s = 0; s < n_stages; ++s) {
            const uint8_t* cur = smem + (s & 1) * kStageBytes;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                half8_t wf[4], xf[2];
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
                    wf[mb] = *reinterpret_cast<const half8_t*>(cur + wfrag + mb * 32 * kRowBytes + j * 32);
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
                    xf[nb] = *reinterpret_cast<const half8_t*>(cur + xfrag + nb * 32 * kRowBytes + j * 32);
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[mb], xf[nb], acc[mb][nb], 0, 0, 0);
            }
            __syncthreads();
        }
    }

    // epilogue: accumulators -> fp16 -> LDS as [token][row] -> coalesced 16-byte stores
    // C[i][j] of a 32x32 block: i = row (8 * (v / 4) + 4 * h + v % 4), j = token (lane % 32)
    constexpr int kOutRow = kTM * 2 + 16;  // bytes per token row of the output tile in LDS
    uint8_t* otile = smem;                 // 256 * 528 = 135,168 bytes, the stage buffers are free now
    if (wave < kConsumerWaves)
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
    for (int piece = tid; piece < kTN * (kTM / 8); piece += kThreads) {
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
    hipLaunchKernelGGL((mpgemm_kernel<B, GQ, HZ>), grid, dim3(kThreads), kGemmLdsBytes, st, a);
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
