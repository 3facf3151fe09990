// The lookup kernel of decoding (Sec. 2.2 "Bit-serial table lookup", Sec. 4.3), as a template over the weight
// format, the padded token count and the kind of table entries (fp16 numbers, or 16-bit integers with integer
// aggregation inside a quantization block); tman_mpgemv.hip and tman_mpgemv_i16.hip instantiate it.
#pragma once
#include "tman_gemv_device.h"

namespace tman {


// Requests tile kt: its weights, its slice of the lookup tables and its group sums (same rule for `live`).
template <int B, int NP, int GQ, bool HZ>
__device__ __forceinline__ void issue_tile(Stage<B, NP, GemvCfg<B, NP, GQ, HZ>::MPL>& s, const Streams& src, bool live,
                                           int kt, int lane) {
    using Cfg = GemvCfg<B, NP, GQ, HZ>;
    issue_weights<B, NP, GQ, HZ>(s, src, live, kt, lane);
    const rsrc_t rt = make_rsrc(src.t, live ? src.t_bytes : 0u);
    const rsrc_t rs = make_rsrc(src.s, live ? src.s_bytes : 0u);
    const int to = kt * Cfg::T_BYTES;
#pragma unroll
    for (int q = 0; q < NP; ++q) s.tt[q] = __builtin_amdgcn_raw_buffer_load_b128(rt, q * 1024 + lane * 16, to, 0);
    // every lane loads one float from the tile's group sums on (no divergent branch: the tile's code
    // stays one basic block); `rs` ends with the array, lanes reaching past it read zero
    s.sv = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (kt * Cfg::S_FLOATS + lane) * 4, 0, 0));
}

// A table entry as it comes out of LDS: NP 16-bit values (the NP tokens of one pattern), fp16 numbers or, with
// integer tables, int16 numbers.
template <int NP, bool INT> struct EntryT;
template <> struct EntryT<1, false> { typedef _Float16 type; };
template <> struct EntryT<2, false> { typedef half2_t type; };
template <> struct EntryT<4, false> { typedef half4_t type; };
template <> struct EntryT<8, false> { typedef half8_t type; };
template <> struct EntryT<1, true> { typedef int16_t type; };   // (a sign-extending LDS read)
template <> struct EntryT<2, true> { typedef uint32_t type; };
template <> struct EntryT<4, true> { typedef u32x2 type; };
template <> struct EntryT<8, true> { typedef u32x4 type; };

typedef float float4_t __attribute__((ext_vector_type(4)));

// Plane weights 2^i ("shift and accumulate") in the two forms the accumulation uses.
//
// One or two tokens: a uniform float, the entry is added with a mixed-precision FMA.
// Four or eight tokens: a lookup returns the entries of 4 (8) tokens for the lane's row, and adding them with
// one FMA per token makes the kernel bound by vector instruction issue.  The matrix pipe does the same
// additions in one 4x4x4 MFMA per four tokens: with the 64 lanes as 16 blocks of 4, lane (b, j) supplies as
// B[k][j] its own four entries (k = token) and as A[i][k] row i = j of 2^plane times the identity, so
// D[i][j] = 2^plane * (entry of token i in lane (b, j)): register i of the lane's accumulator is token i of
// its own row.  fp16 inputs, exact products, fp32 accumulation, as with the FMA.
template <int B, int NP>
struct PlaneWeights {
    float pw[B];
    half4_t hot[B];  // NP >= 4: row (lane % 4) of 2^i * identity
};

template <int B, int NP>
__device__ __forceinline__ PlaneWeights<B, NP> make_plane_weights(int lane) {
    PlaneWeights<B, NP> w;
#pragma unroll
    for (int i = 0; i < B; ++i) {
        w.pw[i] = opaque((float)(1 << i));
#pragma unroll
        for (int k = 0; k < 4; ++k) w.hot[i][k] = (lane & 3) == k ? (_Float16)(float)(1 << i) : (_Float16)0.f;
    }
    return w;
}

template <int NP, bool INT>
struct Accum;

template <int NP>
struct Accum<NP, false> {
    float a[NP < 4 ? NP : 1];
    float4_t q[NP >= 4 ? NP / 4 : 1];
    __device__ __forceinline__ void clear() {
        if constexpr (NP < 4) {
#pragma unroll
            for (int n = 0; n < NP; ++n) a[n] = 0.f;
        } else {
#pragma unroll
            for (int h = 0; h < NP / 4; ++h) q[h] = float4_t{0.f, 0.f, 0.f, 0.f};
        }
    }
    template <int B>
    __device__ __forceinline__ void add(const typename EntryT<NP, false>::type& e, const PlaneWeights<B, NP>& w, int plane) {
        if constexpr (NP == 1) {
            a[0] = fmaf(w.pw[plane], (float)e, a[0]);
        } else if constexpr (NP == 2) {
#pragma unroll
            for (int n = 0; n < NP; ++n) a[n] = fmaf(w.pw[plane], (float)e[n], a[n]);
        } else if constexpr (NP == 4) {
            q[0] = __builtin_amdgcn_mfma_f32_4x4x4f16(w.hot[plane], e, q[0], 0, 0, 0);
        } else {
            const half4_t lo = {e[0], e[1], e[2], e[3]}, hi = {e[4], e[5], e[6], e[7]};
            q[0] = __builtin_amdgcn_mfma_f32_4x4x4f16(w.hot[plane], lo, q[0], 0, 0, 0);
            q[1] = __builtin_amdgcn_mfma_f32_4x4x4f16(w.hot[plane], hi, q[1], 0, 0, 0);
        }
    }
    __device__ __forceinline__ float get(int n) const {
        if constexpr (NP < 4) return a[n];
        else return q[n / 4][n % 4];
    }
};

// Integer tables (Sec. 4.3: entries are aggregated at low precision inside a quantization block, floating point
// only across blocks; Sec. 6.1 A_INT16): 16-bit integer entries, "shift and accumulate" as a shift-add into a
// 32-bit integer per token.  The sum over a block stays below 2^24 (15 * 32 lookups * 32764), so it converts to
// fp32 exactly when the block's scale is applied.
template <int NP>
struct Accum<NP, true> {
    int a[NP];
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int n = 0; n < NP; ++n) a[n] = 0;
    }
    static __device__ __forceinline__ int low_half(uint32_t w) { return (int)(int16_t)(w & 0xffffu); }
    static __device__ __forceinline__ int high_half(uint32_t w) { return (int)w >> 16; }
    template <int B>
    __device__ __forceinline__ void add(const typename EntryT<NP, true>::type& e, const PlaneWeights<B, NP>&, int plane) {
        if constexpr (NP == 1) {
            a[0] += (int)e << plane;
        } else if constexpr (NP == 2) {
            a[0] += low_half(e) << plane;
            a[1] += high_half(e) << plane;
        } else {
#pragma unroll
            for (int w = 0; w < NP / 2; ++w) {
                const uint32_t v = e[w];  // (copy the element out before any cast)
                a[2 * w] += low_half(v) << plane;
                a[2 * w + 1] += high_half(v) << plane;
            }
        }
    }
    __device__ __forceinline__ float get(int n) const { return (float)a[n]; }
};

// Lookups of one tile block for the lane's row.  `lds` is the LDS address of the wave's private slot;
// the callers make it a link-time constant (one copy of the code per wave of the workgroup), so it
// folds, together with the table's offset, into the immediate offset of the LDS load and the address
// register is just the index byte.  The 4*B plane words of the tile are handled
// one after the other, software pipelined: the eight lookups of word w+1 are issued before the eight
// results of word w are accumulated, so LDS latency overlaps the arithmetic with few live registers.
template <int B, int NP, int GQ, bool HZ, bool INT>
__device__ __forceinline__ void consume_tile(const Stage<B, NP, GemvCfg<B, NP, GQ, HZ>::MPL>& s, uint32_t lds, int lane,
                                             const PlaneWeights<B, NP>& pw, float (&y)[NP]) {
    using Cfg = GemvCfg<B, NP, GQ, HZ>;
    typedef typename EntryT<NP, INT>::type entry_t;
    constexpr int EB = 2 * NP;                                       // bytes per table entry
    constexpr int SH = EB == 2 ? 1 : EB == 4 ? 2 : EB == 8 ? 3 : 4;  // log2(EB)
    constexpr uint32_t NIB = 0x0F0F0F0Fu << SH;                      // index * EB, one per byte
    constexpr int TSTRIDE = 16 * EB;                                 // bytes per table
    constexpr int W = 4 * B;                                         // plane words per tile
    constexpr int WPG = (GQ / 32) * B;                               // plane words per quantization block
    // table slice and group sums -> LDS (wave private; LDS operations of one wave execute in order)
    wave_lds_sync();  // every lane is done reading the previous slice
#pragma unroll
    for (int q = 0; q < NP; ++q) store_lds<u32x4>(lds + q * 1024 + lane * 16, s.tt[q]);
    store_lds<float>(lds + Cfg::T_BYTES + lane * 4, s.sv);  // the first S_FLOATS lanes hold the tile's sums
    wave_lds_sync();


    // word wi: 32-weight block kb32 = wi / B of the tile, bit-plane i = wi % B
    auto fetch = [&](int wi, entry_t (&e)[8]) {
        const int kb32 = wi / B, i = wi % B;
        const int v = (kb32 * 32) / Cfg::CH;
        const int ksub = ((kb32 * 32) % Cfg::CH) / 32;
        const int tb = (kb32 * 8) * TSTRIDE;  // the 8 tables of this block
        const uint32_t w = word_of(s.c[v], ksub * B + i);
        // the eight 4-bit indices of the word, pre-multiplied by the entry size: even nibbles in the
        // bytes of xe, odd nibbles in the bytes of xo
        const uint32_t xe = (w << SH) & NIB;
        const uint32_t xo = SH == 4 ? (w & NIB) : ((w >> (4 - SH)) & NIB);
        e[0] = load_lds<entry_t>(byte_of<0>(xe) + (lds + tb + 0 * TSTRIDE));
        e[1] = load_lds<entry_t>(byte_of<0>(xo) + (lds + tb + 1 * TSTRIDE));
        e[2] = load_lds<entry_t>(byte_of<1>(xe) + (lds + tb + 2 * TSTRIDE));
        e[3] = load_lds<entry_t>(byte_of<1>(xo) + (lds + tb + 3 * TSTRIDE));
        e[4] = load_lds<entry_t>(byte_of<2>(xe) + (lds + tb + 4 * TSTRIDE));
        e[5] = load_lds<entry_t>(byte_of<2>(xo) + (lds + tb + 5 * TSTRIDE));
        e[6] = load_lds<entry_t>(byte_of<3>(xe) + (lds + tb + 6 * TSTRIDE));
        e[7] = load_lds<entry_t>(byte_of<3>(xo) + (lds + tb + 7 * TSTRIDE));
    };

    entry_t e[2][8];
    Accum<NP, INT> a;
    fetch(0, e[0]);
#pragma unroll
    for (int wi = 0; wi < W; ++wi) {
        if (wi + 1 < W) fetch(wi + 1, e[(wi + 1) & 1]);
        if (wi % WPG == 0) a.clear();
#pragma unroll
        for (int u = 0; u < 8; ++u) a.template add<B>(e[wi & 1][u], pw, wi % B);
        if (wi % WPG == WPG - 1) {
            // scale and zero of the quantization block just finished
            const int gi = wi / WPG;
            const int mo = gi * Cfg::MSZ;
            const uint32_t mw = s.meta[mo / 4];
            const float sc = half_bits_to_float((mo % 4) ? (mw >> 16) : (mw & 0xffffu));
            const uint32_t sg = lds + Cfg::T_BYTES + gi * NP * 4;
            // the block's activation sums: fp32, or (integer tables) int32, exact in fp32 (128 * 8191 < 2^24)
            auto block_sum = [&](int n) {
                if constexpr (INT) return (float)load_lds<int>(sg + n * 4);
                else return load_lds<float>(sg + n * 4);
            };
            if constexpr (HZ) {
                const float z = half_bits_to_float(mw >> 16);  // 4-byte entry: scale low, zero high
#pragma unroll
                for (int n = 0; n < NP; ++n) y[n] = fmaf(sc, fmaf(-z, block_sum(n), a.get(n)), y[n]);
            } else {
#pragma unroll
                for (int n = 0; n < NP; ++n) y[n] = fmaf(sc, fmaf(2.f, a.get(n), -block_sum(n)), y[n]);
            }
        }
        // keep the pipeline order, which bounds the live registers: the first stops the compiler from
        // collecting the lookups of later words up front, the second the instruction scheduler
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int B, int NP, int GQ, bool HZ, bool SINGLE, bool INT>
__global__ void __launch_bounds__(kWaves * 64) mpgemv_kernel(KernelArgs<SINGLE> a) {
    using Cfg = GemvCfg<B, NP, GQ, HZ>;
    constexpr int D = Cfg::D;
    __shared__ __attribute__((aligned(1024))) uint8_t slots[kWaves * Cfg::SLOT];
    __shared__ float red[kWaves][NP][kRows];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const PlaneWeights<B, NP> pw = make_plane_weights<B, NP>(lane);

    // The grid is (workgroups of the largest GEMV) x (GEMVs): a workgroup knows its GEMV from its block
    // index, without searching the descriptor table (every workgroup of a launch starts at the same time,
    // so a chain of dependent loads here delays the whole launch); surplus workgroups leave at once.
    const int g = SINGLE ? 0 : (int)blockIdx.y;
    const GemvDesc& d = desc_of<SINGLE>(a, g);
    const int n_seg = uniform(d.n_seg), n_ktiles = uniform(d.n_ktiles);
    const int wg_local = (int)blockIdx.x;
    if (wg_local >= uniform(d.n_row_blocks) * n_seg) return;
    if constexpr (SINGLE) {
        // a blob packed for another shape or layout: leave y alone and say so (a batch is checked when its
        // descriptor table is written, which empties the descriptor of such a GEMV)
        if (!header_matches(uniform(d.tiles), uniform(d.M), uniform(d.K), B, GQ, HZ ? 1 : 0)) {
            if (wg_local == 0 && threadIdx.x == 0) report_header_mismatch(a.status);
            return;
        }
    }
    const int rb = wg_local / n_seg, seg = wg_local % n_seg;
    const int seg_tiles = uniform(d.seg_tiles);
    const int k0 = seg * seg_tiles;
    const int k1 = min(k0 + seg_tiles, n_ktiles);
    const int per_wave = (k1 - k0 + kWaves - 1) / kWaves;
    const int t0 = min(k0 + wave * per_wave, k1);  // this wave's K tiles [t0, t1)
    const int t1 = min(t0 + per_wave, k1);
    Streams src;
    src.w = uniform(d.tiles) + (size_t)rb * n_ktiles * Cfg::TB;  // this row block's tiles
    src.t = uniform(d.lut_t);
    src.s = uniform(d.lut_s);
    src.w_bytes = (uint32_t)(n_ktiles * Cfg::TB);
    src.t_bytes = (uint32_t)(n_ktiles * Cfg::T_BYTES);
    src.s_bytes = (uint32_t)(n_ktiles * Cfg::S_FLOATS * 4);

    float y[NP];
#pragma unroll
    for (int n = 0; n < NP; ++n) y[n] = 0.f;

    // The wave's tiles, with the LDS address of its slot known to the compiler (see consume_tile).
    auto stream_tiles = [&](auto wave_tag) {
        constexpr int WAVE = decltype(wave_tag)::value;
        const uint32_t lds = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr<uint8_t>)slots)) + WAVE * Cfg::SLOT;
        Stage<B, NP, Cfg::MPL> st[D] = {};
#pragma unroll
        for (int s = 0; s < D; ++s)
            issue_tile<B, NP, GQ, HZ>(st[s], src, t0 + s < t1, t0 + s, lane);
        for (int base = t0; base < t1; base += D) {
#pragma unroll
            for (int s = 0; s < D; ++s) {
                const int t = base + s;
                if (t < t1) {
                    {   // the more tiles a wave still has to do, the higher its issue priority: the waves
                        // of a SIMD then finish together instead of leaving the youngest to run alone
                        const int rem = t1 - t;
                        if (rem >= 7) __builtin_amdgcn_s_setprio(3);
                        else if (rem >= 5) __builtin_amdgcn_s_setprio(2);
                        else if (rem >= 3) __builtin_amdgcn_s_setprio(1);
                        else __builtin_amdgcn_s_setprio(0);
                    }
                    consume_tile<B, NP, GQ, HZ, INT>(st[s], lds, lane, pw, y);
                    issue_tile<B, NP, GQ, HZ>(st[s], src, t + D < t1, t + D, lane);
                }
            }
        }
    };
    static_assert(kWaves == 4, "one copy of the tile loop per wave");
    switch (wave) {
        case 0: stream_tiles(std::integral_constant<int, 0>{}); break;
        case 1: stream_tiles(std::integral_constant<int, 1>{}); break;
        case 2: stream_tiles(std::integral_constant<int, 2>{}); break;
        default: stream_tiles(std::integral_constant<int, 3>{}); break;
    }

    // the four quarters of the segment meet in LDS
#pragma unroll
    for (int n = 0; n < NP; ++n) red[wave][n][lane] = y[n];
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int n = 0; n < NP; ++n) y[n] = ((red[0][n][lane] + red[1][n][lane]) + red[2][n][lane]) + red[3][n][lane];

    // integer tables: the tokens' power-of-two steps (behind the block sums in the table buffer) scale the result
    float step[NP];
#pragma unroll
    for (int n = 0; n < NP; ++n) step[n] = 1.f;
    if constexpr (INT) {
        const int* ex = reinterpret_cast<const int*>(uniform(d.lut_s) + (size_t)n_ktiles * Cfg::S_FLOATS * 4);
#pragma unroll
        for (int n = 0; n < NP; ++n) step[n] = ldexpf(1.f, uniform(ex[n]));
    }
    finish_rows<NP>(d, rb, seg, n_seg, lane, y, step);
}

// ---------------------------------------------------------------------------------------------
// launch

template <int B, int NP, int GQ, bool HZ, bool SINGLE, bool INT>
static int launch_cfg(const KernelArgs<SINGLE>& a, int n_workgroups, hipStream_t st) {
    hipLaunchKernelGGL((mpgemv_kernel<B, NP, GQ, HZ, SINGLE, INT>), dim3((unsigned)n_workgroups, (unsigned)a.n_gemv), dim3(kWaves * 64),
                       0, st, a);
    return launch_status();
}

template <int B, int NP, bool HZ, bool SINGLE, bool INT>
static int launch_group(int group, const KernelArgs<SINGLE>& a, int n_wg, hipStream_t st) {
    switch (group) {
        case 32: return launch_cfg<B, NP, 32, HZ, SINGLE, INT>(a, n_wg, st);
        case 64: return launch_cfg<B, NP, 64, HZ, SINGLE, INT>(a, n_wg, st);
        default: return launch_cfg<B, NP, 128, HZ, SINGLE, INT>(a, n_wg, st);
    }
}

template <int B, bool HZ, bool SINGLE, bool INT>
static int launch_tokens(int np, int group, const KernelArgs<SINGLE>& a, int n_wg, hipStream_t st) {
    switch (np) {
        case 1: return launch_group<B, 1, HZ, SINGLE, INT>(group, a, n_wg, st);
        case 2: return launch_group<B, 2, HZ, SINGLE, INT>(group, a, n_wg, st);
        case 4: return launch_group<B, 4, HZ, SINGLE, INT>(group, a, n_wg, st);
        default: return launch_group<B, 8, HZ, SINGLE, INT>(group, a, n_wg, st);
    }
}

template <bool SINGLE, bool INT>
static int launch_format(int bits, int has_zero, int np, int group, const KernelArgs<SINGLE>& a, int n_wg,
                         hipStream_t st) {
    if (bits == 1) {
        return has_zero ? launch_tokens<1, true, SINGLE, INT>(np, group, a, n_wg, st)
                        : launch_tokens<1, false, SINGLE, INT>(np, group, a, n_wg, st);
    }
    if (bits == 2) return launch_tokens<2, true, SINGLE, INT>(np, group, a, n_wg, st);
    return launch_tokens<4, true, SINGLE, INT>(np, group, a, n_wg, st);
}

}  // namespace tman
