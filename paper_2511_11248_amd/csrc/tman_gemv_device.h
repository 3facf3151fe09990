// Device-side building blocks shared by the decoding kernels (table lookup by packed weight index, Sec. 2.2
// and Sec. 4.3): streaming of tile blocks through buffer loads, LDS access with explicit address spaces, the
// lookups of one tile block against tables that sit in LDS.
#pragma once
#include <hip/hip_fp16.h>

#include <type_traits>

#include "tman_internal.h"

namespace tman {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 4;  // waves per workgroup

template <int B, int NP, int GQ, bool HZ>
struct GemvCfg {
    static constexpr int CH = kKTile / B;    // weights per 16-byte chunk
    static constexpr int GPT = kKTile / GQ;  // quantization groups per tile
    static constexpr int MSZ = HZ ? 4 : 2;
    static constexpr int MPL = GPT * MSZ;    // group-parameter bytes per lane and tile
    static constexpr int TB = B * 1024 + 64 * MPL;
    static constexpr int T_BYTES = kTableBytesPerKTile * NP;
    static constexpr int S_FLOATS = GPT * NP;
    static constexpr int SLOT = T_BYTES + 256;  // table slice + group sums, per wave (multiple of 256)
    // tile blocks in flight per wave.  Measured: more do not help (the waves of a compute unit together
    // keep enough requests in flight) and cost time.
    static constexpr int D = NP >= 4 ? 1 : (B == 4 ? 1 : (B == 2 ? 2 : 3));
};

template <int B, int NP, int MPL>
struct Stage {
    u32x4 c[B];                    // bit-plane chunks
    uint32_t meta[(MPL + 3) / 4];  // scales / zeros of the lane's groups
    u32x4 tt[NP];                  // this lane's 16 bytes of each 1 KB of the table slice
    float sv;                      // one group sum (lanes < S_FLOATS)
};


__device__ __forceinline__ uint32_t word_of(const u32x4& v, int w) {
    return w == 0 ? v.x : w == 1 ? v.y : w == 2 ? v.z : v.w;
}

// Lanes of one wave exchange data through the wave's private LDS slot.  The hardware executes the
// LDS operations of a wave in order; this keeps the compiler from moving them across the exchange.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
}

__device__ __forceinline__ float half_bits_to_float(uint32_t bits16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
}

// values every lane agrees on, made visibly scalar for the compiler
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T>
__device__ __forceinline__ T* uniform(T* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<T*>(((uint64_t)hi << 32) | lo);
}

// explicit address spaces: descriptor pointers come out of memory as generic pointers, which would
// turn every access into a flat instruction
template <typename T>
using global_ptr = const T __attribute__((address_space(1)))*;
template <typename T>
using lds_ptr = T __attribute__((address_space(3)))*;

// wave-uniform base pointer + 32-bit per-lane byte offset: the form that needs no per-lane
// 64-bit address arithmetic
template <typename T>
__device__ __forceinline__ T load_global(const uint8_t* base, uint32_t off) {
    global_ptr<uint8_t> b = reinterpret_cast<global_ptr<uint8_t>>(reinterpret_cast<uintptr_t>(base));
    return *reinterpret_cast<global_ptr<T>>(b + off);
}
template <typename T>
__device__ __forceinline__ T load_lds(uint32_t addr) {
    return *reinterpret_cast<lds_ptr<const T>>(static_cast<uintptr_t>(addr));
}
template <typename T>
__device__ __forceinline__ void store_lds(uint32_t addr, T v) {
    *reinterpret_cast<lds_ptr<T>>(static_cast<uintptr_t>(addr)) = v;
}

// byte K of x, zero extended, in one full-rate VALU instruction
template <int K>
__device__ __forceinline__ uint32_t byte_of(uint32_t x) {
    uint32_t r;
    if constexpr (K == 0)
        asm("v_and_b32 %0, 0xff, %1" : "=v"(r) : "v"(x));
    else if constexpr (K == 3)
        asm("v_lshrrev_b32 %0, 24, %1" : "=v"(r) : "v"(x));
    else if constexpr (K == 1)
        asm("v_bfe_u32 %0, %1, 8, 8" : "=v"(r) : "v"(x));
    else
        asm("v_bfe_u32 %0, %1, 16, 8" : "=v"(r) : "v"(x));
    return r;
}

// a uniform float the compiler cannot constant-fold, so x * w + acc with fp16 x stays one
// mixed-precision FMA also for w == 1
__device__ __forceinline__ float opaque(float v) {
    asm("" : "+s"(v));
    return v;
}

// Buffer resource over a wave-uniform base: loads then take a 32-bit per-lane offset (constant for
// the whole kernel) plus a scalar offset (the tile), so streaming costs no address arithmetic.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr int kStreamAux = 2;  // non-temporal: weights are read once, keep them from evicting the tables in L2
__device__ __forceinline__ rsrc_t make_rsrc(const uint8_t* base, uint32_t bytes = 0xFFFFFFFFu) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, bytes, 0x00020000);
}

// The three streams a wave reads: its row block's tile blocks, the table slices and the group sums.
struct Streams {
    const uint8_t *w, *t, *s;
    uint32_t w_bytes, t_bytes, s_bytes;
};

// Requests the weights of tile kt: bit-plane chunks and group parameters of the lane's row.  With `live`
// false nothing is fetched and the stage reads as zeros: the caller needs no branch around the request, so
// a tile's lookups and the next request stay one basic block.
template <int B, int NP, int GQ, bool HZ>
__device__ __forceinline__ void issue_weights(Stage<B, NP, GemvCfg<B, NP, GQ, HZ>::MPL>& s, const Streams& src, bool live,
                                              int kt, int lane) {
    using Cfg = GemvCfg<B, NP, GQ, HZ>;
    const rsrc_t rw = make_rsrc(src.w, live ? src.w_bytes : 0u);
    const int so = kt * Cfg::TB;  // scalar offset of the tile block inside the row block
#pragma unroll
    for (int v = 0; v < B; ++v) s.c[v] = __builtin_amdgcn_raw_buffer_load_b128(rw, v * 1024 + lane * 16, so, kStreamAux);
    const int mo = B * 1024 + lane * Cfg::MPL;
    if constexpr (Cfg::MPL == 2) {
        s.meta[0] = __builtin_amdgcn_raw_buffer_load_b16(rw, mo, so, kStreamAux);
    } else if constexpr (Cfg::MPL == 4) {
        s.meta[0] = __builtin_amdgcn_raw_buffer_load_b32(rw, mo, so, kStreamAux);
    } else if constexpr (Cfg::MPL == 8) {
        u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rw, mo, so, kStreamAux);
        s.meta[0] = v.x;
        s.meta[1] = v.y;
    } else {
        u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, mo, so, kStreamAux);
        s.meta[0] = v.x;
        s.meta[1] = v.y;
        s.meta[2] = v.z;
        s.meta[3] = v.w;
    }
}


__device__ __forceinline__ uint32_t index_into(uint32_t idx_word, uint32_t base, uint32_t selector) {
    uint32_t r;
    asm("v_perm_b32 %0, %1, %2, %3" : "=v"(r) : "v"(idx_word), "v"(base), "s"(selector));
    return r;
}

// Sum over blocks of W consecutive lanes (W = 8, 16 or 32), every lane of a block receiving the block's sum.
// A butterfly: at each step a lane adds the sum of the neighbouring sub-block, which all lanes of that
// sub-block hold, so the mirror permutations of DPP serve as well as an exchange with lane ^ d.
template <int CTRL>
__device__ __forceinline__ float add_dpp(float v) {
    return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int W>
__device__ __forceinline__ float sum_over_lanes(float v) {
    v = add_dpp<0xB1>(v);   // quad_perm [1,0,3,2]: lane ^ 1
    v = add_dpp<0x4E>(v);   // quad_perm [2,3,0,1]: lane ^ 2
    v = add_dpp<0x141>(v);  // row_half_mirror: the other quad of 8 lanes
    if constexpr (W >= 16) v = add_dpp<0x140>(v);  // row_mirror: the other half of 16 lanes
    if constexpr (W >= 32)  // lane ^ 16 (crosses DPP rows)
        v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
    return v;
}

// One table of the one-token kernels: `xw` holds the table's four fp16 activations; the 16 entries (entry p = sum
// of the activations whose bit of p is set, added in ascending order, rounded to fp16 once) go to LDS at
// lt + j * 32, and the sum of every quantization group (TPG consecutive tables, held by TPG consecutive lanes)
// to ls + (j / TPG) * 4.  All lanes take part in the lane sum; `live` false stores nothing.
template <int TPG>
__device__ __forceinline__ void store_table(const u32x2& xw, int j, bool live, uint32_t lt, uint32_t ls) {
    // (copy the elements out first: a bit cast applied directly to a vector element reads element 0)
    const uint32_t w01 = xw.x, w23 = xw.y;
    const half2_t x01 = __builtin_bit_cast(half2_t, w01), x23 = __builtin_bit_cast(half2_t, w23);
    const float v[4] = {(float)x01[0], (float)x01[1], (float)x23[0], (float)x23[1]};
    float e[16];
    e[0] = 0.f;
    e[1] = v[0];
    e[2] = v[1];
    e[3] = v[0] + v[1];
#pragma unroll
    for (int p = 4; p < 8; ++p) e[p] = p == 4 ? v[2] : e[p - 4] + v[2];
#pragma unroll
    for (int p = 8; p < 16; ++p) e[p] = p == 8 ? v[3] : e[p - 8] + v[3];
    half8_t lo, hi;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        lo[p] = (_Float16)e[p];
        hi[p] = (_Float16)e[p + 8];
    }
    const float gs = sum_over_lanes<TPG>((v[0] + v[1]) + (v[2] + v[3]));
    if (live) {
        store_lds<u32x4>(lt + j * 32, __builtin_bit_cast(u32x4, lo));
        store_lds<u32x4>(lt + j * 32 + 16, __builtin_bit_cast(u32x4, hi));
        if (j % TPG == 0) store_lds<float>(ls + (j / TPG) * 4, gs);
    }
}

// Lookups of one tile block; `tbase` is the LDS address of the tile's 32 tables, `sbase` of its group sums.
template <int B, int GQ, bool HZ>
__device__ __forceinline__ void consume_weights(const Stage<B, 1, GemvCfg<B, 1, GQ, HZ>::MPL>& s, uint32_t tbase,
                                                uint32_t sbase, const uint32_t (&sel)[4], const float (&pw)[B],
                                                float& y) {
    using Cfg = GemvCfg<B, 1, GQ, HZ>;
    constexpr uint32_t NIB = 0x1E1E1E1Eu;  // index * 2 bytes, one per byte
    constexpr int TSTRIDE = 32;
    constexpr int W = 4 * B;
    constexpr int WPG = (GQ / 32) * B;
    auto fetch = [&](int wi, _Float16 (&e)[8]) {
        const int kb32 = wi / B, i = wi % B;
        const int v = (kb32 * 32) / Cfg::CH;
        const int ksub = ((kb32 * 32) % Cfg::CH) / 32;
        const int tb = (kb32 * 8) * TSTRIDE;
        const uint32_t w = word_of(s.c[v], ksub * B + i);
        const uint32_t xe = (w << 1) & NIB;
        const uint32_t xo = (w >> 3) & NIB;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            e[2 * k] = load_lds<_Float16>(index_into(xe, tbase, sel[k]) + (tb + (2 * k) * TSTRIDE));
            e[2 * k + 1] = load_lds<_Float16>(index_into(xo, tbase, sel[k]) + (tb + (2 * k + 1) * TSTRIDE));
        }
    };
    _Float16 e[2][8];
    float a = 0.f;
    fetch(0, e[0]);
#pragma unroll
    for (int wi = 0; wi < W; ++wi) {
        if (wi + 1 < W) fetch(wi + 1, e[(wi + 1) & 1]);
        if (wi % WPG == 0) a = 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) a = fmaf(pw[wi % B], (float)e[wi & 1][u], a);
        if (wi % WPG == WPG - 1) {
            const int gi = wi / WPG;
            const int mo = gi * Cfg::MSZ;
            const uint32_t mw = s.meta[mo / 4];
            const float sc = half_bits_to_float((mo % 4) ? (mw >> 16) : (mw & 0xffffu));
            const float gs = load_lds<float>(sbase + gi * 4);
            if constexpr (HZ) {
                const float z = half_bits_to_float(mw >> 16);
                y = fmaf(sc, fmaf(-z, gs, a), y);
            } else {
                y = fmaf(sc, fmaf(2.f, a, -gs), y);
            }
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    }
}


// kernel arguments: the descriptor itself for a single GEMV, the device table for a batch
template <bool SINGLE>
struct KernelArgs;
template <>
struct KernelArgs<true> {
    GemvDesc single;
    int n_gemv;   // 1
    int* status;  // the library's status word
};
template <>
struct KernelArgs<false> {
    const GemvDesc* descs;
    int n_gemv;
};

// A batch launch whose workgroups are numbered by the host: workgroup id -> (GEMV, workgroup within the GEMV).
// When all workgroups of a launch are resident at once, this chip's dispatcher hands workgroup i to compute unit
// i mod 256 (measured: ids 8, 264, 520, 776 share a unit), so the numbering decides which workgroups share a
// unit, and the host numbers them so that every unit gets the same amount of work (order_workgroups).
struct OrderedArgs {
    const GemvDesc* descs;
    const uint16_t* order;  // per workgroup id: GEMV in bits 13..15, workgroup within the GEMV in bits 0..12
    int n_gemv;
};
template <bool SINGLE>
__device__ __forceinline__ const GemvDesc& desc_of(const OrderedArgs& a, int g) {
    return a.descs[g];
}
// (GEMV, workgroup of the GEMV) of this workgroup: from the numbering, or from the 2-D grid
template <bool SINGLE, typename Args>
__device__ __forceinline__ void workgroup_of(const Args& a, int& g, int& wg_local) {
    if constexpr (__is_same(Args, OrderedArgs)) {
        const uint32_t e = (uint32_t)__builtin_amdgcn_readfirstlane((int)a.order[blockIdx.x]);
        g = (int)(e >> 13);
        wg_local = (int)(e & 0x1fffu);
    } else {
        g = SINGLE ? 0 : (int)blockIdx.y;
        wg_local = (int)blockIdx.x;
    }
}

template <bool SINGLE>
__device__ __forceinline__ const GemvDesc& desc_of(const KernelArgs<SINGLE>& a, int g) {
    if constexpr (SINGLE) {
        return a.single;
    } else {
        return a.descs[g];
    }
}

// Output of one row block by its first wave: y holds the sums of the workgroup's K segment for the lane's
// row; `step` is a factor per token applied to the final sum (1, or the power-of-two step of integer tables).  With one segment they are the result; otherwise the segments meet through memory (see above).
template <int NP>
__device__ __forceinline__ void finish_rows(const GemvDesc& d, int rb, int seg, int n_seg, int lane, float (&y)[NP],
                                            const float (&step)[NP]) {
    const int m = rb * kRows + lane;
    const int M = d.M, N = d.N;
    _Float16* out = static_cast<_Float16*>(d.y);
    if (n_seg == 1) {
        if (m < M) {
#pragma unroll
            for (int n = 0; n < NP; ++n)
                if (n < N) out[(size_t)n * M + m] = (_Float16)(y[n] * step[n]);
        }
        return;
    }

    // K longer than one segment: publish this segment's partial sums and take a ticket
    float* base_p = d.partial + (size_t)rb * n_seg * NP * kRows;
    float* mine = base_p + (size_t)seg * NP * kRows;
#pragma unroll
    for (int n = 0; n < NP; ++n)
        __hip_atomic_store(mine + n * kRows + lane, y[n], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the partials have reached device-coherent memory
    int32_t* ticket = d.tickets + rb;
    int prev = 0;
    if (lane == 0) prev = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    prev = __builtin_amdgcn_readfirstlane(prev);
    if (prev != n_seg - 1) return;
    // last ticket: every segment of this row block has been published; add them in segment order
    float acc[NP];
#pragma unroll
    for (int n = 0; n < NP; ++n) acc[n] = 0.f;
    for (int p0 = 0; p0 < n_seg; p0 += 4) {
        float v[4][NP];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int n = 0; n < NP; ++n)
                v[q][n] = (p0 + q < n_seg) ? __hip_atomic_load(base_p + ((size_t)(p0 + q) * NP + n) * kRows + lane,
                                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                           : 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int n = 0; n < NP; ++n) acc[n] += v[q][n];
    }
    if (m < M) {
#pragma unroll
        for (int n = 0; n < NP; ++n)
            if (n < N) out[(size_t)n * M + m] = (_Float16)(acc[n] * step[n]);
    }
    if (lane == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace tman
