// Decoding mpGEMV through bit-serial table lookup (Sec. 2.2 "Bit-serial table lookup", Sec. 4.3
// "Mapping of LUT-based Decoding").
//
//   y[n][m] = sum_G scale[m][G] * ( sum_i 2^i sum_{j in G} T[n][j][idx_i[m][j]] - zero[m][G] * S[n][G] )
//
// Mapping onto a CDNA4 compute unit.  As in the paper's vector-core mapping the lookups are
// vectorised along the output rows: the 64 lanes of a wave hold 64 different rows and index the SAME
// 16-entry table, so the table (32 bytes = 8 LDS banks) is read by broadcast without bank conflicts,
// every lane keeps a private fp32 accumulator for its row, and nothing crosses lanes in the loop.
// The paper's two-level tiling appears as: inner tile = one quantization block (table entries summed
// in fp32, then one scale/zero application), outer tile = a 128-column tile whose 32 tables sit in LDS.
//
// Scheduling.  A decode GEMV streams each weight byte once and a whole layer lasts microseconds, so
// the kernel is organised around keeping HBM requests in flight and around short dependency chains:
//   - a workgroup of four waves owns one row block (64 rows) and one K segment of at most 32 tiles;
//     each wave takes a quarter of the segment and walks it with one or two tile blocks in flight
//     (coalesced 16-byte loads of the bit-plane chunks, the group parameters and the 1 KB table
//     slice of the tile); the table slice goes to the wave's private LDS slot, so waves do not
//     synchronise while streaming;
//   - the four partial sums of a row meet in LDS (one barrier, fixed order);
//   - only when K is longer than one segment do segments meet through memory: each publishes its
//     fp32 partial and takes a ticket, the last one adds the partials in segment order (so the result
//     does not depend on timing).  Partials and tickets use device-scope memory operations, which are
//     coherent across the chip without cache write-back or invalidation.
// All GEMVs of a decode step can share one launch (descriptor table), so the machine is filled even
// though one layer alone is too small.
//
// Two kernels follow.  mpgemv_kernel serves 1 to 8 tokens and reads the tables tman_build_lut made
// (Sec. 5: the precompute as a kernel of its own, shared by the layers fed from one activation).
// mpgemv_x_kernel serves one token and builds the tables of its K segment itself, in LDS, from the
// activations: the same lookups, but a decode step is a single launch and no table ever reaches memory.
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

// ---------------------------------------------------------------------------------------------
// host-side planning

static GemvPlan plan_segments(const Layout& L, int np, int max_seg) {
    GemvPlan p;
    p.np = np;
    p.n_seg = (L.n_ktiles + max_seg - 1) / max_seg;
    p.seg_tiles = (L.n_ktiles + p.n_seg - 1) / p.n_seg;
    p.n_seg = (L.n_ktiles + p.seg_tiles - 1) / p.seg_tiles;
    p.n_workgroups = L.n_row_blocks * p.n_seg;
    p.ticket_bytes = ((size_t)L.n_row_blocks * sizeof(int32_t) + 255) / 256 * 256;
    p.partial_bytes = p.n_seg > 1 ? (size_t)L.n_row_blocks * p.n_seg * p.np * kRows * sizeof(float) : 0;
    return p;
}

GemvPlan plan_gemv(const Layout& L, int N) {
    const int np = padded_tokens(N);
    // with four or eight tokens a tile takes about twice as long: shorter segments, more workgroups (measured)
    return plan_segments(L, np, np >= 4 ? kGemvManyTokensSegmentTiles : kGemvSegmentTiles);
}

// Segments of the kernel that builds its own tables (measured on the 7B and 3.8B layer sets): a K that one
// workgroup can take whole - up to 32 tiles and about 80 KB of packed weights per row block - is one segment,
// which spares the exchange of partial sums; a longer K is cut into segments of at most 24 tiles.
GemvPlan plan_gemv_x(const Layout& L) {
    int whole = 81920 / L.tile_bytes;
    if (whole > kGemvXSegmentTiles) whole = kGemvXSegmentTiles;
    return plan_segments(L, 1, L.n_ktiles <= whole ? whole : kGemvXLongSegmentTiles);
}

static void fill_desc_plan(GemvDesc& d, const Layout& L, const GemvPlan& p, const void* packed, const void* lut, int N,
                           void* y, void* workspace, int wg_begin) {
    d.tiles = static_cast<const uint8_t*>(packed) + kHeaderBytes;
    d.lut_t = static_cast<const uint8_t*>(lut);
    d.lut_s = d.lut_t + (size_t)L.n_ktiles * kTableBytesPerKTile * p.np;
    d.y = y;
    d.tickets = static_cast<int32_t*>(workspace);
    d.partial = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + p.ticket_bytes);
    d.M = L.M;
    d.N = N;
    d.n_row_blocks = L.n_row_blocks;
    d.n_ktiles = L.n_ktiles;
    d.wg_begin = wg_begin;
    d.n_seg = p.n_seg;
    d.seg_tiles = p.seg_tiles;
    d.K = L.K;
}

void fill_desc(GemvDesc& d, const Layout& L, const void* packed, const void* lut, int N, void* y, void* workspace,
               int wg_begin) {
    fill_desc_plan(d, L, plan_gemv(L, N), packed, lut, N, y, workspace, wg_begin);
}

void fill_desc_x(GemvDesc& d, const Layout& L, const void* packed, const void* x, void* y, void* workspace) {
    fill_desc_plan(d, L, plan_gemv_x(L), packed, x, 1, y, workspace, 0);
    d.lut_s = nullptr;
}

// ---------------------------------------------------------------------------------------------
// device side

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

// kernel arguments: the descriptor itself for a single GEMV, the device table for a batch
template <bool SINGLE>
struct KernelArgs;
template <>
struct KernelArgs<true> {
    GemvDesc single;
    int n_gemv;  // 1
};
template <>
struct KernelArgs<false> {
    const GemvDesc* descs;
    int n_gemv;
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

// A table entry as it comes out of LDS: NP fp16 values (the NP tokens of one pattern).
template <int NP> struct EntryT;
template <> struct EntryT<1> { typedef _Float16 type; };
template <> struct EntryT<2> { typedef half2_t type; };
template <> struct EntryT<4> { typedef half4_t type; };
template <> struct EntryT<8> { typedef half8_t type; };

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

template <int NP>
struct Accum {
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
    __device__ __forceinline__ void add(const typename EntryT<NP>::type& e, const PlaneWeights<B, NP>& w, int plane) {
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

// Lookups of one tile block for the lane's row.  `lds` is the LDS address of the wave's private slot;
// the callers make it a link-time constant (one copy of the code per wave of the workgroup), so it
// folds, together with the table's offset, into the immediate offset of the LDS load and the address
// register is just the index byte.  The 4*B plane words of the tile are handled
// one after the other, software pipelined: the eight lookups of word w+1 are issued before the eight
// results of word w are accumulated, so LDS latency overlaps the arithmetic with few live registers.
template <int B, int NP, int GQ, bool HZ>
__device__ __forceinline__ void consume_tile(const Stage<B, NP, GemvCfg<B, NP, GQ, HZ>::MPL>& s, uint32_t lds, int lane,
                                             const PlaneWeights<B, NP>& pw, float (&y)[NP]) {
    using Cfg = GemvCfg<B, NP, GQ, HZ>;
    typedef typename EntryT<NP>::type entry_t;
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
    Accum<NP> a;
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
            if constexpr (HZ) {
                const float z = half_bits_to_float(mw >> 16);  // 4-byte entry: scale low, zero high
#pragma unroll
                for (int n = 0; n < NP; ++n) y[n] = fmaf(sc, fmaf(-z, load_lds<float>(sg + n * 4), a.get(n)), y[n]);
            } else {
#pragma unroll
                for (int n = 0; n < NP; ++n) y[n] = fmaf(sc, fmaf(2.f, a.get(n), -load_lds<float>(sg + n * 4)), y[n]);
            }
        }
        // keep the pipeline order, which bounds the live registers: the first stops the compiler from
        // collecting the lookups of later words up front, the second the instruction scheduler
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
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
// row.  With one segment they are the result; otherwise the segments meet through memory (see above).
template <int NP>
__device__ __forceinline__ void finish_rows(const GemvDesc& d, int rb, int seg, int n_seg, int lane, float (&y)[NP]) {
    const int m = rb * kRows + lane;
    const int M = d.M, N = d.N;
    _Float16* out = static_cast<_Float16*>(d.y);
    if (n_seg == 1) {
        if (m < M) {
#pragma unroll
            for (int n = 0; n < NP; ++n)
                if (n < N) out[(size_t)n * M + m] = (_Float16)y[n];
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
            if (n < N) out[(size_t)n * M + m] = (_Float16)acc[n];
    }
    if (lane == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int B, int NP, int GQ, bool HZ, bool SINGLE>
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
                    consume_tile<B, NP, GQ, HZ>(st[s], lds, lane, pw, y);
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

    finish_rows<NP>(d, rb, seg, n_seg, lane, y);
}

// ---------------------------------------------------------------------------------------------
// One token, tables built in the kernel.
//
// With a single token the tables of a whole K segment (at most 32 tiles = 1024 tables = 32 KB) fit in LDS
// next to three or more other workgroups.  The workgroup builds them itself from the activations of its
// segment (at most 8 KB) while its first weight tiles are on their way, so a decode step needs no launch for
// the table precompute, no table traffic between the two kernels, and no per-tile copy of a table
// slice into LDS.  The entries have the values build_lut_kernel computes (fp32 sums in ascending order,
// one rounding to fp16), as have the group sums (same tree of additions).
//
// A lookup address is tile base | index byte: one v_perm_b32 takes byte k of the prepared index word as
// byte 0 and bytes 1..3 of the tile's table base (a multiple of 1024), the table's place inside the
// tile is the immediate offset of the LDS load.  One instruction per lookup, as in the kernel above.

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

template <int B, int GQ, bool HZ, bool SINGLE>
__global__ void __launch_bounds__(kWaves * 64) mpgemv_x_kernel(KernelArgs<SINGLE> a) {
    using Cfg = GemvCfg<B, 1, GQ, HZ>;
    constexpr int D = Cfg::D;
    constexpr int TPG = GQ / kLutGroup;  // tables per quantization group: 8, 16 or 32 consecutive lanes
    // LDS of a workgroup: the tables of its segment, their group sums, the four partial sums of each row.  The
    // launch sizes it for the longest segment among its GEMVs, so short segments leave room for more workgroups.
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds_x[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    float pw[B];
#pragma unroll
    for (int i = 0; i < B; ++i) pw[i] = opaque((float)(1 << i));

    const int g = SINGLE ? 0 : (int)blockIdx.y;
    const GemvDesc& d = desc_of<SINGLE>(a, g);
    const int n_seg = uniform(d.n_seg), n_ktiles = uniform(d.n_ktiles);
    const int wg_local = (int)blockIdx.x;
    if (wg_local >= uniform(d.n_row_blocks) * n_seg) return;
    // (the division runs on the vector unit: bring its results back to scalar registers, or every buffer
    // resource derived from them is taken for lane dependent)
    const int rb = uniform(wg_local / n_seg), seg = uniform(wg_local % n_seg);
    const int seg_tiles = uniform(d.seg_tiles);
    const int k0 = seg * seg_tiles;
    const int k1 = min(k0 + seg_tiles, n_ktiles);
    const int per_wave = (k1 - k0 + kWaves - 1) / kWaves;
    const int t0 = min(k0 + wave * per_wave, k1);
    const int t1 = min(t0 + per_wave, k1);
    Streams src;
    src.w = uniform(d.tiles) + (size_t)rb * n_ktiles * Cfg::TB;
    src.t = src.s = nullptr;
    src.w_bytes = (uint32_t)(n_ktiles * Cfg::TB);
    src.t_bytes = src.s_bytes = 0;

    const uint32_t lt = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr<uint8_t>)lds_x));
    const uint32_t ls = lt + (uint32_t)seg_tiles * kTableBytesPerKTile;  // group sums follow the tables
    const uint32_t lr = ls + (uint32_t)seg_tiles * Cfg::GPT * 4;         // then the partial sums [wave][row]

    // first weight tiles on their way before anything else
    Stage<B, 1, Cfg::MPL> st[D] = {};
#pragma unroll
    for (int s = 0; s < D; ++s) issue_weights<B, 1, GQ, HZ>(st[s], src, t0 + s < t1, t0 + s, lane);

    // tables and group sums of the segment: thread -> tables tid, tid + 256, ... (x beyond K reads as zero).
    // The range check of a buffer load covers the per-lane offset only, not the scalar offset, so the resource
    // starts at the segment's first activation and ends with x: K * 2 bytes less the segment's start.
    {
        const uint32_t x_start = (uint32_t)(k0 * kKTile * 2);  // k0 < n_ktiles, so this lies inside x
        const rsrc_t rx = make_rsrc(uniform(d.lut_t) + x_start, (uint32_t)uniform(d.K) * 2u - x_start);
        const int n_tab = (k1 - k0) * kTablesPerKTile;
        constexpr int kPasses = kGemvXSegmentTiles * kTablesPerKTile / (kWaves * 64);
        static_assert(kPasses * kWaves * 64 == kGemvXSegmentTiles * kTablesPerKTile, "whole passes");
        u32x2 xv[kPasses];  // all requests first (a pass beyond the segment reads activations nobody uses)
#pragma unroll
        for (int i = 0; i < kPasses; ++i)
            xv[i] = __builtin_amdgcn_raw_buffer_load_b64(rx, (i * kWaves * 64 + tid) * 8, 0, 0);
#pragma unroll
        for (int i = 0; i < kPasses; ++i) {
            if (i * kWaves * 64 >= n_tab) break;
            const int j = i * kWaves * 64 + tid;
            // (copy the elements out first: a bit cast applied directly to a vector element reads element 0)
            const uint32_t w01 = xv[i].x, w23 = xv[i].y;
            const half2_t x01 = __builtin_bit_cast(half2_t, w01), x23 = __builtin_bit_cast(half2_t, w23);
            const float v[4] = {(float)x01[0], (float)x01[1], (float)x23[0], (float)x23[1]};
            // entry p = sum of the v[t] with bit t of p set, added in ascending t
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
            if (j < n_tab) {
                store_lds<u32x4>(lt + j * 32, __builtin_bit_cast(u32x4, lo));
                store_lds<u32x4>(lt + j * 32 + 16, __builtin_bit_cast(u32x4, hi));
                if (j % TPG == 0) store_lds<float>(ls + (j / TPG) * 4, gs);
            }
        }
    }
    __syncthreads();

    uint32_t sel[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) sel[k] = 0x03020100u | (uint32_t)(4 + k);
    float y = 0.f;
    for (int base = t0; base < t1; base += D) {
#pragma unroll
        for (int s = 0; s < D; ++s) {
            const int t = base + s;
            if (t < t1) {
                {
                    const int rem = t1 - t;
                    if (rem >= 7) __builtin_amdgcn_s_setprio(3);
                    else if (rem >= 5) __builtin_amdgcn_s_setprio(2);
                    else if (rem >= 3) __builtin_amdgcn_s_setprio(1);
                    else __builtin_amdgcn_s_setprio(0);
                }
                consume_weights<B, GQ, HZ>(st[s], lt + (t - k0) * kTableBytesPerKTile, ls + (t - k0) * Cfg::GPT * 4, sel, pw, y);
                issue_weights<B, 1, GQ, HZ>(st[s], src, t + D < t1, t + D, lane);
            }
        }
    }

    store_lds<float>(lr + (wave * kRows + lane) * 4, y);
    __syncthreads();
    if (wave != 0) return;
    y = ((load_lds<float>(lr + lane * 4) + load_lds<float>(lr + (kRows + lane) * 4)) +
         load_lds<float>(lr + (2 * kRows + lane) * 4)) + load_lds<float>(lr + (3 * kRows + lane) * 4);
    float yy[1] = {y};
    finish_rows<1>(d, rb, seg, n_seg, lane, yy);
}

// ---------------------------------------------------------------------------------------------
// launch

template <int B, int NP, int GQ, bool HZ, bool SINGLE>
static int launch_cfg(const KernelArgs<SINGLE>& a, int n_workgroups, hipStream_t st) {
    hipLaunchKernelGGL((mpgemv_kernel<B, NP, GQ, HZ, SINGLE>), dim3((unsigned)n_workgroups, (unsigned)a.n_gemv), dim3(kWaves * 64),
                       0, st, a);
    return launch_status();
}

template <int B, int NP, bool HZ, bool SINGLE>
static int launch_group(int group, const KernelArgs<SINGLE>& a, int n_wg, hipStream_t st) {
    switch (group) {
        case 32: return launch_cfg<B, NP, 32, HZ, SINGLE>(a, n_wg, st);
        case 64: return launch_cfg<B, NP, 64, HZ, SINGLE>(a, n_wg, st);
        default: return launch_cfg<B, NP, 128, HZ, SINGLE>(a, n_wg, st);
    }
}

template <int B, bool HZ, bool SINGLE>
static int launch_tokens(int np, int group, const KernelArgs<SINGLE>& a, int n_wg, hipStream_t st) {
    switch (np) {
        case 1: return launch_group<B, 1, HZ, SINGLE>(group, a, n_wg, st);
        case 2: return launch_group<B, 2, HZ, SINGLE>(group, a, n_wg, st);
        case 4: return launch_group<B, 4, HZ, SINGLE>(group, a, n_wg, st);
        default: return launch_group<B, 8, HZ, SINGLE>(group, a, n_wg, st);
    }
}

template <bool SINGLE>
static int launch_format(int bits, int has_zero, int np, int group, const KernelArgs<SINGLE>& a, int n_wg,
                         hipStream_t st) {
    if (bits == 1) {
        return has_zero ? launch_tokens<1, true, SINGLE>(np, group, a, n_wg, st)
                        : launch_tokens<1, false, SINGLE>(np, group, a, n_wg, st);
    }
    if (bits == 2) return launch_tokens<2, true, SINGLE>(np, group, a, n_wg, st);
    return launch_tokens<4, true, SINGLE>(np, group, a, n_wg, st);
}

int launch_mpgemv(const Layout& L, const void* packed, const void* lut, int N, void* y, void* workspace,
                  hipStream_t st) {
    KernelArgs<true> a;
    fill_desc(a.single, L, packed, lut, N, y, workspace, 0);
    a.n_gemv = 1;
    return launch_format<true>(L.bits, L.has_zero, padded_tokens(N), L.group, a, plan_gemv(L, N).n_workgroups, st);
}

int launch_mpgemv_batch(int bits, int group, int has_zero, int N, const GemvDesc* descs_dev, int n_gemv,
                        int max_workgroups, hipStream_t st) {
    KernelArgs<false> a;
    a.descs = descs_dev;
    a.n_gemv = n_gemv;
    return launch_format<false>(bits, has_zero, padded_tokens(N), group, a, max_workgroups, st);
}

// LDS of a workgroup whose segment has `seg_tiles` tiles: tables, group sums (at most 4 per tile), partial sums
static unsigned x_lds_bytes(int seg_tiles) {
    return (unsigned)seg_tiles * (kTableBytesPerKTile + 4 * 4) + kWaves * kRows * 4;
}

template <int B, bool HZ, bool SINGLE>
static int launch_x_group(int group, const KernelArgs<SINGLE>& a, int n_wg, int max_seg_tiles, hipStream_t st) {
    const dim3 grid((unsigned)n_wg, (unsigned)a.n_gemv), block(kWaves * 64);
    const unsigned lds = x_lds_bytes(max_seg_tiles);
    switch (group) {
        case 32: hipLaunchKernelGGL((mpgemv_x_kernel<B, 32, HZ, SINGLE>), grid, block, lds, st, a); break;
        case 64: hipLaunchKernelGGL((mpgemv_x_kernel<B, 64, HZ, SINGLE>), grid, block, lds, st, a); break;
        default: hipLaunchKernelGGL((mpgemv_x_kernel<B, 128, HZ, SINGLE>), grid, block, lds, st, a); break;
    }
    return launch_status();
}

template <bool SINGLE>
static int launch_x_format(int bits, int has_zero, int group, const KernelArgs<SINGLE>& a, int n_wg, int max_seg_tiles,
                           hipStream_t st) {
    if (bits == 1) {
        return has_zero ? launch_x_group<1, true, SINGLE>(group, a, n_wg, max_seg_tiles, st)
                        : launch_x_group<1, false, SINGLE>(group, a, n_wg, max_seg_tiles, st);
    }
    if (bits == 2) return launch_x_group<2, true, SINGLE>(group, a, n_wg, max_seg_tiles, st);
    return launch_x_group<4, true, SINGLE>(group, a, n_wg, max_seg_tiles, st);
}

int launch_mpgemv_x(const Layout& L, const void* packed, const void* x, void* y, void* workspace, hipStream_t st) {
    KernelArgs<true> a;
    fill_desc_x(a.single, L, packed, x, y, workspace);
    a.n_gemv = 1;
    const GemvPlan p = plan_gemv_x(L);
    return launch_x_format<true>(L.bits, L.has_zero, L.group, a, p.n_workgroups, p.seg_tiles, st);
}

int launch_mpgemv_x_batch(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv, int max_workgroups,
                          int max_seg_tiles, hipStream_t st) {
    KernelArgs<false> a;
    a.descs = descs_dev;
    a.n_gemv = n_gemv;
    return launch_x_format<false>(bits, has_zero, group, a, max_workgroups, max_seg_tiles, st);
}

// copies up to 16 descriptors per launch from the kernel arguments into the device table
struct DescChunk {
    GemvDesc d[16];
};
__global__ void write_descs_kernel(DescChunk c, int count, GemvDesc* __restrict__ out) {
    if ((int)threadIdx.x < count) out[threadIdx.x] = c.d[threadIdx.x];
}

int launch_write_descs(const GemvDesc* host, int count, GemvDesc* dev, hipStream_t st) {
    for (int i = 0; i < count; i += 16) {
        DescChunk c;
        int n = count - i < 16 ? count - i : 16;
        for (int j = 0; j < 16; ++j) c.d[j] = host[i + (j < n ? j : 0)];
        hipLaunchKernelGGL(write_descs_kernel, dim3(1), dim3(64), 0, st, c, n, dev + i);
    }
    return launch_status();
}

}  // namespace tman
