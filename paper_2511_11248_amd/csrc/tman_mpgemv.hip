// Decoding mpGEMV through bit-serial table lookup (Sec. 2.2 "Bit-serial table lookup", Sec. 4.3
// "Mapping of LUT-based Decoding").
//
//   y[n][m] = sum_G scale[m][G] * ( sum_i 2^i sum_{j in G} T[n][j][idx_i[m][j]] - zero[m][G] * S[n][G] )
//
// Mapping onto a CDNA4 compute unit.  Like the paper's vector-core mapping the lookups are vectorised
// along the output rows: the 32 lanes of a half wave hold 32 different rows and index the SAME
// 16-entry table, so the table (32 bytes, 8 LDS banks) is read by broadcast without bank conflicts
// and every lane keeps a private accumulator for its row -- no cross-lane traffic in the loop.  The
// two half waves cover the two 128-column halves of a 256-column K tile; one cross-half add at the
// end joins them.  The paper's two-level tiling appears as: inner tile = one quantization block
// (sums of table entries in fp32, then one scale/zero application), outer tile = the K slice whose
// tables sit in LDS.
//
// A workgroup of four waves owns four row blocks and one slice of K tiles: it copies the slice of the
// precomputed tables into LDS once, then each wave streams the tile blocks of its row block with
// 16-byte coalesced loads (next tile in flight while the current one is consumed).  When K is
// split over several workgroups the fp32 partial sums go through the workspace and the last
// workgroup to arrive adds them in slice order, so results do not depend on timing.
#include <hip/hip_fp16.h>

#include "tman_internal.h"

namespace tman {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

constexpr int kGemvLdsBudget = 64 * 1024;
constexpr int kGemvTargetWorkgroups = 1024;

GemvPlan plan_gemv(const Layout& L, int N) {
    GemvPlan p;
    p.np = padded_tokens(N);
    int per_ktile = kTableBytesPerKTile * p.np + (kKTile / L.group) * p.np * (int)sizeof(float);
    int max_kts = kGemvLdsBudget / per_ktile;
    p.n_row_groups = (L.n_row_blocks + 3) / 4;
    int want = (kGemvTargetWorkgroups + p.n_row_groups - 1) / p.n_row_groups;
    if (want < 1) want = 1;
    if (want > L.n_ktiles) want = L.n_ktiles;
    int kts = (L.n_ktiles + want - 1) / want;
    if (kts > max_kts) kts = max_kts;
    if (kts < 1) kts = 1;
    p.ktiles_per_slice = kts;
    p.n_slices = (L.n_ktiles + kts - 1) / kts;
    p.lds_bytes = (size_t)kts * per_ktile;
    p.ticket_bytes = ((size_t)p.n_row_groups * sizeof(int32_t) + 255) / 256 * 256;
    p.partial_bytes = p.n_slices > 1 ? (size_t)p.n_slices * p.np * L.n_row_blocks * kRows * sizeof(float) : 0;
    return p;
}

struct GemvArgs {
    const uint8_t* tiles;  // first tile block (past the header)
    const uint8_t* lut_t;  // fp16 tables
    const uint8_t* lut_s;  // fp32 group sums
    _Float16* y;
    int32_t* tickets;
    float* partial;
    int M, N, n_row_blocks, n_ktiles, ktiles_per_slice, n_slices;
};

template <int B, int NP, int GQ, bool HZ>
struct GemvCfg {
    static constexpr int CH = kHalf / B;  // weights per 16-byte chunk
    static constexpr int GPH = kHalf / GQ;  // quantization groups per lane and K tile
    static constexpr int MSZ = HZ ? 4 : 2;
    static constexpr int MPL = GPH * MSZ;  // metadata bytes per lane and K tile
    static constexpr int TB = B * 1024 + 64 * MPL;
    static constexpr int T_BYTES = kTableBytesPerKTile * NP;
    static constexpr int S_BYTES = (kKTile / GQ) * NP * 4;
};

template <int B, int MPL>
struct TileRegs {
    uint4 c[B];
    uint32_t meta[(MPL + 3) / 4];
};

template <int B, int MPL>
__device__ __forceinline__ void load_tile(TileRegs<B, MPL>& t, const uint8_t* tile, int lane) {
#pragma unroll
    for (int v = 0; v < B; ++v) t.c[v] = *reinterpret_cast<const uint4*>(tile + v * 1024 + lane * 16);
    const uint8_t* mp = tile + B * 1024 + lane * MPL;
    if constexpr (MPL == 2) {
        t.meta[0] = *reinterpret_cast<const uint16_t*>(mp);
    } else if constexpr (MPL == 4) {
        t.meta[0] = *reinterpret_cast<const uint32_t*>(mp);
    } else if constexpr (MPL == 8) {
        uint2 v = *reinterpret_cast<const uint2*>(mp);
        t.meta[0] = v.x;
        t.meta[1] = v.y;
    } else {
        uint4 v = *reinterpret_cast<const uint4*>(mp);
        t.meta[0] = v.x;
        t.meta[1] = v.y;
        t.meta[2] = v.z;
        t.meta[3] = v.w;
    }
}

__device__ __forceinline__ uint32_t word_of(const uint4& v, int w) {
    return w == 0 ? v.x : w == 1 ? v.y : w == 2 ? v.z : v.w;
}

__device__ __forceinline__ float half_bits_to_float(uint32_t bits16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
}

// One tile block (32 rows x 256 columns) for the lane's row and half: look up, accumulate per
// quantization group, apply scale and zero.  `tl` points at this K tile's tables in LDS, `sl` at its
// group sums.
template <int B, int NP, int GQ, bool HZ>
__device__ __forceinline__ void consume_tile(const TileRegs<B, GemvCfg<B, NP, GQ, HZ>::MPL>& t,
                                             const uint8_t* tl, const float* sl, int h, float (&y)[NP]) {
    using Cfg = GemvCfg<B, NP, GQ, HZ>;
    const uint8_t* th = tl + h * (32 * 16 * NP * 2);  // tables of this half
#pragma unroll
    for (int gi = 0; gi < Cfg::GPH; ++gi) {
        float a[NP];
#pragma unroll
        for (int n = 0; n < NP; ++n) a[n] = 0.f;
#pragma unroll
        for (int kb = 0; kb < GQ / 32; ++kb) {
            const int kb32 = gi * (GQ / 32) + kb;  // 32-weight block inside the lane's 128 weights
            const int v = (kb32 * 32) / Cfg::CH;
            const int ksub = ((kb32 * 32) % Cfg::CH) / 32;
#pragma unroll
            for (int i = 0; i < B; ++i) {
                const uint32_t w = word_of(t.c[v], ksub * B + i);
                const uint8_t* tb = th + (kb32 * 8) * 16 * NP * 2;
                if constexpr (NP == 1) {
                    const _Float16 pw = (_Float16)(float)(1 << i);
                    const half2_t pw2 = {pw, pw};
#pragma unroll
                    for (int u = 0; u < 8; u += 2) {
                        const uint32_t i0 = (w >> (4 * u)) & 15u, i1 = (w >> (4 * u + 4)) & 15u;
                        half2_t e;
                        e.x = *reinterpret_cast<const _Float16*>(tb + (u * 16 + i0) * 2);
                        e.y = *reinterpret_cast<const _Float16*>(tb + ((u + 1) * 16 + i1) * 2);
                        a[0] = __builtin_amdgcn_fdot2(e, pw2, a[0], false);
                    }
                } else {
                    const float pw = (float)(1 << i);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const uint32_t idx = (w >> (4 * u)) & 15u;
                        const uint8_t* ep = tb + (u * 16 + idx) * NP * 2;
                        if constexpr (NP == 2) {
                            half2_t e = *reinterpret_cast<const half2_t*>(ep);
                            a[0] = fmaf(pw, (float)e.x, a[0]);
                            a[1] = fmaf(pw, (float)e.y, a[1]);
                        } else if constexpr (NP == 4) {
                            half4_t e = *reinterpret_cast<const half4_t*>(ep);
#pragma unroll
                            for (int n = 0; n < 4; ++n) a[n] = fmaf(pw, (float)e[n], a[n]);
                        } else {
                            half8_t e = *reinterpret_cast<const half8_t*>(ep);
#pragma unroll
                            for (int n = 0; n < 8; ++n) a[n] = fmaf(pw, (float)e[n], a[n]);
                        }
                    }
                }
            }
        }
        // scale and zero of this quantization block
        const int mo = gi * Cfg::MSZ;  // byte offset inside the lane's metadata
        const uint32_t mw = t.meta[mo / 4];
        const float s = half_bits_to_float((mo % 4) ? (mw >> 16) : (mw & 0xffffu));
        const float* sg = sl + (h * Cfg::GPH + gi) * NP;
        if constexpr (HZ) {
            const float z = half_bits_to_float(mw >> 16);  // entry is 4 bytes: scale low, zero high
#pragma unroll
            for (int n = 0; n < NP; ++n) y[n] = fmaf(s, fmaf(-z, sg[n], a[n]), y[n]);
        } else {
#pragma unroll
            for (int n = 0; n < NP; ++n) y[n] = fmaf(s, fmaf(2.f, a[n], -sg[n]), y[n]);
        }
    }
}

template <int B, int NP, int GQ, bool HZ>
__global__ void __launch_bounds__(256) mpgemv_kernel(GemvArgs a) {
    using Cfg = GemvCfg<B, NP, GQ, HZ>;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    __shared__ int s_last;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, h = lane >> 5;
    const int rbg = blockIdx.x / a.n_slices, ks = blockIdx.x % a.n_slices;
    const int kt0 = ks * a.ktiles_per_slice;
    const int kt1 = min(kt0 + a.ktiles_per_slice, a.n_ktiles);
    const int nkt = kt1 - kt0;
    const int rb = rbg * 4 + wave;
    const bool valid = rb < a.n_row_blocks;

    TileRegs<B, Cfg::MPL> cur, nxt;
    const uint8_t* tile = a.tiles + ((size_t)(valid ? rb : 0) * a.n_ktiles + kt0) * Cfg::TB;
    if (valid) load_tile<B, Cfg::MPL>(cur, tile, lane);  // weights in flight while the tables are staged

    {  // copy this slice of the tables and group sums into LDS
        const uint4* src = reinterpret_cast<const uint4*>(a.lut_t + (size_t)kt0 * Cfg::T_BYTES);
        uint4* dst = reinterpret_cast<uint4*>(smem);
        const int n16 = nkt * (Cfg::T_BYTES / 16);
        for (int i = threadIdx.x; i < n16; i += 256) dst[i] = src[i];
        const uint32_t* ssrc = reinterpret_cast<const uint32_t*>(a.lut_s + (size_t)kt0 * Cfg::S_BYTES);
        uint32_t* sdst = reinterpret_cast<uint32_t*>(smem + (size_t)a.ktiles_per_slice * Cfg::T_BYTES);
        const int n4 = nkt * (Cfg::S_BYTES / 4);
        for (int i = threadIdx.x; i < n4; i += 256) sdst[i] = ssrc[i];
    }
    __syncthreads();

    float y[NP];
#pragma unroll
    for (int n = 0; n < NP; ++n) y[n] = 0.f;

    if (valid) {
        const float* sbase = reinterpret_cast<const float*>(smem + (size_t)a.ktiles_per_slice * Cfg::T_BYTES);
        for (int t = 0; t < nkt; ++t) {
            if (t + 1 < nkt) load_tile<B, Cfg::MPL>(nxt, tile + (size_t)(t + 1) * Cfg::TB, lane);
            consume_tile<B, NP, GQ, HZ>(cur, smem + (size_t)t * Cfg::T_BYTES, sbase + t * (Cfg::S_BYTES / 4), h, y);
            cur = nxt;
        }
    }
    // join the two K halves of each row: lane r and lane r + 32 hold the same row
#pragma unroll
    for (int n = 0; n < NP; ++n) y[n] += __shfl_xor(y[n], 32, 64);

    const int m = rb * kRows + (lane & 31);
    const int m_pad = a.n_row_blocks * kRows;
    if (a.n_slices == 1) {
        if (valid && lane < 32 && m < a.M) {
#pragma unroll
            for (int n = 0; n < NP; ++n)
                if (n < a.N) a.y[(size_t)n * a.M + m] = (_Float16)y[n];
        }
        return;
    }

    // split K: publish this slice's partial sums, the last workgroup of the row group reduces them
    if (valid && lane < 32) {
#pragma unroll
        for (int n = 0; n < NP; ++n) a.partial[((size_t)ks * NP + n) * m_pad + m] = y[n];
    }
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        int prev = __hip_atomic_fetch_add(&a.tickets[rbg], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == a.n_slices - 1);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    if (threadIdx.x < 128) {
        const int mm = rbg * 128 + threadIdx.x;
        if (mm < a.M) {
            for (int n = 0; n < a.N; ++n) {
                float acc = 0.f;
                for (int s = 0; s < a.n_slices; ++s)
                    acc += __hip_atomic_load(&a.partial[((size_t)s * NP + n) * m_pad + mm], __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
                a.y[(size_t)n * a.M + mm] = (_Float16)acc;
            }
        }
    }
    if (threadIdx.x == 0) __hip_atomic_store(&a.tickets[rbg], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int B, int NP, int GQ, bool HZ>
static int launch_cfg(const GemvArgs& a, const GemvPlan& p, hipStream_t st) {
    dim3 grid((unsigned)(p.n_row_groups * p.n_slices));
    hipLaunchKernelGGL((mpgemv_kernel<B, NP, GQ, HZ>), grid, dim3(256), p.lds_bytes, st, a);
    return launch_status();
}

template <int B, int NP, bool HZ>
static int launch_group(int group, const GemvArgs& a, const GemvPlan& p, hipStream_t st) {
    switch (group) {
        case 32: return launch_cfg<B, NP, 32, HZ>(a, p, st);
        case 64: return launch_cfg<B, NP, 64, HZ>(a, p, st);
        default: return launch_cfg<B, NP, 128, HZ>(a, p, st);
    }
}

template <int B, bool HZ>
static int launch_tokens(int np, int group, const GemvArgs& a, const GemvPlan& p, hipStream_t st) {
    switch (np) {
        case 1: return launch_group<B, 1, HZ>(group, a, p, st);
        case 2: return launch_group<B, 2, HZ>(group, a, p, st);
        case 4: return launch_group<B, 4, HZ>(group, a, p, st);
        default: return launch_group<B, 8, HZ>(group, a, p, st);
    }
}

int launch_mpgemv(const Layout& L, const void* packed, const void* lut, int N, void* y, void* workspace,
                  hipStream_t st) {
    GemvPlan p = plan_gemv(L, N);
    GemvArgs a;
    a.tiles = static_cast<const uint8_t*>(packed) + kHeaderBytes;
    a.lut_t = static_cast<const uint8_t*>(lut);
    a.lut_s = a.lut_t + (size_t)L.n_ktiles * kTableBytesPerKTile * p.np;
    a.y = static_cast<_Float16*>(y);
    a.tickets = static_cast<int32_t*>(workspace);
    a.partial = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + p.ticket_bytes);
    a.M = L.M;
    a.N = N;
    a.n_row_blocks = L.n_row_blocks;
    a.n_ktiles = L.n_ktiles;
    a.ktiles_per_slice = p.ktiles_per_slice;
    a.n_slices = p.n_slices;
    if (L.bits == 1) {
        return L.has_zero ? launch_tokens<1, true>(p.np, L.group, a, p, st)
                          : launch_tokens<1, false>(p.np, L.group, a, p, st);
    }
    if (L.bits == 2) return launch_tokens<2, true>(p.np, L.group, a, p, st);
    return launch_tokens<4, true>(p.np, L.group, a, p, st);
}

}  // namespace tman
