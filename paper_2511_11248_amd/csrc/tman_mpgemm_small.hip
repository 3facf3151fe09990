// mpGEMM for a handful of tokens (2 .. 32): two-level table dequantization in registers feeding the matrix
// cores (Sec. 4.1 "Fused LUT-based dequantization", Sec. 4.2), organised like the decoding kernel because with
// so few tokens the product is bound by the weight stream, not by the matrix cores.
//
// Why not the lookup kernel for 4 or 8 tokens: a lookup then returns 8 or 16 bytes per lane and the vector
// lookups are bound by LDS bandwidth (16 bytes per lane and lookup), three to four times the time the weight
// stream needs.  Dequantizing a weight once and multiplying it with all tokens in one MFMA costs the same
// vector work for 2 tokens as for 32.
//
// Mapping.  The weights stay in the bit-serial layout the decoding kernel streams (lane = row of a 64-row
// tile block, 16-byte chunks of bit-plane words, group scales and zeros behind them): a wave requests whole
// tile blocks exactly as mpgemv_kernel does.  Per 32-column step it dequantizes the lane's 32 weights into
// four 16-byte pieces of 8 fp16 (level 1: bit-field transposition, level 2: the block's affine map as one
// FMA on a code placed in an fp16 mantissa).  v_mfma_f32_32x32x16_f16 wants, per operand, lane l to hold row
// l % 32 and the 8 columns of half l / 32; a lane holds ONE row and all columns, so two pieces (a, b) are
// exchanged between the wave's halves with v_permlane32_swap: one result has rows 0..31 with columns a | b,
// the other rows 32..63 with columns a | b -- two ready operands from four swaps.  The activations of the same
// 16 columns come straight from memory (L2): lane l reads 16 bytes of token l % 32 at column half l / 32;
// tokens beyond N and columns beyond K lie outside the buffer resource and read as zero.
// Accumulators: 64 rows x 32 tokens per wave in fp32.
//
// Scheduling is that of the decoding kernels: a workgroup of four waves owns a row block and a K segment, the
// four quarters meet in LDS, segments of a long K meet through the workspace (tickets, partial sums added in
// segment order, so results do not depend on timing).
#include <vector>

#include "tman_dequant_device.h"
#include "tman_gemv_device.h"

namespace tman {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));

constexpr int kSmallTokens = TMAN_MAX_SMALL_TOKENS;  // 32: the token extent of one MFMA
constexpr int kRedStride = kRows + 4;                  // floats per token in the LDS reduction buffer (bank spread)

GemvPlan plan_small(const Layout& L) {
    // a dequantized tile takes about as long as a looked-up tile of one token: the same segment lengths
    GemvPlan p = plan_segments(L, 1, current_tiling().small_seg_tiles);
    p.np = kSmallTokens;
    p.partial_bytes = p.n_seg > 1 ? (size_t)L.n_row_blocks * p.n_seg * kSmallTokens * kRows * sizeof(float) : 0;
    return p;
}

void fill_desc_small(GemvDesc& d, const Layout& L, const void* packed, const void* x, int N, void* y, void* workspace) {
    fill_desc_plan(d, L, plan_small(L), packed, x, N, y, workspace, 0);
    d.lut_s = nullptr;
}

template <int B, int GQ, bool HZ, bool SINGLE, typename Args>
__global__ void __launch_bounds__(kWaves * 64) mpgemm_small_kernel(Args a) {
    using Cfg = GemvCfg<B, 1, GQ, HZ>;
    constexpr int D = 2;  // weight tile blocks in flight per wave
    __shared__ __attribute__((aligned(16))) float red[kWaves][kSmallTokens][kRedStride];
    __shared__ int last_flag;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    int g, wg_local;
    workgroup_of<SINGLE>(a, g, wg_local);
    const GemvDesc& d = desc_of<SINGLE>(a, g);
    const int n_seg = uniform(d.n_seg), n_ktiles = uniform(d.n_ktiles);
    // Exits: surplus workgroups of the grid, and (single call) a blob packed for another shape or layout, which
    // is reported and leaves y alone (a batch is checked when its descriptor table is written).
    int n_wg = uniform(d.n_row_blocks) * n_seg;
    if constexpr (SINGLE) {
        if (!header_matches(uniform(d.tiles), uniform(d.M), uniform(d.K), B, GQ, HZ ? 1 : 0)) {
            if (wg_local == 0 && tid == 0) report_header_mismatch(a.status);
            n_wg = 0;
        }
    }
    if (wg_local >= n_wg) return;
    const int rb = uniform(wg_local / n_seg), seg = uniform(wg_local % n_seg);
    const int seg_tiles = uniform(d.seg_tiles);
    const int k0 = seg * seg_tiles;
    const int k1 = min(k0 + seg_tiles, n_ktiles);
    const int per_wave = (k1 - k0 + kWaves - 1) / kWaves;
    const int t0 = min(k0 + wave * per_wave, k1);  // this wave's K tiles [t0, t1)
    const int t1 = min(t0 + per_wave, k1);
    const int N = uniform(d.N), K = uniform(d.K), M = uniform(d.M);
    Streams src;
    src.w = uniform(d.tiles) + (size_t)rb * n_ktiles * Cfg::TB;
    src.t = src.s = nullptr;
    src.w_bytes = (uint32_t)(n_ktiles * Cfg::TB);
    src.t_bytes = src.s_bytes = 0;

    // Activations: lane l reads token l % 32, column half l / 32 of each 16-column step.  A token beyond N lies
    // past the end of the resource (N * K * 2 bytes); a column beyond K is sent there explicitly, because inside
    // the buffer it would be the next token's data.
    const rsrc_t rx = make_rsrc(uniform(d.lut_t), (uint32_t)N * (uint32_t)K * 2u);
    const uint32_t xlane = (uint32_t)(lane & 31) * (uint32_t)K * 2u + (uint32_t)(lane >> 5) * 16u;
    const int kcol_lane = (lane >> 5) * 8;
    constexpr uint32_t kOutside = 0xFFFFFFF0u;
    // The activations of a tile are requested in two halves of 64 columns, each half a tile ahead of its use.
    struct XHalf {
        u32x4 v[4];  // step s (16 columns) of the half
    };
    auto issue_x = [&](XHalf& xh, bool live, int kt, int half) {
        const rsrc_t r = live ? rx : make_rsrc(uniform(d.lut_t), 0u);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int c0 = kt * kKTile + half * 64 + s * 16;
            const uint32_t off = c0 + kcol_lane < K ? xlane + (uint32_t)c0 * 2u : kOutside;
            xh.v[s] = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
        }
    };

    float16_t acc[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[h][v] = 0.f;

    // One 32-column step: the lane's 32 weights of block kb32 of the tile, against steps 2 (kb32 % 2) and + 1
    // of the activation half.
    auto step32 = [&](const Stage<B, 1, Cfg::MPL>& cur, const XHalf& xh, int kb32) {
        WRegs<B> r;
        const int v = (kb32 * 32) / Cfg::CH, ksub = ((kb32 * 32) % Cfg::CH) / 32;
#pragma unroll
        for (int i = 0; i < B; ++i) r.plane[i] = word_of(cur.c[v], ksub * B + i);
        const int mo = ((kb32 * 32) / GQ) * Cfg::MSZ;
        const uint32_t mw = cur.meta[mo / 4];
        r.meta = HZ ? mw : ((mo % 4) ? (mw >> 16) : (mw & 0xffffu));
        Dequant<B, HZ> dq;
        dq.start(r);
        dq.insert();
#pragma unroll
        for (int pair = 0; pair < 2; ++pair) {
            const u32x4 pa = dq.piece(2 * pair), pb = dq.piece(2 * pair + 1);
            u32x4 lo, hi;  // operands of rows 0..31 and rows 32..63: columns pa | pb
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const u32x2v sw = __builtin_amdgcn_permlane32_swap(pa[e], pb[e], false, false);
                lo[e] = sw.x;
                hi[e] = sw.y;
            }
            const half8_t xo = __builtin_bit_cast(half8_t, xh.v[(kb32 & 1) * 2 + pair]);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, lo), xo, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, hi), xo, acc[1], 0, 0, 0);
        }
    };

    Stage<B, 1, Cfg::MPL> st[D] = {};
    XHalf xa, xb;
#pragma unroll
    for (int s = 0; s < D; ++s) issue_weights<B, 1, GQ, HZ>(st[s], src, t0 + s < t1, t0 + s, lane);
    issue_x(xa, t0 < t1, t0, 0);
    issue_x(xb, t0 < t1, t0, 1);
    for (int base = t0; base < t1; base += D) {
#pragma unroll
        for (int s = 0; s < D; ++s) {
            const int t = base + s;
            if (t < t1) {
                step32(st[s], xa, 0);
                step32(st[s], xa, 1);
                issue_x(xa, t + 1 < t1, t + 1, 0);
                step32(st[s], xb, 2);
                step32(st[s], xb, 3);
                issue_x(xb, t + 1 < t1, t + 1, 1);
                issue_weights<B, 1, GQ, HZ>(st[s], src, t + D < t1, t + D, lane);
            }
        }
    }

    // The four quarters of the segment meet in LDS.  acc[h][v] is row 32 h + 8 (v / 4) + 4 (lane / 32) + v % 4 of
    // the row block for token lane % 32: four consecutive rows per group of four registers.
    {
        const int token = lane & 31, hh = lane >> 5;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float* dst = &red[wave][token][32 * h + 8 * q + 4 * hh];
#pragma unroll
                for (int e = 0; e < 4; ++e) dst[e] = acc[h][4 * q + e];
            }
    }
    __syncthreads();
    // thread -> token tid / 8, rows 8 (tid % 8) .. + 7
    const int token = tid >> 3, r8 = (tid & 7) * 8;
    float sum[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
        sum[e] = ((red[0][token][r8 + e] + red[1][token][r8 + e]) + red[2][token][r8 + e]) + red[3][token][r8 + e];

    const int m0 = rb * kRows + r8;
    _Float16* out = static_cast<_Float16*>(uniform(d.y));
    auto store_rows = [&](const float (&v)[8]) {
        if (token >= N) return;
        _Float16* dst = out + (size_t)token * M + m0;
        if (m0 + 8 <= M && (M % 8) == 0) {
            half8_t h;
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = (_Float16)v[e];
            *reinterpret_cast<half8_t*>(dst) = h;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (m0 + e < M) dst[e] = (_Float16)v[e];
        }
    };
    if (n_seg == 1) {
        store_rows(sum);
        return;
    }

    // K longer than one segment: publish this segment's sums, take a ticket; the last one adds in segment order
    float* base_p = uniform(d.partial) + (size_t)rb * n_seg * kSmallTokens * kRows;
    float* mine = base_p + (size_t)seg * kSmallTokens * kRows + token * kRows + r8;
    if (token < N) {
#pragma unroll
        for (int e = 0; e < 8; ++e) __hip_atomic_store(mine + e, sum[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the sums have reached device-coherent memory
    __syncthreads();
    int32_t* ticket = uniform(d.tickets) + rb;
    if (tid == 0) last_flag = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_seg - 1;
    __syncthreads();
    if (!last_flag) return;
    float total[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) total[e] = 0.f;
    if (token < N) {
        for (int p = 0; p < n_seg; ++p) {
            const float* src_p = base_p + (size_t)p * kSmallTokens * kRows + token * kRows + r8;
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = __hip_atomic_load(src_p + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int e = 0; e < 8; ++e) total[e] += v[e];
        }
    }
    store_rows(total);
    if (tid == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------------------------------------
// launch

template <int B, bool HZ, bool SINGLE, typename Args>
static int launch_small_group(int group, const Args& a, int n_wg, hipStream_t st) {
    const dim3 grid((unsigned)n_wg, __is_same(Args, OrderedArgs) ? 1u : (unsigned)a.n_gemv), block(kWaves * 64);
    switch (group) {
        case 32: hipLaunchKernelGGL((mpgemm_small_kernel<B, 32, HZ, SINGLE, Args>), grid, block, 0, st, a); break;
        case 64: hipLaunchKernelGGL((mpgemm_small_kernel<B, 64, HZ, SINGLE, Args>), grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL((mpgemm_small_kernel<B, 128, HZ, SINGLE, Args>), grid, block, 0, st, a); break;
    }
    return launch_status();
}

template <bool SINGLE, typename Args>
static int launch_small_format(int bits, int has_zero, int group, const Args& a, int n_wg, hipStream_t st) {
    if (bits == 1) {
        return has_zero ? launch_small_group<1, true, SINGLE>(group, a, n_wg, st)
                        : launch_small_group<1, false, SINGLE>(group, a, n_wg, st);
    }
    if (bits == 2) return launch_small_group<2, true, SINGLE>(group, a, n_wg, st);
    return launch_small_group<4, true, SINGLE>(group, a, n_wg, st);
}

int launch_mpgemm_small(const Layout& L, const void* packed, const void* x, int N, void* y, void* workspace,
                        hipStream_t st) {
    KernelArgs<true> a;
    fill_desc_small(a.single, L, packed, x, N, y, workspace);
    a.n_gemv = 1;
    a.status = device_status_word();
    if (!a.status) return TMAN_ERR_LAUNCH;
    return launch_small_format<true>(L.bits, L.has_zero, L.group, a, plan_small(L).n_workgroups, st);
}

int launch_mpgemm_small_batch(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv, int max_workgroups,
                              hipStream_t st) {
    KernelArgs<false> a;
    a.descs = descs_dev;
    a.n_gemv = n_gemv;
    return launch_small_format<false>(bits, has_zero, group, a, max_workgroups, st);
}

// The numbered launch of a batch (see order_workgroups_of): the reduction buffer of a workgroup takes 34.8 KB of LDS,
// four workgroups are resident per compute unit.
constexpr int kSmallResident = (int)(160u * 1024u / (sizeof(float) * kWaves * kSmallTokens * kRedStride + 64));
int ordered_workgroups_small(int count, const Layout* L, int n_units) {
    if (count > 8) return 0;
    std::vector<GemvPlan> plans(count);
    for (int g = 0; g < count; ++g) plans[g] = plan_small(L[g]);
    return ordered_workgroups_of(count, L, plans.data(), n_units, kSmallResident);
}
bool order_workgroups_small(int count, const Layout* L, int n_units, std::vector<uint16_t>* order) {
    if (count > 8) return false;
    std::vector<GemvPlan> plans(count);
    for (int g = 0; g < count; ++g) plans[g] = plan_small(L[g]);
    return order_workgroups_of(count, L, plans.data(), n_units, kSmallResident, order);
}
int launch_mpgemm_small_ordered(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv,
                                const uint16_t* order_dev, int n_wg, hipStream_t st) {
    OrderedArgs a;
    a.descs = descs_dev;
    a.order = order_dev;
    a.n_gemv = n_gemv;
    return launch_small_format<false>(bits, has_zero, group, a, n_wg, st);
}

}  // namespace tman
