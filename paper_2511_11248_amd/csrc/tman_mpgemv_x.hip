// Decoding mpGEMV of ONE token with the table precompute inside the lookup kernel (Sec. 2.2 "Bit-serial table
// lookup" and Sec. 4.3 for the lookups; Sec. 5 makes the precompute a kernel of its own because it is costly on
// the paper's hardware, whereas here a kernel boundary costs more than the precompute).
//
// With a single token the tables of a whole K segment (at most 32 tiles = 1024 tables = 32 KB) fit in LDS
// next to three or more other workgroups.  The workgroup builds them itself from the activations of its
// segment (at most 8 KB) while its first weight tiles are on their way, so a decode step needs no launch for the
// table precompute, no table traffic between the two kernels, and no per-tile copy of a table
// slice into LDS.  The entries have the values build_lut_kernel computes (fp32 sums in ascending order,
// one rounding to fp16), as have the group sums (same tree of additions).
//
// A lookup address is tile base | index byte: one v_perm_b32 takes byte k of the prepared index word as
// byte 0 and bytes 1..3 of the tile's table base (a multiple of 1024), the table's place inside the
// tile is the immediate offset of the LDS load.  One vector instruction and one LDS read per lookup.
//
// Scheduling is that of mpgemv_kernel: a workgroup of four waves owns one row block and one K segment, the four
// quarters meet in LDS, segments of a long K meet through the workspace (tickets, fixed order of addition).
#include <algorithm>
#include <vector>

#include "tman_gemv_device.h"

namespace tman {

// Segments of the kernel that builds its own tables (measured on the 7B and 3.8B layer sets): a K that one
// workgroup can take whole - up to 32 tiles and about 80 KB of packed weights per row block - is one segment,
// which spares the exchange of partial sums; a longer K is cut into segments of at most 24 tiles.
// LDS of a workgroup whose segment has `seg_tiles` tiles: tables, group sums (at most 4 per tile), partial sums
static unsigned x_lds_bytes(int seg_tiles) {
    return (unsigned)seg_tiles * (kTableBytesPerKTile + 4 * 4) + kWaves * kRows * 4;
}

GemvPlan plan_gemv_x(const Layout& L) {
    const tman_tiling_t t = current_tiling();
    int whole = t.decode_x_whole_bytes / L.tile_bytes;
    if (whole > t.decode_x_seg_tiles) whole = t.decode_x_seg_tiles;
    if (whole < 1) whole = 1;
    return plan_segments(L, 1, L.n_ktiles <= whole ? whole : t.decode_x_long_seg_tiles);
}

void fill_desc_x(GemvDesc& d, const Layout& L, const void* packed, const void* x, void* y, void* workspace) {
    fill_desc_plan(d, L, plan_gemv_x(L), packed, x, 1, y, workspace, 0);
    d.lut_s = nullptr;
}

template <int B, int GQ, bool HZ, bool SINGLE, typename Args>
__global__ void __launch_bounds__(kWaves * 64) mpgemv_x_kernel(Args a) {
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

    int g, wg_local;
    workgroup_of<SINGLE>(a, g, wg_local);
    const GemvDesc& d = desc_of<SINGLE>(a, g);
    const int n_seg = uniform(d.n_seg), n_ktiles = uniform(d.n_ktiles);
    // Exits: surplus workgroups of the grid, and (single call) a blob packed for another shape or layout, which is
    // reported and leaves y alone; a batch is checked when its descriptor table is written, which empties the
    // descriptor of such a GEMV.  One exit for both, before any other memory request.
    int n_wg = uniform(d.n_row_blocks) * n_seg;
    if constexpr (SINGLE) {
        if (!header_matches(uniform(d.tiles), uniform(d.M), uniform(d.K), B, GQ, HZ ? 1 : 0)) {
            if (wg_local == 0 && tid == 0) report_header_mismatch(a.status);
            n_wg = 0;
        }
    }
    if (wg_local >= n_wg) return;
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

    // The activations are requested first and the first weight tiles right behind them: a wave's loads return in
    // the order they were issued, so activations queued behind weight tiles (which come from HBM) would hold the
    // tables back until those tiles are in; this way the tables are built while the weights travel.
    const uint32_t x_start = (uint32_t)(k0 * kKTile * 2);  // k0 < n_ktiles, so this lies inside x
    // (the range check of a buffer load covers the per-lane offset only, not the scalar offset, so the resource
    // starts at the segment's first activation and ends with x: K * 2 bytes less the segment's start)
    const rsrc_t rx = make_rsrc(uniform(d.lut_t) + x_start, (uint32_t)uniform(d.K) * 2u - x_start);
    constexpr int kPasses = kGemvXSegmentTiles * kTablesPerKTile / (kWaves * 64);
    static_assert(kPasses * kWaves * 64 == kGemvXSegmentTiles * kTablesPerKTile, "whole passes");
    u32x2 xv[kPasses];  // (a pass beyond the segment reads activations nobody uses; x beyond K reads as zero)
#pragma unroll
    for (int i = 0; i < kPasses; ++i)
        xv[i] = __builtin_amdgcn_raw_buffer_load_b64(rx, (i * kWaves * 64 + tid) * 8, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    Stage<B, 1, Cfg::MPL> st[D] = {};
#pragma unroll
    for (int s = 0; s < D; ++s) issue_weights<B, 1, GQ, HZ>(st[s], src, t0 + s < t1, t0 + s, lane);
    __builtin_amdgcn_sched_barrier(0);

    // tables and group sums of the segment: thread -> tables tid, tid + 256, ...
    {
        const int n_tab = (k1 - k0) * kTablesPerKTile;
#pragma unroll
        for (int i = 0; i < kPasses; ++i) {
            if (i * kWaves * 64 >= n_tab) break;
            const int j = i * kWaves * 64 + tid;
            store_table<TPG>(xv[i], j, j < n_tab, lt, ls);
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
    y = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) y += load_lds<float>(lr + (w * kRows + lane) * 4);
    float yy[1] = {y};
    const float one[1] = {1.f};
    finish_rows<1>(d, rb, seg, n_seg, lane, yy, one);
}

// ---------------------------------------------------------------------------------------------
// launch

template <int B, bool HZ, bool SINGLE, typename Args>
static int launch_x_group(int group, const Args& a, int n_wg, int max_seg_tiles, hipStream_t st) {
    const dim3 grid((unsigned)n_wg, __is_same(Args, OrderedArgs) ? 1u : (unsigned)a.n_gemv), block(kWaves * 64);
    const unsigned lds = x_lds_bytes(max_seg_tiles);
    switch (group) {
        case 32: hipLaunchKernelGGL((mpgemv_x_kernel<B, 32, HZ, SINGLE, Args>), grid, block, lds, st, a); break;
        case 64: hipLaunchKernelGGL((mpgemv_x_kernel<B, 64, HZ, SINGLE, Args>), grid, block, lds, st, a); break;
        default: hipLaunchKernelGGL((mpgemv_x_kernel<B, 128, HZ, SINGLE, Args>), grid, block, lds, st, a); break;
    }
    return launch_status();
}

template <bool SINGLE, typename Args>
static int launch_x_format(int bits, int has_zero, int group, const Args& a, int n_wg, int max_seg_tiles,
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
    a.status = device_status_word();
    if (!a.status) return TMAN_ERR_LAUNCH;
    const GemvPlan p = plan_gemv_x(L);
    return launch_x_format<true>(L.bits, L.has_zero, L.group, a, p.n_workgroups, p.seg_tiles, st);
}

// The numbered launch of a one-token batch (see order_workgroups_of): at most 8 workgroups of four waves are resident
// per compute unit, fewer when the tables of the longest segment take more LDS.
static int x_resident_per_unit(int count, const Layout* L) {
    int max_seg_tiles = 1;
    for (int g = 0; g < count; ++g) max_seg_tiles = std::max(max_seg_tiles, plan_gemv_x(L[g]).seg_tiles);
    return std::min(8, (int)(160u * 1024u / x_lds_bytes(max_seg_tiles)));
}
int ordered_workgroups(int count, const Layout* L, int n_units) {
    if (count > 8) return 0;
    std::vector<GemvPlan> plans(count);
    for (int g = 0; g < count; ++g) plans[g] = plan_gemv_x(L[g]);
    return ordered_workgroups_of(count, L, plans.data(), n_units, x_resident_per_unit(count, L));
}
bool order_workgroups(int count, const Layout* L, int n_units, std::vector<uint16_t>* order) {
    if (count > 8) return false;
    std::vector<GemvPlan> plans(count);
    for (int g = 0; g < count; ++g) plans[g] = plan_gemv_x(L[g]);
    return order_workgroups_of(count, L, plans.data(), n_units, x_resident_per_unit(count, L), order);
}

int launch_mpgemv_x_ordered(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv,
                            const uint16_t* order_dev, int n_wg, int max_seg_tiles, hipStream_t st) {
    OrderedArgs a;
    a.descs = descs_dev;
    a.order = order_dev;
    a.n_gemv = n_gemv;
    return launch_x_format<false>(bits, has_zero, group, a, n_wg, max_seg_tiles, st);
}

int launch_mpgemv_x_batch(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv, int max_workgroups,
                          int max_seg_tiles, hipStream_t st) {
    KernelArgs<false> a;
    a.descs = descs_dev;
    a.n_gemv = n_gemv;
    return launch_x_format<false>(bits, has_zero, group, a, max_workgroups, max_seg_tiles, st);
}

}  // namespace tman
