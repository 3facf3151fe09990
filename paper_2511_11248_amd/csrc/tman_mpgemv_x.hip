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

// A launch whose workgroups are numbered by the host: workgroup id -> (GEMV, workgroup within the GEMV).  When all
// workgroups of a launch are resident at once, this chip's dispatcher hands workgroup i to compute unit i mod 256
// (measured: ids 8, 264, 520, 776 share a unit), so the numbering decides which workgroups share a unit, and the
// host numbers them so that every unit gets the same amount of work (see order_workgroups).
struct OrderedArgs {
    const GemvDesc* descs;
    const uint16_t* order;  // per workgroup id: GEMV in bits 13..15, workgroup within the GEMV in bits 0..12
    int n_gemv;
};
template <bool SINGLE>
__device__ __forceinline__ const GemvDesc& desc_of(const OrderedArgs& a, int g) {
    return a.descs[g];
}

template <int B, int GQ, bool HZ, bool SINGLE, typename Args>
__global__ void __launch_bounds__(kWaves * 64) mpgemv_x_kernel(Args a) {
    constexpr bool ORDERED = __is_same(Args, OrderedArgs);
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

    int g = SINGLE ? 0 : (int)blockIdx.y, wg_local = (int)blockIdx.x;
    if constexpr (ORDERED) {
        const uint32_t e = uniform((int)a.order[blockIdx.x]);
        g = (int)(e >> 13);
        wg_local = (int)(e & 0x1fffu);
    }
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

// Numbers the workgroups of a batch so that, with workgroup i on compute unit i mod n_units, every unit gets the
// same work: the workgroups, largest first, go one by one to the unit with the least work so far that still has a
// free place (unit j has a place for ids j, j + n_units, ...), then the two extreme units exchange workgroups
// while that helps; inside a unit the largest gets the lowest id.  Work of a workgroup = tile blocks of its K
// segment + 2 (start and end of a workgroup cost about that).  Returns false when the batch does not qualify: more
// than 8 GEMVs, or more workgroups than are resident at once (LDS of the longest segment, 8 workgroups of four
// waves per unit at most), in which case the dispatcher no longer goes by position.
int ordered_workgroups(int count, const Layout* L, int n_units) {
    if (count > 8 || n_units < 1 || !current_tiling().decode_x_balance) return 0;
    int n = 0, max_seg_tiles = 0;
    for (int g = 0; g < count; ++g) {
        const GemvPlan p = plan_gemv_x(L[g]);
        if (p.n_workgroups > 0x1fff) return 0;
        n += p.n_workgroups;
        max_seg_tiles = std::max(max_seg_tiles, p.seg_tiles);
    }
    const int per_unit = std::min(8, (int)(160u * 1024u / x_lds_bytes(max_seg_tiles)));
    return n <= per_unit * n_units && n <= kOrderedMaxWorkgroups ? n : 0;
}

bool order_workgroups(int count, const Layout* L, int n_units, std::vector<uint16_t>* order) {
    const int n = ordered_workgroups(count, L, n_units);
    if (!n) return false;
    // unit j runs the ids j, j + n_units, ...
    auto places = [&](int j) { return n / n_units + (j < n % n_units ? 1 : 0); };
    struct Item {
        int cost;
        uint16_t id;
    };
    std::vector<Item> items;
    for (int g = 0; g < count; ++g) {
        const GemvPlan p = plan_gemv_x(L[g]);
        for (int w = 0; w < p.n_workgroups; ++w) {
            const int seg = w % p.n_seg;
            const int tiles = std::min(p.seg_tiles, L[g].n_ktiles - seg * p.seg_tiles);
            items.push_back(Item{tiles + 2, (uint16_t)((g << 13) | w)});
        }
    }
    std::stable_sort(items.begin(), items.end(), [](const Item& a, const Item& b) { return a.cost > b.cost; });
    std::vector<int> load(n_units, 0), used(n_units, 0);
    std::vector<std::vector<uint16_t>> mine(n_units);
    for (const Item& it : items) {
        int best = -1;
        for (int j = 0; j < n_units; ++j)
            if (used[j] < places(j) && (best < 0 || load[j] < load[best])) best = j;
        load[best] += it.cost;
        ++used[best];
        mine[best].push_back(it.id);
    }
    // Local improvement: the fullest unit exchanges a workgroup with another unit as long as that lowers the larger
    // of the two loads (the number of workgroups per unit is fixed by the position rule).
    auto cost_of = [&](uint16_t id) {
        for (const Item& it : items)
            if (it.id == id) return it.cost;
        return 0;
    };
    std::vector<std::vector<int>> cost(n_units);
    for (int j = 0; j < n_units; ++j)
        for (uint16_t id : mine[j]) cost[j].push_back(cost_of(id));
    for (int round = 0; round < 8 * n; ++round) {
        int hi = 0;
        for (int j = 1; j < n_units; ++j)
            if (load[j] > load[hi]) hi = j;
        // the exchange with any other unit that lowers the larger of the two loads most
        int best_j = -1, best_a = -1, best_b = -1, best_max = load[hi];
        for (int j = 0; j < n_units; ++j) {
            if (j == hi || load[j] >= load[hi]) continue;
            for (size_t a = 0; a < cost[hi].size(); ++a) {
                for (size_t b = 0; b < cost[j].size(); ++b) {
                    const int d = cost[hi][a] - cost[j][b];
                    if (d <= 0) continue;
                    const int m = std::max(load[hi] - d, load[j] + d);
                    if (m < best_max) best_max = m, best_j = j, best_a = (int)a, best_b = (int)b;
                }
            }
        }
        if (best_j < 0) break;
        const int lo = best_j;
        {
            const int d = cost[hi][best_a] - cost[lo][best_b];
            std::swap(cost[hi][best_a], cost[lo][best_b]);
            std::swap(mine[hi][best_a], mine[lo][best_b]);
            load[hi] -= d;
            load[lo] += d;
        }
    }
    order->assign(n, 0);
    for (int j = 0; j < n_units; ++j) {
        std::vector<size_t> by_cost(mine[j].size());
        for (size_t r = 0; r < by_cost.size(); ++r) by_cost[r] = r;
        std::stable_sort(by_cost.begin(), by_cost.end(), [&](size_t a, size_t b) { return cost[j][a] > cost[j][b]; });
        for (size_t r = 0; r < by_cost.size(); ++r) (*order)[r * n_units + j] = mine[j][by_cost[r]];
    }
    return true;
}

int launch_mpgemv_x_ordered(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv,
                            const uint16_t* order_dev, int n_wg, int max_seg_tiles, hipStream_t st) {
    OrderedArgs a;
    a.descs = descs_dev;
    a.order = order_dev;
    a.n_gemv = n_gemv;
    return launch_x_format<false>(bits, has_zero, group, a, n_wg, max_seg_tiles, st);
}

// The numbering goes to device memory through kernel arguments, like the descriptors.
struct OrderChunk {
    uint16_t e[1024];
};
__global__ void write_order_kernel(OrderChunk c, int count, uint16_t* __restrict__ out) {
    for (int i = threadIdx.x; i < count; i += blockDim.x) out[i] = c.e[i];
}
int launch_write_order(const std::vector<uint16_t>& order, uint16_t* dev, hipStream_t st) {
    for (size_t i = 0; i < order.size(); i += 1024) {
        OrderChunk c;
        const int n = (int)std::min<size_t>(1024, order.size() - i);
        for (int j = 0; j < 1024; ++j) c.e[j] = j < n ? order[i + j] : 0;
        hipLaunchKernelGGL(write_order_kernel, dim3(1), dim3(256), 0, st, c, n, dev + i);
    }
    return launch_status();
}

int launch_mpgemv_x_batch(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv, int max_workgroups,
                          int max_seg_tiles, hipStream_t st) {
    KernelArgs<false> a;
    a.descs = descs_dev;
    a.n_gemv = n_gemv;
    return launch_x_format<false>(bits, has_zero, group, a, max_workgroups, max_seg_tiles, st);
}

}  // namespace tman
