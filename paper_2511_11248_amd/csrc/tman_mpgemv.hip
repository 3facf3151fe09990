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
// mpgemv_kernel serves 1 to 8 tokens and reads the tables tman_build_lut made (Sec. 5: the precompute as a
// kernel of its own, shared by the layers fed from one activation).  The one-token kernel that builds its
// tables itself is in tman_mpgemv_x.hip.
#include <algorithm>
#include <vector>

#include "tman_mpgemv_kernel.h"

namespace tman {

// ---------------------------------------------------------------------------------------------
// host-side planning

GemvPlan plan_segments(const Layout& L, int np, int max_seg) {
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
    const tman_tiling_t t = current_tiling();
    return plan_segments(L, np, np >= 4 ? t.decode_seg_tiles_many : t.decode_seg_tiles);
}

void fill_desc_plan(GemvDesc& d, const Layout& L, const GemvPlan& p, const void* packed, const void* lut, int N,
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

// ---------------------------------------------------------------------------------------------
// launch (the kernel is in tman_mpgemv_kernel.h)

int launch_mpgemv(const Layout& L, const void* packed, const void* lut, int N, void* y, void* workspace,
                  hipStream_t st) {
    KernelArgs<true> a;
    fill_desc(a.single, L, packed, lut, N, y, workspace, 0);
    a.n_gemv = 1;
    a.status = device_status_word();
    if (!a.status) return TMAN_ERR_LAUNCH;
    return launch_format<true, false>(L.bits, L.has_zero, padded_tokens(N), L.group, a, plan_gemv(L, N).n_workgroups, st);
}

int launch_mpgemv_batch(int bits, int group, int has_zero, int N, const GemvDesc* descs_dev, int n_gemv,
                        int max_workgroups, hipStream_t st) {
    KernelArgs<false> a;
    a.descs = descs_dev;
    a.n_gemv = n_gemv;
    return launch_format<false, false>(bits, has_zero, padded_tokens(N), group, a, max_workgroups, st);
}

// Copies up to 16 descriptors per launch from the kernel arguments into the device table.  A GEMV whose blob
// carries a header for another shape or layout gets an empty descriptor (no workgroup of the lookup launch
// then touches it) and the mismatch is recorded in the library's status word.
struct DescChunk {
    GemvDesc d[16];
};
__global__ void write_descs_kernel(DescChunk c, int count, int bits, int group, int has_zero, GemvDesc* __restrict__ out,
                                   int* status) {
    if ((int)threadIdx.x >= count) return;
    GemvDesc d = c.d[threadIdx.x];
    if (!header_matches(d.tiles, d.M, d.K, bits, group, has_zero)) {
        d.n_row_blocks = 0;
        report_header_mismatch(status);
    }
    out[threadIdx.x] = d;
}

int launch_write_descs(const GemvDesc* host, int count, int bits, int group, int has_zero, GemvDesc* dev, hipStream_t st) {
    int* status = device_status_word();
    if (!status) return TMAN_ERR_LAUNCH;
    for (int i = 0; i < count; i += 16) {
        DescChunk c;
        int n = count - i < 16 ? count - i : 16;
        for (int j = 0; j < 16; ++j) c.d[j] = host[i + (j < n ? j : 0)];
        hipLaunchKernelGGL(write_descs_kernel, dim3(1), dim3(64), 0, st, c, n, bits, group, has_zero, dev + i, status);
    }
    return launch_status();
}

// ---------------------------------------------------------------------------------------------
// Numbering the workgroups of a batch for equal work per compute unit.
//
// With workgroup i on compute unit i mod n_units (what the dispatcher does with a launch that is resident at
// once), the numbering decides which workgroups share a unit.  The workgroups, largest first, go one by one to the
// unit with the least work so far that still has a free place (unit j has a place for ids j, j + n_units, ...);
// then the fullest unit exchanges a workgroup with another unit as long as that lowers the larger of the two
// loads; inside a unit the largest gets the lowest id.  Work of a workgroup = tile blocks of its K segment + 2
// (start and end of a workgroup cost about that).  A batch qualifies with at most 8 GEMVs (three bits of an
// entry) and no more workgroups than are resident at once: `per_unit` per compute unit.
int ordered_workgroups_of(int count, const Layout* L, const GemvPlan* plans, int n_units, int per_unit) {
    (void)L;
    if (count > 8 || n_units < 1 || per_unit < 1 || !current_tiling().decode_balance) return 0;
    int n = 0;
    for (int g = 0; g < count; ++g) {
        if (plans[g].n_workgroups > 0x1fff) return 0;
        n += plans[g].n_workgroups;
    }
    return n <= per_unit * n_units && n <= kOrderedMaxWorkgroups ? n : 0;
}

bool order_workgroups_of(int count, const Layout* L, const GemvPlan* plans, int n_units, int per_unit,
                         std::vector<uint16_t>* order) {
    const int n = ordered_workgroups_of(count, L, plans, n_units, per_unit);
    if (!n) return false;
    auto places = [&](int j) { return n / n_units + (j < n % n_units ? 1 : 0); };
    struct Item {
        int cost;
        uint16_t id;
    };
    std::vector<Item> items;
    for (int g = 0; g < count; ++g) {
        const GemvPlan& p = plans[g];
        for (int w = 0; w < p.n_workgroups; ++w) {
            const int seg = w % p.n_seg;
            const int tiles = std::min(p.seg_tiles, L[g].n_ktiles - seg * p.seg_tiles);
            items.push_back(Item{tiles + 2, (uint16_t)((g << 13) | w)});
        }
    }
    std::stable_sort(items.begin(), items.end(), [](const Item& a, const Item& b) { return a.cost > b.cost; });
    std::vector<int> load(n_units, 0);
    std::vector<std::vector<uint16_t>> mine(n_units);
    std::vector<std::vector<int>> cost(n_units);
    for (const Item& it : items) {
        int best = -1;
        for (int j = 0; j < n_units; ++j)
            if ((int)mine[j].size() < places(j) && (best < 0 || load[j] < load[best])) best = j;
        load[best] += it.cost;
        mine[best].push_back(it.id);
        cost[best].push_back(it.cost);
    }
    for (int round = 0; round < 8 * n; ++round) {
        int hi = 0;
        for (int j = 1; j < n_units; ++j)
            if (load[j] > load[hi]) hi = j;
        int best_j = -1, best_a = -1, best_b = -1, best_max = load[hi];
        for (int j = 0; j < n_units; ++j) {
            if (j == hi || load[j] >= load[hi]) continue;
            for (size_t a = 0; a < cost[hi].size(); ++a)
                for (size_t b = 0; b < cost[j].size(); ++b) {
                    const int d = cost[hi][a] - cost[j][b];
                    if (d <= 0) continue;
                    const int m = std::max(load[hi] - d, load[j] + d);
                    if (m < best_max) best_max = m, best_j = j, best_a = (int)a, best_b = (int)b;
                }
        }
        if (best_j < 0) break;
        const int d = cost[hi][best_a] - cost[best_j][best_b];
        std::swap(cost[hi][best_a], cost[best_j][best_b]);
        std::swap(mine[hi][best_a], mine[best_j][best_b]);
        load[hi] -= d;
        load[best_j] += d;
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

}  // namespace tman
