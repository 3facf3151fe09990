// Decoding mpGEMV of ONE token with the table precompute inside the lookup kernel (Sec. 2.2 "Bit-serial table
// lookup" and Sec. 4.3 for the lookups; Sec. 5 makes the precompute a kernel of its own because it is costly on
// the paper's hardware, whereas here a kernel boundary costs more than the precompute).
//
// With a single token the tables of up to 40 K tiles (1280 tables, 40 KB) fit in LDS next to two other
// workgroups.  A workgroup builds them itself from the activations (at most 10 KB) while its first weight
// tiles are on their way, so a decode step needs no launch for the table precompute, no table traffic, and no
// per-tile copy of a table slice into LDS.  The entries have the values build_lut_kernel computes (fp32 sums in
// ascending order, one rounding to fp16), as have the group sums (same tree of additions).
//
// A lookup address is tile base | index byte: one v_perm_b32 takes byte k of the prepared index word as byte 0
// and bytes 1..3 of the tile's table base (a multiple of 1024), the table's place inside the tile is the
// immediate offset of the LDS load.  One vector instruction and one LDS read per lookup.
//
// Work distribution.  A decode launch lasts microseconds and every workgroup is resident from its start, so
// what matters is that all compute units get the same number of tile blocks.  The tile blocks of the launch
// (GEMV after GEMV, row block after row block, K tile after K tile) are one linear sequence that the host
// cuts into as many slots as workgroups stay resident (three per compute unit, fixed by the LDS request); a
// workgroup walks its slot interval by interval (an interval = what the slot holds of one row block), in
// chunks of at most 40 tiles, keeping the partial sums of an interval in registers.  A row block held by one
// slot is written directly; one that several slots share meets through the workspace: every interval
// publishes its fp32 sums and adds its tile count to the row block's ticket, the one that completes the
// count adds the published sums in interval order (the result does not depend on timing) and returns the
// ticket to zero.  Sums and tickets use device-scope memory operations, coherent across the chip without
// cache write-back or invalidation.
#include <mutex>
#include <vector>

#include "tman_gemv_device.h"

namespace tman {

// ---------------------------------------------------------------------------------------------
// host side: workspace, descriptors, the cut into slots

static size_t x_ticket_bytes(const Layout& L) { return ((size_t)L.n_row_blocks * sizeof(int32_t) + 255) / 256 * 256; }

size_t x_workspace_bytes(const Layout& L) {
    return x_ticket_bytes(L) + (size_t)L.n_row_blocks * x_parts_per_row(L.n_ktiles) * kRows * sizeof(float);
}

void fill_xdesc(XDesc& d, const Layout& L, const void* packed, const void* x, void* y, void* workspace) {
    d.tiles = static_cast<const uint8_t*>(packed) + kHeaderBytes;
    d.x = static_cast<const uint8_t*>(x);
    d.y = y;
    d.tickets = static_cast<int32_t*>(workspace);
    d.partial = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + x_ticket_bytes(L));
    d.M = L.M;
    d.K = L.K;
    d.n_row_blocks = L.n_row_blocks;
    d.n_ktiles = L.n_ktiles;
    d.parts_per_row = x_parts_per_row(L.n_ktiles);
    d.valid = 1;
    d.bits = L.bits;
    d.group = L.group;
    d.has_zero = L.has_zero;
    d.pad = 0;
}

int x_slots_of_device() {
    static std::once_flag once;
    static int n_cu = 256;  // assumed when no device answers
    std::call_once(once, [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            n_cu = n;
    });
    const int s = n_cu * kXSlotsPerCu;
    return s < kXMaxSlots ? s : kXMaxSlots;
}

// One pass of the greedy cut with slots of at most `limit` tile blocks.  A row block that fits a chunk and the
// limit is never split (it then needs no exchange); longer ones fill the open slot to the limit.  With `out`
// set the slots are recorded; the return value is their number.
static int x_cut(const XDesc* d, int count, int limit, XSlot* out, int max_out) {
    int n = 0, fill = 0;
    bool open = false;
    auto begin = [&](int g, int pos) {
        if (out && n < max_out) {
            XSlot s = {};
            s.gemv = g;
            s.first = pos;
            out[n] = s;
        }
        open = true;
        fill = 0;
    };
    auto close = [&]() {
        if (out && n < max_out) out[n].count = fill;
        ++n;
        open = false;
        fill = 0;
    };
    for (int g = 0; g < count; ++g) {
        const int nk = d[g].n_ktiles;
        const bool whole = nk <= kXPieceTiles && nk <= limit;
        for (int rb = 0; rb < d[g].n_row_blocks; ++rb) {
            if (whole) {
                if (open && fill + nk > limit) close();
                if (!open) begin(g, rb * nk);
                fill += nk;
                if (fill == limit) close();
            } else {
                int pos = rb * nk, rem = nk;
                while (rem > 0) {
                    if (!open) begin(g, pos);
                    const int t = rem < limit - fill ? rem : limit - fill;
                    fill += t;
                    pos += t;
                    rem -= t;
                    if (fill == limit) close();
                }
            }
        }
    }
    if (open) close();
    return n;
}

int x_schedule(const XDesc* d, int count, int max_slots, XSlot* slots) {
    long long total = 0;
    for (int g = 0; g < count; ++g) total += (long long)d[g].n_row_blocks * d[g].n_ktiles;
    if (total <= 0 || total > 0x7fffffffLL || max_slots < 1) return 0;
    int limit = (int)((total + max_slots - 1) / max_slots);
    if (limit < kXMinSlotTiles) limit = kXMinSlotTiles;
    // the smallest limit whose cut fits the slots (whole row blocks make the count step a little)
    while (x_cut(d, count, limit, nullptr, 0) > max_slots) limit += 1 + limit / 64;
    const int n = x_cut(d, count, limit, slots, max_slots);
    // Interval bookkeeping.  The intervals of a row block lie in consecutive slots; only the first interval of a
    // slot can continue a row block that an earlier slot began, and only its last one can be continued later.
    int run = 0;               // intervals seen so far of the row block that is still open
    std::vector<int> touching;  // slots that hold an interval of that row block: (slot << 1) | is_last_interval
    for (int s = 0; s < n; ++s) {
        int g = slots[s].gemv, pos = slots[s].first, rem = slots[s].count;
        bool first = true;
        slots[s].pidx0 = 0;
        slots[s].nparts_first = slots[s].nparts_last = 1;
        while (rem > 0) {
            const int nk = d[g].n_ktiles, tiles_g = d[g].n_row_blocks * nk;
            if (pos >= tiles_g) {
                ++g;
                pos = 0;
                continue;
            }
            const int k0 = pos % nk, len = rem < nk - k0 ? rem : nk - k0;
            if (k0 == 0) {
                run = 0;
                touching.clear();
            }
            if (first) slots[s].pidx0 = run;
            ++run;
            touching.push_back((s << 1) | (first ? 0 : 1));
            if (k0 + len == nk) {  // the row block is complete: everyone who holds a part of it learns the count
                for (int t : touching) {
                    if (t & 1) slots[t >> 1].nparts_last = run;
                    else slots[t >> 1].nparts_first = run;
                }
            }
            pos += len;
            rem -= len;
            first = false;
        }
    }
    return n;
}

size_t x_desc_bytes(int count) { return (size_t)count * sizeof(XDesc) + (size_t)kXMaxSlots * sizeof(XSlot); }

// ---------------------------------------------------------------------------------------------
// device side

struct XArgsSingle {
    XDesc d;
    int slot_tiles;  // tile blocks per slot (a multiple of the row block's tiles when row blocks stay whole)
    int* status;     // the library's status word
};
struct XArgsBatch {
    const XDesc* __restrict__ descs;
    const XSlot* __restrict__ slots;
    int n_gemv;
};

// The slot of a single GEMV cut into equal slots of `st` tile blocks, with the bookkeeping x_schedule does on the
// host: the intervals of a row block start at the row block's first tile and at the multiples of `st` inside it.
__device__ __forceinline__ XSlot single_slot(int l, int st, int nk, int total) {
    XSlot s = {};
    s.gemv = 0;
    s.first = l * st;
    const int end = min(s.first + st, total);
    s.count = max(end - s.first, 0);
    if (s.count == 0) return s;
    const int r0 = (s.first / nk) * nk;  // first tile of the row block the slot starts in
    s.pidx0 = s.first / st - r0 / st;
    s.nparts_first = 1 + (r0 + nk - 1) / st - r0 / st;
    const int r1 = ((end - 1) / nk) * nk;  // and of the one it ends in
    s.nparts_last = 1 + (r1 + nk - 1) / st - r1 / st;
    return s;
}

template <int B, int GQ, bool HZ, bool SINGLE>
__global__ void __launch_bounds__(kWaves * 64)
mpgemv_x_kernel(typename std::conditional<SINGLE, XArgsSingle, XArgsBatch>::type a) {
    using Cfg = GemvCfg<B, 1, GQ, HZ>;
    constexpr int D = Cfg::D;
    constexpr int TPG = GQ / kLutGroup;  // tables per quantization group: 8, 16 or 32 consecutive lanes
    // LDS of a workgroup: the tables of a chunk, their group sums, the four partial sums of each row.  Three
    // such workgroups fit a compute unit, which is what the cut into slots counts on.
    constexpr int kTablesBytes = kXPieceTiles * kTableBytesPerKTile;
    constexpr int kSumsBytes = kXPieceTiles * Cfg::GPT * 4;
    __shared__ __attribute__((aligned(1024))) uint8_t lds_x[kTablesBytes + kSumsBytes + kWaves * kRows * 4];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    float pw[B];
#pragma unroll
    for (int i = 0; i < B; ++i) pw[i] = opaque((float)(1 << i));
    uint32_t sel[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) sel[k] = 0x03020100u | (uint32_t)(4 + k);

    const uint32_t lt = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr<uint8_t>)lds_x));
    const uint32_t ls = lt + kTablesBytes;  // group sums follow the tables
    const uint32_t lr = ls + kSumsBytes;    // then the partial sums [wave][row]

    XSlot sl;
    if constexpr (SINGLE) {
        sl = single_slot((int)blockIdx.x, a.slot_tiles, a.d.n_ktiles, a.d.n_row_blocks * a.d.n_ktiles);
        // a blob packed for another shape or layout: leave y alone and say so
        if (!header_matches(a.d.tiles, a.d.M, a.d.K, B, GQ, HZ ? 1 : 0)) {
            if (blockIdx.x == 0 && tid == 0) report_header_mismatch(a.status);
            return;
        }
    } else {
        sl = a.slots[blockIdx.x];
    }
    int g = uniform(sl.gemv), pos = uniform(sl.first), remaining = uniform(sl.count);
    bool first_interval = true;
    bool tables_in_use = false;  // some wave may still read the tables of the previous chunk

    while (remaining > 0) {
        const XDesc* dp;
        if constexpr (SINGLE) dp = &a.d;
        else dp = a.descs + g;
        const XDesc& d = *dp;
        const int nk = uniform(d.n_ktiles);
        if (pos >= uniform(d.n_row_blocks) * nk) {  // the slot continues in the next GEMV
            ++g;
            pos = 0;
            continue;
        }
        const int rb = uniform(pos / nk), k0 = uniform(pos % nk);
        const int len = min(remaining, nk - k0);
        const int pidx = first_interval ? uniform(sl.pidx0) : 0;
        const int nparts = (k0 == 0 && len == nk) ? 1 : uniform(first_interval ? sl.nparts_first : sl.nparts_last);
        pos += len;
        remaining -= len;
        first_interval = false;
        if (!uniform(d.valid)) continue;

        Streams src;
        src.w = uniform(d.tiles) + (size_t)rb * nk * Cfg::TB;
        src.t = src.s = nullptr;
        src.w_bytes = (uint32_t)(nk * Cfg::TB);
        src.t_bytes = src.s_bytes = 0;
        const uint8_t* xbase = uniform(d.x);
        const uint32_t xbytes = (uint32_t)uniform(d.K) * 2u;

        float y = 0.f;
        for (int c0 = k0; c0 < k0 + len; c0 += kXPieceTiles) {
            const int c1 = min(c0 + kXPieceTiles, k0 + len);
            const int per_wave = (c1 - c0 + kWaves - 1) / kWaves;
            const int t0 = min(c0 + wave * per_wave, c1);  // this wave's K tiles [t0, t1)
            const int t1 = min(t0 + per_wave, c1);

            // first weight tiles on their way before anything else
            Stage<B, 1, Cfg::MPL> st[D] = {};
#pragma unroll
            for (int s = 0; s < D; ++s) issue_weights<B, 1, GQ, HZ>(st[s], src, t0 + s < t1, t0 + s, lane);

            // Tables and group sums of the chunk: thread -> tables tid, tid + 256, ...  The range check of a
            // buffer load covers the per-lane offset only, so the resource starts at the chunk's first activation
            // and ends with x: columns beyond K read as zero.
            {
                const uint32_t x_start = (uint32_t)(c0 * kKTile * 2);  // c0 < n_ktiles, so this lies inside x
                const rsrc_t rx = make_rsrc(xbase + x_start, xbytes - x_start);
                const int n_tab = (c1 - c0) * kTablesPerKTile;
                constexpr int kPasses = kXPieceTiles * kTablesPerKTile / (kWaves * 64);
                static_assert(kPasses * kWaves * 64 == kXPieceTiles * kTablesPerKTile, "whole passes");
                u32x2 xv[kPasses];  // all requests first (a pass beyond the chunk reads activations nobody uses)
#pragma unroll
                for (int i = 0; i < kPasses; ++i)
                    xv[i] = __builtin_amdgcn_raw_buffer_load_b64(rx, (i * kWaves * 64 + tid) * 8, 0, 0);
                if (tables_in_use) __syncthreads();  // every wave is done with the previous chunk's tables
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
            tables_in_use = true;

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
                        consume_weights<B, GQ, HZ>(st[s], lt + (t - c0) * kTableBytesPerKTile, ls + (t - c0) * Cfg::GPT * 4, sel, pw, y);
                        issue_weights<B, 1, GQ, HZ>(st[s], src, t + D < t1, t + D, lane);
                    }
                }
            }
        }

        // the four waves' sums of the interval meet in LDS (this barrier also ends the use of the tables)
        store_lds<float>(lr + (wave * kRows + lane) * 4, y);
        __syncthreads();
        tables_in_use = false;
        if (wave == 0) {
            y = ((load_lds<float>(lr + lane * 4) + load_lds<float>(lr + (kRows + lane) * 4)) +
                 load_lds<float>(lr + (2 * kRows + lane) * 4)) + load_lds<float>(lr + (3 * kRows + lane) * 4);
            const int m = rb * kRows + lane;
            const int M = uniform(d.M);
            _Float16* out = static_cast<_Float16*>(uniform(d.y));
            if (nparts == 1) {
                if (m < M) out[m] = (_Float16)y;
            } else {
                // the row block is shared with other slots: publish this interval's sums, add its tiles to the ticket
                float* base_p = uniform(d.partial) + (size_t)rb * uniform(d.parts_per_row) * kRows;
                __hip_atomic_store(base_p + pidx * kRows + lane, y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the sums have reached device-coherent memory
                int32_t* ticket = uniform(d.tickets) + rb;
                int prev = 0;
                if (lane == 0) prev = __hip_atomic_fetch_add(ticket, len, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                prev = __builtin_amdgcn_readfirstlane(prev);
                if (prev + len == nk) {
                    // the count is complete: every interval of this row block has been published; add them in order
                    float acc = 0.f;
                    for (int p0 = 0; p0 < nparts; p0 += 4) {
                        float v[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            v[q] = (p0 + q < nparts) ? __hip_atomic_load(base_p + (p0 + q) * kRows + lane, __ATOMIC_RELAXED,
                                                                        __HIP_MEMORY_SCOPE_AGENT)
                                                     : 0.f;
#pragma unroll
                        for (int q = 0; q < 4; ++q) acc += v[q];
                    }
                    if (m < M) out[m] = (_Float16)acc;
                    if (lane == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
}

// Writes the descriptor table of a batch into device memory and decides, on the device, whether each blob's
// header agrees with its descriptor (a blob packed for another shape is then skipped by the lookup kernel).
struct XDescChunk {
    XDesc d[16];
};
__global__ void x_write_descs_kernel(XDescChunk c, int count, XDesc* __restrict__ out, int* status) {
    const int i = threadIdx.x;
    if (i >= count) return;
    XDesc d = c.d[i];
    d.valid = header_matches(d.tiles, d.M, d.K, d.bits, d.group, d.has_zero) ? 1 : 0;
    if (!d.valid) report_header_mismatch(status);
    out[i] = d;
}
struct XSlotChunk {
    XSlot s[64];
};
__global__ void x_write_slots_kernel(XSlotChunk c, int count, XSlot* __restrict__ out) {
    const int i = threadIdx.x;
    if (i < count) out[i] = c.s[i];
}

// ---------------------------------------------------------------------------------------------
// launch

int launch_mpgemv_x_prepare(const XDesc* host_descs, int count, const XSlot* host_slots, int n_slots, void* desc_dev,
                            hipStream_t st) {
    int* status = device_status_word();
    if (!status) return TMAN_ERR_LAUNCH;
    XDesc* dd = static_cast<XDesc*>(desc_dev);
    XSlot* ds = reinterpret_cast<XSlot*>(dd + count);
    for (int i = 0; i < count; i += 16) {
        XDescChunk c;
        const int n = count - i < 16 ? count - i : 16;
        for (int j = 0; j < 16; ++j) c.d[j] = host_descs[i + (j < n ? j : 0)];
        hipLaunchKernelGGL(x_write_descs_kernel, dim3(1), dim3(64), 0, st, c, n, dd + i, status);
    }
    // every slot of the grid is defined: those beyond the cut are empty
    const int total = x_slots_of_device();
    for (int i = 0; i < total; i += 64) {
        XSlotChunk c = {};
        const int n = total - i < 64 ? total - i : 64;
        for (int j = 0; j < n; ++j)
            if (i + j < n_slots) c.s[j] = host_slots[i + j];
        hipLaunchKernelGGL(x_write_slots_kernel, dim3(1), dim3(64), 0, st, c, n, ds + i);
    }
    return launch_status();
}

template <int B, bool HZ, bool SINGLE, typename Args>
static int launch_x_group(int group, const Args& a, int n_slots, hipStream_t st) {
    const dim3 grid((unsigned)n_slots), block(kWaves * 64);
    switch (group) {
        case 32: hipLaunchKernelGGL((mpgemv_x_kernel<B, 32, HZ, SINGLE>), grid, block, 0, st, a); break;
        case 64: hipLaunchKernelGGL((mpgemv_x_kernel<B, 64, HZ, SINGLE>), grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL((mpgemv_x_kernel<B, 128, HZ, SINGLE>), grid, block, 0, st, a); break;
    }
    return launch_status();
}

template <bool SINGLE, typename Args>
static int launch_x_format(int bits, int has_zero, int group, const Args& a, int n_slots, hipStream_t st) {
    if (bits == 1) {
        return has_zero ? launch_x_group<1, true, SINGLE>(group, a, n_slots, st)
                        : launch_x_group<1, false, SINGLE>(group, a, n_slots, st);
    }
    if (bits == 2) return launch_x_group<2, true, SINGLE>(group, a, n_slots, st);
    return launch_x_group<4, true, SINGLE>(group, a, n_slots, st);
}

int launch_mpgemv_x(const Layout& L, const void* packed, const void* x, void* y, void* workspace, hipStream_t st) {
    XArgsSingle a;
    fill_xdesc(a.d, L, packed, x, y, workspace);
    a.status = device_status_word();
    if (!a.status) return TMAN_ERR_LAUNCH;
    // equal slots: whole row blocks where a row block fits a chunk, else a plain cut of the tile sequence
    const int S = x_slots_of_device(), nk = L.n_ktiles;
    const long long total = (long long)L.n_row_blocks * nk;
    if (total > 0x7fffffffLL) return TMAN_ERR_SHAPE;
    int limit = (int)((total + S - 1) / S);
    if (limit < kXMinSlotTiles) limit = kXMinSlotTiles;
    // a row block that fits a chunk stays whole (no exchange): slots of ceil(limit / nk) row blocks, which are
    // at most S; longer row blocks are cut tile by tile
    const int st_tiles = nk <= kXPieceTiles ? (limit + nk - 1) / nk * nk : limit;
    a.slot_tiles = st_tiles;
    const int n_slots = (int)((total + st_tiles - 1) / st_tiles);
    return launch_x_format<true>(L.bits, L.has_zero, L.group, a, n_slots, st);
}

int launch_mpgemv_x_batch(int bits, int group, int has_zero, const void* desc_dev, int n_gemv, hipStream_t st) {
    XArgsBatch a;
    a.descs = static_cast<const XDesc*>(desc_dev);
    a.slots = reinterpret_cast<const XSlot*>(a.descs + n_gemv);
    a.n_gemv = n_gemv;
    return launch_x_format<false>(bits, has_zero, group, a, x_slots_of_device(), st);
}

}  // namespace tman
