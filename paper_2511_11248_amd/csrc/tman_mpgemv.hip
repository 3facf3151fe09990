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

}  // namespace tman
