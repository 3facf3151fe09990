// Internal definitions shared by the HIP translation units of libtman (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <vector>
#include <stdint.h>

#include "tman.h"

namespace tman {

// Packed-weight geometry.  A tile block is 64 rows x 128 columns; lane (row % 64) owns the 128
// weights of its row.
constexpr int kHeaderBytes = 128;
constexpr int kRows = 64;
constexpr int kKTile = 128;
constexpr int kLayoutVersion = 1;
constexpr int kLutGroup = 4;                       // activations per table (16-entry tables)
constexpr int kTablesPerKTile = kKTile / kLutGroup;  // 32
constexpr int kTableBytesPerKTile = kTablesPerKTile * 16 * 2;  // fp16 entries, one token

struct Layout {
    int M, K, bits, group, has_zero;
    int n_row_blocks, n_ktiles;
    int groups_per_tile;  // 128 / group
    int meta_entry;       // bytes per (scale[, zero]) entry
    int meta_per_lane;    // groups_per_tile * meta_entry
    int tile_bytes;       // bits * 1024 + 64 * meta_per_lane
    size_t total_bytes;
};

inline int check_shape(const tman_shape_t* s) {
    if (!s) return TMAN_ERR_NULL;
    if (s->bits != 1 && s->bits != 2 && s->bits != 4) return TMAN_ERR_BITS;
    if (s->group != 32 && s->group != 64 && s->group != 128) return TMAN_ERR_GROUP;
    if (s->M < 1 || s->K < 1 || s->K % s->group != 0) return TMAN_ERR_SHAPE;
    if (s->flags & ~TMAN_FLAG_HAS_ZERO) return TMAN_ERR_SHAPE;
    if (!(s->flags & TMAN_FLAG_HAS_ZERO) && s->bits != 1) return TMAN_ERR_SHAPE;  // sign form is 1-bit only
    return TMAN_OK;
}

inline Layout make_layout(const tman_shape_t* s) {
    Layout L;
    L.M = s->M;
    L.K = s->K;
    L.bits = s->bits;
    L.group = s->group;
    L.has_zero = (s->flags & TMAN_FLAG_HAS_ZERO) ? 1 : 0;
    L.n_row_blocks = (s->M + kRows - 1) / kRows;
    L.n_ktiles = (s->K + kKTile - 1) / kKTile;
    L.groups_per_tile = kKTile / s->group;
    L.meta_entry = L.has_zero ? 4 : 2;
    L.meta_per_lane = L.groups_per_tile * L.meta_entry;
    L.tile_bytes = s->bits * 1024 + 64 * L.meta_per_lane;
    L.total_bytes = (size_t)kHeaderBytes + (size_t)L.n_row_blocks * L.n_ktiles * L.tile_bytes;
    return L;
}

// tokens are padded to 1, 2, 4 or 8 inside the lookup-table buffer
inline int padded_tokens(int N) { return N <= 1 ? 1 : N <= 2 ? 2 : N <= 4 ? 4 : 8; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int launch_status() { return hipGetLastError() == hipSuccess ? TMAN_OK : TMAN_ERR_LAUNCH; }

// Does the header in front of the tile blocks describe this shape?  The 14 defined words are fetched with one
// 64-byte load and compared without branches, so the check costs one memory round trip.
typedef int32_t header_words_t __attribute__((ext_vector_type(16)));
__device__ __forceinline__ bool header_matches(const uint8_t* tiles, int M, int K, int bits, int group, int has_zero) {
    const header_words_t h = *reinterpret_cast<const header_words_t*>(tiles - kHeaderBytes);
    const int diff = (h[0] ^ 0x4e414d54) | (h[1] ^ 0x00314b50) | (h[2] ^ M) | (h[3] ^ K) | (h[4] ^ bits) | (h[5] ^ group) |
                     (h[6] ^ has_zero) | (h[7] ^ kRows) | (h[8] ^ kKTile) | (h[12] ^ kHeaderBytes) | (h[13] ^ kLayoutVersion);
    return diff == 0;
}

// What a kernel does when it meets a blob whose header disagrees with the shape it was launched for: one thread
// of the launch records TMAN_ERR_HEADER in the library's status word; the outputs are left alone.
__device__ __forceinline__ void report_header_mismatch(int* status) {
    __hip_atomic_store(status, (int)TMAN_ERR_HEADER, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Decode scheduling: a workgroup (four waves) owns one row block and one K segment of at most this
// many tiles; longer K is cut into equal segments that meet through the workspace.
// The tile counts below are the library's tiling (Sec. 4.1 "Unified tiling strategy"): defaults found by the
// measured search in paper_2511_11248_amd/tune.py, replaceable at run time with tman_set_tiling (which checks the
// constraints that play the part of Eq. 1-4 on this machine).
constexpr int kGemvXSegmentTiles = 32;  // tables one workgroup of the one-token kernel can hold (32 KB of LDS)
tman_tiling_t current_tiling();

// One GEMV of a decode launch, as the kernel sees it.
struct GemvDesc {
    const uint8_t* tiles;  // first tile block (past the header)
    const uint8_t* lut_t;  // fp16 tables; for the kernel that builds its own tables: the activations, fp16 [K]
    const uint8_t* lut_s;  // fp32 group sums (unused by that kernel)
    void* y;               // fp16 [N][M]
    int32_t* tickets;      // [n_row_blocks], zero between launches
    float* partial;        // [n_row_blocks][n_seg][NP][64]
    int M, N, n_row_blocks, n_ktiles;
    int wg_begin;          // index of this GEMV's first workgroup in the launch
    int n_seg;             // K segments per row block
    int seg_tiles;         // tiles per segment (the last may be shorter)
    int K;                 // columns of W
};

struct GemvPlan {
    int np;  // padded tokens
    int n_seg, seg_tiles, n_workgroups;
    size_t ticket_bytes;
    size_t partial_bytes;
};
GemvPlan plan_gemv(const Layout& L, int N);
GemvPlan plan_segments(const Layout& L, int np, int max_seg);
// Plan of the one-token kernel that builds its tables itself: at most 32 tiles per segment (32 KB of tables
// in LDS), 24 when K has to be cut anyway.
GemvPlan plan_gemv_x(const Layout& L);
void fill_desc_plan(GemvDesc& d, const Layout& L, const GemvPlan& p, const void* packed, const void* lut, int N, void* y,
                    void* workspace, int wg_begin);
void fill_desc(GemvDesc& d, const Layout& L, const void* packed, const void* lut, int N, void* y, void* workspace,
               int wg_begin);

// launchers (each returns a tman_status)
int launch_pack(const Layout& L, const uint8_t* codes, const void* scales, const void* zeros, void* packed,
                hipStream_t st);
int launch_unpack(const Layout& L, const void* packed, uint8_t* codes, void* scales, void* zeros, hipStream_t st);
int launch_build_lut(const void* x, int N, int K, int group, void* lut, hipStream_t st);
int launch_build_lut_batch(int count, const void* const* x, int N, const int* K, int group, void* const* lut,
                           hipStream_t st);
int launch_build_lut_i16_batch(int count, const void* const* x, int N, const int* K, int group, void* const* lut,
                               hipStream_t st);
int launch_mpgemv_i16(const Layout& L, const void* packed, const void* lut, int N, void* y, void* workspace, hipStream_t st);
int launch_mpgemv_i16_batch(int bits, int group, int has_zero, int N, const GemvDesc* descs_dev, int n_gemv,
                            int max_workgroups, hipStream_t st);
int launch_mpgemv(const Layout& L, const void* packed, const void* lut, int N, void* y, void* workspace,
                  hipStream_t st);
int launch_mpgemv_batch(int bits, int group, int has_zero, int N, const GemvDesc* descs_dev, int n_gemv,
                        int max_workgroups, hipStream_t st);
// one token, tables built inside the lookup kernel from the activations x (fp16 [K])
void fill_desc_x(GemvDesc& d, const Layout& L, const void* packed, const void* x, void* y, void* workspace);
int launch_mpgemv_x(const Layout& L, const void* packed, const void* x, void* y, void* workspace, hipStream_t st);
int launch_mpgemv_x_batch(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv, int max_workgroups,
                          int max_seg_tiles, hipStream_t st);
constexpr int kOrderedMaxWorkgroups = 4096;  // room in a descriptor table for a numbering of the workgroups
// workgroups of a numbered launch (0: plain grid) and the numbering, for the plans of any of the decode kernels
int ordered_workgroups_of(int count, const Layout* L, const GemvPlan* plans, int n_units, int per_unit);
bool order_workgroups_of(int count, const Layout* L, const GemvPlan* plans, int n_units, int per_unit,
                         std::vector<uint16_t>* order);
int launch_write_order(const std::vector<uint16_t>& order, uint16_t* dev, hipStream_t st);
// ... of a one-token batch (tman_mpgemv_x) and of a small-batch mpGEMM batch
int ordered_workgroups(int count, const Layout* L, int n_units);
bool order_workgroups(int count, const Layout* L, int n_units, std::vector<uint16_t>* order);
int ordered_workgroups_small(int count, const Layout* L, int n_units);
bool order_workgroups_small(int count, const Layout* L, int n_units, std::vector<uint16_t>* order);
int launch_mpgemm_small_ordered(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv,
                                const uint16_t* order_dev, int n_wg, hipStream_t st);
int launch_mpgemv_x_ordered(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv,
                            const uint16_t* order_dev, int n_wg, int max_seg_tiles, hipStream_t st);
// a handful of tokens on the matrix cores, scheduled like the decoding kernels (tman_mpgemm with N <= 32, and its batch form)
GemvPlan plan_small(const Layout& L);
void fill_desc_small(GemvDesc& d, const Layout& L, const void* packed, const void* x, int N, void* y, void* workspace);
int launch_mpgemm_small(const Layout& L, const void* packed, const void* x, int N, void* y, void* workspace, hipStream_t st);
int launch_mpgemm_small_batch(int bits, int group, int has_zero, const GemvDesc* descs_dev, int n_gemv, int max_workgroups,
                              hipStream_t st);
// integer matrix cores for formats with one scale and zero per row (tman_quantize_act_i8, tman_mpgemm_i8)
size_t act_i8_bytes(int N, int K);
int launch_quantize_act_i8(const void* x, int N, int K, void* out, hipStream_t st);
// 1 = the 128 x 128 kernel, 3 / 4 / 7 = the wide kernel with that many 32-token blocks per workgroup
int choose_i8_token_blocks(int n_row_blocks, int N, int K);
int launch_mpgemm_i8(const Layout& L, const void* packed, const void* xq_buf, int N, void* y, void* acc_out, hipStream_t st);
int* device_status_word();  // device address of the library's status word on the current device (nullptr on failure)
int launch_write_descs(const GemvDesc* host, int count, int bits, int group, int has_zero, GemvDesc* dev, hipStream_t st);
int launch_mpgemm(const Layout& L, const void* packed, const void* x, int N, void* y, void* workspace, hipStream_t st);
int mpgemm_row_blocks_per_workgroup(const Layout& L, int N);
int mpgemm_splits_k(const Layout& L, int N);

}  // namespace tman
