// The library's tiling and the constraints it must satisfy (Sec. 4.1 "Unified tiling strategy", Eq. 1-4).
//
// In the paper a search picks, per machine, the tile sizes of the prefill and of the decoding loop nest under
// four constraints -- the tables of a decoding tile fit the vector registers (Eq. 1), both loop nests cover the
// same M extent (Eq. 2) and the same K extent (Eq. 3) of the one pre-permuted weight copy, and the pipeline's
// stage buffers fit the on-chip memory (Eq. 4) -- and three heuristics (largest K per table set, ...).  Here the
// shared tile block is fixed by the packed layout: 64 rows x 128 columns for both kernels, which is Eq. 2 and
// Eq. 3 by construction (a prefill workgroup covers 1..4 tile blocks in M and walks K in four 32-column stages
// per tile block; a decoding wave covers one tile block in M and the 32 tables of its 128 columns).  What
// remains free, and what tman_set_tiling can change, is how many tile blocks one workgroup takes:
//   decode_*            K tiles per decoding workgroup (its K segment); the one-token kernel keeps the tables of
//                       its whole segment in LDS, so there the segment is bounded like K_lut in Eq. 1:
//                       seg_tiles x 1 KB of tables <= the 32 KB a workgroup requests;
//   decode_balance    whether the workgroups of a one-token batch are numbered for equal work per compute unit
//                       (not a tile size, but it decides which segment length is best);
//   prefill_row_blocks  tile blocks in M per prefill workgroup; Eq. 4 reads ring (4) x stage bytes <= 160 KB of
//                       LDS, which admits at most 4;
//   prefill_k_split     whether small prefill grids go to the kernel whose waves split K, and with which tile;
//   i8_token_blocks     which integer-matrix-core prefill kernel runs and how many tokens its workgroup takes.
// The defaults are the best of the measured sweep in paper_2511_11248_amd/tune.py over the benchmark shapes.
#include <atomic>
#include <mutex>

#include "tman_internal.h"

namespace tman {

static constexpr tman_tiling_t kDefaultTiling = {32, 24, 32, 17, 81920, 43, 0, 1, 0, 0};
static std::mutex tiling_mutex;
static tman_tiling_t tiling_now = kDefaultTiling;

tman_tiling_t current_tiling() {
    std::lock_guard<std::mutex> lock(tiling_mutex);
    return tiling_now;
}

// Eq. 1 and Eq. 4 in this machine's terms (Eq. 2 and Eq. 3 hold for every value: the tile block is shared).
static int check_tiling(const tman_tiling_t& t) {
    constexpr int kLdsBytes = 160 * 1024, kRing = 4;
    if (t.decode_seg_tiles < 1 || t.decode_seg_tiles_many < 1 || t.small_seg_tiles < 1) return TMAN_ERR_SHAPE;
    if (t.decode_seg_tiles > 4096 || t.decode_seg_tiles_many > 4096 || t.small_seg_tiles > 4096) return TMAN_ERR_SHAPE;
    // Eq. 1: the tables of a one-token segment (1 KB per tile) must fit the workgroup's 32 KB
    if (t.decode_x_seg_tiles < 1 || t.decode_x_seg_tiles * kTableBytesPerKTile > kGemvXSegmentTiles * kTableBytesPerKTile)
        return TMAN_ERR_SHAPE;
    if (t.decode_x_long_seg_tiles < 1 || t.decode_x_long_seg_tiles > t.decode_x_seg_tiles) return TMAN_ERR_SHAPE;
    if (t.decode_x_whole_bytes < 1024) return TMAN_ERR_SHAPE;
    if (t.decode_balance != 0 && t.decode_balance != 1) return TMAN_ERR_SHAPE;
    // Eq. 4: stage ring of the prefill kernel: rows x 80 bytes of fp16 weights + 256 tokens x 64 bytes per stage
    if (t.prefill_row_blocks < 0 || t.prefill_row_blocks > 4) return TMAN_ERR_SHAPE;
    const int rb = t.prefill_row_blocks ? t.prefill_row_blocks : 4;
    if (kRing * (rb * kRows * 80 + 256 * 64) > kLdsBytes) return TMAN_ERR_SHAPE;
    // the prefill kernel whose waves split K: 0 = where it is measured faster, 1 = never, 2 / 3 = always, with its
    // 64 x 256 / 128 x 128 tile (its LDS, 128 KB of activation buffers or 135 KB of partial tiles, fits for both)
    if (t.prefill_k_split < 0 || t.prefill_k_split > 3) return TMAN_ERR_SHAPE;
    // the integer prefill kernel: 0 = chosen per call, 1 = the 128 x 128 kernel, 3 / 4 / 7 = the wide kernel with that
    // many 32-token blocks per workgroup (its output tile, tokens x 528 bytes, fits the LDS for all three), 9 = the
    // kernel whose waves split K
    if (t.i8_token_blocks != 0 && t.i8_token_blocks != 1 && t.i8_token_blocks != 3 && t.i8_token_blocks != 4 &&
        t.i8_token_blocks != 7 && t.i8_token_blocks != 9)
        return TMAN_ERR_SHAPE;
    return TMAN_OK;
}

}  // namespace tman

using namespace tman;

extern "C" {

int tman_get_tiling(tman_tiling_t* out) {
    if (!out) return TMAN_ERR_NULL;
    *out = current_tiling();
    return TMAN_OK;
}

int tman_default_tiling(tman_tiling_t* out) {
    if (!out) return TMAN_ERR_NULL;
    *out = kDefaultTiling;
    return TMAN_OK;
}

int tman_set_tiling(const tman_tiling_t* t) {
    if (!t) return TMAN_ERR_NULL;
    const int rc = check_tiling(*t);
    if (rc != TMAN_OK) return rc;
    std::lock_guard<std::mutex> lock(tiling_mutex);
    tiling_now = *t;
    return TMAN_OK;
}

}  // extern "C"
