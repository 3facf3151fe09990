/*
 * tman.h -- C ABI of the MI355X (gfx950) table-lookup mixed-precision matmul library.
 *
 * The library implements the hot path of T-MAN (arxiv 2511.11248): the product of group-quantized
 * 1/2/4-bit weights with fp16 activations, y = x * dequant(W)^T, computed through table lookup --
 * bit-serial activation tables for decoding (mpGEMV) and a two-level table dequantization feeding
 * the matrix cores for prefill (mpGEMM) -- from ONE bit-serial packed copy of the weights.
 *
 * Conventions for every call
 *   - all data pointers are DEVICE pointers unless stated otherwise; the caller owns every buffer,
 *     the library never allocates, frees or keeps a pointer after the call returns;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); every call only enqueues
 *     work on it and never synchronises with the host;
 *   - tensors are row-major; fp16 means IEEE binary16;
 *   - the return value is TMAN_OK or a negative tman_status; arguments are validated before
 *     anything is launched, so an error means no work was enqueued (except TMAN_ERR_LAUNCH, which
 *     reports the HIP runtime refusing a launch).
 *
 * Accuracy.  The fp16 paths (tman_mpgemv, tman_mpgemv_x, tman_mpgemm) reproduce the exact product
 * y = x * dequant(W)^T to within 2e-3 of max(|y[n][m]|, rms_m y[n][:]) per token.  That figure is a
 * statistical statement, about five standard deviations of the rounding noise the method itself fixes
 * (16-bit table entries or fp16 weights, Sec. 4.1 / 4.3: rms 2-3e-4 of rms(y); the fp16 result: up to
 * 4.9e-4), not a hard bound: among 1500 random shapes one output in 52,000 of one case reached 2.07e-3,
 * and a token whose one or two outputs cancel to nearly zero can exceed it.  In tman_mpgemm a dequantized
 * weight may differ from fp16((code - zero) * scale) by one fp16 step (about 5 % do: the constant
 * (1024 + zero) * scale is rounded to fp32 before the single rounding to fp16).  The integer paths state their
 * own bounds.
 */
#ifndef TMAN_H
#define TMAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tman_status {
    TMAN_OK = 0,
    TMAN_ERR_NULL = -1,      /* a required pointer is NULL */
    TMAN_ERR_BITS = -2,      /* bits not in {1, 2, 4} */
    TMAN_ERR_GROUP = -3,     /* group not in {32, 64, 128} */
    TMAN_ERR_SHAPE = -4,     /* M < 1, K < 1, K % group != 0, N out of range, flags/zeros mismatch */
    TMAN_ERR_WORKSPACE = -5, /* workspace missing or smaller than the *_workspace_bytes query */
    TMAN_ERR_ALIGN = -6,     /* a pointer is not 16-byte aligned */
    TMAN_ERR_LAUNCH = -7,    /* the HIP runtime reported an error when launching */
    TMAN_ERR_HEADER = -8     /* a packed blob's header disagrees with the shape it is used with */
} tman_status;

#define TMAN_FLAG_HAS_ZERO 1 /* weights carry a per-group zero point (affine form) */

/*
 * Problem statement (Sec. 4.1: weights (M, K), activations (N, K); Sec. 2.2 for the formats):
 *   W has M rows (output features) and K columns (input features); code q[m][k] is an unsigned
 *   integer below 2^bits; along K the codes are grouped in blocks of `group` that share one fp16
 *   scale and (flag HAS_ZERO) one fp16 zero point.
 *     HAS_ZERO set:   w[m][k] = (q[m][k] - zero[m][k/group]) * scale[m][k/group]    (Sec. 2.2)
 *     HAS_ZERO clear: w[m][k] = (2 q[m][k] - 1) * scale[m][k/group]                 (sign plane; bits must be 1)
 */
typedef struct tman_shape {
    int32_t M;
    int32_t K;
    int32_t bits;  /* 1, 2 or 4 */
    int32_t group; /* quantization block size along K: 32, 64 or 128; K % group == 0 */
    int32_t flags; /* TMAN_FLAG_* */
} tman_shape_t;

/* Maximum number of tokens one tman_mpgemv call (and one lookup-table buffer) serves. */
#define TMAN_MAX_DECODE_TOKENS 8

/* Size queries (host only, no GPU needed).  Return 0 for an invalid shape / N. */
size_t tman_packed_bytes(const tman_shape_t *shape);
size_t tman_lut_bytes(int32_t N, int32_t K, int32_t group);
size_t tman_mpgemv_workspace_bytes(const tman_shape_t *shape, int32_t N);
size_t tman_mpgemm_workspace_bytes(const tman_shape_t *shape, int32_t N);

/*
 * Offline weight repacking (Sec. 4.1 "Unified Layout": decoding's bit-serial packing is the stored
 * form, pre-permuted so that both kernels fetch contiguous blocks).
 *   codes  : uint8 [M][K], one code per byte (bits above `bits` are ignored)
 *   scales : fp16  [M][K/group]
 *   zeros  : fp16  [M][K/group], required iff HAS_ZERO, must be NULL otherwise
 *   packed : tman_packed_bytes(shape) bytes, 16-byte aligned; fully overwritten (padding is zeroed)
 * The result is position independent (may be copied, saved and reloaded) and starts with a 128-byte
 * header recording the shape.  Layout: rows in blocks of 64, columns in tiles of 128; inside a tile
 * block lane (row % 64) owns the 128 weights of its row, stored as `bits` 16-byte
 * chunks (one 1024-byte coalesced sub-block per chunk index) whose 32-bit words are single bit-planes
 * of 32 consecutive weights (weight t of a 4-bit lookup index in bit t, Sec. 4.1 "Bit repacking"),
 * followed by the lane's group scales/zeros.
 */
int tman_pack_weights(const tman_shape_t *shape, const uint8_t *codes, const void *scales, const void *zeros,
                      void *packed, void *stream);

/* Inverse of tman_pack_weights (test aid and format check): recovers codes [M][K] and, when the
 * pointers are non-NULL, scales / zeros [M][K/group]. */
int tman_unpack_weights(const tman_shape_t *shape, const void *packed, uint8_t *codes, void *scales, void *zeros,
                        void *stream);

/*
 * Lookup-table precompute (Sec. 2.2 "Bit-serial table lookup"; Sec. 5 "Graph optimization": the
 * precompute is a call of its own so layers fed by the same activation share one table).
 *   x   : fp16 [N][K], 1 <= N <= TMAN_MAX_DECODE_TOKENS
 *   lut : tman_lut_bytes(N, K, group) bytes, 16-byte aligned.  Receives, for every group of 4
 *         consecutive activations j and every 4-bit pattern p, the fp16 entry
 *         T[n][j][p] = sum_{t<4, bit t of p set} x[n][4j+t]   (fp32 sum, ascending t, one rounding),
 *         followed by the fp32 sums S[n][G] of x over each quantization block G of `group` columns
 *         (used for the zero-point term).  Entries for tokens / columns beyond N / K are zero.
 * The buffer may be passed to any number of tman_mpgemv calls with the same K and group.
 */
int tman_build_lut(const void *x, int32_t N, int32_t K, int32_t group, void *lut, void *stream);

/* The same for `count` activations (the distinct inputs of a decode step) in one launch.  `x`, `K` and
 * `lut` are HOST arrays of `count` entries (x[i], lut[i] device pointers); all share N and group. */
int tman_build_lut_batch(int32_t count, const void *const *x, int32_t N, const int32_t *K, int32_t group,
                         void *const *lut, void *stream);

/*
 * Decoding mpGEMV through table lookup (Sec. 2.2, Sec. 4.3):
 *   y[n][m] = sum_G scale[m][G] * ( sum_i 2^i sum_{j in G} T[n][j][idx_i[m][j]] - zero[m][G] * S[n][G] )
 * where idx_i[m][j] is the 4-bit pattern of bit-plane i over weights 4j..4j+3 (sign form:
 * scale * (2 * sum_j T - S)).  fp16 table entries, fp32 accumulation, fp16 result.
 *   packed    : from tman_pack_weights for the same shape
 *   lut       : from tman_build_lut(x, N, shape->K, shape->group)
 *   y         : fp16 [N][M]
 *   workspace : tman_mpgemv_workspace_bytes(shape, N) bytes, 16-byte aligned.  It must be zero-filled
 *               once before its first use; every call leaves it ready for the next one.  Calls that
 *               may overlap in time need separate workspaces.
 * Deterministic: the same inputs give bit-identical outputs on every call.
 */
int tman_mpgemv(const tman_shape_t *shape, const void *packed, const void *lut, int32_t N, void *y, void *workspace,
                size_t workspace_bytes, void *stream);

/*
 * Several decoding GEMVs in one launch (Sec. 5 "Graph optimization": layers fed by one activation
 * share one table; the layers of a decode step are too short to be launched one by one).  All
 * GEMVs of a batch have the same bits / group / flags and the same N; each has its own packed
 * weights, lookup-table buffer (buffers may repeat: Q/K/V, gate/up), output and workspace.
 *
 * tman_mpgemv_batch_prepare writes a descriptor table of tman_mpgemv_batch_desc_bytes(count) bytes
 * into `desc` (device memory, 16-byte aligned).  `shapes`, `packed`, `lut`, `y`, `workspace` and
 * `workspace_bytes` are HOST arrays of `count` entries (the entries of all but `shapes` and
 * `workspace_bytes` are device pointers); workspace[i] must hold
 * tman_mpgemv_workspace_bytes(&shapes[i], N) zero-filled bytes and must not be shared between
 * GEMVs.  The table stays valid while those device buffers stay where they are, so it is built once
 * and reused for every decode step.
 * tman_mpgemv_batch_run launches the batch described by `desc`; `count`, `shapes` and `N` must be the
 * ones given to prepare.  Results are identical to `count` separate tman_mpgemv calls up to the
 * order of the fp32 additions across K, and deterministic for a given batch.
 */
#define TMAN_MAX_BATCH 256
size_t tman_mpgemv_batch_desc_bytes(int32_t count);
int tman_mpgemv_batch_prepare(int32_t count, const tman_shape_t *shapes, const void *const *packed,
                              const void *const *lut, int32_t N, void *const *y, void *const *workspace,
                              const size_t *workspace_bytes, void *desc, void *stream);
int tman_mpgemv_batch_run(int32_t count, const tman_shape_t *shapes, int32_t N, const void *desc, void *stream);

/*
 * Integer activations and integer tables (Sec. 6.1 "A_INT16"; Sec. 4.3 two-level tiling: looked-up entries are
 * aggregated at low precision inside a quantization block, in floating point only across blocks; Sec. 5: 16-bit
 * table entries).  The paper gives no quantizer; this library's reading: token n gets the power-of-two step
 * 2^e[n], the smallest with max_k |x[n][k]| / 2^e[n] <= 8191, and integer activations
 * xq[n][k] = round_to_nearest_even(x[n][k] / 2^e[n]) -- 14-bit magnitudes, so that every table entry
 *   Tq[n][j][p] = sum_{t<4, bit t of p} xq[n][4j+t]
 * is an exact 16-bit integer.  tman_mpgemv_i16 then computes
 *   y[n][m] = 2^e[n] * sum_G scale[m][G] * ( sum_i 2^i sum_{j in G} Tq[n][j][idx_i[m][j]] - zero[m][G] * Sq[n][G] )
 * with the inner sums and Sq[n][G] = sum_{k in G} xq[n][k] as exact integers (sign form: scale * (2 sum - Sq)), the
 * scales applied in fp32, fp16 result: the exact product of the weights with the activations xq * 2^e up to the
 * fp32 sum across blocks and the final rounding.  Activations must be finite.
 *   tman_build_lut_i16 : x fp16 [N][K], 1 <= N <= 8 -> lut (tman_lut_i16_bytes(N, K, group) bytes, 16-byte
 *                        aligned): int16 entries laid out as the fp16 tables, int32 block sums, int32 e[n].
 *                        The _batch form follows tman_build_lut_batch.
 *   tman_mpgemv_i16    : arguments, workspace rules and determinism of tman_mpgemv, `lut` from tman_build_lut_i16.
 *   tman_mpgemv_i16_batch_run : launches a batch whose descriptor table tman_mpgemv_batch_prepare wrote with
 *                        integer table buffers in `lut` (the two table buffers have the same geometry).
 */
size_t tman_lut_i16_bytes(int32_t N, int32_t K, int32_t group);
int tman_build_lut_i16(const void *x, int32_t N, int32_t K, int32_t group, void *lut, void *stream);
int tman_build_lut_i16_batch(int32_t count, const void *const *x, int32_t N, const int32_t *K, int32_t group,
                             void *const *lut, void *stream);
int tman_mpgemv_i16(const tman_shape_t *shape, const void *packed, const void *lut, int32_t N, void *y, void *workspace,
                    size_t workspace_bytes, void *stream);
int tman_mpgemv_i16_batch_run(int32_t count, const tman_shape_t *shapes, int32_t N, const void *desc, void *stream);

/*
 * Decoding mpGEMV of ONE token with the table precompute inside the lookup kernel (Sec. 2.2, Sec. 4.3 for
 * the lookups; Sec. 5 moves the precompute into a kernel of its own because it is costly on the paper's
 * hardware, whereas here a kernel boundary costs more than the precompute).  Every workgroup builds the
 * tables of its own K segment (at most 4096 columns: 1024 tables, 32 KB) in LDS from the activations,
 * exactly as tman_build_lut computes them (fp32 sums in ascending order, one rounding to fp16; the same
 * group sums), and then performs the same lookups as tman_mpgemv.  The result is what
 * tman_build_lut + tman_mpgemv give for N = 1, up to the order of the fp32 additions across K.
 *   x         : fp16 [K], device, 16-byte aligned
 *   y         : fp16 [M]
 *   workspace : tman_mpgemv_workspace_bytes(shape, 1) bytes, under the rules of tman_mpgemv (the size for
 *               N = 1 covers both calls, but a workspace is used by one call at a time)
 * The batch forms follow tman_mpgemv_batch_prepare / _run with `x` in place of `lut` (entries may repeat:
 * Q/K/V, gate/up) and N fixed to 1; a descriptor table made by one prepare call is only valid for the run
 * call of the same kind.
 */
int tman_mpgemv_x(const tman_shape_t *shape, const void *packed, const void *x, void *y, void *workspace,
                  size_t workspace_bytes, void *stream);
int tman_mpgemv_x_batch_prepare(int32_t count, const tman_shape_t *shapes, const void *const *packed,
                                const void *const *x, void *const *y, void *const *workspace,
                                const size_t *workspace_bytes, void *desc, void *stream);
int tman_mpgemv_x_batch_run(int32_t count, const tman_shape_t *shapes, const void *desc, void *stream);
/*
 * Balance.  A batch of up to 8 GEMVs whose workgroups (one per 64-row block and K segment) are all resident at
 * once -- at most 8 per compute unit, fewer when the tables of the longest segment take more LDS -- is launched
 * as a one-dimensional grid whose workgroup ids the library assigns: on this chip a launch that fits is dealt out
 * by position, workgroup i to compute unit i mod (number of units), so the numbering decides which workgroups
 * share a unit, and it is chosen so that every unit gets the same number of tile blocks (tiling.decode_balance;
 * the numbering is part of the descriptor table).  Results do not depend on it.
 * tman_mpgemv_x_batch_order returns that numbering without touching the device: `n_units` compute units (0: the
 * current device's); order[i] = (GEMV << 13) | (workgroup of the GEMV: row block * segments + segment) for
 * workgroup id i, room for `max_entries` (order may be NULL to count only), the number of workgroups in
 * *n_entries -- 0 when the batch is launched as a plain grid (GEMVs) x (workgroups of the largest).
 */
int tman_mpgemv_x_batch_order(int32_t count, const tman_shape_t *shapes, int32_t n_units, uint16_t *order,
                              int32_t max_entries, int32_t *n_entries);

/*
 * Packed blobs carry a 128-byte header (shape, tile geometry, layout version).
 * tman_check_packed compares it with `shape` on the host: it copies the header back on `stream` and WAITS for
 * the stream (the one blocking call of the library; meant for load time).  TMAN_ERR_HEADER on disagreement.
 * The compute calls also check on the device: tman_mpgemv, tman_mpgemv_x and tman_mpgemm at kernel entry, the
 * batch forms when their descriptor table is prepared.  A GEMV whose blob disagrees with its shape is
 * skipped (its y is left untouched) and TMAN_ERR_HEADER is stored in a status word in device memory that
 * tman_device_status returns and clears (it waits for `stream`; TMAN_OK when nothing was reported).  The
 * device-side check protects results, not memory: the kernels size their reads from `shape`, so a blob that is
 * SMALLER than the shape says must be caught with tman_check_packed before it is used.
 */
int tman_check_packed(const tman_shape_t *shape, const void *packed, void *stream);
int tman_device_status(void *stream);

/*
 * mpGEMM on the matrix cores (Sec. 4.1 "Fused LUT-based dequantization", Sec. 4.2): bit-planes are repacked to
 * codes (level 1), each code is looked up in its quantization block's table
 * D[c] = fp16((c - zero) * scale) (level 2; sign form fp16((2c - 1) * scale)), and the fp16 weights
 * feed the matrix cores with fp32 accumulation.
 *   x : fp16 [N][K], any N >= 1;   y : fp16 [N][M]
 * Two kernels share the call.  N > TMAN_MAX_SMALL_TOKENS runs the tiled prefill kernel (256 tokens per
 * workgroup, bound by the matrix cores; it needs no workspace).  1 <= N <= TMAN_MAX_SMALL_TOKENS runs a kernel
 * organised like the decoding kernels (bound by the weight stream: every wave dequantizes the tile blocks it
 * streams and multiplies them with all tokens at once), which cuts a long K into segments that meet in the
 * workspace, under the rules of tman_mpgemv: tman_mpgemm_workspace_bytes(shape, N) bytes (0 when K is one
 * segment, then NULL is accepted), 16-byte aligned, zero-filled once before first use, left ready by every
 * call, not shared by calls that may overlap.  Deterministic.
 */
#define TMAN_MAX_SMALL_TOKENS 32
int tman_mpgemm(const tman_shape_t *shape, const void *packed, const void *x, int32_t N, void *y, void *workspace,
                size_t workspace_bytes, void *stream);

/*
 * Several small-batch mpGEMMs (the same N <= TMAN_MAX_SMALL_TOKENS, the same bits / group / flags) in one
 * launch, e.g. the linear layers of a decode step with a few tokens in flight (Sec. 5: layers fed by one
 * activation share it; here entries of `x` may repeat).  Arguments as for tman_mpgemv_batch_prepare / _run with
 * the activations `x` (fp16 [N][K] each) in place of the table buffers; workspace[i] may be NULL where
 * tman_mpgemm_workspace_bytes(&shapes[i], N) is 0; the descriptor table takes
 * tman_mpgemv_batch_desc_bytes(count) bytes.  Batches of up to 8 GEMMs whose workgroups are all resident at once
 * (four per compute unit) are numbered for balance like those of tman_mpgemv_x (tiling.decode_balance).
 */
int tman_mpgemm_batch_prepare(int32_t count, const tman_shape_t *shapes, const void *const *packed,
                              const void *const *x, int32_t N, void *const *y, void *const *workspace,
                              const size_t *workspace_bytes, void *desc, void *stream);
int tman_mpgemm_batch_run(int32_t count, const tman_shape_t *shapes, int32_t N, const void *desc, void *stream);

/*
 * mpGEMM on the INTEGER matrix cores for weights with one scale and one zero per row of W: per-channel formats,
 * and per-tensor ones such as BitNet's ternary weights as 2-bit codes (Sec. 6.1: "per-tensor quantization ...
 * treated as 2-bit"; Sec. 6.2 mpGEMM: "we dequantize to INT8 and perform computation with W_INT8 A_INT8").
 * The packed blob is the ordinary one; the call uses the scale and zero of the FIRST quantization block of every
 * row for the whole row, so it computes y = x * dequant(W)^T only for blobs whose rows repeat one (scale, zero)
 * pair over all their blocks (not checked).
 *   tman_quantize_act_i8 : x fp16 [N][K] (finite) -> xq, tman_act_i8_bytes(N, K) bytes, 16-byte aligned:
 *       per-token absmax quantization (the paper gives no quantizer; this is the one of the BitNet family):
 *       xq[n][k] = round_to_nearest_even(x[n][k] * (127 / max_k |x[n][k]|)), the decision taken in binary32
 *       (inv = 127.0f / max correctly rounded, t = x * inv correctly rounded, rint), stored as int8 [N][K] with
 *       every 32-column group permuted (byte p = 8 o + 4 h + b of a group holds column 8 b + 4 h + o; o < 4,
 *       h < 2, b < 4: the order in which the weights' codes leave the bit-plane transposition), then, each on a
 *       256-byte boundary, float max[N] and int32 sum_k xq[n][k].
 *   tman_mpgemm_i8 : acc[n][m] = sum_k code[m][k] * xq[n][k] on v_mfma_i32_32x32x32_i8 (exact), then
 *       y[n][m] = fp16( scale[m] * max[n] / 127 * (acc[n][m] - zero[m] * sum_k xq[n][k]) )   (sign form:
 *       scale * max / 127 * (2 acc - sum)), the scaling in fp32.  `acc`, if not NULL, receives the integer
 *       accumulators, int32 [N][M] (test aid).  Any N >= 1; K a multiple of 32; N * K < 2^32.
 */
size_t tman_act_i8_bytes(int32_t N, int32_t K);
int tman_quantize_act_i8(const void *x, int32_t N, int32_t K, void *xq, void *stream);
int tman_mpgemm_i8(const tman_shape_t *shape, const void *packed, const void *xq, int32_t N, void *y, int32_t *acc,
                   void *stream);

/*
 * Rows of W (output features) one workgroup of tman_mpgemm covers for this shape and N > 32: 64, 128, 192 or 256,
 * chosen so that the workgroups fill the compute units of the current device best (256 units are
 * assumed when no device is present).  tman_mpgemm_splits_k tells whether the call goes to the kernel whose waves
 * split K (1) or to the tiled kernel (0).  Informational; 0 / -1 for an invalid shape or N < 1.
 */
int32_t tman_mpgemm_tile_rows(const tman_shape_t *shape, int32_t N);
int32_t tman_mpgemm_splits_k(const tman_shape_t *shape, int32_t N);
/*
 * Which kernel tman_mpgemm_i8 runs for this shape and N, in the terms of tiling.i8_token_blocks: 1 = the kernel with
 * 128 x 128 tiles, 3 / 4 / 7 = the kernel whose workgroups take 256 rows x 96 / 128 / 224 tokens and dequantize in
 * registers, 9 = the kernel whose waves split K.  The choice models the time of the grids they give on the current device (256 units are assumed when
 * no device is present); a non-zero tiling.i8_token_blocks overrides it.  Informational; 0 for an invalid shape or
 * N < 1.
 */
int32_t tman_mpgemm_i8_token_blocks(const tman_shape_t *shape, int32_t N);

/*
 * tman_mpgemv for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as tman_mpgemv, but the
 * workspace (tickets and partial sums of the K segments) is a fixed array of TMAN_NOALLOC_SCRATCH_BYTES in
 * device memory that the library owns (each GPU the library runs on holds it until the process ends).  The
 * call allocates and frees nothing.
 *   - shapes / N whose tman_mpgemv_workspace_bytes exceeds TMAN_NOALLOC_SCRATCH_BYTES are refused with
 *     TMAN_ERR_WORKSPACE (nothing is launched);
 *   - every call on a GPU uses that GPU's one array: calls that may overlap in time on one GPU (different
 *     streams, or several host threads) race and must be serialised by the caller, or use tman_mpgemv
 *     with workspaces of their own;
 *   - the array keeps what the last call left: the tickets are back at zero after every call, the partial
 *     sums are overwritten before they are read, so nothing is cleared between calls.
 * tman_noalloc_init resolves the array's device address on the CURRENT device (the first
 * tman_mpgemv_noalloc call on a device does the same); call it once per device at set-up, outside any graph
 * capture.  Both return TMAN_ERR_LAUNCH when the HIP runtime cannot provide the address.
 */
#define TMAN_NOALLOC_SCRATCH_BYTES (2 * 1024 * 1024)
int tman_noalloc_init(void);
int tman_mpgemv_noalloc(const tman_shape_t *shape, const void *packed, const void *lut, int32_t N, void *y,
                        void *stream);

/*
 * The tiling (Sec. 4.1 "Unified tiling strategy", Eq. 1-4: tile sizes searched per machine under register /
 * on-chip-memory constraints, the prefill and the decoding loop nest covering the same M and K extents of the one
 * weight copy).  The shared tile block is fixed by the packed layout (64 rows x 128 columns, which is Eq. 2 and
 * Eq. 3 by construction); free is how many tile blocks one workgroup takes:
 *   decode_seg_tiles / _many   K tiles per workgroup of tman_mpgemv for 1-2 / 4-8 tokens
 *   decode_x_seg_tiles         tman_mpgemv_x: a K of at most this many tiles, and at most decode_x_whole_bytes of
 *                              packed weights per row block, is ONE segment; it is at most 32 (Eq. 1: the tables
 *                              of a segment, 1 KB per tile, live in the workgroup's 32 KB of LDS)
 *   decode_x_long_seg_tiles    ... a longer K is cut into equal segments of at most this many tiles
 *   decode_balance             1: batches of tman_mpgemv_x and of the small-batch tman_mpgemm number their
 *                              workgroups for equal work per compute unit (see tman_mpgemv_x_batch_order),
 *                              0: plain grids
 *   small_seg_tiles            K tiles per workgroup of tman_mpgemm for N <= 32
 *   prefill_row_blocks         tile blocks in M per workgroup of the tiled prefill kernel, 1..4 (Eq. 4: four
 *                              stage buffers of rows x 80 + 256 x 64 bytes within 160 KB of LDS), 0 = chosen per
 *                              call from the grid it gives
 *   prefill_k_split            tman_mpgemm for N > 32: a grid that leaves compute units idle even with one tile block per
 *                              workgroup goes to a kernel whose four waves split K (each dequantizes its own stages in
 *                              registers; the partial sums meet in LDS in a fixed order): 0 = there, when K >= 2048,
 *                              with the tile chosen per call; 1 = never; 2 / 3 = every call, with the 64 rows x 256
 *                              tokens / 128 rows x 128 tokens tile
 *   i8_token_blocks            tman_mpgemm_i8: 1 = the kernel with 128 x 128 tiles (weights and activations through
 *                              LDS), 3 / 4 / 7 = the kernel whose waves dequantize their own 64 rows in registers and
 *                              share 96 / 128 / 224 tokens of activations through LDS, 9 = the kernel whose four waves
 *                              split K (128 rows x 128 tokens per workgroup, for small grids), 0 = chosen per call
 *                              from the grids they give
 * tman_default_tiling gives the built-in values (the best of the measured sweep paper_2511_11248_amd/tune.py
 * makes on the device), tman_get_tiling the current ones; tman_set_tiling checks the constraints
 * (TMAN_ERR_SHAPE if violated) and makes the values current for all later calls of the process.  The tiling
 * enters the workspace size queries and the descriptor tables: set it before sizing workspaces and preparing
 * batches, not between a prepare and its runs.
 */
typedef struct tman_tiling {
    int32_t decode_seg_tiles;
    int32_t decode_seg_tiles_many;
    int32_t decode_x_seg_tiles;
    int32_t decode_x_long_seg_tiles;
    int32_t decode_x_whole_bytes;
    int32_t small_seg_tiles;
    int32_t prefill_row_blocks;
    int32_t decode_balance;
    int32_t i8_token_blocks;
    int32_t prefill_k_split;
} tman_tiling_t;
int tman_default_tiling(tman_tiling_t *out);
int tman_get_tiling(tman_tiling_t *out);
int tman_set_tiling(const tman_tiling_t *tiling);

/* Static, human-readable name of a status code. */
const char *tman_status_string(int status);

/* Layout version of the packed format this build reads and writes (also stored in the header). */
int32_t tman_layout_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TMAN_H */
