// Prefill mpGEMM: two-level dequantization fused in front of the matrix cores
// (Sec. 4.1 "Unified Layout through Fused LUT-based Dequantization", Sec. 4.2 three-stage pipeline).
//
// The weights stay in the bit-serial layout decoding uses (lane = row, 64 rows x 128 columns per tile
// block).  Per 32-column stage a producer wave turns the bit-plane words of its 64 rows into fp16 weights:
//   level 1  bit-serial -> bit-parallel (Sec. 4.1 "Bit repacking"): two rounds of bit-field inserts
//            transpose a 4 x 32 bit matrix in 16 ALU ops, giving for each 32-weight block four words
//            of eight 4-bit codes, word o holding the codes of weights 4f + o;
//   level 2  code -> fp16 weight with the block's scale and zero baked in (Sec. 4.1 "Integer-to-float
//            conversion", "Applying scales and zero-points").  The 16-entry conversion table of the
//            paper collapses on this hardware to inserting the code into the mantissa of 1024.0
//            (fp16 0x6400 | c == 1024 + c exactly), and the baked affine table entry
//            D[c] = fp16((c - zero) * scale) is produced by ONE mixed-precision FMA
//            fp16( (1024 + c) * scale - (1024 + zero) * scale ): product and sum are exact inside the FMA
//            and rounded to fp16 once; the per-block constant -(1024 + zero) * scale, computed once per block,
//            is rounded to fp32 before (it has up to 24 significant bits), which moves the result by at most
//            2^-23 * 1040 * scale ahead of that rounding: about 5 % of the entries come out one fp16 step
//            from fp16((c - zero) * scale).
//            A lookup per weight in LDS would compete with the MFMA operand reads for LDS bandwidth.
// The fp16 weight tile goes to LDS and is shared by the waves of the workgroup (each weight is
// dequantized once per 256 tokens); activations go from global memory straight into LDS.  Pipeline (the
// GPU form of DMA -> vector -> matrix): producer waves keep packed weights four stages ahead in registers
// and fill a ring of four LDS stage buffers; consumer waves feed v_mfma_f32_32x32x16_f16
// (fp32 accumulation) from the ring; one barrier per 32-column stage.
// Grids too small for that kernel (at most one workgroup per compute unit) go to mpgemm_ksplit_kernel, below.
#include <hip/hip_fp16.h>

#include <mutex>

#include "tman_dequant_device.h"

namespace tman {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTN = 256;      // tokens per workgroup
constexpr int kStageK = 32;   // columns per pipeline stage (one 32-weight block of the layout)
constexpr int kRowBytes = kStageK * 2 + 16;  // padded LDS row: 20 dwords, conflict-free 16-byte accesses
constexpr int kRing = 4;      // stage buffers in LDS
constexpr int kSets = 4;      // register sets of the producers = stages of global loads in flight
constexpr int kXcds = 8;      // workgroups are dealt to the chip's 8 XCDs (one L2 each) round robin

// A workgroup covers RB row blocks (64 * RB output features) x 256 tokens; RB = 1 .. 4 is chosen
// per call so that the number of workgroups fills the compute units best.
template <int RB>
struct Tile {
    static constexpr int TM = RB * 64;
    static constexpr int WBytes = TM * kRowBytes;    // fp16 weights of a stage, padded rows
    static constexpr int XBytes = kTN * kStageK * 2; // activations of a stage, 64-byte rows, chunks swizzled
    static constexpr int StageBytes = WBytes + XBytes;
    static constexpr int OutRow = TM * 2 + 16;       // bytes per token of the output tile in LDS
    static constexpr int LdsBytes = kRing * StageBytes > kTN * OutRow ? kRing * StageBytes : kTN * OutRow;
};

struct GemmArgs {
    const uint8_t* tiles;
    const _Float16* x;
    _Float16* y;
    int M, N, K, n_row_blocks, n_ktiles;
    int m_tiles, n_tiles;
    int* status;  // the library's status word
};

typedef __amdgpu_buffer_rsrc_t rsrc_t;
// raw buffer resource: loads at or beyond `bytes` return zero
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// Loads 32-weight block `kb32` of tile block `tile` of this wave's row block.  `rw` covers the row
// block's tiles or nothing (rows beyond M, stages beyond K), in which case everything reads as zero.
template <int B, int GQ, bool HZ>
__device__ __forceinline__ void load_w(WRegs<B>& r, rsrc_t rw, int tile, int kb32, int lane) {
    constexpr int CH = kKTile / B;
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int MPL = (kKTile / GQ) * MSZ;
    constexpr int TB = B * 1024 + 64 * MPL;
    const int v = (kb32 * 32) / CH, ksub = ((kb32 * 32) % CH) / 32;
    const int so = tile * TB + v * 1024 + ksub * B * 4;
    if constexpr (B == 4) {
        const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(rw, lane * 16, so, 0);
        r.plane[0] = w.x; r.plane[1] = w.y; r.plane[2] = w.z; r.plane[3] = w.w;
    } else if constexpr (B == 2) {
        const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rw, lane * 16, so, 0);
        r.plane[0] = w.x; r.plane[1] = w.y;
    } else {
        r.plane[0] = __builtin_amdgcn_raw_buffer_load_b32(rw, lane * 16, so, 0);
    }
    const int mo = tile * TB + B * 1024 + ((kb32 * 32) / GQ) * MSZ;
    if constexpr (HZ) r.meta = __builtin_amdgcn_raw_buffer_load_b32(rw, lane * MPL, mo, 0);
    else r.meta = __builtin_amdgcn_raw_buffer_load_b16(rw, lane * MPL, mo, 0);
}

// Activation staging: the 64 bytes a token contributes to a stage are four 16-byte chunks.  They go
// from global memory straight into LDS (no registers, no LDS store instruction); such a load writes
// the 64 lanes' 16 bytes consecutively, i.e. 16 token rows of 64 bytes per wave instruction.  Rows are
// not padded, so chunk c of token row R is kept at position c ^ ((R >> 2) & 3) of its row: the MFMA
// operand reads of 16 consecutive rows then fall into 16 different 16-byte bank groups.  The
// permutation is applied on the global-address side, where every lane is free to pick its source.

// Workgroup = 12 waves, three per SIMD.  Waves 0..7 are consumers: wave (wm, wn) owns 32 RB rows x 64
// tokens of the tile and does nothing but read MFMA operands from LDS and issue MFMAs.  Waves 8..11
// are producers: wave p < RB turns row block p of each stage into fp16 in LDS, and all four stage the
// activations.  Vector work of the producers and matrix work of the consumers come from different
// waves of a SIMD, so the hardware overlaps them without any help from the instruction schedule.
//
// Ring protocol, one barrier at the end of every stage s: before it the producers have written stage
// s+2 and the consumers have finished reading stage s.  Hence consumers may prefetch operands of stage
// s+1 during stage s, and the buffer written during stage s (stage s+2) was last read in stage s-2.
// The producers hold the global loads of four further stages in registers: at the rates of this kernel
// that many bytes in flight are needed to cover the latency of HBM and L2.
constexpr int kConsumerWaves = 8;
constexpr int kThreads = 768;

template <int B, int GQ, bool HZ, int RB>
__global__ void __launch_bounds__(kThreads, 1) mpgemm_kernel(GemmArgs a) {
    using T = Tile<RB>;
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int TB = B * 1024 + 64 * (kKTile / GQ) * MSZ;

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // Tile of this workgroup.  Consecutive workgroup ids go to consecutive XCDs; the n_tiles workgroups
    // that share the weights of one row tile get ids that are 8 apart, i.e. the same XCD and L2.
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int mt = (slot / a.n_tiles) * kXcds + xcd, nt = slot % a.n_tiles;
    // A blob packed for another shape or layout: say so and leave y alone.  (The check is folded into the one
    // exit below: a second exit after this load makes the compiler keep the dequantization state in scratch
    // memory.)
    const bool header_ok = header_matches(a.tiles, a.M, a.K, B, GQ, HZ ? 1 : 0);
    if (!header_ok && blockIdx.x == 0 && threadIdx.x == 0) report_header_mismatch(a.status);
    if (mt >= (header_ok ? a.m_tiles : 0)) return;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int n0 = nt * kTN;
    // K is a multiple of the quantization group, hence of 32.  The loops run a multiple of four stages
    // (no conditional code between the loads and their use); a stage beyond K holds zero activations.
    // (Eight with one row block, whose producers work in rounds of eight stages.)
    constexpr int kRound = RB == 1 ? 2 * kSets : kSets;
    const int k_stages = a.K / kStageK, n_stages = (k_stages + kRound - 1) & ~(kRound - 1);

    float16_t acc[RB][2];
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;
    const int wm = (wave >> 2) & 1, wn = wave & 3, r = lane & 31, h = lane >> 5;

    if (wave >= kConsumerWaves) {
        // ---------------------------------------------------------------- producer
        const int p = wave - kConsumerWaves;
        // the row block this wave dequantizes (with one row block per workgroup waves 0 and 1 share it)
        const int pb = RB == 1 ? 0 : p;
        const int rbw = mt * RB + pb;
        // the producers' short vector bursts gate every stage: issue them ahead of the consumers' MFMAs
        __builtin_amdgcn_s_setprio(3);
        const bool wvalid = (RB == 1 ? p < 2 : p < RB) && rbw < a.n_row_blocks;
        const uint8_t* wsrc = a.tiles + (size_t)(wvalid ? rbw : 0) * a.n_ktiles * TB;
        const int xrows = a.N - n0 < kTN ? a.N - n0 : kTN;
        const _Float16* xsrc = a.x + (size_t)n0 * a.K;
        const uint32_t xbytes = (uint32_t)xrows * (uint32_t)a.K * 2u;
        // Roles.  With four row blocks every producer wave dequantizes one and issues a quarter of the
        // activation loads.  With fewer, wave 3 has no row block: it issues all activation loads (about 40
        // cycles each) and the dequantizing waves none, which shortens the chain that gates a stage.
        constexpr bool kSplitRoles = RB < 4;
        constexpr int kLoaderWave = 3;
        constexpr int kXAll = kTN / 16;  // activation loads of a stage (16 token rows each)
        const uint32_t xlane = ((lane >> 2) * (uint32_t)a.K + ((lane & 3) ^ ((lane >> 4) & 3)) * 8u) * 2u;
        const uint32_t x16rows = 16u * (uint32_t)a.K * 2u;  // bytes between the sources of consecutive loads
        // load number i of a stage fills token rows 16 i .. 16 i + 15; lane = 4 * row + position
        auto load_x = [&](int t, int first, int count) {
            const rsrc_t rx = make_rsrc(xsrc, t < k_stages ? xbytes : 0u);
            uint8_t* dst = smem + (t & (kRing - 1)) * T::StageBytes + T::WBytes;
#pragma unroll
            for (int i = 0; i < kXAll; ++i)
                if (i < count)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(dst + (first + i) * 1024),
                                                             16, xlane + (uint32_t)(first + i) * x16rows, t * kStageK * 2, 0, 0);
        };
        const int wdst = (pb * 64 + lane) * kRowBytes;  // this lane's 64 bytes in the weight tile

        WRegs<B> wr[kSets];
        // stage t: packed weights global -> register set (a wave without a row block reads nothing)
        auto load_wregs = [&](int set, int t) {
            load_w<B, GQ, HZ>(wr[set], make_rsrc(wsrc, t < k_stages && wvalid ? 0x7fffffffu : 0u), t >> 2, t & 3, lane);
        };
        auto w_to_lds = [&](int set, int t) {
            if (p < RB) dequant_to_lds<B, HZ>(wr[set], smem + (t & (kRing - 1)) * T::StageBytes + wdst);
        };
        // Ring timing, any role: during stage s the activations of stage s+3 are requested (that buffer
        // was last read in stage s-1), the weights of stage s+2 go registers -> ring and the weights of
        // stage s+6 global -> the same registers.  Loads complete in order.  Before the barrier of stage
        // s the activations of stage s+2 must have landed; they were issued first in stage s-1.
        if (kSplitRoles && p == kLoaderWave) {
            load_x(0, 0, kXAll);
            load_x(1, 0, kXAll);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            load_x(2, 0, kXAll);
            asm volatile("s_barrier" ::: "memory");
            for (int s = 0; s < n_stages; ++s) {
                load_x(s + 3, 0, kXAll);
                // younger than the loads of stage s+2: the sixteen just issued
                asm volatile("s_waitcnt vmcnt(16)\n\ts_barrier" ::: "memory");
            }
        } else if constexpr (RB == 1) {
            if (p < 2) {
                // One row block: a stage is short, and what gates it is the chain load -> dequantize ->
                // write -> barrier of a single wave.  Waves 0 and 1 take the even and the odd stages and
                // spread the work of a stage over two stage slots (codes -> fp16 integers in registers
                // during the first, the FMAs and the LDS writes during the second), in antiphase: in every
                // slot one of them is in its first half and the other in its second.  Stage t is written
                // during stage t-2, like in the other roles.
                const uint32_t wlive = wvalid ? 0x7fffffffu : 0u;
                uint8_t* const wrow = smem + wdst;
                Dequant<B, HZ> dq;
                auto load_own = [&](int set, int t) {  // t: a stage of this wave (p, p + 2, ...)
                    load_w<B, GQ, HZ>(wr[set], make_rsrc(wsrc, t < k_stages ? wlive : 0u), t >> 2, t & 3, lane);
                };
                auto first_half = [&](int set) {
                    dq.start(wr[set]);
                    dq.insert();
                };
                auto second_half = [&](int t) {
                    uint8_t* dst = wrow + (t & (kRing - 1)) * T::StageBytes;
#pragma unroll
                    for (int q = 0; q < 4; ++q) dq.emit(q, dst);
                };
                // prologue: this wave's first stage complete in the ring, its next four in the register sets;
                // wave 0 also has the first half of stage 2 done
#pragma unroll
                for (int i = 0; i < kSets; ++i) load_own(i, p + 2 * i);
                first_half(0);
                second_half(p);
                __builtin_amdgcn_sched_barrier(0);
                load_own(0, p + 2 * kSets);
                if (p == 0) {
                    first_half(1);
                    __builtin_amdgcn_sched_barrier(0);
                    load_own(1, 2 + 2 * kSets);
                }
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                // slots t (even) and t + 1.  Wave 0: second half of stage t+2, then first half of t+4.
                // Wave 1: first half of stage t+3, then its second half.
                if (p == 0) {
                    for (int s = 0; s < n_stages; s += 2 * kSets) {
#pragma unroll
                        for (int u = 0; u < kSets; ++u) {
                            const int t = s + 2 * u;
                            second_half(t + 2);
                            __builtin_amdgcn_sched_barrier(0);
                            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                            first_half((u + 2) % kSets);  // stage t + 4, the wave's stage number t / 2 + 2
                            __builtin_amdgcn_sched_barrier(0);
                            load_own((u + 2) % kSets, t + 4 + 2 * kSets);
                            __builtin_amdgcn_sched_barrier(0);
                            asm volatile("s_barrier" ::: "memory");
                        }
                    }
                } else {
                    for (int s = 0; s < n_stages; s += 2 * kSets) {
#pragma unroll
                        for (int u = 0; u < kSets; ++u) {
                            const int t = s + 2 * u;
                            first_half((u + 1) % kSets);  // stage t + 3, the wave's stage number t / 2 + 1
                            __builtin_amdgcn_sched_barrier(0);
                            load_own((u + 1) % kSets, t + 3 + 2 * kSets);
                            __builtin_amdgcn_sched_barrier(0);
                            asm volatile("s_barrier" ::: "memory");
                            second_half(t + 3);
                            __builtin_amdgcn_sched_barrier(0);
                            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                        }
                    }
                }
            } else {  // wave 2 has no work: it only keeps the barriers
                asm volatile("s_barrier" ::: "memory");
                for (int s = 0; s < n_stages; ++s) asm volatile("s_barrier" ::: "memory");
            }
        } else if (kSplitRoles) {
            load_wregs(0, 0);
            load_wregs(1, 1);
            load_wregs(2, 2);
            load_wregs(3, 3);
            w_to_lds(0, 0);
            w_to_lds(1, 1);
            __builtin_amdgcn_sched_barrier(0);
            load_wregs(0, 4);
            load_wregs(1, 5);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            for (int s = 0; s < n_stages; s += kSets) {
#pragma unroll
                for (int u = 0; u < kSets; ++u) {
                    w_to_lds((u + 2) % kSets, s + u + 2);
                    __builtin_amdgcn_sched_barrier(0);
                    load_wregs((u + 2) % kSets, s + u + 6);
                    __builtin_amdgcn_sched_barrier(0);
                    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                }
            }
        } else {
            // prologue: stages 0 and 1 complete in the ring, activations of stage 2 on their way, weights
            // of stages 2..5 in the register sets 2, 3, 0, 1
            load_x(0, 4 * p, 4);
            load_x(1, 4 * p, 4);
            load_wregs(0, 0);
            load_wregs(1, 1);
            load_wregs(2, 2);
            load_wregs(3, 3);
            w_to_lds(0, 0);
            w_to_lds(1, 1);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt vmcnt(4)" ::: "memory");  // all but the weights of stages 2 and 3 (two loads each)
            load_x(2, 4 * p, 4);
            load_wregs(0, 4);
            load_wregs(1, 5);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            for (int s = 0; s < n_stages; s += kSets) {
#pragma unroll
                for (int u = 0; u < kSets; ++u) {
                    load_x(s + u + 3, 4 * p, 4);
                    __builtin_amdgcn_sched_barrier(0);
                    w_to_lds((u + 2) % kSets, s + u + 2);
                    __builtin_amdgcn_sched_barrier(0);
                    load_wregs((u + 2) % kSets, s + u + 6);
                    __builtin_amdgcn_sched_barrier(0);
                    // younger than the activation loads of stage s+2: 2 weight loads of stage s-1, 4
                    // activation loads and 2 weight loads of stage s
                    asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
                }
            }
        }
        // Loads of stages past the end (zero-sized sources: they write zeros) may still be on their way to
        // LDS, which the epilogue reuses: they must have landed before any wave passes the barrier below.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        // ---------------------------------------------------------------- consumer
        // MFMA operand addresses: lanes with h = 0 / 1 take the two 8-column groups of a 16-column step
        const int wfrag = (wm * RB * 32 + r) * kRowBytes + h * 16;
        // activation operand: token row wn * 64 + nb * 32 + r, chunk 2j + h, kept at chunk ^ ((r >> 2) & 3)
        const int xrow = T::WBytes + (wn * 64 + r) * (kStageK * 2);
        const int xchunk[2] = {xrow + ((h ^ ((r >> 2) & 3)) * 16), xrow + (((2 + h) ^ ((r >> 2) & 3)) * 16)};
        // Operand registers: one weight operand per 32-row block, reloaded for the next 16-column step
        // as soon as its two MFMAs are issued (so the read has the other blocks' MFMAs to land), and two
        // pairs of activation operands (this step's and the next one's).
        half8_t wf[RB], xf[2][2];
        auto read_w = [&](int mb, const uint8_t* stage, int j) {
            wf[mb] = *reinterpret_cast<const half8_t*>(stage + wfrag + mb * 32 * kRowBytes + j * 32);
        };
        auto read_x = [&](int set, const uint8_t* stage, int j) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                xf[set][nb] = *reinterpret_cast<const half8_t*>(stage + xchunk[j] + nb * 32 * (kStageK * 2));
        };
        __syncthreads();
        read_x(0, smem, 0);
#pragma unroll
        for (int mb = 0; mb < RB; ++mb) read_w(mb, smem, 0);
        for (int s = 0; s < k_stages; ++s) {
            const uint8_t* cur = smem + (s & (kRing - 1)) * T::StageBytes;
            const uint8_t* nxt = smem + ((s + 1) & (kRing - 1)) * T::StageBytes;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                // operands after this step: step 1 of this stage, or step 0 of stage s+1, which is complete
                // in the ring (past the last stage this reads stale LDS that is never used)
                const uint8_t* ahead = j == 0 ? cur : nxt;
                read_x(j ^ 1, ahead, j ^ 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mb = 0; mb < RB; ++mb) {
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[mb], xf[j][nb], acc[mb][nb], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    read_w(mb, ahead, j ^ 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // Plain barrier: this wave has no LDS writes to publish, and its outstanding reads (stage
            // s+1) need not land before it; everything it read from stage s has been consumed.
            asm volatile("s_barrier" ::: "memory");
        }
        // the producers run a multiple of four stages; meet them at the barriers of the padding stages
        for (int s = k_stages; s < n_stages; ++s) asm volatile("s_barrier" ::: "memory");
    }

    // epilogue: accumulators -> fp16 -> LDS as [token][row] -> coalesced 16-byte stores
    // C[i][j] of a 32x32 block: i = row (8 * (v / 4) + 4 * h + v % 4), j = token (lane % 32)
    // One more barrier between the last stage and the epilogue: the consumers leave the last stage barrier
    // while activation loads of the padding stages, issued by the producers, can still be writing to the ring.
    __syncthreads();
    uint8_t* otile = smem;  // the stage buffers are free now
    if (wave < kConsumerWaves) {
#pragma unroll
        for (int mb = 0; mb < RB; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                uint8_t* col = otile + (wn * 64 + nb * 32 + r) * T::OutRow + ((wm * RB + mb) * 32 + 4 * h) * 2;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    half2_t lo, hi;
                    lo.x = (_Float16)acc[mb][nb][4 * g + 0];
                    lo.y = (_Float16)acc[mb][nb][4 * g + 1];
                    hi.x = (_Float16)acc[mb][nb][4 * g + 2];
                    hi.y = (_Float16)acc[mb][nb][4 * g + 3];
                    u32x2 w = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
                    *reinterpret_cast<u32x2*>(col + g * 16) = w;  // rows 8g + 4h + 0..3
                }
            }
    }
    __syncthreads();
    const int m0 = mt * T::TM;
    const bool fast = (a.M % 8 == 0);  // 16-byte aligned rows of y
    for (int piece = tid; piece < kTN * (T::TM / 8); piece += kThreads) {
        const int n = piece / (T::TM / 8), c8 = piece % (T::TM / 8);
        const int gn = n0 + n, gm = m0 + c8 * 8;
        if (gn >= a.N || gm >= a.M) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(otile + n * T::OutRow + c8 * 16);
        _Float16* dst = a.y + (size_t)gn * a.M + gm;
        if (fast && gm + 8 <= a.M) {
            *reinterpret_cast<u32x4*>(dst) = v;
        } else {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            for (int t = 0; t < 8 && gm + t < a.M; ++t)
                dst[t] = __builtin_bit_cast(_Float16, (uint16_t)(w[t >> 1] >> (16 * (t & 1))));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// One row block per workgroup (grids that would otherwise leave compute units idle): 64 rows x 256 tokens, the
// four waves split K.  Wave w takes the 32-column stages w, w + 4, ... whole: it dequantizes the stage's weights in
// registers (lane = row; v_permlane32_swap makes the MFMA operands, as in the small-batch kernel), brings the
// stage's activations into its own LDS buffers and multiplies them with all 256 tokens.  So every weight is still
// dequantized once per 256 tokens, no weight goes through LDS, a wave reads 0.5 KB of LDS per MFMA instead of
// 1.5 KB, and the waves never wait for one another until the end, where their four partial tiles meet in LDS
// (added in wave order: results do not depend on timing).
// Two shapes of the tile: 64 rows x 256 tokens, or 128 rows x 128 tokens (every wave then dequantizes two row
// blocks per stage and needs half the activation bytes per MFMA; its activation buffers are half as large, so
// four instead of two of them fit and the requests run three own stages ahead instead of one).
constexpr int kKsSets = 4;  // register sets of packed weights = own stages in flight per wave
template <int RBW, int TT>
struct KsTile {
    static constexpr int TN = 32 * TT, TM = 64 * RBW;
    static constexpr int XBytes = TN * kStageK * 2;           // activations of a stage
    static constexpr int NBuf = 128 * 1024 / (4 * XBytes);   // activation buffers per wave
    static constexpr int XLoads = TN / 16;                    // requests per stage (16 token rows each)
    static constexpr int PartRow = TM * 4 + 16;               // bytes per token of a wave's partial tile in LDS
    static constexpr int PartBytes = (TN / 2) * PartRow;      // ... of half of its tokens
    static constexpr int LdsBytes = 4 * NBuf * XBytes > 4 * PartBytes ? 4 * NBuf * XBytes : 4 * PartBytes;
    static_assert(RBW * TT == 8 && NBuf >= 2 && LdsBytes <= 160 * 1024, "tile of the K-split kernel");
};

template <int B, int GQ, bool HZ, int RBW, int TT>
__global__ void __launch_bounds__(256, 1) mpgemm_ksplit_kernel(GemmArgs a) {
    using T = KsTile<RBW, TT>;
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int TB = B * 1024 + 64 * (kKTile / GQ) * MSZ;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int mt = (slot / a.n_tiles) * kXcds + xcd, nt = slot % a.n_tiles;
    const bool header_ok = header_matches(a.tiles, a.M, a.K, B, GQ, HZ ? 1 : 0);
    if (!header_ok && blockIdx.x == 0 && threadIdx.x == 0) report_header_mismatch(a.status);
    if (mt >= (header_ok ? a.m_tiles : 0)) return;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int n0 = nt * T::TN;
    const int k_stages = a.K / kStageK;
    // own stages of this wave: wave, wave + 4, ...; the loop runs whole rounds of kKsSets own stages (a stage past
    // K has empty sources: zero weights, zero activations)
    const int n_own = (k_stages + 3) / 4, n_own_pad = (n_own + kKsSets - 1) & ~(kKsSets - 1);
    const int r = lane & 31, h = lane >> 5;

    float16_t acc[RBW][2][TT];
#pragma unroll
    for (int b = 0; b < RBW; ++b)
#pragma unroll
        for (int hb = 0; hb < 2; ++hb)
#pragma unroll
            for (int nb = 0; nb < TT; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[b][hb][nb][v] = 0.f;

    WRegs<B> wr[kKsSets][RBW];
    auto load_wregs = [&](int set, int i) {  // own stage i = stage 4 i + wave, every row block of the tile
        const int t = 4 * i + wave;
#pragma unroll
        for (int b = 0; b < RBW; ++b) {
            const int rb = mt * RBW + b;
            const bool wvalid = rb < a.n_row_blocks;
            const uint8_t* wsrc = a.tiles + (size_t)(wvalid ? rb : 0) * a.n_ktiles * TB;
            load_w<B, GQ, HZ>(wr[set][b], make_rsrc(wsrc, t < k_stages && wvalid ? 0x7fffffffu : 0u), t >> 2, t & 3, lane);
        }
    };
    // activations of own stage i go to this wave's buffer i % NBuf
    const int xrows = a.N - n0 < T::TN ? a.N - n0 : T::TN;
    const _Float16* xsrc = a.x + (size_t)n0 * a.K;
    const uint32_t xbytes = (uint32_t)xrows * (uint32_t)a.K * 2u;
    const uint32_t xlane = ((lane >> 2) * (uint32_t)a.K + ((lane & 3) ^ ((lane >> 4) & 3)) * 8u) * 2u;
    const uint32_t x16rows = 16u * (uint32_t)a.K * 2u;
    uint8_t* const xbuf = smem + wave * T::NBuf * T::XBytes;
    auto load_x = [&](int i) {
        const int t = 4 * i + wave;
        const rsrc_t rx = make_rsrc(xsrc, t < k_stages ? xbytes : 0u);
        uint8_t* dst = xbuf + (i & (T::NBuf - 1)) * T::XBytes;
#pragma unroll
        for (int q = 0; q < T::XLoads; ++q)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(dst + q * 1024), 16,
                                                     xlane + (uint32_t)q * x16rows, t * kStageK * 2, 0, 0);
    };
    const int xrow = r * (kStageK * 2);
    const int xchunk[2] = {xrow + ((h ^ ((r >> 2) & 3)) * 16), xrow + (((2 + h) ^ ((r >> 2) & 3)) * 16)};
    half8_t xf[2][TT];
    auto read_x = [&](int j, const uint8_t* stage) {
#pragma unroll
        for (int nb = 0; nb < TT; ++nb)
            xf[j][nb] = *reinterpret_cast<const half8_t*>(stage + xchunk[j] + nb * 32 * (kStageK * 2));
    };
    half8_t wf[2][RBW][2][2];  // [set][row block][rows 0..31 / 32..63][16-column step]
    Dequant<B, HZ> dq;
    auto operands = [&](int set, int b, int j) {
        const u32x4 pa = dq.piece(2 * j), pb = dq.piece(2 * j + 1);
        u32x4 lo, hi;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const u32x2 sw = __builtin_amdgcn_permlane32_swap(pa[e], pb[e], false, false);
            lo[e] = sw.x;
            hi[e] = sw.y;
        }
        wf[set][b][0][j] = __builtin_bit_cast(half8_t, lo);
        wf[set][b][1][j] = __builtin_bit_cast(half8_t, hi);
    };
    auto mfmas = [&](int set, int j) {
#pragma unroll
        for (int nb = 0; nb < TT; ++nb)
#pragma unroll
            for (int b = 0; b < RBW; ++b) {
                acc[b][0][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[set][b][0][j], xf[j][nb], acc[b][0][nb], 0, 0, 0);
                acc[b][1][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[set][b][1][j], xf[j][nb], acc[b][1][nb], 0, 0, 0);
            }
    };
    // the vector work of a stage in two parts, one beside each 16-column step of the previous stage: with one row
    // block level 1 / level 2 of it, with two the whole of block 0 / of block 1
    auto dequant_part = [&](int part, int wset, int oset) {
        if constexpr (RBW == 1) {
            if (part == 0) {
                dq.start(wr[wset][0]);
                dq.insert();
            } else {
                operands(oset, 0, 0);
                operands(oset, 0, 1);
            }
        } else {
            dq.start(wr[wset][part]);
            dq.insert();
            operands(oset, part, 0);
            operands(oset, part, 1);
        }
    };

    // prologue: activations of own stage 0 in LDS and those of own stage 1 requested; weights of own stages 1..4 in
    // the register sets, own stage 0 dequantized into operand set 0
    load_x(0);
#pragma unroll
    for (int i = 0; i < kKsSets; ++i) load_wregs(i, i);
    dequant_part(0, 0, 0);
    dequant_part(1, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = 1; i < T::NBuf; ++i) load_x(i);
    __builtin_amdgcn_sched_barrier(0);
    load_wregs(0, kKsSets);
    __builtin_amdgcn_sched_barrier(0);
    read_x(0, xbuf);

    for (int i0 = 0; i0 < n_own_pad; i0 += kKsSets) {
#pragma unroll
        for (int u = 0; u < kKsSets; ++u) {
            const int i = i0 + u;
            const uint8_t* cur = xbuf + (i & (T::NBuf - 1)) * T::XBytes;
            const uint8_t* nxt = xbuf + ((i + 1) & (T::NBuf - 1)) * T::XBytes;
            // first half: 16-column step 0 of own stage i; meanwhile the activations of step 1 and level 1 of the
            // next own stage
            read_x(1, cur);
            dequant_part(0, (u + 1) % kKsSets, (u + 1) & 1);
            mfmas(u & 1, 0);
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, RBW == 1 ? 3 : 6, 0);
                if (q < TT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            // second half: step 1; meanwhile the rest of the next own stage's vector work
            dequant_part(1, (u + 1) % kKsSets, (u + 1) & 1);
            mfmas(u & 1, 1);
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, RBW == 1 ? 5 : 6, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            // The buffer of own stage i is free now (its operand reads are consumed): request own stage i + NBuf
            // into it.  Before the reads that follow, the activations of own stage i + 1 must be in: what was
            // requested after them is at least the activations of NBuf - 2 stages and one stage's weights (requests
            // complete in order; older weight requests are long in by then).
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((T::NBuf - 2) * T::XLoads + 2 * RBW) : "memory");
            load_x(i + T::NBuf);
            __builtin_amdgcn_sched_barrier(0);
            load_wregs((u + 1) % kKsSets, i + 1 + kKsSets);
            __builtin_amdgcn_sched_barrier(0);
            read_x(0, nxt);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // requests of own stages past the end may still be writing zeros to LDS, which the partial tiles reuse
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // The four partial tiles meet in LDS, half of the tokens at a time: wave w writes its fp32 sums as
    // [token][row], then thread -> (token, 8 rows) adds the four in wave order and stores fp16.
    // acc[b][hb][nb][v] is row 64 b + 32 hb + 8 (v / 4) + 4 h + v % 4 for token 32 nb + r.
    const int m0 = mt * T::TM;
    const bool fast = (a.M % 8 == 0);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        uint8_t* mine = smem + wave * T::PartBytes;
#pragma unroll
        for (int nq = 0; nq < TT / 2; ++nq) {
            const int nb = half * (TT / 2) + nq;
#pragma unroll
            for (int b = 0; b < RBW; ++b)
#pragma unroll
                for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float* dst = reinterpret_cast<float*>(mine + (nq * 32 + r) * T::PartRow + (64 * b + 32 * hb + 8 * g + 4 * h) * 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) dst[e] = acc[b][hb][nb][4 * g + e];
                    }
        }
        __syncthreads();
        for (int piece = tid; piece < (T::TN / 2) * (T::TM / 8); piece += 256) {
            const int n = piece / (T::TM / 8), c8 = piece % (T::TM / 8);
            const int gn = n0 + half * (T::TN / 2) + n, gm = m0 + c8 * 8;
            float sum[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) sum[e] = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float* src = reinterpret_cast<const float*>(smem + w * T::PartBytes + n * T::PartRow + c8 * 32);
#pragma unroll
                for (int e = 0; e < 8; ++e) sum[e] += src[e];
            }
            if (gn >= a.N || gm >= a.M) continue;
            _Float16* dst = a.y + (size_t)gn * a.M + gm;
            if (fast && gm + 8 <= a.M) {
                half8_t o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (_Float16)sum[e];
                *reinterpret_cast<half8_t*>(dst) = o;
            } else {
                for (int t = 0; t < 8 && gm + t < a.M; ++t) dst[t] = (_Float16)sum[t];
            }
        }
        __syncthreads();
    }
}

template <int B, int GQ, bool HZ, int RBW, int TT>
static int launch_ksplit(GemmArgs a, hipStream_t st) {
    using T = KsTile<RBW, TT>;
    static std::once_flag once;
    static hipError_t attr_rc = hipSuccess;
    std::call_once(once, [] {
        attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&mpgemm_ksplit_kernel<B, GQ, HZ, RBW, TT>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, T::LdsBytes);
    });
    if (attr_rc != hipSuccess) return TMAN_ERR_LAUNCH;
    a.m_tiles = (a.n_row_blocks + RBW - 1) / RBW;
    a.n_tiles = (a.N + T::TN - 1) / T::TN;
    const unsigned grid = (unsigned)((a.m_tiles + kXcds - 1) / kXcds * kXcds * a.n_tiles);
    hipLaunchKernelGGL((mpgemm_ksplit_kernel<B, GQ, HZ, RBW, TT>), dim3(grid), dim3(256), T::LdsBytes, st, a);
    return launch_status();
}

template <int B, int GQ, bool HZ, int RB>
static int launch_tile(GemmArgs a, hipStream_t st) {
    // once per kernel instantiation, also when several host threads make their first call together
    static std::once_flag once;
    static hipError_t attr_rc = hipSuccess;
    std::call_once(once, [] {
        attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&mpgemm_kernel<B, GQ, HZ, RB>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, Tile<RB>::LdsBytes);
    });
    if (attr_rc != hipSuccess) return TMAN_ERR_LAUNCH;
    a.m_tiles = (a.n_row_blocks + RB - 1) / RB;
    a.n_tiles = (a.N + kTN - 1) / kTN;
    const unsigned grid = (unsigned)((a.m_tiles + kXcds - 1) / kXcds * kXcds * a.n_tiles);
    hipLaunchKernelGGL((mpgemm_kernel<B, GQ, HZ, RB>), dim3(grid), dim3(kThreads), Tile<RB>::LdsBytes, st, a);
    return launch_status();
}

// Which kernel and tile: 1 .. 4 = the tiled kernel with that many row blocks per workgroup; kSplitWide /
// kSplitTall = the K-split kernel with 64 rows x 256 tokens / 128 rows x 128 tokens.
// Tiled kernel: the row blocks that need the least time, counted as rounds of workgroups over the compute units
// times rows per workgroup, with a small bonus for larger tiles (fewer operand reads and less dequantization per
// MFMA).  A grid that leaves compute units idle even with one row block per workgroup goes to the K-split kernel
// (measured 10 - 40 % faster there) unless K is short: the tall tile when the workgroups' activation streams are
// what limits them (more than 256 tokens, or a full 256 with at least half of the units busy), else the wide one.
constexpr int kSplitWide = 5, kSplitTall = 6;
static int choose_tile(int n_row_blocks, int N, int K) {
    static std::once_flag once;
    static int n_cu = 256;  // assumed when no device answers
    std::call_once(once, [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            n_cu = n;
    });
    const tman_tiling_t t = current_tiling();
    if (t.prefill_k_split == 2) return kSplitWide;
    if (t.prefill_k_split == 3) return kSplitTall;
    const int forced = t.prefill_row_blocks;
    if (forced >= 1 && forced <= 4) return forced;
    const int n_tiles = (N + kTN - 1) / kTN;
    if ((long long)n_row_blocks * n_tiles <= n_cu) {
        if (t.prefill_k_split == 1 || K < 2048) return 1;
        return N > 256 || (N > 192 && (long long)n_row_blocks * n_tiles * 2 >= n_cu) ? kSplitTall : kSplitWide;
    }
    const double penalty[5] = {0, 0, 1.10, 1.03, 1.0};
    int best = 4;
    double best_cost = 1e30;
    for (int rb = 4; rb >= 2; --rb) {
        const long long wgs = (long long)((n_row_blocks + rb - 1) / rb) * n_tiles;
        const double cost = (double)((wgs + n_cu - 1) / n_cu) * rb * penalty[rb];
        if (cost < best_cost) {
            best_cost = cost;
            best = rb;
        }
    }
    return best;
}

template <int B, int GQ, bool HZ>
static int launch_cfg(const GemmArgs& a, hipStream_t st) {
    switch (choose_tile(a.n_row_blocks, a.N, a.K)) {
        case kSplitWide: return launch_ksplit<B, GQ, HZ, 1, 8>(a, st);
        case kSplitTall: return launch_ksplit<B, GQ, HZ, 2, 4>(a, st);
        case 1: return launch_tile<B, GQ, HZ, 1>(a, st);
        case 2: return launch_tile<B, GQ, HZ, 2>(a, st);
        case 3: return launch_tile<B, GQ, HZ, 3>(a, st);
        default: return launch_tile<B, GQ, HZ, 4>(a, st);
    }
}

template <int B, bool HZ>
static int launch_group(int group, const GemmArgs& a, hipStream_t st) {
    switch (group) {
        case 32: return launch_cfg<B, 32, HZ>(a, st);
        case 64: return launch_cfg<B, 64, HZ>(a, st);
        default: return launch_cfg<B, 128, HZ>(a, st);
    }
}

int mpgemm_row_blocks_per_workgroup(const Layout& L, int N) {
    const int c = choose_tile(L.n_row_blocks, N, L.K);
    return c == kSplitWide ? 1 : c == kSplitTall ? 2 : c;
}
int mpgemm_splits_k(const Layout& L, int N) {
    const int c = choose_tile(L.n_row_blocks, N, L.K);
    return c == kSplitWide || c == kSplitTall;
}

int launch_mpgemm(const Layout& L, const void* packed, const void* x, int N, void* y, void* workspace,
                  hipStream_t st) {
    (void)workspace;
    GemmArgs a;
    a.tiles = static_cast<const uint8_t*>(packed) + kHeaderBytes;
    a.x = static_cast<const _Float16*>(x);
    a.y = static_cast<_Float16*>(y);
    a.M = L.M;
    a.N = N;
    a.K = L.K;
    a.n_row_blocks = L.n_row_blocks;
    a.n_ktiles = L.n_ktiles;
    a.m_tiles = a.n_tiles = 0;
    a.status = device_status_word();
    if (!a.status) return TMAN_ERR_LAUNCH;
    if (L.bits == 1) return L.has_zero ? launch_group<1, true>(L.group, a, st) : launch_group<1, false>(L.group, a, st);
    if (L.bits == 2) return launch_group<2, true>(L.group, a, st);
    return launch_group<4, true>(L.group, a, st);
}

}  // namespace tman
