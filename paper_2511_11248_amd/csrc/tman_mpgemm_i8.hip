// mpGEMM on the integer matrix cores for formats with ONE scale and zero per row of W -- per-channel, or
// per-tensor such as BitNet's ternary weights (Sec. 6.1: "per-tensor quantization ... treated as 2-bit";
// Sec. 6.2 mpGEMM: such models are dequantized to INT8 and computed as W_INT8 x A_INT8).
//
//   xq[n][k]  = rint(x[n][k] * 127 / max_k |x[n][k]|)                      int8, per token (tman_quantize_act_i8)
//   acc[n][m] = sum_k c[m][k] * xq[n][k]                                     int32, exact (v_mfma_i32_32x32x32_i8)
//   y[n][m]   = scale[m] * (max_n / 127) * (acc[n][m] - zero[m] * sum_k xq[n][k])      fp32, rounded once to fp16
//
// Level 1 of the paper's dequantization (bit-serial -> bit-parallel) is all the weights need here: the matrix
// unit multiplies the unsigned codes themselves, the zero point moves to the epilogue through the token's sum of
// integer activations.  The codes of a 32-weight block come out of the bit-field transposition as four words
// of eight nibbles, word o nibble f = weight 4 f + o; two masks per word turn them into bytes in the order
//   position p = 8 o + 4 h + b  <->  column 8 b + 4 h + o          (o < 4, h < 2, b < 4)
// and instead of sorting the weights the ACTIVATIONS are stored in that order: the quantizer writes every
// 32-column group of a token permuted accordingly, so both MFMA operands are plain 16-byte LDS reads.
//
// Three kernels, chosen per call from the grids they give (choose_i8_token_blocks).  The first:
// workgroup = 4 waves = 128 rows x 128 tokens; wave (wm, wn) accumulates 64 x 64 as four 32 x 32 tiles.  Per
// 64-column stage every wave transposes one 32-weight block of one of the two row blocks into LDS (lane = row),
// the 128 x 64 bytes of activations go through registers into LDS, one barrier, eight MFMAs per wave.  Two stage
// buffers: a wave writes stage s + 1 while others still read stage s.
// The second (mpgemm_i8_wide_kernel, below) keeps the weights out of LDS altogether; in the third
// (mpgemm_i8_ksplit_kernel) the waves of a workgroup also split K, for grids too small for the other two.
#include <hip/hip_fp16.h>

#include <mutex>

#include "tman_dequant_device.h"

namespace tman {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x16 __attribute__((ext_vector_type(16)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;

constexpr int kI8Rows = 128, kI8Tokens = 128, kI8StageK = 64;
constexpr int kI8Ahead = 4;  // stages of global loads in flight per wave
constexpr int kI8RowBytes = kI8StageK + 16;  // padded LDS row: 20 dwords, conflict-free 16-byte accesses
constexpr int kI8StageBytes = (kI8Rows + kI8Tokens) * kI8RowBytes;
constexpr int kI8OutRow = kI8Rows * 2 + 16;  // bytes per token of the fp16 output tile in LDS
constexpr int kI8LdsBytes = 2 * kI8StageBytes > kI8Tokens * kI8OutRow ? 2 * kI8StageBytes : kI8Tokens * kI8OutRow;

__device__ __forceinline__ rsrc_t rsrc_of(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// ---------------------------------------------------------------------------------------------
// activation quantizer: one workgroup per token

// byte position p of a 32-column group holds column sigma(p) (see above)
__host__ __device__ constexpr int sigma(int p) { return 8 * (p & 3) + 4 * ((p >> 2) & 1) + (p >> 3); }

struct ActI8Layout {
    size_t q_bytes;     // int8 [N][K], every 32-column group permuted
    size_t absmax_off;  // float [N]
    size_t sum_off;     // int32 [N]
    size_t total;
};
static ActI8Layout act_i8_layout(int N, int K) {
    ActI8Layout l;
    l.q_bytes = ((size_t)N * K + 255) / 256 * 256;
    l.absmax_off = l.q_bytes;
    l.sum_off = l.absmax_off + (((size_t)N * 4 + 255) / 256 * 256);
    l.total = l.sum_off + (((size_t)N * 4 + 255) / 256 * 256);
    return l;
}
size_t act_i8_bytes(int N, int K) { return act_i8_layout(N, K).total; }

__global__ void __launch_bounds__(256) quantize_act_i8_kernel(const uint16_t* __restrict__ x, int K, int8_t* __restrict__ q,
                                                              float* __restrict__ absmax, int32_t* __restrict__ sums) {
    __shared__ unsigned wave_max[4];
    __shared__ int wave_sum[4];
    const int n = blockIdx.x, tid = threadIdx.x;
    const uint16_t* xb = x + (size_t)n * K;
    unsigned mx = 0;  // magnitudes compare like their bit patterns
    for (int k = tid; k < K; k += 256) mx = max(mx, (unsigned)(xb[k] & 0x7fffu));
    for (int d = 1; d < 64; d <<= 1) mx = max(mx, (unsigned)__shfl_xor((int)mx, d, 64));
    if ((tid & 63) == 0) wave_max[tid >> 6] = mx;
    __syncthreads();
    mx = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
    const float amax = (float)__builtin_bit_cast(_Float16, (uint16_t)mx);
    // the decision is taken in binary32: one correctly rounded division, one product, round to nearest even
    const float inv = amax > 0.f ? __fdiv_rn(127.0f, amax) : 0.f;
    int s = 0;
    for (int g = tid; g < K / 32; g += 256) {
        int v[32];
#pragma unroll
        for (int c = 0; c < 32; ++c) {
            v[c] = (int)rintf(__fmul_rn((float)__builtin_bit_cast(_Float16, xb[g * 32 + c]), inv));
            s += v[c];
        }
        uint32_t w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            w[i] = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) w[i] |= (uint32_t)(v[sigma(4 * i + b)] & 0xff) << (8 * b);
        }
        uint32_t* dst = reinterpret_cast<uint32_t*>(q + (size_t)n * K + (size_t)g * 32);
#pragma unroll
        for (int i = 0; i < 8; ++i) dst[i] = w[i];
    }
    for (int d = 1; d < 64; d <<= 1) s += __shfl_xor(s, d, 64);
    if ((tid & 63) == 0) wave_sum[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) {
        absmax[n] = amax;
        sums[n] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
    }
}

// The same for activations that start on a 16-byte boundary (every row then does: K is a multiple of 32): thread t
// reads group t of the token (32 columns, 64 bytes) once, with four 16-byte loads, and keeps it in registers from
// the search for the maximum to the rounding; only tokens longer than 8192 columns read their further groups twice.
__global__ void __launch_bounds__(256) quantize_act_i8_aligned_kernel(const uint16_t* __restrict__ x, int K,
                                                                      int8_t* __restrict__ q, float* __restrict__ absmax,
                                                                      int32_t* __restrict__ sums) {
    __shared__ unsigned wave_max[4];
    __shared__ int wave_sum[4];
    const int n = blockIdx.x, tid = threadIdx.x;
    const uint16_t* xb = x + (size_t)n * K;
    const int n_groups = K / 32;
    auto load_group = [&](u32x4 (&c)[4], int g) {
        const u32x4* src = reinterpret_cast<const u32x4*>(xb + (size_t)g * 32);
#pragma unroll
        for (int i = 0; i < 4; ++i) c[i] = src[i];
    };
    auto group_max = [&](const u32x4 (&c)[4], unsigned mx) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) mx = max(mx, max(c[i][e] & 0x7fffu, (c[i][e] >> 16) & 0x7fffu));
        return mx;
    };
    u32x4 mine[4] = {};
    const bool have = tid < n_groups;
    if (have) load_group(mine, tid);
    unsigned mx = group_max(mine, 0u);  // magnitudes compare like their bit patterns
    for (int g = tid + 256; g < n_groups; g += 256) {
        u32x4 c[4];
        load_group(c, g);
        mx = group_max(c, mx);
    }
    for (int d = 1; d < 64; d <<= 1) mx = max(mx, (unsigned)__shfl_xor((int)mx, d, 64));
    if ((tid & 63) == 0) wave_max[tid >> 6] = mx;
    __syncthreads();
    mx = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
    const float amax = (float)__builtin_bit_cast(_Float16, (uint16_t)mx);
    // the decision is taken in binary32: one correctly rounded division, one product, round to nearest even
    const float inv = amax > 0.f ? __fdiv_rn(127.0f, amax) : 0.f;
    int s = 0;
    auto quantize_group = [&](const u32x4 (&c)[4], int g) {
        int v[32];
#pragma unroll
        for (int col = 0; col < 32; ++col) {
            const uint32_t word = c[col >> 3][(col >> 1) & 3];
            const uint16_t bits = (uint16_t)((col & 1) ? word >> 16 : word);
            v[col] = (int)rintf(__fmul_rn((float)__builtin_bit_cast(_Float16, bits), inv));
            s += v[col];
        }
        u32x4 out[2];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t w = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) w |= (uint32_t)(v[sigma(4 * i + b)] & 0xff) << (8 * b);
            out[i >> 2][i & 3] = w;
        }
        u32x4* dst = reinterpret_cast<u32x4*>(q + (size_t)n * K + (size_t)g * 32);
        dst[0] = out[0];
        dst[1] = out[1];
    };
    if (have) quantize_group(mine, tid);
    for (int g = tid + 256; g < n_groups; g += 256) {
        u32x4 c[4];
        load_group(c, g);
        quantize_group(c, g);
    }
    for (int d = 1; d < 64; d <<= 1) s += __shfl_xor(s, d, 64);
    if ((tid & 63) == 0) wave_sum[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) {
        absmax[n] = amax;
        sums[n] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
    }
}

int launch_quantize_act_i8(const void* x, int N, int K, void* out, hipStream_t st) {
    const ActI8Layout l = act_i8_layout(N, K);
    uint8_t* o = static_cast<uint8_t*>(out);
    const auto kernel = (reinterpret_cast<uintptr_t>(x) & 15u) == 0 ? quantize_act_i8_aligned_kernel : quantize_act_i8_kernel;
    hipLaunchKernelGGL(kernel, dim3((unsigned)N), dim3(256), 0, st, static_cast<const uint16_t*>(x), K,
                       reinterpret_cast<int8_t*>(o), reinterpret_cast<float*>(o + l.absmax_off),
                       reinterpret_cast<int32_t*>(o + l.sum_off));
    return launch_status();
}

// ---------------------------------------------------------------------------------------------
// the product

struct GemmI8Args {
    const uint8_t* tiles;
    const int8_t* xq;
    const float* absmax;
    const int32_t* sums;
    _Float16* y;
    int32_t* acc_out;  // optional: the integer accumulators [N][M]
    int M, N, K, n_row_blocks, n_ktiles;
    int m_tiles, n_tiles;
    int* status;
};

// The codes of one 32-weight block as 32 bytes in sigma order.
template <int B>
__device__ __forceinline__ void codes_to_bytes(const uint32_t (&plane)[B], u32x4& lo, u32x4& hi) {
    uint32_t codes[4];
    planes_to_codes<B>(plane, codes);
    constexpr uint32_t kMask = ((1u << B) - 1u) * 0x01010101u;
    // word o: even nibbles -> bytes 8 o .. 8 o + 3, odd nibbles -> bytes 8 o + 4 .. 8 o + 7
    lo = u32x4{codes[0] & kMask, (codes[0] >> 4) & kMask, codes[1] & kMask, (codes[1] >> 4) & kMask};
    hi = u32x4{codes[2] & kMask, (codes[2] >> 4) & kMask, codes[3] & kMask, (codes[3] >> 4) & kMask};
}

template <int B, int GQ, bool HZ>
__global__ void __launch_bounds__(256) mpgemm_i8_kernel(GemmI8Args a) {
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int MPL = (kKTile / GQ) * MSZ;
    constexpr int TB = B * 1024 + 64 * MPL;
    constexpr int CH = kKTile / B;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    __shared__ float row_scale[kI8Rows], row_zs[kI8Rows];  // scale[m] and zero[m] * scale[m]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mt = blockIdx.x / a.n_tiles, nt = blockIdx.x % a.n_tiles;
    // a blob packed for another shape or layout: say so and leave y alone (one exit)
    const bool header_ok = header_matches(a.tiles, a.M, a.K, B, GQ, HZ ? 1 : 0);
    if (!header_ok && blockIdx.x == 0 && tid == 0) report_header_mismatch(a.status);
    if (mt >= (header_ok ? a.m_tiles : 0)) return;
    const int n0 = nt * kI8Tokens;
    const int k_stages = (a.K + kI8StageK - 1) / kI8StageK;  // K is a multiple of 32; a last half stage reads zeros

    // roles in the weight transposition: wave w -> row block w / 2 of the tile, 32-weight block w % 2 of the stage
    const int wrb = mt * 2 + (wave >> 1), wblk = wave & 1;
    const bool wvalid = wrb < a.n_row_blocks;
    const uint8_t* wsrc = a.tiles + (size_t)(wvalid ? wrb : 0) * a.n_ktiles * TB;
    const uint32_t wbytes = wvalid ? (uint32_t)(a.n_ktiles * TB) : 0u;
    const int k32_total = a.K / 32;
    auto load_planes = [&](uint32_t (&plane)[B], int stage) {
        const int k32 = stage * 2 + wblk;  // 32-weight block along K
        const rsrc_t rw = rsrc_of(wsrc, k32 < k32_total ? wbytes : 0u);
        const int tile = k32 >> 2, kb32 = k32 & 3;
        const int v = (kb32 * 32) / CH, ksub = ((kb32 * 32) % CH) / 32;
        const int so = tile * TB + v * 1024 + ksub * B * 4;
        if constexpr (B == 4) {
            const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(rw, lane * 16, so, 0);
            plane[0] = w.x; plane[1] = w.y; plane[2] = w.z; plane[3] = w.w;
        } else if constexpr (B == 2) {
            const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rw, lane * 16, so, 0);
            plane[0] = w.x; plane[1] = w.y;
        } else {
            plane[0] = __builtin_amdgcn_raw_buffer_load_b32(rw, lane * 16, so, 0);
        }
    };
    // activations of a stage: thread -> token tid / 2, 32 bytes at column half tid % 2; tokens beyond N and columns
    // beyond K lie outside the resource and read as zero
    const int xtok = tid >> 1, xhalf = tid & 1;
    const rsrc_t rx = rsrc_of(a.xq, (uint32_t)a.N * (uint32_t)a.K);
    auto load_x = [&](u32x4 (&xv)[2], int stage) {
        const int col = stage * kI8StageK + xhalf * 32;
        const bool in = (n0 + xtok) < a.N && col < a.K;
        const uint32_t off = in ? (uint32_t)(n0 + xtok) * (uint32_t)a.K + (uint32_t)col : 0xFFFFFFF0u;
        xv[0] = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 0);
        xv[1] = __builtin_amdgcn_raw_buffer_load_b128(rx, in ? off + 16u : 0xFFFFFFF0u, 0, 0);
    };

    i32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    const int wm = wave >> 1, wn = wave & 1, r = lane & 31, h = lane >> 5;

    // Global loads run kI8Ahead stages ahead of their use, in a ring of register sets (a stage of MFMAs is far
    // shorter than the latency of a load); stages past K read zeros, so the loop runs whole rings.
    uint32_t plane[kI8Ahead][B];
    u32x4 xv[kI8Ahead][2];
#pragma unroll
    for (int u = 0; u < kI8Ahead; ++u) {
        load_planes(plane[u], u);
        load_x(xv[u], u);
    }
    // scale and zero of the tile's rows (the first quantization block of a row stands for the whole row)
    if (tid < kI8Rows) {
        const int rb = mt * 2 + (tid >> 6), l = tid & 63;
        float sc = 0.f, zs = 0.f;
        if (rb < a.n_row_blocks) {
            const uint8_t* meta = a.tiles + (size_t)rb * a.n_ktiles * TB + B * 1024 + l * MPL;
            sc = (float)*reinterpret_cast<const _Float16*>(meta);
            zs = HZ ? (float)*reinterpret_cast<const _Float16*>(meta + 2) * sc : 0.f;
        }
        row_scale[tid] = sc;
        row_zs[tid] = zs;
    }
    const int n_stages = (k_stages + kI8Ahead - 1) / kI8Ahead * kI8Ahead;
    for (int s0 = 0; s0 < n_stages; s0 += kI8Ahead) {
#pragma unroll
        for (int u = 0; u < kI8Ahead; ++u) {
            const int s = s0 + u;
            uint8_t* buf = smem + (s & 1) * kI8StageBytes;
            {
                u32x4 lo, hi;
                codes_to_bytes<B>(plane[u], lo, hi);
                uint8_t* wrow = buf + ((wave >> 1) * 64 + lane) * kI8RowBytes + wblk * 32;
                *reinterpret_cast<u32x4*>(wrow) = lo;
                *reinterpret_cast<u32x4*>(wrow + 16) = hi;
                uint8_t* xrow = buf + (kI8Rows + xtok) * kI8RowBytes + xhalf * 32;
                *reinterpret_cast<u32x4*>(xrow) = xv[u][0];
                *reinterpret_cast<u32x4*>(xrow + 16) = xv[u][1];
            }
            load_planes(plane[u], s + kI8Ahead);
            load_x(xv[u], s + kI8Ahead);
            __syncthreads();
            const uint8_t* wbase = buf + (wm * 64 + r) * kI8RowBytes + h * 16;
            const uint8_t* xbase = buf + (kI8Rows + wn * 64 + r) * kI8RowBytes + h * 16;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                i32x4 wf[2], xf[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    wf[i] = *reinterpret_cast<const i32x4*>(wbase + i * 32 * kI8RowBytes + ks * 32);
                    xf[i] = *reinterpret_cast<const i32x4*>(xbase + i * 32 * kI8RowBytes + ks * 32);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[i], xf[j], acc[i][j], 0, 0, 0);
            }
        }
    }
    __syncthreads();  // every wave is done with the stage buffers, which the output tile reuses

    // epilogue: C[i][j] of a 32 x 32 tile: i = row 8 (v / 4) + 4 h + v % 4, j = token lane % 32
    uint8_t* otile = smem;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int tok = wn * 64 + j * 32 + r, gn = n0 + tok;
        const bool live = gn < a.N;
        const float delta = live ? a.absmax[gn] * (1.0f / 127.0f) : 0.f;
        const float sx = live ? (float)a.sums[gn] : 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int row = wm * 64 + i * 32 + 8 * g4 + 4 * h;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float av = (float)acc[i][j][4 * g4 + e];
                    // (c - z) s summed: s acc - (z s) sum(xq); sign form (2 c - 1) s: 2 s acc - s sum(xq)
                    v[e] = HZ ? delta * fmaf(row_scale[row + e], av, -row_zs[row + e] * sx)
                              : delta * row_scale[row + e] * fmaf(2.f, av, -sx);
                }
                half2_t p0, p1;
                p0.x = (_Float16)v[0]; p0.y = (_Float16)v[1];
                p1.x = (_Float16)v[2]; p1.y = (_Float16)v[3];
                u32x2 w = {__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1)};
                *reinterpret_cast<u32x2*>(otile + tok * kI8OutRow + row * 2) = w;
                if (a.acc_out && live) {
                    const int gm = mt * kI8Rows + row;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (gm + e < a.M) a.acc_out[(size_t)gn * a.M + gm + e] = acc[i][j][4 * g4 + e];
                }
            }
        }
    }
    __syncthreads();
    const int m0 = mt * kI8Rows;
    const bool fast = (a.M % 8 == 0);  // 16-byte aligned rows of y
    for (int piece = tid; piece < kI8Tokens * (kI8Rows / 8); piece += 256) {
        const int n = piece / (kI8Rows / 8), c8 = piece % (kI8Rows / 8);
        const int gn = n0 + n, gm = m0 + c8 * 8;
        if (gn >= a.N || gm >= a.M) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(otile + n * kI8OutRow + c8 * 16);
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
// Wide variant for long token ranges: no weight tile in LDS.  A wave owns 64 rows x 32 TT tokens; it turns the bit
// planes of its rows into bytes in registers (lane = row) and makes the two MFMA operands of a 32-column step with
// four v_permlane32_swap (rows 0..31 and rows 32..63, each with the lane halves holding bytes 0..15 and 16..31 of
// the step).  Only the activations go through LDS, straight from memory, shared by the four waves (256 rows) of
// the workgroup.  Per MFMA this reads half the LDS bytes of the 128 x 128 kernel and dequantizes each weight once
// per 32 TT tokens instead of once per 128.
constexpr int kI8WRing = 4;   // stage buffers of activations in LDS
constexpr int kI8WSets = 4;   // register sets of bit planes = stages of weight loads in flight
constexpr int kI8WStageK = 32;
constexpr int kI8WRows = 256;

template <int TT>
struct I8Wide {
    static constexpr int TN = TT * 32;
    static constexpr int XLoads = (TT + 3) / 4;        // activation loads of a stage per wave (32 token rows each)
    static constexpr int XBytes = XLoads * 4 * 1024;   // stage buffer: whole loads of all four waves
    static constexpr int OutRow = kI8WRows * 2 + 16;   // bytes per token of the fp16 output tile in LDS
    static constexpr int LdsBytes = kI8WRing * XBytes > TN * OutRow ? kI8WRing * XBytes : TN * OutRow;
};

template <int B, bool HZ, int TT>
__global__ void __launch_bounds__(256, (TT <= 4 ? 2 : 1)) mpgemm_i8_wide_kernel(GemmI8Args a, int group) {
    using T = I8Wide<TT>;
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int CH = kKTile / B;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    __shared__ float row_scale[kI8WRows], row_zs[kI8WRows];

    const int MPL = (kKTile / group) * MSZ, TB = B * 1024 + 64 * MPL;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mt = blockIdx.x / a.n_tiles, nt = blockIdx.x % a.n_tiles;
    const bool header_ok = header_matches(a.tiles, a.M, a.K, B, group, HZ ? 1 : 0);
    if (!header_ok && blockIdx.x == 0 && tid == 0) report_header_mismatch(a.status);
    if (mt >= (header_ok ? a.m_tiles : 0)) return;
    const int n0 = nt * T::TN;
    const int k_stages = a.K / kI8WStageK, n_stages = (k_stages + kI8WSets - 1) & ~(kI8WSets - 1);
    const int r = lane & 31, h = lane >> 5;

    i32x16 acc[2][TT];
#pragma unroll
    for (int hb = 0; hb < 2; ++hb)
#pragma unroll
        for (int nb = 0; nb < TT; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[hb][nb][v] = 0;

    // bit planes of this wave's row block, one 32-weight block per stage
    const int wrb = mt * 4 + wave;
    const bool wvalid = wrb < a.n_row_blocks;
    const uint8_t* wsrc = a.tiles + (size_t)(wvalid ? wrb : 0) * a.n_ktiles * TB;
    const uint32_t wbytes = wvalid ? (uint32_t)(a.n_ktiles * TB) : 0u;
    uint32_t plane[kI8WSets][B];
    auto load_planes = [&](uint32_t (&pl)[B], int t) {
        const rsrc_t rw = rsrc_of(wsrc, t < k_stages ? wbytes : 0u);
        const int tile = t >> 2, kb32 = t & 3;
        const int v = (kb32 * 32) / CH, ksub = ((kb32 * 32) % CH) / 32;
        const int so = tile * TB + v * 1024 + ksub * B * 4;
        if constexpr (B == 4) {
            const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(rw, lane * 16, so, 0);
            pl[0] = w.x; pl[1] = w.y; pl[2] = w.z; pl[3] = w.w;
        } else if constexpr (B == 2) {
            const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rw, lane * 16, so, 0);
            pl[0] = w.x; pl[1] = w.y;
        } else {
            pl[0] = __builtin_amdgcn_raw_buffer_load_b32(rw, lane * 16, so, 0);
        }
    };
    // activations: load i of a stage brings 32 token rows x 32 bytes straight into LDS (lane -> row lane / 2, half
    // lane % 2); wave w issues loads w, w + 4, ...; rows beyond the tile's tokens lie outside the resource (zeros)
    const int xrows = a.N - n0 < T::TN ? a.N - n0 : T::TN;
    const int8_t* xsrc = a.xq + (size_t)n0 * a.K;
    const uint32_t xbytes = (uint32_t)xrows * (uint32_t)a.K;
    const uint32_t xlane = (uint32_t)(lane >> 1) * (uint32_t)a.K + (uint32_t)(lane & 1) * 16u;
    const uint32_t x32rows = 32u * (uint32_t)a.K;
    auto load_x = [&](int t) {
        const rsrc_t rx = rsrc_of(xsrc, t < k_stages ? xbytes : 0u);
        uint8_t* dst = smem + (t & (kI8WRing - 1)) * T::XBytes;
#pragma unroll
        for (int i = 0; i < T::XLoads; ++i) {
            const int li = wave + 4 * i;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(dst + li * 1024), 16,
                                                     xlane + (uint32_t)li * x32rows, t * kI8WStageK, 0, 0);
        }
    };
    const int xoff = r * 32 + h * 16;  // operand of token block nb: token nb * 32 + r, bytes 16 h .. 16 h + 15
    i32x4 xf[2][TT];
    auto read_x = [&](int set, const uint8_t* stage) {
#pragma unroll
        for (int nb = 0; nb < TT; ++nb) xf[set][nb] = *reinterpret_cast<const i32x4*>(stage + xoff + nb * 1024);
    };
    i32x4 wf[2][2];  // [set][rows 0..31 / 32..63]
    auto operands = [&](int set, const uint32_t (&pl)[B]) {
        u32x4 lo, hi;
        codes_to_bytes<B>(pl, lo, hi);
        u32x4 o0, o1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const u32x2 sw = __builtin_amdgcn_permlane32_swap(lo[e], hi[e], false, false);
            o0[e] = sw.x;
            o1[e] = sw.y;
        }
        wf[set][0] = __builtin_bit_cast(i32x4, o0);
        wf[set][1] = __builtin_bit_cast(i32x4, o1);
    };

    load_x(0);
    load_x(1);
#pragma unroll
    for (int u = 0; u < kI8WSets; ++u) load_planes(plane[u], u);
    // scale and zero of the tile's rows (the first quantization block of a row stands for the whole row)
    {
        const int rb = mt * 4 + (tid >> 6), l = tid & 63;
        float sc = 0.f, zs = 0.f;
        if (rb < a.n_row_blocks) {
            const uint8_t* meta = a.tiles + (size_t)rb * a.n_ktiles * TB + B * 1024 + l * MPL;
            sc = (float)*reinterpret_cast<const _Float16*>(meta);
            zs = HZ ? (float)*reinterpret_cast<const _Float16*>(meta + 2) * sc : 0.f;
        }
        row_scale[tid] = sc;
        row_zs[tid] = zs;
    }
    operands(0, plane[0]);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    load_x(2);
    __builtin_amdgcn_sched_barrier(0);
    load_planes(plane[0], kI8WSets);  // (after the activations of stage 2: the waits of the loop count requests in this order)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_barrier" ::: "memory");
    read_x(0, smem);

    for (int s0 = 0; s0 < n_stages; s0 += kI8WSets) {
#pragma unroll
        for (int u = 0; u < kI8WSets; ++u) {
            const int s = s0 + u;
            const uint8_t* nxt = smem + ((s + 1) & (kI8WRing - 1)) * T::XBytes;
            load_x(s + 3);
            __builtin_amdgcn_sched_barrier(0);
            // the MFMAs of stage s; meanwhile the activations and the weight operands of stage s + 1
            read_x((u + 1) & 1, nxt);
            operands((u + 1) & 1, plane[(u + 1) % kI8WSets]);
#pragma unroll
            for (int nb = 0; nb < TT; ++nb) {
                acc[0][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[u & 1][0], xf[u & 1][nb], acc[0][nb], 0, 0, 0);
                acc[1][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[u & 1][1], xf[u & 1][nb], acc[1][nb], 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < 2 * TT; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
                if (i < TT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            load_planes(plane[(u + 1) % kI8WSets], s + 1 + kI8WSets);
            __builtin_amdgcn_sched_barrier(0);
            // the activations of stage s + 2 (requested during stage s - 1) are in before any wave goes on: younger
            // are the weight request of stage s - 1 and the requests just above
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(T::XLoads + 2) : "memory");
        }
    }
    // requests of stages past the end may still be writing zeros to the ring, which the output tile reuses
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // epilogue: C[i][j] of a 32 x 32 tile: i = row 8 (v / 4) + 4 h + v % 4, j = token lane % 32
    uint8_t* otile = smem;
#pragma unroll
    for (int nb = 0; nb < TT; ++nb) {
        const int tok = nb * 32 + r, gn = n0 + tok;
        const bool live = gn < a.N;
        const float delta = live ? a.absmax[gn] * (1.0f / 127.0f) : 0.f;
        const float sx = live ? (float)a.sums[gn] : 0.f;
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int row = wave * 64 + hb * 32 + 8 * g4 + 4 * h;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float av = (float)acc[hb][nb][4 * g4 + e];
                    v[e] = HZ ? delta * fmaf(row_scale[row + e], av, -row_zs[row + e] * sx)
                              : delta * row_scale[row + e] * fmaf(2.f, av, -sx);
                }
                half2_t p0, p1;
                p0.x = (_Float16)v[0]; p0.y = (_Float16)v[1];
                p1.x = (_Float16)v[2]; p1.y = (_Float16)v[3];
                u32x2 w = {__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1)};
                *reinterpret_cast<u32x2*>(otile + tok * T::OutRow + row * 2) = w;
                if (a.acc_out && live) {
                    const int gm = mt * kI8WRows + row;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (gm + e < a.M) a.acc_out[(size_t)gn * a.M + gm + e] = acc[hb][nb][4 * g4 + e];
                }
            }
        }
    }
    __syncthreads();
    const int m0 = mt * kI8WRows;
    const bool fast = (a.M % 8 == 0);  // 16-byte aligned rows of y
    for (int piece = tid; piece < T::TN * (kI8WRows / 8); piece += 256) {
        const int n = piece / (kI8WRows / 8), c8 = piece % (kI8WRows / 8);
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

template <int B, bool HZ, int TT>
static int launch_i8_wide(GemmI8Args a, int group, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_rc = hipSuccess;
    std::call_once(once, [] {
        attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&mpgemm_i8_wide_kernel<B, HZ, TT>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, I8Wide<TT>::LdsBytes);
    });
    if (attr_rc != hipSuccess) return TMAN_ERR_LAUNCH;
    a.m_tiles = (a.n_row_blocks + 3) / 4;
    a.n_tiles = (a.N + I8Wide<TT>::TN - 1) / I8Wide<TT>::TN;
    hipLaunchKernelGGL((mpgemm_i8_wide_kernel<B, HZ, TT>), dim3((unsigned)(a.m_tiles * a.n_tiles)), dim3(256),
                       I8Wide<TT>::LdsBytes, st, a, group);
    return launch_status();
}

// ---------------------------------------------------------------------------------------------
// Third kernel, for grids that leave compute units idle even with 64-row workgroups: the four waves of a workgroup
// split K.  Wave w takes the 32-column stages w, w + 4, ... whole: bit planes -> bytes in registers -> operands
// by v_permlane32_swap (as in the wide kernel), the stage's activations into LDS buffers of its own, MFMAs with all
// tokens of the tile; no wave waits for another until the end, where the four partial integer tiles are added in
// LDS (integers: the result does not depend on the grouping, so every kernel of this file gives the same bits).
// Tile: 128 rows x 128 tokens (two row blocks per wave); the 64 x 256 tile the template also allows was slower
// everywhere here, where the dequantization is cheap and the activation stream is what a wave waits for.
constexpr int kI8KsSets = 4;  // register sets of bit planes = own stages in flight per wave

template <int RBW, int TT>
struct I8KsTile {
    static constexpr int TN = 32 * TT, TM = 64 * RBW;
    static constexpr int XBytes = TN * kI8WStageK;            // activations of a stage, 32 bytes per token
    static constexpr int NBuf = 4;                             // activation buffers per wave
    static constexpr int XLoads = TN / 32;                     // requests per stage (32 token rows each)
    static constexpr int PartRow = TM * 4 + 16;                // bytes per token of a wave's partial tile in LDS
    static constexpr int PartBytes = (TN / 2) * PartRow;       // ... of half of its tokens
    static constexpr int LdsBytes = 4 * NBuf * XBytes > 4 * PartBytes ? 4 * NBuf * XBytes : 4 * PartBytes;
    static_assert(RBW * TT == 8 && LdsBytes + 2 * TM * 4 <= 160 * 1024, "tile of the K-split kernel");
};

template <int B, bool HZ, int RBW, int TT>
__global__ void __launch_bounds__(256, 1) mpgemm_i8_ksplit_kernel(GemmI8Args a, int group) {
    using T = I8KsTile<RBW, TT>;
    constexpr int MSZ = HZ ? 4 : 2;
    constexpr int CH = kKTile / B;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    __shared__ float row_scale[T::TM], row_zs[T::TM];

    const int MPL = (kKTile / group) * MSZ, TB = B * 1024 + 64 * MPL;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mt = blockIdx.x / a.n_tiles, nt = blockIdx.x % a.n_tiles;
    const bool header_ok = header_matches(a.tiles, a.M, a.K, B, group, HZ ? 1 : 0);
    if (!header_ok && blockIdx.x == 0 && tid == 0) report_header_mismatch(a.status);
    if (mt >= (header_ok ? a.m_tiles : 0)) return;
    const int n0 = nt * T::TN;
    const int k_stages = a.K / kI8WStageK;
    const int n_own = (k_stages + 3) / 4, n_own_pad = (n_own + kI8KsSets - 1) & ~(kI8KsSets - 1);
    const int r = lane & 31, h = lane >> 5;

    i32x16 acc[RBW][2][TT];
#pragma unroll
    for (int b = 0; b < RBW; ++b)
#pragma unroll
        for (int hb = 0; hb < 2; ++hb)
#pragma unroll
            for (int nb = 0; nb < TT; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[b][hb][nb][v] = 0;

    uint32_t plane[kI8KsSets][RBW][B];
    auto load_planes = [&](int set, int i) {  // own stage i = stage 4 i + wave, every row block of the tile
        const int t = 4 * i + wave;
        const int tile = t >> 2, kb32 = t & 3;
        const int v = (kb32 * 32) / CH, ksub = ((kb32 * 32) % CH) / 32;
        const int so = tile * TB + v * 1024 + ksub * B * 4;
#pragma unroll
        for (int b = 0; b < RBW; ++b) {
            const int rb = mt * RBW + b;
            const bool wvalid = rb < a.n_row_blocks;
            const uint8_t* wsrc = a.tiles + (size_t)(wvalid ? rb : 0) * a.n_ktiles * TB;
            const rsrc_t rw = rsrc_of(wsrc, t < k_stages && wvalid ? (uint32_t)(a.n_ktiles * TB) : 0u);
            uint32_t (&pl)[B] = plane[set][b];
            if constexpr (B == 4) {
                const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(rw, lane * 16, so, 0);
                pl[0] = w.x; pl[1] = w.y; pl[2] = w.z; pl[3] = w.w;
            } else if constexpr (B == 2) {
                const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rw, lane * 16, so, 0);
                pl[0] = w.x; pl[1] = w.y;
            } else {
                pl[0] = __builtin_amdgcn_raw_buffer_load_b32(rw, lane * 16, so, 0);
            }
        }
    };
    // activations of own stage i go to this wave's buffer i % NBuf: lane -> token row lane / 2, half lane % 2
    const int xrows = a.N - n0 < T::TN ? a.N - n0 : T::TN;
    const int8_t* xsrc = a.xq + (size_t)n0 * a.K;
    const uint32_t xbytes = (uint32_t)xrows * (uint32_t)a.K;
    const uint32_t xlane = (uint32_t)(lane >> 1) * (uint32_t)a.K + (uint32_t)(lane & 1) * 16u;
    const uint32_t x32rows = 32u * (uint32_t)a.K;
    uint8_t* const xbuf = smem + wave * T::NBuf * T::XBytes;
    auto load_x = [&](int i) {
        const int t = 4 * i + wave;
        const rsrc_t rx = rsrc_of(xsrc, t < k_stages ? xbytes : 0u);
        uint8_t* dst = xbuf + (i & (T::NBuf - 1)) * T::XBytes;
#pragma unroll
        for (int q = 0; q < T::XLoads; ++q)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void*)(dst + q * 1024), 16,
                                                     xlane + (uint32_t)q * x32rows, t * kI8WStageK, 0, 0);
    };
    const int xoff = r * 32 + h * 16;
    i32x4 xf[2][TT];
    auto read_x = [&](int set, const uint8_t* stage) {
#pragma unroll
        for (int nb = 0; nb < TT; ++nb) xf[set][nb] = *reinterpret_cast<const i32x4*>(stage + xoff + nb * 1024);
    };
    i32x4 wf[2][RBW][2];  // [set][row block][rows 0..31 / 32..63]
    auto operands = [&](int set, int wset) {
#pragma unroll
        for (int b = 0; b < RBW; ++b) {
            u32x4 lo, hi;
            codes_to_bytes<B>(plane[wset][b], lo, hi);
            u32x4 o0, o1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const u32x2 sw = __builtin_amdgcn_permlane32_swap(lo[e], hi[e], false, false);
                o0[e] = sw.x;
                o1[e] = sw.y;
            }
            wf[set][b][0] = __builtin_bit_cast(i32x4, o0);
            wf[set][b][1] = __builtin_bit_cast(i32x4, o1);
        }
    };

    load_x(0);
#pragma unroll
    for (int i = 0; i < kI8KsSets; ++i) load_planes(i, i);
    // scale and zero of the tile's rows (the first quantization block of a row stands for the whole row)
    if (tid < T::TM) {
        const int rb = mt * RBW + (tid >> 6), l = tid & 63;
        float sc = 0.f, zs = 0.f;
        if (rb < a.n_row_blocks) {
            const uint8_t* meta = a.tiles + (size_t)rb * a.n_ktiles * TB + B * 1024 + l * MPL;
            sc = (float)*reinterpret_cast<const _Float16*>(meta);
            zs = HZ ? (float)*reinterpret_cast<const _Float16*>(meta + 2) * sc : 0.f;
        }
        row_scale[tid] = sc;
        row_zs[tid] = zs;
    }
    operands(0, 0);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = 1; i < T::NBuf; ++i) load_x(i);
    __builtin_amdgcn_sched_barrier(0);
    load_planes(0, kI8KsSets);
    __builtin_amdgcn_sched_barrier(0);
    read_x(0, xbuf);

    for (int i0 = 0; i0 < n_own_pad; i0 += kI8KsSets) {
#pragma unroll
        for (int u = 0; u < kI8KsSets; ++u) {
            const int i = i0 + u;
            const uint8_t* nxt = xbuf + ((i + 1) & (T::NBuf - 1)) * T::XBytes;
            // the MFMAs of own stage i; meanwhile the weight operands of own stage i + 1
            operands((u + 1) & 1, (u + 1) % kI8KsSets);
#pragma unroll
            for (int nb = 0; nb < TT; ++nb)
#pragma unroll
                for (int b = 0; b < RBW; ++b) {
                    acc[b][0][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[u & 1][b][0], xf[u & 1][nb], acc[b][0][nb], 0, 0, 0);
                    acc[b][1][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[u & 1][b][1], xf[u & 1][nb], acc[b][1][nb], 0, 0, 0);
                }
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, RBW == 1 ? 2 : 4, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            // The buffer of own stage i is free now: request own stage i + NBuf into it.  Before the reads that
            // follow, the activations of own stage i + 1 must be in: what was requested after them is at least the
            // activations of NBuf - 2 stages and one stage's bit planes (requests complete in order).
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((T::NBuf - 2) * T::XLoads + RBW) : "memory");
            load_x(i + T::NBuf);
            __builtin_amdgcn_sched_barrier(0);
            load_planes((u + 1) % kI8KsSets, i + 1 + kI8KsSets);
            __builtin_amdgcn_sched_barrier(0);
            read_x((u + 1) & 1, nxt);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // requests of own stages past the end may still be writing zeros to LDS, which the partial tiles reuse
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // The four partial tiles meet in LDS, half of the tokens at a time: wave w writes its int32 sums as
    // [token][row], then thread -> (token, 8 rows) adds the four, scales and stores fp16.
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
                        int32_t* dst = reinterpret_cast<int32_t*>(mine + (nq * 32 + r) * T::PartRow + (64 * b + 32 * hb + 8 * g + 4 * h) * 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) dst[e] = acc[b][hb][nb][4 * g + e];
                    }
        }
        __syncthreads();
        for (int piece = tid; piece < (T::TN / 2) * (T::TM / 8); piece += 256) {
            const int n = piece / (T::TM / 8), c8 = piece % (T::TM / 8);
            const int gn = n0 + half * (T::TN / 2) + n, gm = m0 + c8 * 8;
            int32_t sum[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) sum[e] = 0;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const int32_t* src = reinterpret_cast<const int32_t*>(smem + w * T::PartBytes + n * T::PartRow + c8 * 32);
#pragma unroll
                for (int e = 0; e < 8; ++e) sum[e] += src[e];
            }
            if (gn >= a.N || gm >= a.M) continue;
            const float delta = a.absmax[gn] * (1.0f / 127.0f);
            const float sx = (float)a.sums[gn];
            _Float16 o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float av = (float)sum[e];
                const int row = c8 * 8 + e;
                o[e] = (_Float16)(HZ ? delta * fmaf(row_scale[row], av, -row_zs[row] * sx)
                                     : delta * row_scale[row] * fmaf(2.f, av, -sx));
            }
            _Float16* dst = a.y + (size_t)gn * a.M + gm;
            if (fast && gm + 8 <= a.M) {
                half8_t v;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = o[e];
                *reinterpret_cast<half8_t*>(dst) = v;
            } else {
                for (int t = 0; t < 8 && gm + t < a.M; ++t) dst[t] = o[t];
            }
            if (a.acc_out) {
                for (int t = 0; t < 8 && gm + t < a.M; ++t) a.acc_out[(size_t)gn * a.M + gm + t] = sum[t];
            }
        }
        __syncthreads();
    }
}

template <int B, bool HZ, int RBW, int TT>
static int launch_i8_ksplit(GemmI8Args a, int group, hipStream_t st) {
    using T = I8KsTile<RBW, TT>;
    static std::once_flag once;
    static hipError_t attr_rc = hipSuccess;
    std::call_once(once, [] {
        attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&mpgemm_i8_ksplit_kernel<B, HZ, RBW, TT>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, T::LdsBytes);
    });
    if (attr_rc != hipSuccess) return TMAN_ERR_LAUNCH;
    a.m_tiles = (a.n_row_blocks + RBW - 1) / RBW;
    a.n_tiles = (a.N + T::TN - 1) / T::TN;
    hipLaunchKernelGGL((mpgemm_i8_ksplit_kernel<B, HZ, RBW, TT>), dim3((unsigned)(a.m_tiles * a.n_tiles)), dim3(256),
                       T::LdsBytes, st, a, group);
    return launch_status();
}

template <int B, int GQ, bool HZ>
static int launch_i8_cfg(GemmI8Args a, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_rc = hipSuccess;
    std::call_once(once, [] {
        attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&mpgemm_i8_kernel<B, GQ, HZ>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, kI8LdsBytes);
    });
    if (attr_rc != hipSuccess) return TMAN_ERR_LAUNCH;
    a.m_tiles = (a.n_row_blocks + 1) / 2;
    a.n_tiles = (a.N + kI8Tokens - 1) / kI8Tokens;
    hipLaunchKernelGGL((mpgemm_i8_kernel<B, GQ, HZ>), dim3((unsigned)(a.m_tiles * a.n_tiles)), dim3(256), kI8LdsBytes, st, a);
    return launch_status();
}

template <int B, bool HZ>
static int launch_i8_group(int group, const GemmI8Args& a, hipStream_t st) {
    switch (group) {
        case 32: return launch_i8_cfg<B, 32, HZ>(a, st);
        case 64: return launch_i8_cfg<B, 64, HZ>(a, st);
        default: return launch_i8_cfg<B, 128, HZ>(a, st);
    }
}

template <int B, bool HZ>
static int launch_i8_wide_tokens(int tt, const GemmI8Args& a, int group, hipStream_t st) {
    switch (tt) {
        case 3: return launch_i8_wide<B, HZ, 3>(a, group, st);
        case 4: return launch_i8_wide<B, HZ, 4>(a, group, st);
        case 9: return launch_i8_ksplit<B, HZ, 2, 4>(a, group, st);
        default: return launch_i8_wide<B, HZ, 7>(a, group, st);
    }
}

// Which kernel, and for the wide one how many 32-token blocks per workgroup: the choice with the least modelled
// time.  The model counts rounds of workgroups over the compute units with the time one workgroup took on this
// chip at K = 4096 (microseconds; alone on its unit / sharing it with a second one, which the 96- and 128-token
// tiles allow), scaled by K; the 128 x 128 kernel's time grows linearly with its workgroups.  1 = that kernel,
// 3 / 4 / 7 = the wide kernel with that many 32-token blocks, 9 = the kernel whose waves split K.
int choose_i8_token_blocks(int n_row_blocks, int N, int K) {
    static std::once_flag once;
    static int n_cu = 256;  // assumed when no device answers
    std::call_once(once, [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            n_cu = n;
    });
    const int forced = current_tiling().i8_token_blocks;
    if (forced == 1 || forced == 3 || forced == 4 || forced == 7 || forced == 9) return forced;
    const double k = (double)K / 4096.0;
    const long long old_wgs = (long long)((n_row_blocks + 1) / 2) * ((N + kI8Tokens - 1) / kI8Tokens);
    double best_cost = (17.0 + 0.08 * (double)old_wgs * 256.0 / n_cu) * k;
    int best = 1;
    const int tts[3] = {7, 4, 3};
    const double alone[3] = {59.0, 40.0, 35.0}, shared[3] = {0.0, 58.0, 52.0};
    for (int i = 0; i < 3; ++i) {
        const long long wgs = (long long)((n_row_blocks + 3) / 4) * ((N + 32 * tts[i] - 1) / (32 * tts[i]));
        double cost;
        if (tts[i] > 4) {
            cost = (double)((wgs + n_cu - 1) / n_cu) * alone[i];
        } else {
            const long long full = wgs / (2 * n_cu), rem = wgs % (2 * n_cu);
            cost = (double)full * shared[i] + (rem == 0 ? 0.0 : rem > n_cu ? shared[i] : alone[i]);
        }
        cost *= k;
        if (cost < best_cost) {
            best_cost = cost;
            best = tts[i];
        }
    }
    // the kernel whose waves split K (128 rows x 128 tokens, one workgroup per unit): 19 us per round on an almost
    // empty chip, 25 when every unit streams activations
    if (K >= 2048) {
        const long long wgs = (long long)((n_row_blocks + 1) / 2) * ((N + 127) / 128);
        const double fill = wgs >= n_cu ? 1.0 : (double)wgs / n_cu;
        const double cost = (double)((wgs + n_cu - 1) / n_cu) * (19.0 + 6.0 * fill) * k;
        if (cost < best_cost) {
            best_cost = cost;
            best = 9;
        }
    }
    return best;
}

int launch_mpgemm_i8(const Layout& L, const void* packed, const void* xq_buf, int N, void* y, void* acc_out, hipStream_t st) {
    const ActI8Layout al = act_i8_layout(N, L.K);
    const uint8_t* xb = static_cast<const uint8_t*>(xq_buf);
    GemmI8Args a;
    a.tiles = static_cast<const uint8_t*>(packed) + kHeaderBytes;
    a.xq = reinterpret_cast<const int8_t*>(xb);
    a.absmax = reinterpret_cast<const float*>(xb + al.absmax_off);
    a.sums = reinterpret_cast<const int32_t*>(xb + al.sum_off);
    a.y = static_cast<_Float16*>(y);
    a.acc_out = static_cast<int32_t*>(acc_out);
    a.M = L.M;
    a.N = N;
    a.K = L.K;
    a.n_row_blocks = L.n_row_blocks;
    a.n_ktiles = L.n_ktiles;
    a.m_tiles = a.n_tiles = 0;
    a.status = device_status_word();
    if (!a.status) return TMAN_ERR_LAUNCH;
    const int tt = choose_i8_token_blocks(L.n_row_blocks, N, L.K);
    if (tt > 1) {
        if (L.bits == 1)
            return L.has_zero ? launch_i8_wide_tokens<1, true>(tt, a, L.group, st) : launch_i8_wide_tokens<1, false>(tt, a, L.group, st);
        if (L.bits == 2) return launch_i8_wide_tokens<2, true>(tt, a, L.group, st);
        return launch_i8_wide_tokens<4, true>(tt, a, L.group, st);
    }
    if (L.bits == 1) return L.has_zero ? launch_i8_group<1, true>(L.group, a, st) : launch_i8_group<1, false>(L.group, a, st);
    if (L.bits == 2) return launch_i8_group<2, true>(L.group, a, st);
    return launch_i8_group<4, true>(L.group, a, st);
}

}  // namespace tman
