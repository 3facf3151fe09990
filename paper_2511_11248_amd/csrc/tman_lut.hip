// Lookup-table precompute for decoding (Sec. 2.2 "Bit-serial table lookup"; Sec. 5 "Graph
// optimization" makes it a kernel of its own so several GEMVs share one table).
//
// For every group j of 4 consecutive activations and every 4-bit pattern p the table holds
//   T[n][j][p] = sum_{t<4, bit t of p} x[n][4j+t]
// as a 16-bit entry (Sec. 5: 16-entry tables with 16-bit entries), here fp16 rounded once from an
// fp32 sum taken in ascending t.  The fp32 sums S[n][G] of x over each quantization block follow;
// the GEMV needs them for the zero-point term.
//
// Buffer layout (tokens padded to NP = 1, 2, 4 or 8; K padded to a multiple of 128 with zeros):
//   fp16 element (j * 16 + p) * NP + n          for j < n_ktiles * 32
//   fp32 element  G * NP + n                    at byte offset n_ktiles * 1024 * NP, G < n_ktiles * 128 / group
// so the slice of one K tile is contiguous and can be copied to LDS as it is.
//
// One launch serves up to 8 activations (the distinct inputs of a decode step): the second grid
// dimension is the activation; a thread builds one table of one token and takes part in
// the sum of its quantization block.
#include <hip/hip_fp16.h>

#include "tman_internal.h"

namespace tman {

struct LutJob {
    const _Float16* x;
    _Float16* T;
    float* S;
    int K, n_tables;
};
constexpr int kLutJobsPerLaunch = 8;  // kernel arguments stay small
struct LutJobs {
    LutJob job[kLutJobsPerLaunch];
    int count, N, NP, group;
};

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

// One thread per (table j, token n).  Consecutive lanes own consecutive tables of one token, so the
// group sum of a quantization block (group / 4 tables) is a butterfly over adjacent lanes.
__global__ void __launch_bounds__(256) build_lut_kernel(LutJobs a) {
    // grid = (blocks of the longest activation) x (activations): no search for the job
    const LutJob& jb = a.job[blockIdx.y];
    const int N = a.N, NP = a.NP, K = jb.K;
    if ((int)blockIdx.x * 256 >= jb.n_tables * NP) return;
    const int tid = (int)blockIdx.x * 256 + threadIdx.x;
    const int n = tid / jb.n_tables, j = tid % jb.n_tables;  // n_tables is a multiple of 32
    const bool live = n < NP;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (live && n < N) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int k = 4 * j + t;
            if (k < K) v[t] = (float)jb.x[(size_t)n * K + k];
        }
    }
    _Float16 e[16];
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if ((p >> t) & 1) s += v[t];
        e[p] = (_Float16)s;  // round to nearest even
    }
    if (live) {
        if (NP == 1) {
            half8_t lo, hi;
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                lo[p] = e[p];
                hi[p] = e[p + 8];
            }
            half8_t* dst = reinterpret_cast<half8_t*>(jb.T + (size_t)j * 16);
            dst[0] = lo;
            dst[1] = hi;
        } else {
            _Float16* dst = jb.T + ((size_t)j * 16) * NP + n;
#pragma unroll
            for (int p = 0; p < 16; ++p) dst[(size_t)p * NP] = e[p];
        }
    }
    // group sums: add the four activations, then the group / 4 tables of the block
    float s = (v[0] + v[1]) + (v[2] + v[3]);
    const int tables_per_group = a.group / kLutGroup;  // 8, 16 or 32: within one wave
    for (int d = 1; d < tables_per_group; d <<= 1) s += __shfl_xor(s, d, 64);
    if (live && (j % tables_per_group) == 0) jb.S[(size_t)(j / tables_per_group) * NP + n] = s;
}

int launch_build_lut_batch(int count, const void* const* x, int N, const int* K, int group, void* const* lut,
                           hipStream_t st) {
    const int NP = padded_tokens(N);
    for (int i0 = 0; i0 < count; i0 += kLutJobsPerLaunch) {
        LutJobs a;
        a.count = count - i0 < kLutJobsPerLaunch ? count - i0 : kLutJobsPerLaunch;
        a.N = N;
        a.NP = NP;
        a.group = group;
        int blocks = 0;  // of the longest activation
        for (int i = 0; i < kLutJobsPerLaunch; ++i) {
            const int src = i0 + (i < a.count ? i : 0);
            const int nkt = (K[src] + kKTile - 1) / kKTile;
            LutJob& jb = a.job[i];
            jb.x = static_cast<const _Float16*>(x[src]);
            jb.T = static_cast<_Float16*>(lut[src]);
            jb.S = reinterpret_cast<float*>(static_cast<uint8_t*>(lut[src]) + (size_t)nkt * kTableBytesPerKTile * NP);
            jb.K = K[src];
            jb.n_tables = nkt * kTablesPerKTile;
            const int b = (jb.n_tables * NP + 255) / 256;
            if (i < a.count && b > blocks) blocks = b;
        }
        hipLaunchKernelGGL(build_lut_kernel, dim3((unsigned)blocks, (unsigned)a.count), dim3(256), 0, st, a);
    }
    return launch_status();
}

// ---------------------------------------------------------------------------------------------
// Integer tables (Sec. 6.1 "A_INT16"; Sec. 5: 16-bit table entries).
//
// Every token gets a power-of-two step 2^e, the smallest for which all |x| / 2^e <= 8191, and integer
// activations xq = round_to_nearest_even(x / 2^e); four of them always sum to a 16-bit integer, so the table
//   Tq[n][j][p] = sum_{t<4, bit t of p} xq[n][4j+t]
// is exact.  Dividing an fp16 number by a power of two is exact in fp32, so xq does not depend on the precision
// it is computed in.  With the largest |x| = m * 2^E (0.5 <= m < 1), e = E - 13; a token of zeros gets e = 0.
// The activations must be finite.
//
// Buffer layout: as the fp16 tables (int16 element (j * 16 + p) * NP + n, then the int32 block sums, element
// G * NP + n), followed by the int32 exponents e[n], n < NP.
//
// grid = (blocks of 256 tables) x (padded tokens) x (activations); every block first finds its token's largest
// magnitude (K fp16 numbers: a few KB from L2), then builds 256 tables.
__global__ void __launch_bounds__(256) build_lut_i16_kernel(LutJobs a) {
    __shared__ unsigned wave_max[4];
    const LutJob& jb = a.job[blockIdx.z];
    const int N = a.N, NP = a.NP, K = jb.K;
    if ((int)blockIdx.x * 256 >= jb.n_tables) return;
    const int n = blockIdx.y, j = (int)blockIdx.x * 256 + threadIdx.x;
    const uint16_t* xb = reinterpret_cast<const uint16_t*>(jb.x) + (size_t)n * K;
    // magnitudes compare like their bit patterns
    unsigned mx = 0;
    if (n < N) {
        // 16 bytes per thread and step where the row allows it (K is a multiple of 32; the row start is 16-byte
        // aligned when x is and K * 2 is a multiple of 16, which it is)
        if ((reinterpret_cast<uintptr_t>(xb) & 15u) == 0) {
            typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
            const u32x4_t* x16 = reinterpret_cast<const u32x4_t*>(xb);
            for (int c = threadIdx.x; c < K / 8; c += 256) {
                const u32x4_t w = x16[c];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t d = w[i] & 0x7fff7fffu;
                    mx = max(mx, max(d & 0xffffu, d >> 16));
                }
            }
        } else {
            for (int k = threadIdx.x; k < K; k += 256) mx = max(mx, (unsigned)(xb[k] & 0x7fffu));
        }
    }
    for (int d = 1; d < 64; d <<= 1) mx = max(mx, (unsigned)__shfl_xor((int)mx, d, 64));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
    int e = 0;
    if (mx != 0) {
        const int eb = (int)(mx >> 10), f = (int)(mx & 0x3ffu);
        // normal: (1024 + f) * 2^(eb - 25) lies in [2^(eb - 15), 2^(eb - 14)); subnormal: f * 2^-24
        const int E = eb != 0 ? eb - 14 : (32 - __builtin_clz((unsigned)f)) - 24;
        e = E - 13;
    }
    int* S = reinterpret_cast<int*>(jb.S);
    int* ex = S + (size_t)(jb.n_tables / kTablesPerKTile) * (kKTile / a.group) * NP;
    if (blockIdx.x == 0 && threadIdx.x == 0) ex[n] = e;

    const bool live = j < jb.n_tables;
    int v[4] = {0, 0, 0, 0};
    if (live && n < N) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int k = 4 * j + t;
            if (k < K) v[t] = (int)rintf(ldexpf((float)__builtin_bit_cast(_Float16, xb[k]), -e));
        }
    }
    int16_t q[16];
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        int s = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if ((p >> t) & 1) s += v[t];
        q[p] = (int16_t)s;
    }
    if (live) {
        int16_t* dst = reinterpret_cast<int16_t*>(jb.T) + ((size_t)j * 16) * NP + n;
#pragma unroll
        for (int p = 0; p < 16; ++p) dst[(size_t)p * NP] = q[p];
    }
    int s = (v[0] + v[1]) + (v[2] + v[3]);
    const int tables_per_group = a.group / kLutGroup;  // 8, 16 or 32: within one wave
    for (int d = 1; d < tables_per_group; d <<= 1) s += __shfl_xor(s, d, 64);
    if (live && (j % tables_per_group) == 0) S[(size_t)(j / tables_per_group) * NP + n] = s;
}

int launch_build_lut_i16_batch(int count, const void* const* x, int N, const int* K, int group, void* const* lut,
                               hipStream_t st) {
    const int NP = padded_tokens(N);
    for (int i0 = 0; i0 < count; i0 += kLutJobsPerLaunch) {
        LutJobs a;
        a.count = count - i0 < kLutJobsPerLaunch ? count - i0 : kLutJobsPerLaunch;
        a.N = N;
        a.NP = NP;
        a.group = group;
        int blocks = 0;  // of the longest activation
        for (int i = 0; i < kLutJobsPerLaunch; ++i) {
            const int src = i0 + (i < a.count ? i : 0);
            const int nkt = (K[src] + kKTile - 1) / kKTile;
            LutJob& jb = a.job[i];
            jb.x = static_cast<const _Float16*>(x[src]);
            jb.T = static_cast<_Float16*>(lut[src]);
            jb.S = reinterpret_cast<float*>(static_cast<uint8_t*>(lut[src]) + (size_t)nkt * kTableBytesPerKTile * NP);
            jb.K = K[src];
            jb.n_tables = nkt * kTablesPerKTile;
            const int b = (jb.n_tables + 255) / 256;
            if (i < a.count && b > blocks) blocks = b;
        }
        hipLaunchKernelGGL(build_lut_i16_kernel, dim3((unsigned)blocks, (unsigned)NP, (unsigned)a.count), dim3(256), 0, st, a);
    }
    return launch_status();
}

int launch_build_lut(const void* x, int N, int K, int group, void* lut, hipStream_t st) {
    return launch_build_lut_batch(1, &x, N, &K, group, &lut, st);
}

}  // namespace tman
