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
#include <hip/hip_fp16.h>

#include "tman_internal.h"

namespace tman {

__global__ void __launch_bounds__(256) build_tables_kernel(const _Float16* __restrict__ x, int N, int K, int NP,
                                                           int n_tables, _Float16* __restrict__ T) {
    int tid = blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= n_tables * NP) return;
    int j = tid / NP, n = tid % NP;
    float a[4] = {0.f, 0.f, 0.f, 0.f};
    if (n < N) {
        for (int t = 0; t < 4; ++t) {
            int k = 4 * j + t;
            if (k < K) a[t] = (float)x[(size_t)n * K + k];
        }
    }
    _Float16* dst = T + ((size_t)j * 16) * NP + n;
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if ((p >> t) & 1) s += a[t];
        dst[(size_t)p * NP] = (_Float16)s;  // round to nearest even
    }
}

__global__ void __launch_bounds__(256) group_sums_kernel(const _Float16* __restrict__ x, int N, int K, int NP,
                                                         int group, int n_groups, float* __restrict__ S) {
    int tid = blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= n_groups * NP) return;
    int G = tid / NP, n = tid % NP;
    float s = 0.f;
    if (n < N) {
        int k0 = G * group;
        for (int t = 0; t < group; ++t)
            if (k0 + t < K) s += (float)x[(size_t)n * K + k0 + t];
    }
    S[(size_t)G * NP + n] = s;
}

int launch_build_lut(const void* x, int N, int K, int group, void* lut, hipStream_t st) {
    int NP = padded_tokens(N);
    int nkt = (K + kKTile - 1) / kKTile;
    int n_tables = nkt * kTablesPerKTile;
    int n_groups = nkt * (kKTile / group);
    _Float16* T = static_cast<_Float16*>(lut);
    float* S = reinterpret_cast<float*>(static_cast<uint8_t*>(lut) + (size_t)nkt * kTableBytesPerKTile * NP);
    hipLaunchKernelGGL(build_tables_kernel, dim3((n_tables * NP + 255) / 256), dim3(256), 0, st,
                       static_cast<const _Float16*>(x), N, K, NP, n_tables, T);
    hipLaunchKernelGGL(group_sums_kernel, dim3((n_groups * NP + 255) / 256), dim3(256), 0, st,
                       static_cast<const _Float16*>(x), N, K, NP, group, n_groups, S);
    return launch_status();
}

}  // namespace tman
