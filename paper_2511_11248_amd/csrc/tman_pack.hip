// Offline weight repacking into the unified bit-serial layout, and its inverse.
//
// Sec. 4.1 ("Unified Layout through Fused LUT-based Dequantization") stores the weights bit-serially,
// the form decoding needs, and pre-permutes them so both kernels fetch contiguous blocks.  Here one
// thread owns 32 consecutive weights of one row: it splits their codes into `bits` one-bit planes
// (Sec. 2.2 one-bit decomposition) and writes one 32-bit word per plane at the position the layout
// function assigns.  The padded domain (rows up to a multiple of 64, columns up to a multiple of
// 128) is covered too, so the blob is completely defined.
#include "tman_internal.h"

namespace tman {

struct PackGeom {
    int M, K, bits, group, has_zero;
    int n_ktiles, n_row_blocks, tile_bytes, meta_per_lane, meta_entry;
};

static PackGeom geom_of(const Layout& L) {
    return PackGeom{L.M, L.K, L.bits, L.group, L.has_zero, L.n_ktiles, L.n_row_blocks, L.tile_bytes, L.meta_per_lane,
                    L.meta_entry};
}

// byte offset (from the blob start) of the 32-bit word holding plane i of weights k32*32 .. +31 of row m
__device__ __forceinline__ size_t word_offset(const PackGeom& g, int m, int k32, int i) {
    int rb = m / kRows, lane = m % kRows;
    int k = k32 << 5;
    int kt = k / kKTile, kk = k % kKTile;
    int chunk = kKTile / g.bits;  // weights per 16-byte chunk
    int v = kk / chunk, kc = kk % chunk;
    int ksub = kc >> 5;
    return (size_t)kHeaderBytes + ((size_t)rb * g.n_ktiles + kt) * g.tile_bytes + v * 1024 + lane * 16 +
           (ksub * g.bits + i) * 4;
}

// byte offset of the scale of (row m, quantization group G); the zero follows at +2
__device__ __forceinline__ size_t meta_offset(const PackGeom& g, int m, int G) {
    int rb = m / kRows, lane = m % kRows;
    int k0 = G * g.group;
    int kt = k0 / kKTile, gi = (k0 % kKTile) / g.group;
    return (size_t)kHeaderBytes + ((size_t)rb * g.n_ktiles + kt) * g.tile_bytes + g.bits * 1024 +
           lane * g.meta_per_lane + gi * g.meta_entry;
}

__global__ void __launch_bounds__(256) pack_codes_kernel(PackGeom g, const uint8_t* __restrict__ codes,
                                                         uint8_t* __restrict__ packed) {
    int k32_pad = g.n_ktiles * (kKTile / 32);
    long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = (long long)g.n_row_blocks * kRows * k32_pad;
    if (tid >= total) return;
    int m = (int)(tid / k32_pad), k32 = (int)(tid % k32_pad);
    uint32_t plane[4] = {0u, 0u, 0u, 0u};
    if (m < g.M && k32 * 32 < g.K) {  // K is a multiple of 32, so a block is entirely inside or outside
        const uint8_t* src = codes + (size_t)m * g.K + (size_t)k32 * 32;
        for (int t = 0; t < 32; ++t) {
            uint32_t c = src[t];
            for (int i = 0; i < g.bits; ++i) plane[i] |= ((c >> i) & 1u) << t;
        }
    }
    for (int i = 0; i < g.bits; ++i) *reinterpret_cast<uint32_t*>(packed + word_offset(g, m, k32, i)) = plane[i];
}

__global__ void __launch_bounds__(256) pack_meta_kernel(PackGeom g, const uint16_t* __restrict__ scales,
                                                        const uint16_t* __restrict__ zeros,
                                                        uint8_t* __restrict__ packed) {
    int G_pad = g.n_ktiles * (kKTile / g.group);
    int G_real = g.K / g.group;
    long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = (long long)g.n_row_blocks * kRows * G_pad;
    if (tid >= total) return;
    int m = (int)(tid / G_pad), G = (int)(tid % G_pad);
    uint16_t s = 0, z = 0;
    if (m < g.M && G < G_real) {
        s = scales[(size_t)m * G_real + G];
        if (g.has_zero) z = zeros[(size_t)m * G_real + G];
    }
    uint16_t* dst = reinterpret_cast<uint16_t*>(packed + meta_offset(g, m, G));
    dst[0] = s;
    if (g.has_zero) dst[1] = z;
}

__global__ void write_header_kernel(PackGeom g, int32_t* __restrict__ hdr) {
    int t = threadIdx.x;  // 32 threads, one int32 each
    int32_t v = 0;
    switch (t) {
        case 0: v = 0x4e414d54; break;  // "TMAN"
        case 1: v = 0x00314b50; break;  // "PK1\0"
        case 2: v = g.M; break;
        case 3: v = g.K; break;
        case 4: v = g.bits; break;
        case 5: v = g.group; break;
        case 6: v = g.has_zero; break;
        case 7: v = kRows; break;
        case 8: v = kKTile; break;
        case 9: v = g.n_row_blocks; break;
        case 10: v = g.n_ktiles; break;
        case 11: v = g.tile_bytes; break;
        case 12: v = kHeaderBytes; break;
        case 13: v = kLayoutVersion; break;
        default: v = 0;
    }
    hdr[t] = v;
}

__global__ void __launch_bounds__(256) unpack_codes_kernel(PackGeom g, const uint8_t* __restrict__ packed,
                                                           uint8_t* __restrict__ codes) {
    int k32_n = g.K / 32;
    long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = (long long)g.M * k32_n;
    if (tid >= total) return;
    int m = (int)(tid / k32_n), k32 = (int)(tid % k32_n);
    uint32_t plane[4] = {0u, 0u, 0u, 0u};
    for (int i = 0; i < g.bits; ++i) plane[i] = *reinterpret_cast<const uint32_t*>(packed + word_offset(g, m, k32, i));
    uint8_t* dst = codes + (size_t)m * g.K + (size_t)k32 * 32;
    for (int t = 0; t < 32; ++t) {
        uint32_t c = 0;
        for (int i = 0; i < g.bits; ++i) c |= ((plane[i] >> t) & 1u) << i;
        dst[t] = (uint8_t)c;
    }
}

__global__ void __launch_bounds__(256) unpack_meta_kernel(PackGeom g, const uint8_t* __restrict__ packed,
                                                          uint16_t* __restrict__ scales, uint16_t* __restrict__ zeros) {
    int G_real = g.K / g.group;
    long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    long long total = (long long)g.M * G_real;
    if (tid >= total) return;
    int m = (int)(tid / G_real), G = (int)(tid % G_real);
    const uint16_t* src = reinterpret_cast<const uint16_t*>(packed + meta_offset(g, m, G));
    if (scales) scales[(size_t)m * G_real + G] = src[0];
    if (zeros && g.has_zero) zeros[(size_t)m * G_real + G] = src[1];
}

static unsigned blocks_for(long long total) { return (unsigned)((total + 255) / 256); }

int launch_pack(const Layout& L, const uint8_t* codes, const void* scales, const void* zeros, void* packed,
                hipStream_t st) {
    PackGeom g = geom_of(L);
    uint8_t* out = static_cast<uint8_t*>(packed);
    hipLaunchKernelGGL(write_header_kernel, dim3(1), dim3(32), 0, st, g, reinterpret_cast<int32_t*>(out));
    long long n_words = (long long)L.n_row_blocks * kRows * L.n_ktiles * (kKTile / 32);
    hipLaunchKernelGGL(pack_codes_kernel, dim3(blocks_for(n_words)), dim3(256), 0, st, g, codes, out);
    long long n_meta = (long long)L.n_row_blocks * kRows * L.n_ktiles * (kKTile / L.group);
    hipLaunchKernelGGL(pack_meta_kernel, dim3(blocks_for(n_meta)), dim3(256), 0, st, g,
                       static_cast<const uint16_t*>(scales), static_cast<const uint16_t*>(zeros), out);
    return launch_status();
}

int launch_unpack(const Layout& L, const void* packed, uint8_t* codes, void* scales, void* zeros, hipStream_t st) {
    PackGeom g = geom_of(L);
    const uint8_t* in = static_cast<const uint8_t*>(packed);
    long long n_words = (long long)L.M * (L.K / 32);
    hipLaunchKernelGGL(unpack_codes_kernel, dim3(blocks_for(n_words)), dim3(256), 0, st, g, in, codes);
    if (scales || zeros) {
        long long n_meta = (long long)L.M * (L.K / L.group);
        hipLaunchKernelGGL(unpack_meta_kernel, dim3(blocks_for(n_meta)), dim3(256), 0, st, g, in,
                           static_cast<uint16_t*>(scales), static_cast<uint16_t*>(zeros));
    }
    return launch_status();
}

}  // namespace tman
