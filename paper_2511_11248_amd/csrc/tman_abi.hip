// C ABI of libtman: argument validation, size queries and dispatch to the kernel launchers.
// Everything here runs on the host and validates before anything is enqueued.
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "tman_internal.h"

namespace tman {

// The library's device status word: kernels that find a packed blob whose header disagrees with the shape they
// were launched for store TMAN_ERR_HEADER here (and leave their outputs alone); tman_device_status reads it.
// The array's name is a host-side stand-in for the symbol; kernels receive its device address, looked up once
// per device.
static __device__ int status_word;
static std::mutex status_mutex;
static int* status_ptr[64];

int* device_status_word() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(status_mutex);
    if (!status_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(status_word)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        status_ptr[dev] = static_cast<int*>(p);
    }
    return status_ptr[dev];
}

}  // namespace tman

using namespace tman;

extern "C" {

size_t tman_packed_bytes(const tman_shape_t* shape) {
    if (check_shape(shape) != TMAN_OK) return 0;
    return make_layout(shape).total_bytes;
}

size_t tman_lut_bytes(int32_t N, int32_t K, int32_t group) {
    if (N < 1 || N > TMAN_MAX_DECODE_TOKENS || K < 1) return 0;
    if (group != 32 && group != 64 && group != 128) return 0;
    if (K % group != 0) return 0;
    size_t nkt = (size_t)(K + kKTile - 1) / kKTile;
    size_t np = (size_t)padded_tokens(N);
    return nkt * kTableBytesPerKTile * np + nkt * (kKTile / group) * np * sizeof(float);
}

size_t tman_lut_i16_bytes(int32_t N, int32_t K, int32_t group) {
    const size_t b = tman_lut_bytes(N, K, group);  // 16-bit entries and 32-bit block sums, as the fp16 tables
    return b ? b + 32 : 0;                          // + the tokens' exponents (8 x int32)
}

size_t tman_mpgemv_workspace_bytes(const tman_shape_t* shape, int32_t N) {
    if (check_shape(shape) != TMAN_OK || N < 1 || N > TMAN_MAX_DECODE_TOKENS) return 0;
    const Layout L = make_layout(shape);
    GemvPlan p = plan_gemv(L, N);
    size_t need = p.ticket_bytes + p.partial_bytes;
    if (N == 1) {  // also serves tman_mpgemv_x, which cuts K into shorter segments
        GemvPlan px = plan_gemv_x(L);
        if (px.ticket_bytes + px.partial_bytes > need) need = px.ticket_bytes + px.partial_bytes;
    }
    return need;
}

size_t tman_mpgemm_workspace_bytes(const tman_shape_t* shape, int32_t N) {
    if (check_shape(shape) != TMAN_OK || N < 1) return 0;
    if (N > TMAN_MAX_SMALL_TOKENS) return 0;  // the tiled prefill kernel needs no scratch memory
    const GemvPlan p = plan_small(make_layout(shape));  // a long K is cut into segments that meet in the workspace
    return p.n_seg > 1 ? p.ticket_bytes + p.partial_bytes : 0;
}

int tman_pack_weights(const tman_shape_t* shape, const uint8_t* codes, const void* scales, const void* zeros,
                      void* packed, void* stream) {
    int rc = check_shape(shape);
    if (rc != TMAN_OK) return rc;
    if (!codes || !scales || !packed) return TMAN_ERR_NULL;
    bool hz = shape->flags & TMAN_FLAG_HAS_ZERO;
    if (hz && !zeros) return TMAN_ERR_NULL;
    if (!hz && zeros) return TMAN_ERR_SHAPE;
    if (!aligned16(packed)) return TMAN_ERR_ALIGN;
    return launch_pack(make_layout(shape), codes, scales, zeros, packed, (hipStream_t)stream);
}

int tman_unpack_weights(const tman_shape_t* shape, const void* packed, uint8_t* codes, void* scales, void* zeros,
                        void* stream) {
    int rc = check_shape(shape);
    if (rc != TMAN_OK) return rc;
    if (!packed || !codes) return TMAN_ERR_NULL;
    if (!aligned16(packed)) return TMAN_ERR_ALIGN;
    if (zeros && !(shape->flags & TMAN_FLAG_HAS_ZERO)) return TMAN_ERR_SHAPE;
    return launch_unpack(make_layout(shape), packed, codes, scales, zeros, (hipStream_t)stream);
}

int tman_build_lut(const void* x, int32_t N, int32_t K, int32_t group, void* lut, void* stream) {
    if (!x || !lut) return TMAN_ERR_NULL;
    if (group != 32 && group != 64 && group != 128) return TMAN_ERR_GROUP;
    if (N < 1 || N > TMAN_MAX_DECODE_TOKENS || K < 1 || K % group != 0) return TMAN_ERR_SHAPE;
    if (!aligned16(lut)) return TMAN_ERR_ALIGN;
    return launch_build_lut(x, N, K, group, lut, (hipStream_t)stream);
}

int tman_build_lut_batch(int32_t count, const void* const* x, int32_t N, const int32_t* K, int32_t group,
                         void* const* lut, void* stream) {
    if (!x || !K || !lut) return TMAN_ERR_NULL;
    if (group != 32 && group != 64 && group != 128) return TMAN_ERR_GROUP;
    if (count < 1 || count > TMAN_MAX_BATCH || N < 1 || N > TMAN_MAX_DECODE_TOKENS) return TMAN_ERR_SHAPE;
    for (int i = 0; i < count; ++i) {
        if (!x[i] || !lut[i]) return TMAN_ERR_NULL;
        if (K[i] < 1 || K[i] % group != 0) return TMAN_ERR_SHAPE;
        if (!aligned16(lut[i])) return TMAN_ERR_ALIGN;
    }
    return launch_build_lut_batch(count, x, N, K, group, lut, (hipStream_t)stream);
}

int tman_build_lut_i16(const void* x, int32_t N, int32_t K, int32_t group, void* lut, void* stream) {
    if (!x || !lut) return TMAN_ERR_NULL;
    if (group != 32 && group != 64 && group != 128) return TMAN_ERR_GROUP;
    if (N < 1 || N > TMAN_MAX_DECODE_TOKENS || K < 1 || K % group != 0) return TMAN_ERR_SHAPE;
    if (!aligned16(lut)) return TMAN_ERR_ALIGN;
    return launch_build_lut_i16_batch(1, &x, N, &K, group, &lut, (hipStream_t)stream);
}

int tman_build_lut_i16_batch(int32_t count, const void* const* x, int32_t N, const int32_t* K, int32_t group,
                             void* const* lut, void* stream) {
    if (!x || !K || !lut) return TMAN_ERR_NULL;
    if (group != 32 && group != 64 && group != 128) return TMAN_ERR_GROUP;
    if (count < 1 || count > TMAN_MAX_BATCH || N < 1 || N > TMAN_MAX_DECODE_TOKENS) return TMAN_ERR_SHAPE;
    for (int i = 0; i < count; ++i) {
        if (!x[i] || !lut[i]) return TMAN_ERR_NULL;
        if (K[i] < 1 || K[i] % group != 0) return TMAN_ERR_SHAPE;
        if (!aligned16(lut[i])) return TMAN_ERR_ALIGN;
    }
    return launch_build_lut_i16_batch(count, x, N, K, group, lut, (hipStream_t)stream);
}

int tman_mpgemv_i16(const tman_shape_t* shape, const void* packed, const void* lut, int32_t N, void* y, void* workspace,
                    size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != TMAN_OK) return rc;
    if (!packed || !lut || !y) return TMAN_ERR_NULL;
    if (N < 1 || N > TMAN_MAX_DECODE_TOKENS) return TMAN_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(lut)) return TMAN_ERR_ALIGN;
    size_t need = tman_mpgemv_workspace_bytes(shape, N);
    if (need && (!workspace || workspace_bytes < need)) return TMAN_ERR_WORKSPACE;
    if (workspace && !aligned16(workspace)) return TMAN_ERR_ALIGN;
    return launch_mpgemv_i16(make_layout(shape), packed, lut, N, y, workspace, (hipStream_t)stream);
}

int tman_mpgemv(const tman_shape_t* shape, const void* packed, const void* lut, int32_t N, void* y, void* workspace,
                size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != TMAN_OK) return rc;
    if (!packed || !lut || !y) return TMAN_ERR_NULL;
    if (N < 1 || N > TMAN_MAX_DECODE_TOKENS) return TMAN_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(lut)) return TMAN_ERR_ALIGN;
    size_t need = tman_mpgemv_workspace_bytes(shape, N);
    if (need && (!workspace || workspace_bytes < need)) return TMAN_ERR_WORKSPACE;
    if (workspace && !aligned16(workspace)) return TMAN_ERR_ALIGN;
    return launch_mpgemv(make_layout(shape), packed, lut, N, y, workspace, (hipStream_t)stream);
}

// A descriptor table: the GEMV descriptors, then (one-token batches whose workgroups are numbered for balance) the
// numbering.
static size_t desc_table_bytes(int count) { return ((size_t)count * sizeof(GemvDesc) + 255) / 256 * 256; }
static uint16_t* order_of(void* desc, int count) {
    return reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(desc) + desc_table_bytes(count));
}
static int device_units() {
    static std::once_flag once;
    static int n_units = 0;
    std::call_once(once, [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            n_units = n;
    });
    return n_units;
}

size_t tman_mpgemv_batch_desc_bytes(int32_t count) {
    if (count < 1 || count > TMAN_MAX_BATCH) return 0;
    return desc_table_bytes(count) + (size_t)kOrderedMaxWorkgroups * sizeof(uint16_t);
}

static int check_batch(int32_t count, const tman_shape_t* shapes, int32_t N) {
    if (!shapes) return TMAN_ERR_NULL;
    if (count < 1 || count > TMAN_MAX_BATCH) return TMAN_ERR_SHAPE;
    if (N < 1 || N > TMAN_MAX_DECODE_TOKENS) return TMAN_ERR_SHAPE;
    long long total = 0;
    for (int i = 0; i < count; ++i) {
        int rc = check_shape(&shapes[i]);
        if (rc != TMAN_OK) return rc;
        if (shapes[i].bits != shapes[0].bits || shapes[i].group != shapes[0].group ||
            shapes[i].flags != shapes[0].flags)
            return TMAN_ERR_SHAPE;  // one launch runs one weight format
        total += plan_gemv(make_layout(&shapes[i]), N).n_workgroups;
    }
    if (total > 0x7fffffffLL) return TMAN_ERR_SHAPE;
    return TMAN_OK;
}

int tman_mpgemv_batch_prepare(int32_t count, const tman_shape_t* shapes, const void* const* packed,
                              const void* const* lut, int32_t N, void* const* y, void* const* workspace,
                              const size_t* workspace_bytes, void* desc, void* stream) {
    int rc = check_batch(count, shapes, N);
    if (rc != TMAN_OK) return rc;
    if (!packed || !lut || !y || !workspace || !workspace_bytes || !desc) return TMAN_ERR_NULL;
    if (!aligned16(desc)) return TMAN_ERR_ALIGN;
    GemvDesc host[TMAN_MAX_BATCH];
    int wg_begin = 0;
    for (int i = 0; i < count; ++i) {
        if (!packed[i] || !lut[i] || !y[i] || !workspace[i]) return TMAN_ERR_NULL;
        if (!aligned16(packed[i]) || !aligned16(lut[i]) || !aligned16(workspace[i])) return TMAN_ERR_ALIGN;
        if (workspace_bytes[i] < tman_mpgemv_workspace_bytes(&shapes[i], N)) return TMAN_ERR_WORKSPACE;
        for (int j = 0; j < i; ++j)
            if (workspace[j] == workspace[i]) return TMAN_ERR_WORKSPACE;  // every GEMV needs its own
        Layout L = make_layout(&shapes[i]);
        fill_desc(host[i], L, packed[i], lut[i], N, y[i], workspace[i], wg_begin);
        wg_begin += plan_gemv(L, N).n_workgroups;
    }
    return launch_write_descs(host, count, shapes[0].bits, shapes[0].group, (shapes[0].flags & TMAN_FLAG_HAS_ZERO) ? 1 : 0,
                              static_cast<GemvDesc*>(desc), (hipStream_t)stream);
}

int tman_mpgemv_batch_run(int32_t count, const tman_shape_t* shapes, int32_t N, const void* desc, void* stream) {
    int rc = check_batch(count, shapes, N);
    if (rc != TMAN_OK) return rc;
    if (!desc) return TMAN_ERR_NULL;
    if (!aligned16(desc)) return TMAN_ERR_ALIGN;
    int max_wg = 0;  // the launch grid is (workgroups of the largest GEMV) x count
    for (int i = 0; i < count; ++i) {
        const int n = plan_gemv(make_layout(&shapes[i]), N).n_workgroups;
        if (n > max_wg) max_wg = n;
    }
    return launch_mpgemv_batch(shapes[0].bits, shapes[0].group, shapes[0].flags & TMAN_FLAG_HAS_ZERO, N,
                               static_cast<const GemvDesc*>(desc), count, max_wg, (hipStream_t)stream);
}

int tman_mpgemv_i16_batch_run(int32_t count, const tman_shape_t* shapes, int32_t N, const void* desc, void* stream) {
    int rc = check_batch(count, shapes, N);
    if (rc != TMAN_OK) return rc;
    if (!desc) return TMAN_ERR_NULL;
    if (!aligned16(desc)) return TMAN_ERR_ALIGN;
    int max_wg = 0;
    for (int i = 0; i < count; ++i) {
        const int n = plan_gemv(make_layout(&shapes[i]), N).n_workgroups;
        if (n > max_wg) max_wg = n;
    }
    return launch_mpgemv_i16_batch(shapes[0].bits, shapes[0].group, shapes[0].flags & TMAN_FLAG_HAS_ZERO, N,
                                   static_cast<const GemvDesc*>(desc), count, max_wg, (hipStream_t)stream);
}

int tman_mpgemv_x(const tman_shape_t* shape, const void* packed, const void* x, void* y, void* workspace,
                  size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != TMAN_OK) return rc;
    if (!packed || !x || !y) return TMAN_ERR_NULL;
    if (!aligned16(packed) || !aligned16(x)) return TMAN_ERR_ALIGN;
    size_t need = tman_mpgemv_workspace_bytes(shape, 1);
    if (need && (!workspace || workspace_bytes < need)) return TMAN_ERR_WORKSPACE;
    if (workspace && !aligned16(workspace)) return TMAN_ERR_ALIGN;
    return launch_mpgemv_x(make_layout(shape), packed, x, y, workspace, (hipStream_t)stream);
}

int tman_mpgemv_x_batch_prepare(int32_t count, const tman_shape_t* shapes, const void* const* packed,
                                const void* const* x, void* const* y, void* const* workspace,
                                const size_t* workspace_bytes, void* desc, void* stream) {
    int rc = check_batch(count, shapes, 1);
    if (rc != TMAN_OK) return rc;
    if (!packed || !x || !y || !workspace || !workspace_bytes || !desc) return TMAN_ERR_NULL;
    if (!aligned16(desc)) return TMAN_ERR_ALIGN;
    GemvDesc host[TMAN_MAX_BATCH];
    for (int i = 0; i < count; ++i) {
        if (!packed[i] || !x[i] || !y[i] || !workspace[i]) return TMAN_ERR_NULL;
        if (!aligned16(packed[i]) || !aligned16(x[i]) || !aligned16(workspace[i])) return TMAN_ERR_ALIGN;
        if (workspace_bytes[i] < tman_mpgemv_workspace_bytes(&shapes[i], 1)) return TMAN_ERR_WORKSPACE;
        for (int j = 0; j < i; ++j)
            if (workspace[j] == workspace[i]) return TMAN_ERR_WORKSPACE;  // every GEMV needs its own
        fill_desc_x(host[i], make_layout(&shapes[i]), packed[i], x[i], y[i], workspace[i]);
    }
    rc = launch_write_descs(host, count, shapes[0].bits, shapes[0].group, (shapes[0].flags & TMAN_FLAG_HAS_ZERO) ? 1 : 0,
                            static_cast<GemvDesc*>(desc), (hipStream_t)stream);
    if (rc != TMAN_OK) return rc;
    // a launch whose workgroups are all resident at once gets them numbered for equal work per compute unit
    std::vector<Layout> L(count);
    for (int i = 0; i < count; ++i) L[i] = make_layout(&shapes[i]);
    std::vector<uint16_t> order;
    if (!order_workgroups(count, L.data(), device_units(), &order)) return TMAN_OK;
    return launch_write_order(order, order_of(desc, count), (hipStream_t)stream);
}

int tman_mpgemv_x_batch_order(int32_t count, const tman_shape_t* shapes, int32_t n_units, uint16_t* order,
                              int32_t max_entries, int32_t* n_entries) {
    int rc = check_batch(count, shapes, 1);
    if (rc != TMAN_OK) return rc;
    if (!n_entries) return TMAN_ERR_NULL;
    if (n_units < 0 || max_entries < 0) return TMAN_ERR_SHAPE;
    std::vector<Layout> L(count);
    for (int i = 0; i < count; ++i) L[i] = make_layout(&shapes[i]);
    std::vector<uint16_t> o;
    if (!order_workgroups(count, L.data(), n_units > 0 ? n_units : device_units(), &o)) o.clear();
    *n_entries = (int32_t)o.size();
    if (order)
        for (size_t i = 0; i < o.size() && i < (size_t)max_entries; ++i) order[i] = o[i];
    return TMAN_OK;
}

int tman_mpgemv_x_batch_run(int32_t count, const tman_shape_t* shapes, const void* desc, void* stream) {
    int rc = check_batch(count, shapes, 1);
    if (rc != TMAN_OK) return rc;
    if (!desc) return TMAN_ERR_NULL;
    if (!aligned16(desc)) return TMAN_ERR_ALIGN;
    int max_wg = 0, max_seg_tiles = 0;  // grid = (workgroups of the largest GEMV) x count; LDS for the longest segment
    for (int i = 0; i < count; ++i) {
        const GemvPlan p = plan_gemv_x(make_layout(&shapes[i]));
        if (p.n_workgroups > max_wg) max_wg = p.n_workgroups;
        if (p.seg_tiles > max_seg_tiles) max_seg_tiles = p.seg_tiles;
    }
    {
        Layout L[8];
        for (int i = 0; i < count && i < 8; ++i) L[i] = make_layout(&shapes[i]);
        if (const int n_wg = ordered_workgroups(count, L, device_units()))
            return launch_mpgemv_x_ordered(shapes[0].bits, shapes[0].group, shapes[0].flags & TMAN_FLAG_HAS_ZERO,
                                           static_cast<const GemvDesc*>(desc), count,
                                           order_of(const_cast<void*>(desc), count), n_wg, max_seg_tiles,
                                           (hipStream_t)stream);
    }
    return launch_mpgemv_x_batch(shapes[0].bits, shapes[0].group, shapes[0].flags & TMAN_FLAG_HAS_ZERO,
                                 static_cast<const GemvDesc*>(desc), count, max_wg, max_seg_tiles, (hipStream_t)stream);
}

int32_t tman_mpgemm_tile_rows(const tman_shape_t* shape, int32_t N) {
    if (check_shape(shape) != TMAN_OK || N < 1) return 0;
    return kRows * mpgemm_row_blocks_per_workgroup(make_layout(shape), N);
}

int32_t tman_mpgemm_splits_k(const tman_shape_t* shape, int32_t N) {
    if (check_shape(shape) != TMAN_OK || N < 1) return -1;
    return mpgemm_splits_k(make_layout(shape), N);
}

int32_t tman_mpgemm_i8_token_blocks(const tman_shape_t* shape, int32_t N) {
    if (check_shape(shape) != TMAN_OK || N < 1) return 0;
    const Layout L = make_layout(shape);
    return choose_i8_token_blocks(L.n_row_blocks, N, L.K);
}

int tman_mpgemm(const tman_shape_t* shape, const void* packed, const void* x, int32_t N, void* y, void* workspace,
                size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != TMAN_OK) return rc;
    if (!packed || !x || !y) return TMAN_ERR_NULL;
    if (N < 1) return TMAN_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(x)) return TMAN_ERR_ALIGN;
    size_t need = tman_mpgemm_workspace_bytes(shape, N);
    if (need && (!workspace || workspace_bytes < need)) return TMAN_ERR_WORKSPACE;
    if (need && !aligned16(workspace)) return TMAN_ERR_ALIGN;
    const Layout L = make_layout(shape);
    if (N <= TMAN_MAX_SMALL_TOKENS) {
        if ((long long)N * L.K * 2 > 0xFFFFFFF0LL) return TMAN_ERR_SHAPE;  // the activations are one buffer resource
        return launch_mpgemm_small(L, packed, x, N, y, need ? workspace : nullptr, (hipStream_t)stream);
    }
    return launch_mpgemm(L, packed, x, N, y, workspace, (hipStream_t)stream);
}

int tman_mpgemm_batch_prepare(int32_t count, const tman_shape_t* shapes, const void* const* packed,
                              const void* const* x, int32_t N, void* const* y, void* const* workspace,
                              const size_t* workspace_bytes, void* desc, void* stream) {
    int rc = check_batch(count, shapes, 1);
    if (rc != TMAN_OK) return rc;
    if (N < 1 || N > TMAN_MAX_SMALL_TOKENS) return TMAN_ERR_SHAPE;
    if (!packed || !x || !y || !workspace || !workspace_bytes || !desc) return TMAN_ERR_NULL;
    if (!aligned16(desc)) return TMAN_ERR_ALIGN;
    GemvDesc host[TMAN_MAX_BATCH];
    for (int i = 0; i < count; ++i) {
        if (!packed[i] || !x[i] || !y[i]) return TMAN_ERR_NULL;
        if (!aligned16(packed[i]) || !aligned16(x[i])) return TMAN_ERR_ALIGN;
        const size_t need = tman_mpgemm_workspace_bytes(&shapes[i], N);
        if (need) {
            if (!workspace[i] || workspace_bytes[i] < need) return TMAN_ERR_WORKSPACE;
            if (!aligned16(workspace[i])) return TMAN_ERR_ALIGN;
            for (int j = 0; j < i; ++j)
                if (workspace[j] == workspace[i]) return TMAN_ERR_WORKSPACE;  // every GEMM needs its own
        }
        if ((long long)N * shapes[i].K * 2 > 0xFFFFFFF0LL) return TMAN_ERR_SHAPE;
        fill_desc_small(host[i], make_layout(&shapes[i]), packed[i], x[i], N, y[i], need ? workspace[i] : nullptr);
    }
    rc = launch_write_descs(host, count, shapes[0].bits, shapes[0].group, (shapes[0].flags & TMAN_FLAG_HAS_ZERO) ? 1 : 0,
                            static_cast<GemvDesc*>(desc), (hipStream_t)stream);
    if (rc != TMAN_OK) return rc;
    std::vector<Layout> L(count);
    for (int i = 0; i < count; ++i) L[i] = make_layout(&shapes[i]);
    std::vector<uint16_t> order;
    if (!order_workgroups_small(count, L.data(), device_units(), &order)) return TMAN_OK;
    return launch_write_order(order, order_of(desc, count), (hipStream_t)stream);
}

int tman_mpgemm_batch_run(int32_t count, const tman_shape_t* shapes, int32_t N, const void* desc, void* stream) {
    int rc = check_batch(count, shapes, 1);
    if (rc != TMAN_OK) return rc;
    if (N < 1 || N > TMAN_MAX_SMALL_TOKENS) return TMAN_ERR_SHAPE;
    if (!desc) return TMAN_ERR_NULL;
    if (!aligned16(desc)) return TMAN_ERR_ALIGN;
    {
        Layout L[8];
        for (int i = 0; i < count && i < 8; ++i) L[i] = make_layout(&shapes[i]);
        if (const int n_wg = ordered_workgroups_small(count, L, device_units()))
            return launch_mpgemm_small_ordered(shapes[0].bits, shapes[0].group, shapes[0].flags & TMAN_FLAG_HAS_ZERO,
                                               static_cast<const GemvDesc*>(desc), count,
                                               order_of(const_cast<void*>(desc), count), n_wg, (hipStream_t)stream);
    }
    int max_wg = 0;  // the launch grid is (workgroups of the largest GEMM) x count
    for (int i = 0; i < count; ++i) {
        const int n = plan_small(make_layout(&shapes[i])).n_workgroups;
        if (n > max_wg) max_wg = n;
    }
    return launch_mpgemm_small_batch(shapes[0].bits, shapes[0].group, shapes[0].flags & TMAN_FLAG_HAS_ZERO,
                                     static_cast<const GemvDesc*>(desc), count, max_wg, (hipStream_t)stream);
}

size_t tman_act_i8_bytes(int32_t N, int32_t K) {
    if (N < 1 || K < 1 || K % 32 != 0 || (long long)N * K > 0xFFFFFFF0LL) return 0;
    return act_i8_bytes(N, K);
}

int tman_quantize_act_i8(const void* x, int32_t N, int32_t K, void* xq, void* stream) {
    if (!x || !xq) return TMAN_ERR_NULL;
    if (tman_act_i8_bytes(N, K) == 0) return TMAN_ERR_SHAPE;
    if (!aligned16(xq)) return TMAN_ERR_ALIGN;
    return launch_quantize_act_i8(x, N, K, xq, (hipStream_t)stream);
}

int tman_mpgemm_i8(const tman_shape_t* shape, const void* packed, const void* xq, int32_t N, void* y, int32_t* acc,
                   void* stream) {
    int rc = check_shape(shape);
    if (rc != TMAN_OK) return rc;
    if (!packed || !xq || !y) return TMAN_ERR_NULL;
    if (tman_act_i8_bytes(N, shape->K) == 0) return TMAN_ERR_SHAPE;
    if (!aligned16(packed) || !aligned16(xq)) return TMAN_ERR_ALIGN;
    return launch_mpgemm_i8(make_layout(shape), packed, xq, N, y, acc, (hipStream_t)stream);
}

int tman_check_packed(const tman_shape_t* shape, const void* packed, void* stream) {
    int rc = check_shape(shape);
    if (rc != TMAN_OK) return rc;
    if (!packed) return TMAN_ERR_NULL;
    int32_t h[32];
    if (hipMemcpyAsync(h, packed, sizeof(h), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess ||
        hipStreamSynchronize((hipStream_t)stream) != hipSuccess) {
        (void)hipGetLastError();
        return TMAN_ERR_LAUNCH;
    }
    const Layout L = make_layout(shape);
    const int32_t want[14] = {0x4e414d54, 0x00314b50, L.M, L.K, L.bits, L.group, L.has_zero, kRows, kKTile,
                              L.n_row_blocks, L.n_ktiles, L.tile_bytes, kHeaderBytes, kLayoutVersion};
    for (int i = 0; i < 14; ++i)
        if (h[i] != want[i]) return TMAN_ERR_HEADER;
    return TMAN_OK;
}

int tman_device_status(void* stream) {
    int* word = device_status_word();
    if (!word) return TMAN_ERR_LAUNCH;
    int v = 0;
    const int zero = 0;
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(&v, word, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipMemcpyAsync(word, &zero, sizeof(int), hipMemcpyHostToDevice, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        (void)hipGetLastError();
        return TMAN_ERR_LAUNCH;
    }
    return v;
}

const char* tman_status_string(int status) {
    switch (status) {
        case TMAN_OK: return "ok";
        case TMAN_ERR_NULL: return "null pointer";
        case TMAN_ERR_BITS: return "bits must be 1, 2 or 4";
        case TMAN_ERR_GROUP: return "group must be 32, 64 or 128";
        case TMAN_ERR_SHAPE: return "invalid shape, token count or flags";
        case TMAN_ERR_WORKSPACE: return "workspace missing or too small";
        case TMAN_ERR_ALIGN: return "pointer not 16-byte aligned";
        case TMAN_ERR_LAUNCH: return "HIP launch failed";
        case TMAN_ERR_HEADER: return "packed blob's header disagrees with the shape";
        default: return "unknown status";
    }
}

int32_t tman_layout_version(void) { return kLayoutVersion; }

}  // extern "C"
