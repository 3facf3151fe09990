// Decoding mpGEMV through lookups in INTEGER tables (Sec. 6.1 "A_INT16": activations as 16-bit integers;
// Sec. 4.3 two-level tiling: the looked-up entries are aggregated at low precision -- here as exact integers --
// inside a quantization block, and in floating point only across blocks).  The tables come from
// tman_build_lut_i16; the kernel is mpgemv_kernel with integer entries (tman_mpgemv_kernel.h), the scheduling,
// the workspace and the descriptor tables are those of tman_mpgemv.
#include "tman_mpgemv_kernel.h"

namespace tman {

int launch_mpgemv_i16(const Layout& L, const void* packed, const void* lut, int N, void* y, void* workspace,
                      hipStream_t st) {
    KernelArgs<true> a;
    fill_desc(a.single, L, packed, lut, N, y, workspace, 0);
    a.n_gemv = 1;
    a.status = device_status_word();
    if (!a.status) return TMAN_ERR_LAUNCH;
    return launch_format<true, true>(L.bits, L.has_zero, padded_tokens(N), L.group, a, plan_gemv(L, N).n_workgroups, st);
}

int launch_mpgemv_i16_batch(int bits, int group, int has_zero, int N, const GemvDesc* descs_dev, int n_gemv,
                            int max_workgroups, hipStream_t st) {
    KernelArgs<false> a;
    a.descs = descs_dev;
    a.n_gemv = n_gemv;
    return launch_format<false, true>(bits, has_zero, padded_tokens(N), group, a, max_workgroups, st);
}

}  // namespace tman
