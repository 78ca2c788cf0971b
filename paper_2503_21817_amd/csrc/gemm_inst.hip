// Instantiations and launcher of the bf16 MFMA GEMM core.
#include "kernels.hpp"

namespace skipffn {

template <bool A_KC, bool B_KC, int EPI, bool NARROW = false>
static hipError_t set_lds_limit() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<A_KC, B_KC, EPI, NARROW>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS_BYTES);
}

hipError_t gemm_init() {
    hipError_t e;
    if ((e = set_lds_limit<true, true, EPI_SWIGLU>()) != hipSuccess) return e;
    if ((e = set_lds_limit<true, true, EPI_PARTIAL>()) != hipSuccess) return e;
    if ((e = set_lds_limit<true, true, EPI_RESID_SCATTER>()) != hipSuccess) return e;
    if ((e = set_lds_limit<true, true, EPI_STORE>()) != hipSuccess) return e;
    if ((e = set_lds_limit<true, true, EPI_SWIGLU, true>()) != hipSuccess) return e;
    if ((e = set_lds_limit<true, true, EPI_PARTIAL, true>()) != hipSuccess) return e;
    if ((e = set_lds_limit<true, true, EPI_RESID_SCATTER, true>()) != hipSuccess) return e;
    if ((e = set_lds_limit<true, true, EPI_PARTIAL_GU, true>()) != hipSuccess) return e;
    if ((e = set_lds_limit<true, true, EPI_PARTIAL_GU>()) != hipSuccess) return e;
    if ((e = set_lds_limit<true, false, EPI_PARTIAL>()) != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_dual_kernel<true, false, EPI_SWIGLU_BWD, true, true, EPI_STORE>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS_BYTES);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_streamk_kernel<true, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS_BYTES);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_streamk_kernel<true, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS_BYTES);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_selfsim_kernel<EPI_STORE>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS_BYTES);
    if (e != hipSuccess) return e;
    return hipSuccess;
}

static void finish_args(int epi, GemmArgs& a) {
    const int tm_rows = a.narrow ? BM / 2 : BM;
    a.tiles_m = (a.M + tm_rows - 1) / tm_rows;
    a.tiles_n = (epi == EPI_SWIGLU || epi == EPI_PARTIAL_GU) ? (a.N + BN / 2 - 1) / (BN / 2) : (a.N + BN - 1) / BN;
    if (a.splits < 1) a.splits = 1;
    if (a.batch < 1) a.batch = 1;
    // a last tile row of at most 128 rows runs on 128-row tiles (host-side row count, one
    // workgroup per tile: the gate/up GEMM)
    const int rem = a.M % BM;
    a.tail_narrow = (!a.narrow && epi == EPI_SWIGLU && a.m_dev == nullptr &&
                     a.splits == 1 && a.batch == 1 && rem > 0 && rem <= BM / 2) ? 1 : 0;
    if (a.tail_narrow) a.tiles_m = a.M / BM;           // full tile rows only; the tail row is extra
}
// workgroups of a one-tile-per-workgroup launch
static unsigned grid_blocks(const GemmArgs& a) {
    return (unsigned)(a.tiles_m * a.tiles_n * a.splits * a.batch + (a.tail_narrow ? a.tiles_n : 0));
}

template <bool A_KC, bool B_KC, int EPI, bool NARROW = false>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s) {
    const unsigned blocks = grid_blocks(a);
    hipLaunchKernelGGL((gemm_bf16_kernel<A_KC, B_KC, EPI, NARROW>), dim3(blocks), dim3(GEMM_THREADS),
                       GEMM_LDS_BYTES, s, a);
    return hipGetLastError();
}

hipError_t launch_gemm_dual(int which, GemmArgs& a0, GemmArgs& a1, hipStream_t s) {
    if (which != DUAL_DH_DWDOWN) return hipErrorInvalidValue;
    finish_args(EPI_SWIGLU_BWD, a0);
    finish_args(EPI_STORE, a1);
    const int real0 = (int)grid_blocks(a0);
    const int n0 = (real0 + 7) / 8 * 8;
    const int n1 = a1.tiles_m * a1.tiles_n * a1.splits * a1.batch;
    if (real0 <= 0 || n1 <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL((gemm_bf16_dual_kernel<true, false, EPI_SWIGLU_BWD, true, true, EPI_STORE>),
                       dim3((unsigned)(n0 + n1)), dim3(GEMM_THREADS), GEMM_LDS_BYTES, s, a0, a1, n0, real0);
    return hipGetLastError();
}

hipError_t launch_gemm_streamk(bool a_kc, bool b_kc, GemmArgs& a, int nbg, hipStream_t s) {
    finish_args(EPI_PARTIAL, a);
    if (a.tiles_m <= 0 || a.tiles_n <= 0) return hipSuccess;
    if (nbg < 1 || !a_kc || a.batch != 1) return hipErrorInvalidValue;
    a.splits = nbg;
    const unsigned blocks = (unsigned)(a.tiles_n * nbg);
    if (b_kc)
        hipLaunchKernelGGL((gemm_bf16_streamk_kernel<true, true>), dim3(blocks), dim3(GEMM_THREADS),
                           GEMM_LDS_BYTES, s, a);
    else
        hipLaunchKernelGGL((gemm_bf16_streamk_kernel<true, false>), dim3(blocks), dim3(GEMM_THREADS),
                           GEMM_LDS_BYTES, s, a);
    return hipGetLastError();
}

hipError_t launch_gemm_selfsim(const bf16_t* xn, int C, const SegTable& st, int n_max, float* sim, int ld,
                               int64_t sim_stride, hipStream_t s) {
    if (st.count <= 0 || n_max <= 0) return hipSuccess;
    GemmArgs a{};
    a.M = n_max; a.N = n_max; a.K = C;
    a.A0 = xn; a.lda = C; a.B0 = xn; a.ldb = C;
    a.pairs = 1; a.splits = 1; a.batch = 1;
    a.out0 = sim; a.ldo = ld; a.out_f32 = 1; a.accumulate = 0;
    const int tiles_1d = (n_max + BM - 1) / BM;
    a.tiles_m = a.tiles_n = tiles_1d;
    const unsigned blocks = (unsigned)(st.count * tiles_1d * tiles_1d);
    hipLaunchKernelGGL(gemm_bf16_selfsim_kernel<EPI_STORE>, dim3(blocks), dim3(GEMM_THREADS), GEMM_LDS_BYTES, s, a, st,
                       tiles_1d, sim_stride);
    return hipGetLastError();
}

hipError_t launch_gemm(bool a_kc, bool b_kc, int epi, GemmArgs& a, hipStream_t s) {
    finish_args(epi, a);
    if (grid_blocks(a) == 0 || a.tiles_n <= 0) return hipSuccess;
    if (a.narrow) {
        if (a_kc && b_kc && epi == EPI_SWIGLU) return launch_one<true, true, EPI_SWIGLU, true>(a, s);
        if (a_kc && b_kc && epi == EPI_PARTIAL) return launch_one<true, true, EPI_PARTIAL, true>(a, s);
        if (a_kc && b_kc && epi == EPI_RESID_SCATTER) return launch_one<true, true, EPI_RESID_SCATTER, true>(a, s);
        if (a_kc && b_kc && epi == EPI_PARTIAL_GU) return launch_one<true, true, EPI_PARTIAL_GU, true>(a, s);
        return hipErrorInvalidValue;
    }
    if (a_kc && b_kc && epi == EPI_SWIGLU) return launch_one<true, true, EPI_SWIGLU>(a, s);
    if (a_kc && b_kc && epi == EPI_PARTIAL) return launch_one<true, true, EPI_PARTIAL>(a, s);
    if (a_kc && b_kc && epi == EPI_PARTIAL_GU) return launch_one<true, true, EPI_PARTIAL_GU>(a, s);
    if (a_kc && b_kc && epi == EPI_RESID_SCATTER) return launch_one<true, true, EPI_RESID_SCATTER>(a, s);
    if (a_kc && b_kc && epi == EPI_STORE) return launch_one<true, true, EPI_STORE>(a, s);
    if (a_kc && !b_kc && epi == EPI_PARTIAL) return launch_one<true, false, EPI_PARTIAL>(a, s);
    return hipErrorInvalidValue;
}

}  // namespace skipffn
