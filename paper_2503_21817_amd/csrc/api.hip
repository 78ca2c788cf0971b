// C ABI of the Skip-FFN block and of the operations around it (skip KV-cache, adaptive
// summary layer, retained-token selection, token merge): argument validation, workspace
// carving and the launch sequences.  Declarations and the contract of every entry point are
// in include/skipffn.h.
#include <algorithm>
#include <atomic>
#include <mutex>
#include <vector>

#include "../../include/skipffn.h"
#include "kernels.hpp"
#include "layout.hpp"

using namespace skipffn;

namespace {

thread_local int g_last_hip = 0;

int hip_fail(hipError_t e) {
    g_last_hip = (int)e;
    return SKIPFFN_EHIP;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool bad_ptr(const void* p) { return p == nullptr || !aligned16(p); }
constexpr int64_t kMaxTensorBytes = (int64_t)1 << 31;

// ---- event profiler -----------------------------------------------------------------
struct ProfRec { int kc; hipEvent_t a, b; };
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfRec> g_prof_recs;
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_prof_pool;

std::once_flag g_gemm_once;
hipError_t g_gemm_init_err = hipSuccess;
hipError_t ensure_gemm_init() {
    std::call_once(g_gemm_once, [] { g_gemm_init_err = gemm_init(); });
    return g_gemm_init_err;
}

// Compute units of the current device (one workgroup of the GEMM core occupies one CU), read once
// per device; 256 - an MI355X - when no device can be queried (size queries on a host without a GPU).
constexpr int kDefaultCus = 256;
int num_cus() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { (void)hipGetLastError(); return kDefaultCus; }
    int v = cached[dev].load(std::memory_order_relaxed);
    if (v > 0) return v;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        return kDefaultCus;
    }
    cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

int check_common(int64_t T, int64_t C, int64_t I, int64_t R, const int32_t* num_retained,
                 uint32_t flags) {
    if (flags & ~SKIPFFN_FLAG_ALL) return SKIPFFN_EUNSUPPORTED;
    if (T < 0 || C <= 0 || I <= 0 || R < -1 || R > T) return SKIPFFN_EINVAL;
    if (R == -1 && num_retained == nullptr) return SKIPFFN_EINVAL;
    if ((C & 7) || (I & 7)) return SKIPFFN_ESHAPE;
    int64_t Rb = R < 0 ? T : R;
    if (T * C * 2 >= kMaxTensorBytes || I * C * 2 >= kMaxTensorBytes ||
        Rb * I * 2 >= kMaxTensorBytes || T > 0x7fffffff)
        return SKIPFFN_ESHAPE;
    return SKIPFFN_OK;
}

// SKIPFFN_FLAG_VALIDATE_IDX: run the check, wait for it and read the verdict back
int validate_idx_now(const int32_t* idx, int64_t Rb, const int32_t* r_dev, int64_t T, void* status_dev,
                     hipStream_t s) {
    int32_t* st = static_cast<int32_t*>(status_dev);
    hipError_t e = launch_validate_idx(idx, (int)Rb, r_dev, T, st, s);
    if (e != hipSuccess) return hip_fail(e);
    int32_t host[2] = {0, 0};
    if ((e = hipMemcpyAsync(host, st, sizeof(host), hipMemcpyDeviceToHost, s)) != hipSuccess) return hip_fail(e);
    if ((e = hipStreamSynchronize(s)) != hipSuccess) return hip_fail(e);
    return host[0] == 0 ? SKIPFFN_OK : SKIPFFN_EIDX;
}

bool partial_overlap(const void* a, const void* b, size_t bytes) {
    if (a == b) return false;
    uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + bytes && y < x + bytes;
}

}  // namespace

namespace skipffn {

const char* kernel_class_name(int kc) {
    static const char* names[KC_COUNT] = {
        "compact", "gather_rmsnorm", "gemm_gate_up_swiglu", "gemm_down", "resid_scatter",
        "passthrough_copy", "gather_rows", "gemm_dh_swiglu_bwd+dw_down", "gemm_dw_gate_up",
        "gemm_dxn", "rmsnorm_bwd_scatter", "fill_zero", "kv_compact", "summary_fwd", "summary_bwd", "select_retained", "token_merge"};
    return (kc >= 0 && kc < KC_COUNT) ? names[kc] : "?";
}

void profile_mark_begin(int kc, hipStream_t s) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    ProfRec r; r.kc = kc;
    if (!g_prof_pool.empty()) {
        r.a = g_prof_pool.back().first; r.b = g_prof_pool.back().second;
        g_prof_pool.pop_back();
    } else {
        if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
    }
    (void)hipEventRecord(r.a, s);
    g_prof_recs.push_back(r);
}

void profile_mark_end(int kc, hipStream_t s) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (size_t i = g_prof_recs.size(); i-- > 0;) {
        if (g_prof_recs[i].kc == kc) { (void)hipEventRecord(g_prof_recs[i].b, s); break; }
    }
}

}  // namespace skipffn

extern "C" {

const char* skipffn_status_string(int status) {
    switch (status) {
        case SKIPFFN_OK: return "ok";
        case SKIPFFN_EINVAL: return "invalid argument (null or misaligned pointer, negative size, R > T)";
        case SKIPFFN_ESHAPE: return "unsupported shape (C, I must be multiples of 8; tensors below 2 GiB; skipffn_compact_static: T above skipffn_compact_static_max_tokens())";
        case SKIPFFN_EWORKSPACE: return "workspace too small";
        case SKIPFFN_EHIP: return "HIP runtime error";
        case SKIPFFN_EUNSUPPORTED: return "unsupported flag";
        case SKIPFFN_EIDX: return "idx is not strictly ascending inside [0, T)";
        default: return "unknown status";
    }
}

int skipffn_last_hip_error(void) { return g_last_hip; }
int skipffn_version(void) { return 20100; }   // 2.1.0: leading dimension of the transposed saved copies

int skipffn_profile_begin(void) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto& r : g_prof_recs) g_prof_pool.emplace_back(r.a, r.b);
    g_prof_recs.clear();
    g_prof_on = true;
    return SKIPFFN_OK;
}

int skipffn_profile_end(const char** names, double* ms, int64_t* launches, int cap) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = false;
    double tot[KC_COUNT] = {0};
    int64_t cnt[KC_COUNT] = {0};
    for (auto& r : g_prof_recs) {
        if (hipEventSynchronize(r.b) != hipSuccess) continue;
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) { tot[r.kc] += t; cnt[r.kc] += 1; }
    }
    for (auto& r : g_prof_recs) g_prof_pool.emplace_back(r.a, r.b);
    g_prof_recs.clear();
    int n = KC_COUNT < cap ? KC_COUNT : cap;
    for (int i = 0; i < n; ++i) {
        if (names) names[i] = kernel_class_name(i);
        if (ms) ms[i] = tot[i];
        if (launches) launches[i] = cnt[i];
    }
    return KC_COUNT;
}

// ---- compaction ------------------------------------------------------------------------
size_t skipffn_compact_workspace_bytes(int64_t T) { return compact_workspace_bytes(T); }

int skipffn_compact(const uint8_t* skip_mask, int64_t T, int32_t* idx, int32_t* num_retained,
                    int32_t* pos, void* workspace, size_t workspace_bytes, void* stream) {
    if (T < 0 || T > 0x7fffffff || num_retained == nullptr) return SKIPFFN_EINVAL;
    if (T > 0 && (bad_ptr(skip_mask) || idx == nullptr)) return SKIPFFN_EINVAL;
    if ((reinterpret_cast<uintptr_t>(idx) & 3u) || (reinterpret_cast<uintptr_t>(pos) & 3u) ||
        (reinterpret_cast<uintptr_t>(num_retained) & 3u))
        return SKIPFFN_EINVAL;
    size_t need = compact_workspace_bytes(T);
    if (workspace_bytes < need || (need > 0 && workspace == nullptr)) return SKIPFFN_EWORKSPACE;
    hipError_t e = launch_compact(skip_mask, T, idx, num_retained, pos, workspace, (hipStream_t)stream);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

int64_t skipffn_compact_static_max_tokens(void) { return compact_static_max_tokens(); }

int skipffn_compact_static(const uint8_t* skip_mask, int64_t T, int32_t* idx, int32_t* num_retained,
                           int32_t* pos, void* stream) {
    if (T < 0 || T > 0x7fffffff || num_retained == nullptr) return SKIPFFN_EINVAL;
    if (T > compact_static_max_tokens()) return SKIPFFN_ESHAPE;      // beyond the built-in scratch
    if (T > 0 && (bad_ptr(skip_mask) || idx == nullptr)) return SKIPFFN_EINVAL;
    if ((reinterpret_cast<uintptr_t>(idx) & 3u) || (reinterpret_cast<uintptr_t>(pos) & 3u) ||
        (reinterpret_cast<uintptr_t>(num_retained) & 3u))
        return SKIPFFN_EINVAL;
    hipError_t e = launch_compact_static(skip_mask, T, idx, num_retained, pos, (hipStream_t)stream);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

// ---- sizes --------------------------------------------------------------------------------
size_t skipffn_saved_bytes(int64_t R_max, int64_t C, int64_t I) {
    if (R_max < 0 || C <= 0 || I <= 0) return 0;
    return saved_layout(R_max, C, I).total + 256;
}
int skipffn_saved_layout(int64_t R_max, int64_t C, int64_t I, size_t* offsets) {
    if (R_max < 0 || C <= 0 || I <= 0 || offsets == nullptr) return SKIPFFN_EINVAL;
    SavedLayout L = saved_layout(R_max, C, I);
    for (int i = 0; i < 8; ++i) offsets[i] = L.off[i];
    return SKIPFFN_OK;
}
size_t skipffn_forward_workspace_bytes(int64_t R_max, int64_t C, int64_t I, int has_saved) {
    if (R_max < 0 || C <= 0 || I <= 0) return 0;
    return fwd_ws(R_max, C, I, has_saved != 0, num_cus()).total + 256;
}
size_t skipffn_backward_workspace_bytes(int64_t R_max, int64_t C, int64_t I) {
    if (R_max < 0 || C <= 0 || I <= 0) return 0;
    return bwd_ws(R_max, C, I).total + 256;
}

// ---- forward ---------------------------------------------------------------------------------
int skipffn_forward(int64_t T, int64_t C, int64_t I, float eps, const void* hidden, void* out,
                    const int32_t* idx, int64_t R, const int32_t* num_retained,
                    const void* rms_gain, const void* w_gate, const void* w_up, const void* w_down,
                    void* saved, void* workspace, size_t workspace_bytes, uint32_t flags,
                    void* stream) {
    int st = check_common(T, C, I, R, num_retained, flags);
    if (st != SKIPFFN_OK) return st;
    if (!(eps >= 0.0f)) return SKIPFFN_EINVAL;
    const int64_t Rb = R < 0 ? T : R;
    if (T > 0 && (bad_ptr(hidden) || bad_ptr(out))) return SKIPFFN_EINVAL;
    if (T > 0 && partial_overlap(hidden, out, (size_t)T * C * 2)) return SKIPFFN_EINVAL;
    if (rms_gain != nullptr && !aligned16(rms_gain)) return SKIPFFN_EINVAL;
    if (saved != nullptr && !aligned16(saved)) return SKIPFFN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int32_t* r_dev = R < 0 ? num_retained : nullptr;

    if (Rb > 0) {
        if (idx == nullptr || (reinterpret_cast<uintptr_t>(idx) & 3u)) return SKIPFFN_EINVAL;
        if (bad_ptr(w_gate) || bad_ptr(w_up) || bad_ptr(w_down)) return SKIPFFN_EINVAL;
        FwdWs W = fwd_ws(Rb, C, I, saved != nullptr, num_cus());
        if (workspace == nullptr || !aligned16(workspace)) return SKIPFFN_EWORKSPACE;
        if (workspace_bytes < W.total) return SKIPFFN_EWORKSPACE;
    }
    if (T == 0) return SKIPFFN_OK;
    if ((flags & SKIPFFN_FLAG_VALIDATE_IDX) && Rb > 0) {
        st = validate_idx_now(idx, Rb, r_dev, T, static_cast<char*>(workspace) + fwd_ws(Rb, C, I, saved != nullptr, num_cus()).status, s);
        if (st != SKIPFFN_OK) return st;
    }

    hipError_t e;
    if (out != hidden) {
        e = launch_passthrough(hidden, out, T, C * 2, idx, (int)Rb, r_dev, s);
        if (e != hipSuccess) return hip_fail(e);
    }
    if (Rb == 0) return SKIPFFN_OK;
    if ((e = ensure_gemm_init()) != hipSuccess) return hip_fail(e);

    FwdWs W = fwd_ws(Rb, C, I, saved != nullptr, num_cus());
    char* ws = static_cast<char*>(workspace);
    bf16_t *xrows = nullptr, *xn, *xnT = nullptr, *G = nullptr, *U = nullptr, *H, *HT = nullptr;
    float* rstd;
    if (saved != nullptr) {
        SavedLayout L = saved_layout(Rb, C, I);
        char* sv = static_cast<char*>(saved);
        xrows = reinterpret_cast<bf16_t*>(sv + L.off[0]);
        xn = reinterpret_cast<bf16_t*>(sv + L.off[1]);
        rstd = reinterpret_cast<float*>(sv + L.off[2]);
        G = reinterpret_cast<bf16_t*>(sv + L.off[3]);
        U = reinterpret_cast<bf16_t*>(sv + L.off[4]);
        H = reinterpret_cast<bf16_t*>(sv + L.off[5]);
        xnT = reinterpret_cast<bf16_t*>(sv + L.off[6]);
        HT = reinterpret_cast<bf16_t*>(sv + L.off[7]);
    } else {
        xn = reinterpret_cast<bf16_t*>(ws + W.xn);
        rstd = reinterpret_cast<float*>(ws + W.rstd);
        H = reinterpret_cast<bf16_t*>(ws + W.h);
    }
    float* partial = reinterpret_cast<float*>(ws + W.partial);

    // (2) gather + RMSNorm
    e = launch_gather_rmsnorm(static_cast<const bf16_t*>(hidden), idx, (int)Rb, r_dev, (int)C, eps,
                              static_cast<const bf16_t*>(rms_gain), xrows, xn, rstd, s);
    if (e != hipSuccess) return hip_fail(e);
    if (xnT != nullptr) {   // K-contiguous copy of the normalised rows for the dW_gate / dW_up GEMMs
        e = launch_gather_transpose(xn, (int)C, nullptr, (int)Rb, r_dev, nullptr, xnT,
                                    (int)ld_transposed(Rb), s);
        if (e != hipSuccess) return hip_fail(e);
    }

    // (3) gate/up GEMM + SiLU*mul
    {
        GemmArgs a{};
        a.M = (int)Rb; a.N = (int)I; a.K = (int)C; a.m_dev = r_dev;
        a.A0 = xn; a.lda = (int)C; a.a_bytes = (uint32_t)(Rb * C * 2);
        a.B0 = static_cast<const bf16_t*>(w_gate); a.B1 = static_cast<const bf16_t*>(w_up);
        a.ldb = (int)C; a.b_bytes = (uint32_t)(I * C * 2);
        a.pairs = 1; a.splits = 1;
        a.out0 = H; a.out1 = G; a.out2 = U; a.ldo = (int)I;
        const int gu_splits = gate_up_splits(Rb, C, I, num_cus());
        profile_mark_begin(KC_GEMM_GATE_UP, s);
        if (gu_splits) {
            // few rows: split K on 128-row tiles, fp32 partial sums, SwiGLU in the reducing kernel
            a.narrow = 1;
            a.splits = gu_splits;
            a.partial = reinterpret_cast<float*>(ws + W.gu_partial);
            e = launch_gemm(true, true, EPI_PARTIAL_GU, a, s);
            if (e == hipSuccess)
                e = launch_swiglu_reduce(a.partial, gu_splits, (int)Rb, r_dev, (int)I, a.tiles_n * BN, H, G, U, s);
            profile_mark_end(KC_GEMM_GATE_UP, s);
            // few rows: the K-contiguous copy of H for the dW_down GEMM comes from a copy kernel
            if (e == hipSuccess && HT != nullptr)
                e = launch_gather_transpose(H, (int)I, nullptr, (int)Rb, r_dev, nullptr, HT, (int)ld_transposed(Rb), s);
        } else {
            a.narrow = narrow_rows(Rb) ? 1 : 0;
            a.outT0 = HT; a.ldt = (int)ld_transposed(Rb);     // written by the epilogue when training
            e = launch_gemm(true, true, EPI_SWIGLU, a, s);
            profile_mark_end(KC_GEMM_GATE_UP, s);
        }
        if (e != hipSuccess) return hip_fail(e);
    }

    // (4) down GEMM + residual scatter-add
    {
        GemmArgs a{};
        a.M = (int)Rb; a.N = (int)C; a.K = (int)I; a.m_dev = r_dev;
        a.A0 = H; a.lda = (int)I; a.a_bytes = (uint32_t)(Rb * I * 2);
        a.B0 = static_cast<const bf16_t*>(w_down); a.ldb = (int)I; a.b_bytes = (uint32_t)(C * I * 2);
        a.pairs = 1;
        const bool balanced = (flags & SKIPFFN_FLAG_BALANCED_SPLIT) != 0;
        a.narrow = (narrow_rows(Rb) && !balanced) ? 1 : 0;
        const int tile_rows = a.narrow ? BM / 2 : BM;
        const int tiles_m = (int)((Rb + tile_rows - 1) / tile_rows), tiles_n = (int)((C + BN - 1) / BN);
        const int ktiles = (int)((I + BK - 1) / BK);
        const KPartition kp = a.narrow ? choose_k_split_narrow(tiles_m, tiles_n, ktiles, num_cus())
                                       : choose_k_partition(tiles_m, tiles_n, ktiles, balanced, num_cus());
        a.splits = kp.splits;
        a.idx = idx; a.ldo = (int)C;
        a.no_residual = (flags & SKIPFFN_FLAG_NO_RESIDUAL) ? 1 : 0;
        profile_mark_begin(KC_GEMM_DOWN, s);
        if (kp.splits == 1 && kp.sk_nbg == 0) {
            a.out0 = out; a.e0 = static_cast<const bf16_t*>(hidden);
            e = launch_gemm(true, true, EPI_RESID_SCATTER, a, s);
            profile_mark_end(KC_GEMM_DOWN, s);
            if (e != hipSuccess) return hip_fail(e);
        } else {
            a.partial = partial;
            e = kp.sk_nbg > 0 ? launch_gemm_streamk(true, true, a, kp.sk_nbg, s)
                              : launch_gemm(true, true, EPI_PARTIAL, a, s);
            profile_mark_end(KC_GEMM_DOWN, s);
            if (e != hipSuccess) return hip_fail(e);
            const PartialLayout pl{kp.splits, kp.sk_nbg, ktiles};
            e = launch_resid_scatter(partial, pl, (int)Rb, r_dev, (int)C, idx,
                                     static_cast<const bf16_t*>(hidden), static_cast<bf16_t*>(out),
                                     a.no_residual, s);
            if (e != hipSuccess) return hip_fail(e);
        }
    }
    return SKIPFFN_OK;
}

// ---- backward --------------------------------------------------------------------------------
int skipffn_backward(int64_t T, int64_t C, int64_t I, float eps, const void* grad_out,
                     void* grad_hidden, const int32_t* idx, int64_t R,
                     const int32_t* num_retained, const void* rms_gain, const void* w_gate,
                     const void* w_up, const void* w_down, const void* saved, void* dw_gate,
                     void* dw_up, void* dw_down, void* d_rms_gain, void* workspace,
                     size_t workspace_bytes, uint32_t flags, void* stream) {
    int st = check_common(T, C, I, R, num_retained, flags);
    if (st != SKIPFFN_OK) return st;
    (void)eps;
    if (d_rms_gain != nullptr && !aligned16(d_rms_gain)) return SKIPFFN_EINVAL;
    const int64_t Rb = R < 0 ? T : R;
    if (T > 0 && (bad_ptr(grad_out) || bad_ptr(grad_hidden))) return SKIPFFN_EINVAL;
    if (T > 0 && partial_overlap(grad_out, grad_hidden, (size_t)T * C * 2)) return SKIPFFN_EINVAL;
    if (bad_ptr(dw_gate) || bad_ptr(dw_up) || bad_ptr(dw_down)) return SKIPFFN_EINVAL;
    if (rms_gain != nullptr && !aligned16(rms_gain)) return SKIPFFN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int32_t* r_dev = R < 0 ? num_retained : nullptr;
    const bool f32 = (flags & SKIPFFN_FLAG_DW_FP32) != 0;
    const bool accum = (flags & SKIPFFN_FLAG_DW_ACCUMULATE) != 0;

    if (Rb > 0) {
        if (idx == nullptr || (reinterpret_cast<uintptr_t>(idx) & 3u)) return SKIPFFN_EINVAL;
        if (bad_ptr(w_gate) || bad_ptr(w_up) || bad_ptr(w_down) || bad_ptr(saved)) return SKIPFFN_EINVAL;
        BwdWs W = bwd_ws(Rb, C, I);
        if (workspace == nullptr || !aligned16(workspace)) return SKIPFFN_EWORKSPACE;
        if (workspace_bytes < W.total) return SKIPFFN_EWORKSPACE;
    }

    if ((flags & SKIPFFN_FLAG_VALIDATE_IDX) && Rb > 0 && T > 0) {
        st = validate_idx_now(idx, Rb, r_dev, T, static_cast<char*>(workspace) + bwd_ws(Rb, C, I).status, s);
        if (st != SKIPFFN_OK) return st;
    }
    hipError_t e;
    if (T > 0 && grad_hidden != grad_out) {
        e = launch_passthrough(grad_out, grad_hidden, T, C * 2, idx, (int)Rb, r_dev, s);
        if (e != hipSuccess) return hip_fail(e);
    }
    if (Rb == 0) {
        if (!accum) {
            size_t wbytes = (size_t)I * C * (f32 ? 4 : 2);
            if ((e = launch_fill_zero(dw_gate, wbytes, s)) != hipSuccess) return hip_fail(e);
            if ((e = launch_fill_zero(dw_up, wbytes, s)) != hipSuccess) return hip_fail(e);
            if ((e = launch_fill_zero(dw_down, wbytes, s)) != hipSuccess) return hip_fail(e);
            if (d_rms_gain != nullptr &&
                (e = launch_fill_zero(d_rms_gain, (size_t)C * 4, s)) != hipSuccess) return hip_fail(e);
        }
        return SKIPFFN_OK;
    }
    if ((e = ensure_gemm_init()) != hipSuccess) return hip_fail(e);

    SavedLayout L = saved_layout(Rb, C, I);
    const char* sv = static_cast<const char*>(saved);
    const bf16_t* xrows = reinterpret_cast<const bf16_t*>(sv + L.off[0]);
    // L.off[1] and L.off[5] (the normalised rows and silu(gate)*up, row-major) are not read here: the
    // weight-gradient GEMMs take the transposed copies
    const float* rstd = reinterpret_cast<const float*>(sv + L.off[2]);
    const bf16_t* G = reinterpret_cast<const bf16_t*>(sv + L.off[3]);
    const bf16_t* U = reinterpret_cast<const bf16_t*>(sv + L.off[4]);
    const bf16_t* xnT = reinterpret_cast<const bf16_t*>(sv + L.off[6]);
    const bf16_t* HT = reinterpret_cast<const bf16_t*>(sv + L.off[7]);
    BwdWs W = bwd_ws(Rb, C, I);
    char* ws = static_cast<char*>(workspace);
    bf16_t* dY = reinterpret_cast<bf16_t*>(ws + W.dy);
    bf16_t* dG = reinterpret_cast<bf16_t*>(ws + W.dg);
    bf16_t* dU = reinterpret_cast<bf16_t*>(ws + W.du);
    float* partial = reinterpret_cast<float*>(ws + W.partial);

    // dY = dOut[idx], and its transposed copy dY^T [C][ldT] for the dW_down GEMM
    bf16_t* dYT = reinterpret_cast<bf16_t*>(ws + W.dyT);
    const int ldT = (int)ld_transposed(Rb);
    e = launch_gather_transpose(static_cast<const bf16_t*>(grad_out), (int)C, idx, (int)Rb, r_dev, dY,
                                dYT, ldT, s);
    if (e != hipSuccess) return hip_fail(e);

    // dH = dY * W_down fused with the SiLU*mul backward (-> dG, dU and their transposed copies),
    // and, in the same grid (it depends only on dY and H), dW_down [C, I] = dY^T * H with both
    // operands in their K-contiguous (R-contiguous) copies
    bf16_t* dGT = reinterpret_cast<bf16_t*>(ws + W.dgT);
    bf16_t* dUT = reinterpret_cast<bf16_t*>(ws + W.duT);
    {
        GemmArgs a{};
        a.M = (int)Rb; a.N = (int)I; a.K = (int)C; a.m_dev = r_dev;
        a.A0 = dY; a.lda = (int)C; a.a_bytes = (uint32_t)(Rb * C * 2);
        a.B0 = static_cast<const bf16_t*>(w_down); a.ldb = (int)I; a.b_bytes = (uint32_t)(C * I * 2);
        a.pairs = 1; a.splits = 1;
        a.out0 = dG; a.out1 = dU; a.ldo = (int)I; a.e0 = G; a.e1 = U; a.lde = (int)I;
        a.outT0 = dGT; a.outT1 = dUT; a.ldt = ldT;
        GemmArgs b{};
        b.M = (int)C; b.N = (int)I; b.K = (int)Rb; b.k_dev = r_dev;
        b.A0 = dYT; b.lda = ldT; b.a_bytes = (uint32_t)(C * (int64_t)ldT * 2);   // K (= R) contiguous
        b.B0 = HT; b.ldb = ldT; b.b_bytes = (uint32_t)(I * (int64_t)ldT * 2);
        b.pairs = 1; b.splits = 1;
        b.out0 = dw_down; b.ldo = (int)I; b.out_f32 = f32; b.accumulate = accum;
        profile_mark_begin(KC_GEMM_DH_DWDOWN, s);
        e = launch_gemm_dual(DUAL_DH_DWDOWN, a, b, s);
        profile_mark_end(KC_GEMM_DH_DWDOWN, s);
        if (e != hipSuccess) return hip_fail(e);
    }
    // dW_gate [I, C] = dG^T * xn ; dW_up [I, C] = dU^T * xn : one launch, two problems sharing
    // the B operand, every operand in its K-contiguous (R-contiguous) copy
    {
        GemmArgs a{};
        a.M = (int)I; a.N = (int)C; a.K = (int)Rb; a.k_dev = r_dev;
        a.A0 = dGT; a.A1 = dUT; a.lda = ldT; a.a_bytes = (uint32_t)(I * (int64_t)ldT * 2);
        a.B0 = xnT; a.ldb = ldT; a.b_bytes = (uint32_t)(C * (int64_t)ldT * 2);
        a.pairs = 1; a.splits = 1; a.batch = 2;
        a.out0 = dw_gate; a.out1 = dw_up; a.ldo = (int)C; a.out_f32 = f32; a.accumulate = accum;
        profile_mark_begin(KC_GEMM_DW_GATE_UP, s);
        e = launch_gemm(true, true, EPI_STORE, a, s);
        profile_mark_end(KC_GEMM_DW_GATE_UP, s);
        if (e != hipSuccess) return hip_fail(e);
    }
    // dxn = dG * W_gate + dU * W_up  (K runs over both pairs), fp32 split-K slabs.  (Sharing a
    // grid with the dW GEMMs above was measured slower: both are already well balanced.)
    PartialLayout pl{1, 0, 0};
    {
        GemmArgs a{};
        a.M = (int)Rb; a.N = (int)C; a.K = (int)I; a.m_dev = r_dev;
        a.A0 = dG; a.A1 = dU; a.lda = (int)I; a.a_bytes = (uint32_t)(Rb * I * 2);
        a.B0 = static_cast<const bf16_t*>(w_gate); a.B1 = static_cast<const bf16_t*>(w_up);
        a.ldb = (int)C; a.b_bytes = (uint32_t)(I * C * 2);
        a.pairs = 2;
        const int tiles_m = (int)((Rb + BM - 1) / BM), tiles_n = (int)((C + BN - 1) / BN);
        const int ktiles = 2 * (int)((I + BK - 1) / BK);
        const KPartition kp = choose_k_partition(tiles_m, tiles_n, ktiles, (flags & SKIPFFN_FLAG_BALANCED_SPLIT) != 0,
                                                 num_cus());
        a.splits = kp.splits;
        pl = PartialLayout{kp.splits, kp.sk_nbg, ktiles};
        a.partial = partial;
        profile_mark_begin(KC_GEMM_DXN, s);
        e = kp.sk_nbg > 0 ? launch_gemm_streamk(true, false, a, kp.sk_nbg, s)
                          : launch_gemm(true, false, EPI_PARTIAL, a, s);
        profile_mark_end(KC_GEMM_DXN, s);
        if (e != hipSuccess) return hip_fail(e);
    }
    // RMSNorm backward + residual gradient, scattered to the retained rows
    e = launch_rmsnorm_bwd_scatter(partial, pl, (int)Rb, r_dev, (int)C, xrows, rstd,
                                   static_cast<const bf16_t*>(rms_gain), dY, idx,
                                   static_cast<bf16_t*>(grad_hidden),
                                   reinterpret_cast<float*>(ws + W.gainp),
                                   static_cast<float*>(d_rms_gain), accum ? 1 : 0, s);
    if (e != hipSuccess) return hip_fail(e);
    return SKIPFFN_OK;
}

int skipffn_validate_idx(const int32_t* idx, int64_t R, const int32_t* num_retained, int64_t T,
                         int32_t* status, void* stream) {
    if (T < 0 || T > 0x7fffffff || R < -1 || R > T) return SKIPFFN_EINVAL;
    if (R == -1 && num_retained == nullptr) return SKIPFFN_EINVAL;
    if (status == nullptr || (reinterpret_cast<uintptr_t>(status) & 3u)) return SKIPFFN_EINVAL;
    const int64_t Rb = R < 0 ? T : R;
    if (Rb > 0 && (idx == nullptr || (reinterpret_cast<uintptr_t>(idx) & 3u))) return SKIPFFN_EINVAL;
    hipError_t e = launch_validate_idx(idx, (int)Rb, R < 0 ? num_retained : nullptr, T, status, (hipStream_t)stream);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

// ---- skip KV-cache row gather -------------------------------------------------------------------
int skipffn_gather_rows(const void* src, void* dst, int64_t T, int64_t row_bytes,
                        const int32_t* idx, int64_t R, const int32_t* num_retained, void* stream) {
    if (T < 0 || row_bytes < 0 || R < -1 || R > T) return SKIPFFN_EINVAL;
    if (R == -1 && num_retained == nullptr) return SKIPFFN_EINVAL;
    if (row_bytes & 15) return SKIPFFN_ESHAPE;
    const int64_t Rb = R < 0 ? T : R;
    if (Rb == 0 || row_bytes == 0) return SKIPFFN_OK;
    if (bad_ptr(src) || bad_ptr(dst) || idx == nullptr) return SKIPFFN_EINVAL;
    if (T > 0x7fffffff) return SKIPFFN_ESHAPE;
    hipError_t e = launch_gather_rows(src, dst, row_bytes, idx, (int)Rb, R < 0 ? num_retained : nullptr,
                                      (hipStream_t)stream);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

int skipffn_kv_compact(const void* src, void* dst, int64_t n_slabs, int64_t T, int64_t row_bytes,
                       int64_t src_slab_bytes, int64_t dst_slab_bytes, const int32_t* idx,
                       int64_t R, const int32_t* num_retained, void* stream) {
    if (n_slabs < 0 || T < 0 || row_bytes < 0 || R < -1 || R > T) return SKIPFFN_EINVAL;
    if (R == -1 && num_retained == nullptr) return SKIPFFN_EINVAL;
    if ((row_bytes & 15) || (src_slab_bytes & 15) || (dst_slab_bytes & 15)) return SKIPFFN_ESHAPE;
    const int64_t Rb = R < 0 ? T : R;
    if (Rb == 0 || row_bytes == 0 || n_slabs == 0) return SKIPFFN_OK;
    if (bad_ptr(src) || bad_ptr(dst) || idx == nullptr) return SKIPFFN_EINVAL;
    if (T > 0x7fffffff || row_bytes > ((int64_t)1 << 24)) return SKIPFFN_ESHAPE;
    if (Rb * (row_bytes / 16) >= ((int64_t)1 << 31) * (int64_t)256) return SKIPFFN_ESHAPE;
    if (src_slab_bytes < T * row_bytes || dst_slab_bytes < Rb * row_bytes) return SKIPFFN_EINVAL;
    // the two caches may not overlap
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(src), b0 = reinterpret_cast<uintptr_t>(dst);
    const uintptr_t a1 = a0 + (uintptr_t)((n_slabs - 1) * src_slab_bytes + T * row_bytes);
    const uintptr_t b1 = b0 + (uintptr_t)((n_slabs - 1) * dst_slab_bytes + Rb * row_bytes);
    if (a0 < b1 && b0 < a1) return SKIPFFN_EINVAL;
    hipError_t e = launch_kv_compact(src, dst, n_slabs, row_bytes, src_slab_bytes, dst_slab_bytes, idx,
                                     (int)Rb, R < 0 ? num_retained : nullptr, (hipStream_t)stream);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

// ---- adaptive summary layer ------------------------------------------------------------------
namespace {
struct SumSaved { size_t scores, lse, xs, total; };
SumSaved sum_saved(int64_t n_tok, int64_t S, int64_t C) {
    SumSaved L; size_t o = 0;
    L.scores = o; o += align_up((size_t)n_tok * 4);
    L.lse = o;    o += align_up((size_t)S * 4);
    L.xs = o;     o += align_up((size_t)S * C * 4);
    L.total = o;
    return L;
}
struct SumWs { size_t acc, md, total; };
SumWs sum_ws(int64_t n_tok, int64_t S, int64_t C) {
    const size_t nq = (size_t)summary_max_chunks(n_tok, S);
    SumWs W; size_t o = 0;
    W.acc = o; o += align_up(nq * (size_t)C * 4);     // forward: weighted row sums; backward: dw
    W.md = o;  o += align_up(nq * 2 * 4);
    W.total = o;
    return W;
}
int check_summary(int64_t T, int64_t C, int64_t n_tok, int64_t S) {
    if (T < 0 || C <= 0 || n_tok < 0 || S < 0) return SKIPFFN_EINVAL;
    if (C & 7) return SKIPFFN_ESHAPE;
    if (T * C * 2 >= kMaxTensorBytes || T > 0x7fffffff || n_tok > 0x7fffffff || S > 65535 ||
        summary_max_chunks(n_tok, S) * C * 4 >= ((int64_t)1 << 40))
        return SKIPFFN_ESHAPE;
    return SKIPFFN_OK;
}
}  // namespace

size_t skipffn_summary_saved_bytes(int64_t n_tok, int64_t S, int64_t C) {
    if (n_tok < 0 || S < 0 || C <= 0) return 0;
    return sum_saved(n_tok, S, C).total + 256;
}
size_t skipffn_summary_workspace_bytes(int64_t n_tok, int64_t S, int64_t C) {
    if (n_tok < 0 || S < 0 || C <= 0) return 0;
    return sum_ws(n_tok, S, C).total + 256;
}

int skipffn_summary_forward(int64_t T, int64_t C, const void* hidden, const int32_t* tok,
                            const int32_t* seg, int64_t n_tok, int64_t S, const void* w, void* out,
                            void* saved, void* workspace, size_t workspace_bytes, void* stream) {
    int st = check_summary(T, C, n_tok, S);
    if (st != SKIPFFN_OK) return st;
    if (S == 0) return SKIPFFN_OK;
    if (bad_ptr(out) || bad_ptr(w) || seg == nullptr || (reinterpret_cast<uintptr_t>(seg) & 3u)) return SKIPFFN_EINVAL;
    if (n_tok > 0 && (tok == nullptr || (reinterpret_cast<uintptr_t>(tok) & 3u))) return SKIPFFN_EINVAL;
    if (T > 0 && bad_ptr(hidden)) return SKIPFFN_EINVAL;
    if (saved != nullptr && !aligned16(saved)) return SKIPFFN_EINVAL;
    const SumWs W = sum_ws(n_tok, S, C);
    if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < W.total) return SKIPFFN_EWORKSPACE;
    const SumSaved L = sum_saved(n_tok, S, C);
    char* sv = static_cast<char*>(saved);
    char* ws = static_cast<char*>(workspace);
    // with no token rows at all every set is empty (the kernels read row 0 for an absent token)
    if (T == 0) n_tok = 0;
    hipError_t e = launch_summary_forward(
        static_cast<const bf16_t*>(hidden), T, (int)C, tok, seg, n_tok, (int)S,
        static_cast<const bf16_t*>(w), static_cast<bf16_t*>(out),
        sv ? reinterpret_cast<float*>(sv + L.scores) : nullptr,
        sv ? reinterpret_cast<float*>(sv + L.lse) : nullptr,
        sv ? reinterpret_cast<float*>(sv + L.xs) : nullptr,
        reinterpret_cast<float*>(ws + W.acc), reinterpret_cast<float*>(ws + W.md), (hipStream_t)stream);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

int skipffn_summary_backward(int64_t T, int64_t C, const void* hidden, const int32_t* tok,
                             const int32_t* seg, int64_t n_tok, int64_t S, const void* w,
                             const void* saved, const void* grad_out, void* grad_hidden, void* dw,
                             void* workspace, size_t workspace_bytes, uint32_t flags, void* stream) {
    int st = check_summary(T, C, n_tok, S);
    if (st != SKIPFFN_OK) return st;
    if (flags & ~SKIPFFN_FLAG_DW_ACCUMULATE) return SKIPFFN_EUNSUPPORTED;
    if (bad_ptr(dw)) return SKIPFFN_EINVAL;
    const bool accum = (flags & SKIPFFN_FLAG_DW_ACCUMULATE) != 0;
    hipStream_t s = (hipStream_t)stream;
    if (S == 0) {
        if (!accum) {
            hipError_t e0 = launch_fill_zero(dw, (size_t)C * 4, s);
            if (e0 != hipSuccess) return hip_fail(e0);
        }
        return SKIPFFN_OK;
    }
    if (bad_ptr(w) || bad_ptr(saved) || bad_ptr(grad_out) || seg == nullptr ||
        (reinterpret_cast<uintptr_t>(seg) & 3u))
        return SKIPFFN_EINVAL;
    if (n_tok > 0 && (tok == nullptr || (reinterpret_cast<uintptr_t>(tok) & 3u))) return SKIPFFN_EINVAL;
    if (T > 0 && (bad_ptr(hidden) || bad_ptr(grad_hidden))) return SKIPFFN_EINVAL;
    const SumWs W = sum_ws(n_tok, S, C);
    if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < W.total) return SKIPFFN_EWORKSPACE;
    const SumSaved L = sum_saved(n_tok, S, C);
    const char* sv = static_cast<const char*>(saved);
    char* ws = static_cast<char*>(workspace);
    if (T == 0) n_tok = 0;
    hipError_t e = launch_summary_backward(
        static_cast<const bf16_t*>(hidden), T, (int)C, tok, seg, n_tok, (int)S,
        static_cast<const bf16_t*>(w), reinterpret_cast<const float*>(sv + L.xs),
        reinterpret_cast<const float*>(sv + L.scores), reinterpret_cast<const float*>(sv + L.lse),
        static_cast<const bf16_t*>(grad_out), static_cast<bf16_t*>(grad_hidden),
        reinterpret_cast<float*>(ws + W.acc), static_cast<float*>(dw), accum ? 1 : 0, s);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

// ---- retained-token selection --------------------------------------------------------------------
int skipffn_select_retained(const void* features, const void* cls, const int32_t* seq_off,
                            int64_t n_feat, int64_t B, int64_t Cv, int64_t n_keep,
                            const int32_t* n_keep_dev, uint8_t* mask, float* sim,
                            const int32_t* token_pos, uint8_t* skip_mask, int64_t T, void* stream) {
    if (n_feat < 0 || B < 0 || Cv <= 0 || n_keep < 0 || T < 0) return SKIPFFN_EINVAL;
    if (Cv & 7) return SKIPFFN_ESHAPE;
    if (n_feat > 0x7fffffff || B > 65535 || n_keep > 0x7fffffff || T > 0x7fffffff ||
        n_feat * Cv * 2 >= kMaxTensorBytes)
        return SKIPFFN_ESHAPE;
    if (B == 0 || n_feat == 0) return SKIPFFN_OK;
    if (bad_ptr(features) || bad_ptr(cls) || seq_off == nullptr || mask == nullptr || sim == nullptr)
        return SKIPFFN_EINVAL;
    if ((reinterpret_cast<uintptr_t>(seq_off) & 3u) || (reinterpret_cast<uintptr_t>(sim) & 3u)) return SKIPFFN_EINVAL;
    if ((token_pos == nullptr) != (skip_mask == nullptr)) return SKIPFFN_EINVAL;
    hipError_t e = launch_select_retained(static_cast<const bf16_t*>(features), static_cast<const bf16_t*>(cls),
                                          seq_off, n_feat, (int)B, (int)Cv, (int)n_keep, n_keep_dev, mask,
                                          sim, token_pos, skip_mask, T, (hipStream_t)stream);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

// ---- token merge -----------------------------------------------------------------------------------
namespace {
// sets handled per launch group: bounded by the kernel-argument table and by the size of the
// similarity buffer (256 MB)
int merge_group_sets(int64_t n_max) {
    const int64_t ld = (n_max + 7) / 8 * 8;
    const int64_t per_set = std::max<int64_t>(n_max * ld * 4, 1);
    int64_t g = ((int64_t)256 << 20) / per_set;
    g = std::max<int64_t>(1, std::min<int64_t>(g, SEG_TABLE_MAX));
    return (int)g;
}
struct MergeWs { size_t xn, sim, slot, kept, total; };
MergeWs merge_ws(int64_t n_tok, int64_t n_max, int64_t C) {
    MergeWs W; size_t o = 0;
    const size_t ld = (size_t)(n_max + 7) / 8 * 8;
    W.xn = o;   o += align_up((size_t)n_tok * C * 2);
    W.sim = o;  o += align_up((size_t)merge_group_sets(n_max) * n_max * ld * 4);
    W.slot = o; o += align_up((size_t)n_tok * 4);
    W.kept = o; o += align_up((size_t)n_tok);
    W.total = o;
    return W;
}
}  // namespace

size_t skipffn_token_merge_workspace_bytes(int64_t n_tok, int64_t n_max, int64_t C) {
    if (n_tok < 0 || n_max < 0 || C <= 0) return 0;
    return merge_ws(n_tok, n_max, C).total + 256;
}

int skipffn_token_merge(const void* x, const int32_t* seg_host, int64_t S, int64_t C, int64_t k,
                        void* out, int32_t* kept_idx, int32_t* assign, float* avg_sim,
                        void* workspace, size_t workspace_bytes, void* stream) {
    if (S < 0 || C <= 0 || k < 0) return SKIPFFN_EINVAL;
    if (C & 7) return SKIPFFN_ESHAPE;
    if (S == 0) return SKIPFFN_OK;
    if (seg_host == nullptr) return SKIPFFN_EINVAL;
    int64_t n_max = 0;
    for (int64_t i = 0; i < S; ++i) {
        if (seg_host[i] < 0 || seg_host[i + 1] < seg_host[i]) return SKIPFFN_EINVAL;
        n_max = std::max<int64_t>(n_max, seg_host[i + 1] - seg_host[i]);
    }
    const int64_t n_tok = seg_host[S];
    if (n_max > MERGE_MAX_N || k > MERGE_MAX_N || S > 65535) return SKIPFFN_ESHAPE;
    if (n_tok * C * 2 >= kMaxTensorBytes || S * k * C * 2 >= kMaxTensorBytes) return SKIPFFN_ESHAPE;
    if (k > 0 && (bad_ptr(out) || kept_idx == nullptr)) return SKIPFFN_EINVAL;
    if (n_tok > 0 && (bad_ptr(x) || assign == nullptr || avg_sim == nullptr)) return SKIPFFN_EINVAL;
    const MergeWs W = merge_ws(n_tok, n_max, C);
    if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < W.total) return SKIPFFN_EWORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if ((e = ensure_gemm_init()) != hipSuccess) return hip_fail(e);
    char* ws = static_cast<char*>(workspace);
    bf16_t* xn = reinterpret_cast<bf16_t*>(ws + W.xn);
    float* sim = reinterpret_cast<float*>(ws + W.sim);
    int32_t* slot_of = reinterpret_cast<int32_t*>(ws + W.slot);
    uint8_t* kept = reinterpret_cast<uint8_t*>(ws + W.kept);
    const bf16_t* xb = static_cast<const bf16_t*>(x);
    const int ld = (int)((n_max + 7) / 8 * 8);
    const int64_t sim_stride = n_max * ld;
    const int group = merge_group_sets(n_max);
    profile_mark_begin(KC_MERGE, s);
    e = launch_row_normalize(xb, n_tok, (int)C, xn, s);
    for (int64_t g0 = 0; g0 < S && e == hipSuccess; g0 += group) {
        SegTable st;
        st.count = (int)std::min<int64_t>(group, S - g0);
        int gmax = 0;
        for (int i = 0; i <= st.count; ++i) st.off[i] = seg_host[g0 + i];
        for (int i = st.count + 1; i <= SEG_TABLE_MAX; ++i) st.off[i] = st.off[st.count];
        for (int i = 0; i < st.count; ++i) gmax = std::max(gmax, st.off[i + 1] - st.off[i]);
        // S_i = Xn_i Xn_i^T  [n_i, n_i] fp32 on the MFMA core, every set of the group in one grid
        e = launch_gemm_selfsim(xn, (int)C, st, gmax, sim, ld, sim_stride, s);
        if (e != hipSuccess) break;
        e = launch_merge_group(xb, st, gmax, (int)C, (int)k, (int)g0, sim, ld, sim_stride, avg_sim, kept,
                               slot_of, kept_idx, assign, static_cast<bf16_t*>(out), s);
    }
    profile_mark_end(KC_MERGE, s);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

int skipffn_token_merge_backward(const void* grad_out, const int32_t* seg_host, int64_t S, int64_t C,
                                 int64_t k, const int32_t* assign, void* grad_x, void* stream) {
    if (S < 0 || C <= 0 || k < 0) return SKIPFFN_EINVAL;
    if (C & 7) return SKIPFFN_ESHAPE;
    if (S == 0) return SKIPFFN_OK;
    if (seg_host == nullptr) return SKIPFFN_EINVAL;
    int64_t n_max = 0;
    for (int64_t i = 0; i < S; ++i) {
        if (seg_host[i] < 0 || seg_host[i + 1] < seg_host[i]) return SKIPFFN_EINVAL;
        n_max = std::max<int64_t>(n_max, seg_host[i + 1] - seg_host[i]);
    }
    const int64_t n_tok = seg_host[S];
    if (n_max > MERGE_MAX_N || k > MERGE_MAX_N || S > 65535) return SKIPFFN_ESHAPE;
    if (n_tok * C * 2 >= kMaxTensorBytes || S * k * C * 2 >= kMaxTensorBytes) return SKIPFFN_ESHAPE;
    if (n_max == 0) return SKIPFFN_OK;
    if (bad_ptr(grad_x) || assign == nullptr || (k > 0 && bad_ptr(grad_out))) return SKIPFFN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    profile_mark_begin(KC_MERGE, s);
    for (int64_t g0 = 0; g0 < S && e == hipSuccess; g0 += SEG_TABLE_MAX) {
        SegTable st;
        st.count = (int)std::min<int64_t>(SEG_TABLE_MAX, S - g0);
        int gmax = 0;
        for (int i = 0; i <= st.count; ++i) st.off[i] = seg_host[g0 + i];
        for (int i = st.count + 1; i <= SEG_TABLE_MAX; ++i) st.off[i] = st.off[st.count];
        for (int i = 0; i < st.count; ++i) gmax = std::max(gmax, st.off[i + 1] - st.off[i]);
        e = launch_merge_bwd_group(static_cast<const bf16_t*>(grad_out), st, gmax, (int)C, (int)k, (int)g0,
                                   assign, static_cast<bf16_t*>(grad_x), s);
    }
    profile_mark_end(KC_MERGE, s);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

// ---- measurement aid ---------------------------------------------------------------------------------
int skipffn_probe_mfma(int64_t blocks, int64_t iters, int random_operands, float* out, int64_t* clocks,
                       void* stream) {
    if (blocks < 0 || iters < 0 || blocks > (1 << 20) || iters > (1 << 24)) return SKIPFFN_EINVAL;
    if (blocks == 0 || iters == 0) return SKIPFFN_OK;
    if (out == nullptr || clocks == nullptr || (reinterpret_cast<uintptr_t>(out) & 3u) ||
        (reinterpret_cast<uintptr_t>(clocks) & 7u))
        return SKIPFFN_EINVAL;
    hipError_t e = launch_mfma_probe((int)blocks, (int)iters, random_operands ? 1 : 0, out,
                                     reinterpret_cast<long long*>(clocks), (hipStream_t)stream);
    return e == hipSuccess ? SKIPFFN_OK : hip_fail(e);
}

}  // extern "C"
