// Host-side launchers of the Skip-FFN kernels.  Every launcher only enqueues
// work on `stream` and returns the hipError_t of the launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "gemm.hpp"

namespace skipffn {

// kernel classes for the built-in event profiler
enum KernelClass : int {
    KC_COMPACT = 0,
    KC_GATHER_RMSNORM,
    KC_GEMM_GATE_UP,
    KC_GEMM_DOWN,
    KC_RESID_SCATTER,
    KC_PASSTHROUGH,
    KC_GATHER_ROWS,
    KC_GEMM_DH_DWDOWN,      // dH + SwiGLU backward and dW_down in one grid
    KC_GEMM_DW_GATE_UP,     // dW_gate and dW_up, batched in one grid
    KC_GEMM_DXN,
    KC_RMSNORM_BWD,
    KC_FILL,
    KC_KV_COMPACT,
    KC_SUMMARY_FWD,
    KC_SUMMARY_BWD,
    KC_SELECT,
    KC_MERGE,
    KC_COUNT
};
const char* kernel_class_name(int kc);
void profile_mark_begin(int kc, hipStream_t s);
void profile_mark_end(int kc, hipStream_t s);

// ---- compaction ---------------------------------------------------------------
size_t compact_workspace_bytes(int64_t T);
hipError_t launch_compact(const uint8_t* mask, int64_t T, int32_t* idx, int32_t* num_retained,
                          int32_t* pos, void* ws, hipStream_t s);

// the same with the library's own per-GPU scratch (no workspace, nothing allocated), T <= compact_static_max_tokens()
int64_t compact_static_max_tokens();
hipError_t launch_compact_static(const uint8_t* mask, int64_t T, int32_t* idx, int32_t* num_retained,
                                 int32_t* pos, hipStream_t s);
// status[0] = 0 if idx[0..R) is strictly ascending inside [0, T) else 1; status[1] = first bad position
hipError_t launch_validate_idx(const int32_t* idx, int R, const int32_t* r_dev, int64_t T, int32_t* status,
                               hipStream_t s);

// ---- row kernels ---------------------------------------------------------------
// x rows (optional copy), normalised rows and 1/rms for rows idx[0..R)
hipError_t launch_gather_rmsnorm(const bf16_t* hidden, const int32_t* idx, int R,
                                 const int32_t* r_dev, int C, float eps, const bf16_t* gain,
                                 bf16_t* xrows, bf16_t* xn, float* rstd, hipStream_t s);
// How many fp32 partial slabs a reducing kernel adds per output element: `splits` for a plain
// split-K GEMM (sk_nbg == 0), else the per-tile count of the balanced split (streamk_count)
// with sk_nbg workgroups per n-tile group and sk_kt K slabs per tile.
struct PartialLayout { int splits; int sk_nbg; int sk_kt; };
// out[idx[r]] = bf16(res[idx[r]] + sum_z partial[z][r])
hipError_t launch_resid_scatter(const float* partial, PartialLayout pl, int R, const int32_t* r_dev,
                                int C, const int32_t* idx, const bf16_t* res, bf16_t* out,
                                int no_residual, hipStream_t s);
// SwiGLU over the split-K partial sums of a gate/up GEMM run with EPI_PARTIAL_GU (ldp = tiles_n * 256)
hipError_t launch_swiglu_reduce(const float* partial, int splits, int R, const int32_t* r_dev, int I, int ldp,
                                bf16_t* H, bf16_t* G, bf16_t* U, hipStream_t s);
// dst[r] = src[idx[r]]  (rows of row_bytes, multiple of 16)
hipError_t launch_gather_rows(const void* src, void* dst, int64_t row_bytes, const int32_t* idx,
                              int R, const int32_t* r_dev, hipStream_t s);
// dst[s][r] = src[s][idx[r]] for n_slabs slabs (slab strides in bytes, multiples of 16)
hipError_t launch_kv_compact(const void* src, void* dst, int64_t n_slabs, int64_t row_bytes,
                             int64_t src_slab_bytes, int64_t dst_slab_bytes, const int32_t* idx,
                             int R, const int32_t* r_dev, hipStream_t s);
// dst[r] = src[idx ? idx[r] : r] (dst optional) and the transposed copy dstT[c][r], leading
// dimension ldT (multiple of 8, >= R bound), columns r >= R zero
hipError_t launch_gather_transpose(const bf16_t* src, int C, const int32_t* idx, int R,
                                   const int32_t* r_dev, bf16_t* dst, bf16_t* dstT, int ldT,
                                   hipStream_t s);
// copy every row t of src to dst that is NOT listed in idx (skipped tokens)
hipError_t launch_passthrough(const void* src, void* dst, int64_t T, int64_t row_bytes,
                              const int32_t* idx, int R, const int32_t* r_dev, hipStream_t s);
// dX[idx[r]] = bf16(dY[r] + rmsnorm_bwd(sum_z dxn_partial[z][r], x[r], rstd[r], gain)); with dgain != null
// also dgain[c] (+)= sum_r dxn[r][c] * x[r][c] * rstd[r] (fp32, through gain_partial)
hipError_t launch_rmsnorm_bwd_scatter(const float* dxn_partial, PartialLayout pl, int R,
                                      const int32_t* r_dev, int C, const bf16_t* xrows,
                                      const float* rstd, const bf16_t* gain, const bf16_t* dY,
                                      const int32_t* idx, bf16_t* dX, float* gain_partial,
                                      float* dgain, int accumulate, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);

// ---- adaptive summary layer -------------------------------------------------------------------
constexpr int SUM_CH = 16;        // tokens per workgroup chunk
int64_t summary_max_chunks(int64_t n_tok, int64_t S);      // chunks the launches cover
hipError_t launch_summary_forward(const bf16_t* hidden, int64_t T, int C, const int32_t* tok,
                                  const int32_t* seg, int64_t n_tok, int S, const bf16_t* w,
                                  bf16_t* out, float* scores, float* lse, float* xs_f32,
                                  float* part_acc, float* part_md, hipStream_t s);
hipError_t launch_summary_backward(const bf16_t* hidden, int64_t T, int C, const int32_t* tok,
                                   const int32_t* seg, int64_t n_tok, int S, const bf16_t* w,
                                   const float* xs_f32, const float* scores, const float* lse,
                                   const bf16_t* gout, bf16_t* grad_hidden, float* part_dw, float* dw,
                                   int accumulate, hipStream_t s);

// ---- retained-token selection ---------------------------------------------------------------------
constexpr int SEL_CH = 16;        // tokens per workgroup of the similarity kernel
hipError_t launch_select_retained(const bf16_t* feat, const bf16_t* cls, const int32_t* seq_off,
                                  int64_t n_feat, int B, int Cv, int n_keep, const int32_t* n_keep_dev,
                                  uint8_t* mask, float* sim, const int32_t* token_pos,
                                  uint8_t* skip_mask, int64_t T, hipStream_t s);

// ---- token merge -----------------------------------------------------------------------------------
constexpr int MERGE_MAX_N = 4096;   // tokens per set (the similarity matrix is n x n fp32)
hipError_t launch_row_normalize(const bf16_t* x, int64_t rows, int C, bf16_t* xn, hipStream_t s);
hipError_t launch_gemm_selfsim(const bf16_t* xn, int C, const SegTable& st, int n_max, float* sim, int ld,
                               int64_t sim_stride, hipStream_t s);
hipError_t launch_merge_group(const bf16_t* x, const SegTable& st, int n_max, int C, int k, int set_base,
                              const float* sim, int ld, int64_t sim_stride, float* avg, uint8_t* kept,
                              int32_t* slot_of, int32_t* kept_idx, int32_t* assign, bf16_t* out,
                              hipStream_t s);
hipError_t launch_merge_bwd_group(const bf16_t* dout, const SegTable& st, int n_max, int C, int k, int set_base,
                                  const int32_t* assign, bf16_t* dx, hipStream_t s);

// ---- measurement aid: register-only MFMA loop -------------------------------------------------------
// out: blocks * 256 floats; clocks: 2 * blocks int64 (shader cycles, 100 MHz wall ticks per workgroup)
hipError_t launch_mfma_probe(int blocks, int iters, int random_operands, float* out, long long* clocks,
                             hipStream_t s);

// ---- GEMMs -----------------------------------------------------------------------
hipError_t gemm_init();   // raises the dynamic-LDS limit of every instantiation (once per process)
// layouts: a_kc / b_kc as in gemm.hpp
hipError_t launch_gemm(bool a_kc, bool b_kc, int epi, GemmArgs& args, hipStream_t s);
// two independent GEMMs in one grid (problem 0 is dispatched first)
enum DualKind : int {
    DUAL_DH_DWDOWN = 0    // <KC,MNC,SWIGLU_BWD> (dH -> dG, dU)  +  <KC,KC,STORE> (dW_down = dY^T * H)
};
hipError_t launch_gemm_dual(int which, GemmArgs& a0, GemmArgs& a1, hipStream_t s);
// balanced split-K GEMM into fp32 partial slabs (EPI_PARTIAL): nbg workgroups per n-tile group
hipError_t launch_gemm_streamk(bool a_kc, bool b_kc, GemmArgs& args, int nbg, hipStream_t s);

}  // namespace skipffn
