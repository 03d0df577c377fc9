// Host-side interface between the C ABI layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace kd {

constexpr int kNumCU = 256;            // MI355X: 8 XCDs x 32 CUs; persistent grids are sized for it
constexpr int kTileM = 128;            // vocabulary rows per logit tile
constexpr int kTileN = 256;            // token rows per logit tile
#ifndef KD_GEMM_TILE_M
#define KD_GEMM_TILE_M 128
#endif
constexpr int kGemmTileM = KD_GEMM_TILE_M;        // rows of the first operand per tile of the backward products

// Everything a launch needs, resolved by the planner in kd_api.hip.
struct Problem {
  int T, V, H_s, H_t;
  int kind;
  float tau, beta;
  int grad_f32;
  int accumulate_grad_W;
  float out_weight;        // factor on the loss and the gradients of this call (teacher weight, tau^2)
  int accumulate_loss;     // add to *loss and per_token_loss instead of overwriting them
  const void *h_t, *W_t, *h_s, *W_s;                   // bf16 [rows][K_t or K_s] as the kernels read them
  const void *user_h_t, *user_W_t, *user_h_s, *user_W_s;  // the caller's arrays
  int in_f32;                   // inputs are fp32
  int w_hv;                     // the caller's heads and grad_W_s are stored [H][V]
  int w_hv_inplace;             // ... and the kernels read the heads in that order, in place (else they are
                                // re-packed into [V][K] copies like any operand that needs re-packing)
  long long* clock_out;         // measurement aid, see kd_loss_profile_clock (null unless set)
  int t_fp8;                    // teacher operands are e4m3 bytes (K_t = H_t elements = bytes per row)
  float t_scale;                // ... and z_t = t_scale * (product of the codes)
  int prep_ht, prep_Wt, prep_hs, prep_Ws;   // which operands are re-packed into the workspace
  int K_t, K_s;                 // contraction lengths of the (re-packed) logit operands, multiples of 64
  const uint8_t* mask;
  float* loss;
  float* per_token_loss;
  void *grad_h_s, *grad_W_s;
  // plan
  int T_pad, n_tt, n_vt, n_split, V_c, n_ksplit_h, ksteps_h, n_cu;
  // workspace carve-up
  int* meta;           // device-side plan written by the row-map kernel
  int* rowmap;         // [T_pad] compacted index -> token
  int* inv;            // [T] token -> compacted index or -1
  float* rowinfo;      // [T_pad][4]
  float* akl;          // AKL only: [6][T_pad] per-token values between its passes (null otherwise)
  float* row_loss;     // [T_pad]
  float* partials;     // [n_split*4][5][T_pad]
  void* h_sT;          // bf16 [H_s][T_pad]
  void* dz;            // bf16 [T_pad][V_c]
  float* gh32;         // [n_ksplit_h][T][H_s]
};

// out[n][m] (+)= sum_k A[m][k] B[n][k]; A is [M][lda], B is [N][ldb], both K-contiguous bf16.
struct GemmDesc {
  const void *A, *B;
  int lda, ldb, M, N;
  int K;                  // multiple of 64
  int k_per_split;        // split-K: elements per part, a multiple of 64 (0 = no split); part s writes
                          // out + s * out_split_stride
  void* out;
  int64_t ldo, out_split_stride;
  int out_f32, accumulate;
  const int* meta;        // device-side plan, needed when a flag below is set
  int n_from_meta;        // N = number of valid tokens
  int k_from_meta;        // K = valid tokens rounded up to whole token tiles (no split-K)
  int k_major;            // 0: both K-contiguous; 1: A is stored [K][M] (element (m, k) at A[k * lda + m]);
                          // 2: B is stored [K][N]
  int k_rows;             // rows of the k-major operand that exist; K may round up beyond, the other
                          // operand must be zero there
};

hipError_t launch_rowmap(const Problem& p, hipStream_t st);
hipError_t launch_mfma_probe(const void* operands, int iters, float* sink, long long* clock_out, int n_cu,
                             hipStream_t st);
hipError_t launch_quantize_e4m3(const void* src, int src_f32, int64_t n, float inv_scale, void* dst, hipStream_t st);
hipError_t launch_stats(const Problem& p, hipStream_t st);
hipError_t launch_combine(const Problem& p, hipStream_t st);
hipError_t launch_rows(const Problem& p, hipStream_t st);
hipError_t launch_akl_search(const Problem& p, hipStream_t st);      // one search pass and its merge
hipError_t launch_akl_weights(const Problem& p, hipStream_t st);
constexpr int kAklSearchPasses = 4;    // 17-fold narrowing each: 40 -> 4.8e-4 in base-2 log-probability
constexpr int kAklThresholds = 16;     // per pass (the kernels' AKL_K)
hipError_t launch_combine_rows(const Problem& p, hipStream_t st);
hipError_t launch_finalize(const Problem& p, hipStream_t st);
hipError_t launch_grad_chunk(const Problem& p, int v0, int width, bool accumulate, hipStream_t st);
// dst[c][r] = src[r][c] (zero for R <= r < R_pad); elements of 1 or 2 bytes
hipError_t launch_transpose(const void* src, int64_t ld_src, int R, int C, void* dst, int64_t ld_dst, int R_pad,
                            int elem_bytes, hipStream_t st);
hipError_t launch_gemm(const GemmDesc& d, int n_cu, hipStream_t st);
hipError_t launch_gradh_finish(const Problem& p, hipStream_t st);
const char* build_info();     // compile-time configuration of the kernels (tile shapes, ablation switch)
int build_ablation();
// dst bf16 [R][K]: mode 0 = copy, 1 = fp32 split as [hi|hi|lo], 2 = fp32 split as [hi|lo|hi]; zero-padded to K
hipError_t launch_prepare(const void* src, int src_f32, int R, int H, void* dst, int K, int split_mode,
                          const int* rowmap, const int* meta, int src_transposed, hipStream_t st);

}  // namespace kd
