/*
 * libkdloss - full-vocabulary knowledge-distillation loss, forward + backward,
 * for one AMD MI355X (gfx950).
 *
 * The operation (KDFlow paper, abstract and Sec. 3.2 "Efficient Communication
 * via Hidden States"): a student worker receives the teacher's final hidden
 * states h_t [T,H_t] instead of teacher logits, rebuilds the full teacher
 * logits with a frozen copy of the teacher output head,  z_t = h_t . W_t,
 * and aligns the student's logits  z_s = h_s . W_s  to them with one of the
 * divergences of Sec. 3.4 (forward KL, reverse KL, Jensen-Shannon).  The
 * student's backward pass (Sec. 3.1, StudentActorGroup) then needs
 * dL/dh_s and dL/dW_s.  This library is that computation and nothing else.
 *
 * Definitions (the paper names the divergences; these are the textbook forms
 * it refers to, natural logarithm, p = softmax(z / tau) for both models):
 *   FKL: l_t = KL(p_t || p_s)            RKL: l_t = KL(p_s || p_t)
 *   JSD: l_t = beta KL(p_t || M) + (1-beta) KL(p_s || M),  M = beta p_t + (1-beta) p_s
 *   n = sum_t mask_t,  loss = sum_t mask_t l_t / n   (0 when n == 0)
 *   grad_h_s = dL/dz_s . W_s^T,   grad_W_s = h_s^T . dL/dz_s
 * No tau^2 factor is applied.  Masked tokens are compacted away on the device before any
 * product is formed, so they cost nothing.  Logits are never stored: they are produced
 * vocabulary tile by vocabulary tile in registers, twice (three times for JSD,
 * TVD and the skewed KLs, whose row value needs both log-sum-exps first).
 *
 * Conventions of every entry point
 *  - plain C ABI; no exceptions, no allocation, no device synchronisation.  The
 *    caller owns every buffer.  The entry points of this header read no
 *    environment variable and keep no state from one call to the next, except
 *    that each kernel's launch attribute is set once per process and device, and
 *    that kd_loss_fwd_bwd_static works in a device array owned by the library.
 *    (The measurement aids of kdloss_bench.h keep a per-thread hook.)
 *  - all argument checks run on the host before anything touches the GPU, so
 *    they can be exercised on a machine without one.
 *  - work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and the call returns without waiting.  Only kernels are
 *    enqueued (no memsets, no copies), so a call may be captured into a HIP graph;
 *    the workspace carries nothing from one call to the next.
 */
#ifndef KDLOSS_H
#define KDLOSS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KD_OK = 0,
  KD_ERR_NULL = 1,        /* a required pointer is NULL                          */
  KD_ERR_SHAPE = 2,       /* T, H_t, H_s or V < 1, or beyond the supported range */
  KD_ERR_ALIGN = 3,       /* pointer not 16-byte aligned, or H_t/H_s/V % 8 != 0  */
  KD_ERR_PARAM = 4,       /* tau outside [1e-6, 1e6] or not finite, unknown enum, beta outside (0,1) where it is used */
  KD_ERR_WORKSPACE = 5,   /* workspace_bytes smaller than kd_loss_workspace_size */
  KD_ERR_UNSUPPORTED = 6, /* valid request this build does not implement         */
  KD_ERR_LAUNCH = 7,      /* the HIP runtime refused a launch (see hipGetLastError) */
  KD_ERR_TOO_LARGE = 8    /* kd_loss_fwd_bwd_static only: the problem needs more scratch memory than
                             the library's static array holds (KD_STATIC_SCRATCH_BYTES) */
} kd_status;

/* Sec. 3.4 / Table 1: built-in divergence metrics.
 *   KD_TVD      = 1/2 sum_v |p_t - p_s|
 *   KD_SKEW_FKL = KL(p_t || a p_t + (1-a) p_s),  KD_SKEW_RKL = KL(p_s || (1-a) p_t + a p_s),
 *   with the skew weight a passed in `beta` (0 < a < 1; a -> 0 recovers FKL / RKL).
 *   KD_AKL      = w_f KL(p_t || p_s) + w_r KL(p_s || p_t), the adaptive KL of Table 1 (defined in the paper by
 *                 Wu et al. that the authors cite, not in the paper itself).  Per token the vocabulary is
 *                 split by the teacher: in descending order of p_t, the head is the longest prefix whose
 *                 cumulative teacher mass stays <= mu (the top entry always belongs to it), the tail the
 *                 rest; w_f = g_head / (g_head + g_tail), w_r = g_tail / (g_head + g_tail) with
 *                 g = sum |p_t - p_s| over the part (1/2 each if both vanish).  mu is passed in `beta`
 *                 (0 < mu < 1; the cited method uses 1/2).  The weights are constants for the gradient.
 *                 The head boundary is found by a search over teacher log-probabilities to within 5e-4
 *                 (base 2): entries that close to the boundary may fall on either side.  Costs four
 *                 more passes over the teacher logits and one more over both; not with the fp8 teacher. */
typedef enum { KD_FKL = 0, KD_RKL = 1, KD_JSD = 2, KD_TVD = 3, KD_SKEW_FKL = 4, KD_SKEW_RKL = 5, KD_AKL = 6 } kd_kind;

typedef enum { KD_BF16 = 0, KD_F32 = 1 } kd_dtype;

/* Storage order of an output head W (mathematical shape [H, V]):
 *   KD_W_HV: W[k * V + v]   (V contiguous)
 *   KD_W_VH: W[v * H + k]   (H contiguous; the order lm_head.weight is kept in)
 * The same order applies to W_t, W_s and grad_W_s.  KD_W_VH is the faster one (both logit operands
 * contiguous along the contraction; about 5 % ahead).  KD_W_HV heads are read in place when they are
 * bf16 with H_t, H_s and V multiples of 64; otherwise they are re-packed into the workspace (which then
 * holds copies of both heads) by a slow strided pass, a fallback for small problems.  grad_W_s is written
 * in the caller's order either way.  With the fp8 teacher, KD_W_HV heads always take the re-packing path
 * (better: quantise the frozen head from a [V,H] copy once and pass KD_W_VH). */
typedef enum { KD_W_HV = 0, KD_W_VH = 1 } kd_wlayout;

/* KD_FLAG_TAU2: multiply the loss, the per-token losses and both gradients by tau^2 (the
 * convention that keeps gradient magnitudes independent of the temperature).  Off by default:
 * the paper does not mention it. */
/* KD_FLAG_TEACHER_FP8: h_t and W_t hold OCP e4m3 bytes (one per element) instead of in_dtype values,
 * quantised with one scale per array (kd_quantize_e4m3):  z_t = teacher_scale * sum_k q_h[t,k] q_W[v,k],
 * teacher_scale = scale_h * scale_W.  The teacher logit tiles then run on the fp8 matrix pipe at twice the
 * bf16 rate and half the operand traffic; everything else (student side, divergence, gradients) is unchanged.
 * An extension in the spirit of the paper's FP8 teacher inference (Table 3): the paper does not quantise the
 * head.  Requires in_dtype == KD_BF16 and H_t a multiple of 128.  In the multi-teacher
 * call every teacher is then fp8, each with its own scale (teacher_scales[k]; params->teacher_scale is not read). */
typedef enum { KD_FLAG_TAU2 = 1, KD_FLAG_TEACHER_FP8 = 2 } kd_flags;

typedef struct {
  int64_t T;            /* tokens (batch x sequence, flattened)                     */
  int64_t H_t, H_s;     /* teacher / student hidden sizes, multiples of 8           */
  int64_t V;            /* vocabulary size shared by both heads, multiple of 8      */
  int32_t in_dtype;     /* kd_dtype of h_t, W_t, h_s, W_s                           */
  int32_t grad_dtype;   /* kd_dtype of grad_h_s and grad_W_s                        */
  int32_t w_layout;     /* kd_wlayout                                               */
  int32_t kind;         /* kd_kind                                                  */
  float tau;            /* temperature, 1e-6 <= tau <= 1e6.  The scaled logits z / tau
                           are held in fp32: results are meaningful while |z| / tau
                           stays below about 1e5, and a loss far below 1e-4 (very
                           high temperatures) is resolved to about 1e-7 absolute    */
  float beta;           /* JSD mixing weight on the teacher term, the skew weight of
                           the skewed KLs, or AKL's head mass mu; 0 < beta < 1;
                           ignored for FKL/RKL/TVD                                  */
  int32_t accumulate_grad_W; /* 0: grad_W_s is overwritten. 1: added to (gradient
                           accumulation over micro-batches, Table 3 caption)        */
  int32_t flags;        /* bit set of kd_flags; other bits must be 0                */
  float teacher_scale;  /* KD_FLAG_TEACHER_FP8 only: > 0, finite                    */
  int32_t vocab_chunk;  /* columns of the vocabulary handled per backward chunk (the
                           width of the dL/dz_s staging buffer): 0 = chosen by the
                           library, else a multiple of 256 in [256, 2^20].  Enters
                           the size query and the call alike, so the two cannot
                           disagree.  Results do not depend on it beyond the
                           summation order of grad_h_s                              */
  float loss_scale;     /* finite, non-zero: factor on the loss, the per-token losses
                           and both gradients (1 = the plain masked mean; e.g. 1 /
                           micro-batches under gradient accumulation, or the
                           upstream gradient when it is known before the call)      */
  int32_t reserved;     /* must be 0 (KD_ERR_PARAM otherwise)                       */
} kd_loss_params;

/* Bytes of device workspace kd_loss_fwd_bwd needs for these parameters.
 * (Footnote of Sec. 1: shipping full logits would take about 160 GB per global
 * batch, 2 T V bytes per T tokens; this is what the recomputation needs instead.)
 * Host only.  The size is O(T * V_c + H_s * V_c + T * (H_t + H_s)) for a vocabulary
 * chunk V_c chosen by the library (a few thousand columns) - staging of dL/dz_s,
 * fp32 sums of grad_h_s, compacted copies of the hidden states - plus copies of
 * the heads only when they must be re-packed (fp32 inputs, hidden sizes that are
 * not multiples of 64).  It never grows like T * V.  Returns KD_OK or the status kd_loss_fwd_bwd would return for
 * the same params. */
kd_status kd_loss_workspace_size(const kd_loss_params* params, size_t* bytes);

/* Forward + backward of the distillation loss (paper Sec. 3.2 and 3.4; student
 * backward of Sec. 3.1).
 *
 *  h_t  [T, H_t]  device, read-only, row-major (H contiguous), in_dtype
 *  W_t  head of the teacher, device, read-only, in_dtype, order w_layout
 *  h_s  [T, H_s]  device, read-only
 *  W_s  head of the student, device, read-only
 *  mask [T] uint8 device, non-zero = token counts; NULL = every token counts
 *  loss            device, one float: the masked-mean divergence
 *  per_token_loss  device, [T] floats (l_t; 0 for masked tokens, which are never computed) or NULL
 *  grad_h_s [T, H_s] device, grad_dtype; rows of masked tokens are exactly 0
 *  grad_W_s device, grad_dtype, same order as W_s; overwritten or accumulated
 *  workspace       device, 256-byte aligned, workspace_bytes >= the size query
 *  hip_stream      hipStream_t
 *
 * Pointers must be 16-byte aligned.  Inputs must not alias outputs or the
 * workspace.  Results are bitwise reproducible from call to call (no floating
 * point atomics).  On any status other than KD_OK and KD_ERR_LAUNCH nothing
 * was enqueued. */
kd_status kd_loss_fwd_bwd(const kd_loss_params* params,
                          const void* h_t, const void* W_t,
                          const void* h_s, const void* W_s,
                          const uint8_t* mask,
                          float* loss, float* per_token_loss,
                          void* grad_h_s, void* grad_W_s,
                          void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/* kd_loss_fwd_bwd for callers that cannot allocate device memory or have no workspace to pass: code
 * that runs under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.
 * Same arguments, checks, kernels and results as kd_loss_fwd_bwd, minus the workspace: the scratch memory
 * is a static device array of KD_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs on
 * holds its own copy until the process ends).  The call allocates and frees nothing.
 *  - With params->vocab_chunk == 0 the library picks the widest vocabulary chunk whose plan fits the
 *    array; with a chunk given, that plan must fit.  A problem that does not fit returns
 *    KD_ERR_TOO_LARGE and enqueues nothing (the headline workload, T = 4096, H_t = 4096, H_s = 1024,
 *    V = 151936, fits; T = 32768 with H_s = 4096 does not).
 *  - The array's address is looked up on the first call on each device (current device = the stream's);
 *    make that first call outside a graph capture.
 *  - Nothing in the array has to be zero or survive between calls, but every call on one GPU uses the
 *    same array: calls that overlap in time on one GPU (two streams, two threads) race.  Serialise them,
 *    or give the concurrent ones their own workspace through kd_loss_fwd_bwd. */
#define KD_STATIC_SCRATCH_BYTES ((size_t)128 << 20)
kd_status kd_loss_fwd_bwd_static(const kd_loss_params* params,
                                 const void* h_t, const void* W_t,
                                 const void* h_s, const void* W_s,
                                 const uint8_t* mask,
                                 float* loss, float* per_token_loss,
                                 void* grad_h_s, void* grad_W_s,
                                 void* hip_stream);

/* Forward only: loss and per-token loss, no gradients (the logit tiles are
 * produced once; twice for JSD).  Same arguments and checks as above. */
kd_status kd_loss_fwd(const kd_loss_params* params,
                      const void* h_t, const void* W_t,
                      const void* h_s, const void* W_s,
                      const uint8_t* mask,
                      float* loss, float* per_token_loss,
                      void* workspace, size_t workspace_bytes,
                      void* hip_stream);

/* Quantise n values to OCP e4m3 bytes (KD_FLAG_TEACHER_FP8):  dst[i] = e4m3(src[i] * (1 / scale)), the
 * reciprocal and the product in fp32, round to nearest even, magnitudes beyond 448 saturate, NaN -> 0x7f.
 * src: device, src_dtype (KD_BF16 or KD_F32), n values; dst: device, n bytes; both 16-byte aligned.
 * A good scale is max|src| / 448.  The frozen teacher head is quantised once, hidden states per batch. */
kd_status kd_quantize_e4m3(const void* src, int32_t src_dtype, int64_t n, float scale, void* dst,
                           void* hip_stream);

/* Multi-teacher distillation (Table 1, "Multi-Teacher Distillation"): n_teachers teachers over the
 * same tokens and vocabulary, each with its own hidden states h_t[k] [T, H_t[k]] and head W_t[k];
 *   loss = sum_k weights[k] * D(p_t^k, p_s)      (same divergence, temperature and mask for all)
 * and the gradients are those of that sum.  params->H_t is ignored; h_t, W_t, H_t, weights (and
 * teacher_scales, read only with KD_FLAG_TEACHER_FP8, else may be NULL) are HOST arrays of n_teachers
 * entries (the pointers in h_t / W_t are device pointers).  1 <= n_teachers <= 16.
 * Everything else is as for kd_loss_fwd_bwd; the workspace must satisfy the _multi size query (the
 * single-teacher workspace plus, per teacher, its row statistics and any re-packed operand copies).
 * The token compaction, the student operands and the two backward products are shared: each chunk of
 * dL/dz_s is summed over the teachers (in its bf16 staging buffer) before grad_W_s and grad_h_s are
 * formed once.  The student logit tiles are recomputed with every teacher's tiles. */
kd_status kd_loss_workspace_size_multi(const kd_loss_params* params, int n_teachers, const int64_t* H_t,
                                       size_t* bytes);
kd_status kd_loss_fwd_bwd_multi(const kd_loss_params* params, int n_teachers,
                                const void* const* h_t, const void* const* W_t, const int64_t* H_t,
                                const float* weights, const float* teacher_scales,
                                const void* h_s, const void* W_s, const uint8_t* mask,
                                float* loss, float* per_token_loss, void* grad_h_s, void* grad_W_s,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/* Static, NUL-terminated description of a status code (error reporting of this boundary; nothing of
 * the paper's). */
const char* kd_status_string(kd_status status);

/* For reports: the vocabulary chunk kd_loss_fwd_bwd uses for these params and the number of kernels
 * one call launches (counted as for a call with a mask, whose hidden states are compacted into the
 * workspace).  Either output pointer may be NULL.  Host only. */
kd_status kd_loss_plan_info(const kd_loss_params* params, int64_t* vocab_chunk,
                            int64_t* n_launches);

#ifdef __cplusplus
}
#endif
#endif /* KDLOSS_H */
