// C ABI of libkdloss: argument checks, workspace planning and the launch sequence.
// All checks are host-only and happen before the first HIP call.
#include <hip/hip_runtime.h>

#include "../../include/kdloss.h"
#include "../../include/kdloss_bench.h"
#include "kd_launch.h"

#include <atomic>
#include <cmath>
#ifdef KD_TRACE_ERRORS
#include <cstdio>
#endif

// Scratch memory of kd_loss_fwd_bwd_static: one array per GPU, owned by the library.  In host code this
// name is only a handle for hipGetSymbolAddress; the device address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[KD_STATIC_SCRATCH_BYTES];

namespace {

using kd::Problem;

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Layout {
  size_t meta, rowmap, inv, row_loss, partials, h_sT, dz, gh32;
  size_t prep_h_s, prep_W_s;                       // re-packed student operands (only when needed)
  size_t common;                                   // end of everything above: the same for every teacher
  size_t rowinfo, akl, prep_h_t, prep_W_t;         // per-teacher block (row statistics, re-packed operands)
  size_t total;                                    // end of this teacher's block
};

kd_status check_params(const kd_loss_params* p) {
  if (!p) return KD_ERR_NULL;
  if (p->T < 1 || p->H_t < 1 || p->H_s < 1 || p->V < 1) return KD_ERR_SHAPE;
  if (p->T > (1 << 22) || p->V > (1 << 24) || p->H_t > 65536 || p->H_s > 65536) return KD_ERR_SHAPE;
  if (p->H_t % 8 || p->H_s % 8 || p->V % 8) return KD_ERR_ALIGN;
  if (p->in_dtype != KD_BF16 && p->in_dtype != KD_F32) return KD_ERR_PARAM;
  if (p->grad_dtype != KD_BF16 && p->grad_dtype != KD_F32) return KD_ERR_PARAM;
  if (p->w_layout != KD_W_HV && p->w_layout != KD_W_VH) return KD_ERR_PARAM;
  if (p->kind < KD_FKL || p->kind > KD_AKL) return KD_ERR_PARAM;
  if (!(p->tau >= 1e-6f && p->tau <= 1e6f)) return KD_ERR_PARAM;   // also rejects NaN
  if ((p->kind == KD_JSD || p->kind == KD_SKEW_FKL || p->kind == KD_SKEW_RKL || p->kind == KD_AKL) &&
      !(p->beta > 0.f && p->beta < 1.f))
    return KD_ERR_PARAM;
  if (p->accumulate_grad_W != 0 && p->accumulate_grad_W != 1) return KD_ERR_PARAM;
  if (p->flags & ~(int32_t)(KD_FLAG_TAU2 | KD_FLAG_TEACHER_FP8)) return KD_ERR_PARAM;
  if (p->flags & KD_FLAG_TEACHER_FP8) {
    if (!(p->teacher_scale > 0.f && p->teacher_scale < INFINITY)) return KD_ERR_PARAM;
    if (p->in_dtype != KD_BF16) return KD_ERR_UNSUPPORTED;     // the student side stays bf16
    if (p->H_t % 128) return KD_ERR_ALIGN;                     // fp8 k-steps are 128 elements
  }
  if (p->kind == KD_AKL && (p->flags & KD_FLAG_TEACHER_FP8)) return KD_ERR_UNSUPPORTED;   // its search pass is bf16 only
  if (p->vocab_chunk != 0 && (p->vocab_chunk < 256 || p->vocab_chunk > (1 << 20) || p->vocab_chunk % 256))
    return KD_ERR_PARAM;
  if (!(std::isfinite(p->loss_scale) && p->loss_scale != 0.f)) return KD_ERR_PARAM;
  if (p->reserved != 0) return KD_ERR_PARAM;
  return KD_OK;
}

// Tile counts, vocabulary chunk and split factors.  Depends on the params only.  The per-teacher
// block is placed at `teacher_base` (default: right after the common part).  `repack_hv` makes
// [H][V] heads go through the re-packing path even where they could be read in place (a
// multi-teacher call takes that decision once for all its teachers).
void plan(const kd_loss_params* p, Problem& q, Layout& L, bool with_backward, size_t teacher_base = 0,
          bool repack_hv = false) {
  q.T = (int)p->T; q.V = (int)p->V; q.H_s = (int)p->H_s; q.H_t = (int)p->H_t;
  q.kind = p->kind; q.tau = p->tau; q.beta = p->beta;
  q.grad_f32 = p->grad_dtype == KD_F32;
  q.accumulate_grad_W = p->accumulate_grad_W;
  q.out_weight = p->loss_scale * ((p->flags & KD_FLAG_TAU2) ? p->tau * p->tau : 1.f);
  q.accumulate_loss = 0;
  q.n_cu = kd::kNumCU;
  // Operands as the kernels want them: bf16, K-contiguous, K a multiple of 64.  fp32 inputs are
  // split into bf16 high and low parts laid side by side along K (three products recover all
  // but the low x low term); bf16 inputs with an odd hidden size are zero-padded along K.
  q.in_f32 = p->in_dtype == KD_F32;
  q.w_hv = p->w_layout == KD_W_HV;
  q.t_fp8 = (p->flags & KD_FLAG_TEACHER_FP8) ? 1 : 0;
  q.t_scale = q.t_fp8 ? p->teacher_scale : 1.f;
  q.K_t = (int)round_up(q.in_f32 ? 3 * q.H_t : q.H_t, 64);      // fp8: H_t % 128 == 0, used as it is
  q.K_s = (int)round_up(q.in_f32 ? 3 * q.H_s : q.H_s, 64);
  q.prep_Wt = q.in_f32 || q.K_t != q.H_t;
  q.prep_Ws = q.in_f32 || q.K_s != q.H_s;
  // [H][V] heads are read in place as k-major operands when they are bf16 with whole k-steps and a
  // vocabulary that the K-contiguous operand of the grad_h_s product can walk in whole 64-element
  // steps; otherwise both are re-packed (transposing) and the kernels see [V][K] copies
  // (an fp8 teacher head kept as [H][V] bytes is transposed into a [V][H] copy: the fp8 phase of the tile
  // loop reads K-contiguous rows only)
  q.w_hv_inplace = q.w_hv && !repack_hv && !q.t_fp8 && !q.prep_Wt && !q.prep_Ws && q.V % 64 == 0;
  if (q.w_hv && !q.w_hv_inplace) q.prep_Wt = q.prep_Ws = 1;
  // hidden states are also re-packed when a mask is given: valid tokens are compacted to the front
  // (the workspace is sized as if it were, since the size query does not see the mask)
  q.prep_ht = q.prep_hs = 1;
  q.T_pad = (int)round_up(q.T, kd::kTileN);
  q.n_tt = q.T_pad / kd::kTileN;
  q.n_vt = (int)((q.V + kd::kTileM - 1) / kd::kTileM);
  // Vocabulary splits of the statistics passes.  The device picks the actual number once it knows
  // how many token tiles survive the mask (about n_cu / tiles, at least 8 so that the 32 workgroups
  // co-resident on an XCD form a 4 x 8 block); this is the upper bound the buffers are sized for:
  // enough to keep every CU busy with up to half of the tokens masked.
  int ns = 2 * ((q.n_cu + q.n_tt - 1) / q.n_tt);
  if (ns < 8) ns = 8;
  if (ns > q.n_cu) ns = q.n_cu;          // a single token tile is split over all CUs
  if (ns > q.n_vt) ns = q.n_vt;
  if (ns < 1) ns = 1;
  q.n_split = ns;

  // vocabulary chunk of the backward pass: a power of two.  The [T_pad, V_c] bf16 staging buffer of
  // dL/dz_s is written by the gradient kernel and read back by both products, so it should stay within
  // the 256 MB last-level cache together with the operands (128 MiB: measured best from T = 256 to 4096);
  // but every chunk also re-reads and re-writes the fp32 sums of grad_h_s, so with many tokens a chunk
  // of at least 8192 columns wins as long as the staging buffer stays within 512 MiB.
  int64_t vc = 1 << 20;
  while (vc > 1024 && (int64_t)q.T_pad * vc * 2 > (128ll << 20)) vc >>= 1;
  if (vc < 8192) {
    vc = 8192;
    while (vc > 1024 && (int64_t)q.T_pad * vc * 2 > (512ll << 20)) vc >>= 1;
  }
  if (p->vocab_chunk > 0) vc = p->vocab_chunk;       // the caller's choice (checked: a multiple of 256)
  const int64_t v_all = round_up(q.V, 256);
  if (vc > v_all) vc = v_all;
  q.V_c = (int)vc;

  // split-K of the grad_h_s product so that a chunk offers about one tile per CU
  const int tiles_h = ((q.H_s + kd::kGemmTileM - 1) / kd::kGemmTileM) * q.n_tt;
  int sk = q.n_cu / tiles_h;
  if (sk < 1) sk = 1;
  if (sk > 32) sk = 32;
  while (sk > 1 && q.V_c / sk < 512) --sk;
  const int steps_first = (int)(round_up(q.V < q.V_c ? q.V : q.V_c, 64) / 64);
  if (sk > steps_first) sk = steps_first;
  q.ksteps_h = (steps_first + sk - 1) / sk;
  q.n_ksplit_h = (steps_first + q.ksteps_h - 1) / q.ksteps_h;   // every part is written by the first chunk

  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = (size_t)round_up((int64_t)(off + bytes), 256); return o; };
  L.meta = take(64);
  L.rowmap = take((size_t)q.T_pad * 4);
  L.inv = take((size_t)q.T * 4);
  L.row_loss = take((size_t)q.T_pad * 4);
  // partial sums per (vocabulary split, quarter of a workgroup, token): 5 statistics, 6 for AKL, whose
  // search passes keep one sum per threshold
  const int part_vals = q.kind == KD_AKL ? kd::kAklThresholds : 5;
  L.partials = take((size_t)q.n_split * 4 * part_vals * q.T_pad * 4);
  L.prep_h_t = L.prep_W_t = L.prep_h_s = L.prep_W_s = 0;
  if (q.prep_hs) L.prep_h_s = take((size_t)q.T * q.K_s * 2);
  if (q.prep_Ws) L.prep_W_s = take((size_t)q.V * q.K_s * 2);
  if (with_backward) {
    L.h_sT = take((size_t)q.H_s * q.T_pad * 2);
    L.dz = take((size_t)q.T_pad * q.V_c * 2);
    L.gh32 = take((size_t)q.n_ksplit_h * q.T * q.H_s * 4);
  } else {
    L.h_sT = L.dz = L.gh32 = off;
  }
  // what belongs to one teacher comes last, so that everything above sits at the same offsets for
  // every teacher of a multi-teacher call and the teachers' blocks can lie side by side
  L.common = off;
  if (teacher_base > off) off = teacher_base;
  L.rowinfo = take((size_t)q.T_pad * 16);
  L.akl = q.kind == KD_AKL ? take((size_t)q.T_pad * 6 * 4) : 0;
  const size_t t_es = q.t_fp8 ? 1 : 2;
  if (q.prep_ht) L.prep_h_t = take((size_t)q.T * q.K_t * t_es);
  if (q.prep_Wt) L.prep_W_t = take((size_t)q.V * q.K_t * t_es);
  L.total = off;
}

void carve(Problem& q, const Layout& L, void* ws) {
  char* b = static_cast<char*>(ws);
  q.meta = reinterpret_cast<int*>(b + L.meta);
  q.rowmap = reinterpret_cast<int*>(b + L.rowmap);
  q.inv = reinterpret_cast<int*>(b + L.inv);
  q.rowinfo = reinterpret_cast<float*>(b + L.rowinfo);
  q.akl = q.kind == KD_AKL ? reinterpret_cast<float*>(b + L.akl) : nullptr;
  q.row_loss = reinterpret_cast<float*>(b + L.row_loss);
  q.partials = reinterpret_cast<float*>(b + L.partials);
  q.h_sT = b + L.h_sT;
  q.dz = b + L.dz;
  q.gh32 = reinterpret_cast<float*>(b + L.gh32);
  q.user_h_t = q.h_t; q.user_W_t = q.W_t; q.user_h_s = q.h_s; q.user_W_s = q.W_s;
  // without a mask the hidden states are used in place unless they need re-packing anyway
  if (!q.mask) {
    q.prep_ht = q.prep_Wt;
    q.prep_hs = q.prep_Ws;
  }
  if (q.prep_ht) q.h_t = b + L.prep_h_t;
  if (q.prep_Wt) q.W_t = b + L.prep_W_t;
  if (q.prep_hs) q.h_s = b + L.prep_h_s;
  if (q.prep_Ws) q.W_s = b + L.prep_W_s;
}



// Benchmark aid: bracket the launches of one kernel family with caller-supplied events.
struct ProfileHook {
  int which = -1;
  hipEvent_t* events = nullptr;
  int n_events = 0;
  int used = 0;     // pairs recorded
};
thread_local ProfileHook g_hook;
thread_local long long* g_clock_out = nullptr;   // kd_loss_profile_clock

struct ProfileScope {
  bool on;
  hipStream_t st;
  ProfileScope(int which, hipStream_t s) : on(false), st(s) {
    if (g_hook.which == which && g_hook.events && 2 * g_hook.used + 1 < g_hook.n_events) {
      on = true;
      (void)hipEventRecord(g_hook.events[2 * g_hook.used], st);
    }
  }
  ~ProfileScope() {
    if (on) {
      (void)hipEventRecord(g_hook.events[2 * g_hook.used + 1], st);
      ++g_hook.used;
    }
  }
};

// -DKD_TRACE_ERRORS (a debugging build) names the failing call on stderr.
#ifdef KD_TRACE_ERRORS
#define KD_TRY(expr)                                                                              \
  do {                                                                                            \
    const hipError_t kd_e_ = (expr);                                                              \
    if (kd_e_ != hipSuccess) {                                                                    \
      std::fprintf(stderr, "libkdloss: %s:%d: %s -> %s\n", __FILE__, __LINE__, #expr, hipGetErrorString(kd_e_)); \
      return KD_ERR_LAUNCH;                                                                       \
    }                                                                                             \
  } while (0)
#else
#define KD_TRY(expr)                                \
  do {                                              \
    if ((expr) != hipSuccess) return KD_ERR_LAUNCH; \
  } while (0)
#endif

// Re-pack the operands that need it (fp32 split / K padding / compaction) into the workspace.
kd_status prepare_operands(const Problem& q, hipStream_t st, bool student, bool teacher) {
  const int* map = q.mask ? q.rowmap : nullptr;     // gather valid tokens to the front
  if (teacher && q.prep_ht && q.t_fp8)     // rows of H_t bytes are gathered as rows of H_t / 2 two-byte words
    KD_TRY(kd::launch_prepare(q.user_h_t, 0, q.T, q.H_t / 2, const_cast<void*>(q.h_t), q.K_t / 2, 2, map, q.meta, 0, st));
  else if (teacher && q.prep_ht)
    KD_TRY(kd::launch_prepare(q.user_h_t, q.in_f32, q.T, q.H_t, const_cast<void*>(q.h_t), q.K_t, 2, map, q.meta, 0, st));
  if (teacher && q.prep_Wt && q.t_fp8)      // only ever an [H][V] head of e4m3 bytes: transposed copy
    KD_TRY(kd::launch_transpose(q.user_W_t, q.V, q.H_t, q.V, const_cast<void*>(q.W_t), q.K_t, q.K_t, 1, st));
  else if (teacher && q.prep_Wt)
    KD_TRY(kd::launch_prepare(q.user_W_t, q.in_f32, q.V, q.H_t, const_cast<void*>(q.W_t), q.K_t, 1, nullptr, q.meta, q.w_hv, st));
  if (student && q.prep_hs)
    KD_TRY(kd::launch_prepare(q.user_h_s, q.in_f32, q.T, q.H_s, const_cast<void*>(q.h_s), q.K_s, 2, map, q.meta, 0, st));
  if (student && q.prep_Ws)
    KD_TRY(kd::launch_prepare(q.user_W_s, q.in_f32, q.V, q.H_s, const_cast<void*>(q.W_s), q.K_s, 1, nullptr, q.meta, q.w_hv, st));
  return KD_OK;
}

// Forward pass of one teacher.  The token compaction and the student operands are shared by the
// teachers of a call: only the first one makes them.
kd_status run_forward(const Problem& q, hipStream_t st, bool first_teacher = true) {
  if (first_teacher) KD_TRY(kd::launch_rowmap(q, st));
  {
    kd_status ps = prepare_operands(q, st, first_teacher, true);
    if (ps != KD_OK) return ps;
  }
  {
    ProfileScope ps(KD_PROF_STATS, st);
    KD_TRY(kd::launch_stats(q, st));
  }
  KD_TRY(kd::launch_combine(q, st));
  if (q.kind == KD_AKL) {
    // the teacher probability that splits each token's vocabulary into head and tail, by a multi-way search
    // over the teacher logit tiles; then the head and tail gaps, which weigh the two KLs
    for (int pass = 0; pass < kd::kAklSearchPasses; ++pass) KD_TRY(kd::launch_akl_search(q, st));
    {
      ProfileScope ps(KD_PROF_ROWS, st);
      KD_TRY(kd::launch_rows(q, st));
    }
    KD_TRY(kd::launch_akl_weights(q, st));
  } else if (q.kind >= KD_JSD) {   // divergences that need both log-sum-exps before their row value
    {
      ProfileScope ps(KD_PROF_ROWS, st);
      KD_TRY(kd::launch_rows(q, st));
    }
    KD_TRY(kd::launch_combine_rows(q, st));
  }
  KD_TRY(kd::launch_finalize(q, st));
  return KD_OK;
}

// Backward pass: dL/dz_s chunk by chunk and the two products.  With several teachers the chunk of
// dL/dz_s is the sum over the teachers (each gradient kernel adds its weighted share to the bf16
// staging buffer), so the products run once per chunk whatever the number of teachers.  grad_h_s is
// summed in fp32 over the chunks and converted once at the end.
kd_status run_backward(const Problem* qs, int n_teachers, hipStream_t st) {
  const Problem& q = qs[0];          // everything on the student side is the same for all teachers
  // h_s^T [H_s][T_pad] once (token axis zero-padded): the K-contiguous operand of grad_W_s
  KD_TRY(kd::launch_transpose(q.h_s, q.K_s, q.T, q.H_s, q.h_sT, q.T_pad, q.T_pad, 2, st));

  const size_t gsz = q.grad_f32 ? 4 : 2;
  bool first = true;
  for (int64_t v0 = 0; v0 < q.V; v0 += q.V_c) {
    const int width = (int)((q.V - v0 < q.V_c) ? q.V - v0 : q.V_c);
    for (int k = 0; k < n_teachers; ++k) {
      ProfileScope ps(KD_PROF_GRAD, st);
      KD_TRY(kd::launch_grad_chunk(qs[k], (int)v0, width, k > 0, st));
    }
    kd::GemmDesc gw{}, gh{};
    gw.K = q.T_pad; gw.k_per_split = 0;
    gw.meta = q.meta; gw.k_from_meta = 1;        // only the token tiles that hold valid tokens
    gw.out_split_stride = 0;
    gw.out_f32 = q.grad_f32; gw.accumulate = q.accumulate_grad_W;
    gh.B = q.dz; gh.ldb = q.V_c; gh.N = q.T;
    gh.meta = q.meta; gh.n_from_meta = 1;        // rows = valid tokens
    gh.K = (int)round_up(width, 64); gh.k_per_split = q.ksteps_h * 64;
    gh.out = q.gh32; gh.ldo = q.H_s; gh.out_split_stride = (int64_t)q.T * q.H_s;
    gh.out_f32 = 1; gh.accumulate = first ? 0 : 1;
    if (!q.w_hv) {
      // grad_W_s[v][h] = sum_t h_sT[h][t] dz[t][v]   (dz read token-major as it lies)
      gw.A = q.h_sT; gw.lda = q.T_pad; gw.M = q.H_s;
      gw.B = q.dz; gw.ldb = q.V_c; gw.N = width;
      gw.k_major = 2; gw.k_rows = q.T_pad;
      gw.out = static_cast<char*>(q.grad_W_s) + (size_t)v0 * q.H_s * gsz; gw.ldo = q.H_s;
    } else {
      // the caller keeps grad_W_s as [H][V]: grad_W_s[h][v] = sum_t dz[t][v] h_sT[h][t], dz again read as it
      // lies, now as the first operand so that the output rows run along the vocabulary
      gw.A = q.dz; gw.lda = q.V_c; gw.M = width;
      gw.B = q.h_sT; gw.ldb = q.T_pad; gw.N = q.H_s;
      gw.k_major = 1; gw.k_rows = q.T_pad;
      gw.out = static_cast<char*>(q.grad_W_s) + (size_t)v0 * gsz; gw.ldo = q.V;
    }
    if (!q.w_hv_inplace) {
      // grad_h_s[t][h] += sum_v W_s[v][h] dz[t][v]   (the [V][K] head read vocabulary-major as it lies; dz is
      // zero from the chunk's last valid column to the end of its 128-column tile)
      gh.A = static_cast<const char*>(q.W_s) + (size_t)v0 * q.K_s * 2; gh.lda = q.K_s; gh.M = q.H_s;
      gh.k_major = 1; gh.k_rows = width;
    } else {
      // head read in place as [H][V]: grad_h_s[t][h] += sum_v W_s[h][v] dz[t][v], both operands K-contiguous
      gh.A = static_cast<const char*>(q.W_s) + (size_t)v0 * 2; gh.lda = q.V; gh.M = q.H_s;
      gh.k_major = 0; gh.k_rows = width;
    }
    {
      ProfileScope ps(KD_PROF_GEMM_GRAD_W, st);
      KD_TRY(kd::launch_gemm(gw, q.n_cu, st));
    }
    {
      ProfileScope ps(KD_PROF_GEMM_GRAD_H, st);
      KD_TRY(kd::launch_gemm(gh, q.n_cu, st));
    }
    first = false;
  }
  KD_TRY(kd::launch_gradh_finish(q, st));
  return KD_OK;
}


kd_status check_buffers(const kd_loss_params* params, const void* h_t, const void* W_t, const void* h_s,
                        const void* W_s, const uint8_t* mask, float* loss, void* workspace,
                        size_t workspace_bytes, bool backward, void* grad_h_s, void* grad_W_s,
                        Problem& q, Layout& L, size_t teacher_base = 0, bool repack_hv = false) {
  kd_status s = check_params(params);
  if (s != KD_OK) return s;
  if (!h_t || !W_t || !h_s || !W_s || !loss || !workspace) return KD_ERR_NULL;
  if (backward && (!grad_h_s || !grad_W_s)) return KD_ERR_NULL;
  if (!aligned16(h_t) || !aligned16(W_t) || !aligned16(h_s) || !aligned16(W_s)) return KD_ERR_ALIGN;
  if (backward && (!aligned16(grad_h_s) || !aligned16(grad_W_s))) return KD_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return KD_ERR_ALIGN;
  plan(params, q, L, backward, teacher_base, repack_hv);
  if (workspace_bytes < L.total) return KD_ERR_WORKSPACE;
  q.h_t = h_t; q.W_t = W_t; q.h_s = h_s; q.W_s = W_s; q.mask = mask;
  q.clock_out = g_clock_out;
  q.loss = loss;
  q.grad_h_s = grad_h_s; q.grad_W_s = grad_W_s;
  carve(q, L, workspace);
  return KD_OK;
}

// The student side of a multi-teacher call (how [H][V] heads are read, which student operands are
// re-packed, where the shared buffers lie) must be the same for every teacher.  Whether [H][V] heads can
// be read in place depends on each teacher's hidden size, so the decision is taken here once: if any
// teacher needs the re-packing path, all of them (and the student head) take it.  Also runs the parameter
// checks of every teacher.
kd_status multi_student_plan(const kd_loss_params* params, int n_teachers, const int64_t* H_t, bool& repack_hv) {
  repack_hv = false;
  for (int k = 0; k < n_teachers; ++k) {
    kd_loss_params pk = *params;
    pk.H_t = H_t[k];
    if (pk.flags & KD_FLAG_TEACHER_FP8) pk.teacher_scale = 1.f;   // checked per teacher by the call itself
    kd_status s = check_params(&pk);
    if (s != KD_OK) return s;
    Problem q{};
    Layout L{};
    plan(&pk, q, L, true);
    if (q.w_hv && !q.w_hv_inplace) repack_hv = true;
  }
  return KD_OK;
}

}  // namespace

extern "C" {

kd_status kd_loss_workspace_size(const kd_loss_params* params, size_t* bytes) {
  if (!bytes) return KD_ERR_NULL;
  kd_status s = check_params(params);
  if (s != KD_OK) return s;
  Problem q{};
  Layout L{};
  plan(params, q, L, true);
  *bytes = L.total;
  return KD_OK;
}

kd_status kd_loss_plan_info(const kd_loss_params* params, int64_t* vocab_chunk, int64_t* n_launches) {
  kd_status s = check_params(params);
  if (s != KD_OK) return s;
  Problem q{};
  Layout L{};
  plan(params, q, L, true);
  const int64_t chunks = (q.V + q.V_c - 1) / q.V_c;
  if (vocab_chunk) *vocab_chunk = q.V_c;
  // compaction, operand copies (as with a mask), statistics + merge, row pass + merge, loss,
  // h_s^T, per chunk the gradient kernel and the two products, grad_h_s conversion
  if (n_launches)
    *n_launches = 1 + (q.prep_ht + q.prep_Wt + q.prep_hs + q.prep_Ws) + 2 + (q.kind >= KD_JSD ? 2 : 0) +
                  (q.kind == KD_AKL ? 2 * kd::kAklSearchPasses : 0) + 1 + 1 + chunks * 3 + 1;
  return KD_OK;
}

kd_status kd_loss_fwd(const kd_loss_params* params, const void* h_t, const void* W_t, const void* h_s,
                      const void* W_s, const uint8_t* mask, float* loss, float* per_token_loss,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  Problem q{};
  Layout L{};
  kd_status s = check_buffers(params, h_t, W_t, h_s, W_s, mask, loss, workspace, workspace_bytes, false,
                              nullptr, nullptr, q, L);
  if (s != KD_OK) return s;
  q.per_token_loss = per_token_loss;
  return run_forward(q, static_cast<hipStream_t>(hip_stream));
}

kd_status kd_loss_fwd_bwd(const kd_loss_params* params, const void* h_t, const void* W_t, const void* h_s,
                          const void* W_s, const uint8_t* mask, float* loss, float* per_token_loss,
                          void* grad_h_s, void* grad_W_s, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  Problem q{};
  Layout L{};
  kd_status s = check_buffers(params, h_t, W_t, h_s, W_s, mask, loss, workspace, workspace_bytes, true,
                              grad_h_s, grad_W_s, q, L);
  if (s != KD_OK) return s;
  q.per_token_loss = per_token_loss;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);

  s = run_forward(q, st);
  if (s != KD_OK) return s;
  return run_backward(&q, 1, st);
}

kd_status kd_loss_fwd_bwd_static(const kd_loss_params* params, const void* h_t, const void* W_t, const void* h_s,
                                 const void* W_s, const uint8_t* mask, float* loss, float* per_token_loss,
                                 void* grad_h_s, void* grad_W_s, void* hip_stream) {
  kd_status s = check_params(params);
  if (s != KD_OK) return s;
  // the plan: the caller's chunk, else the widest one that fits the array
  kd_loss_params pp = *params;
  Problem q{};
  Layout L{};
  plan(&pp, q, L, true);
  if (L.total > KD_STATIC_SCRATCH_BYTES && params->vocab_chunk == 0) {
    for (int vc = 1 << 19; vc >= 256 && L.total > KD_STATIC_SCRATCH_BYTES; vc >>= 1) {
      if (vc >= q.V_c) continue;
      pp.vocab_chunk = vc;
      plan(&pp, q, L, true);
    }
  }
  if (L.total > KD_STATIC_SCRATCH_BYTES) return KD_ERR_TOO_LARGE;
  // every remaining host-side check, with a stand-in for the scratch address (nothing is dereferenced)
  q = Problem{};
  s = check_buffers(&pp, h_t, W_t, h_s, W_s, mask, loss, reinterpret_cast<void*>(uintptr_t{256}),
                    KD_STATIC_SCRATCH_BYTES, true, grad_h_s, grad_W_s, q, L);
  if (s != KD_OK) return s;
  // device address of this GPU's copy of the array, looked up once per device
  static void* ptr_of_device[64];
  static std::atomic<uint64_t> have{0};
  int dev = 0;
  KD_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return KD_ERR_UNSUPPORTED;
  const uint64_t bit = 1ull << dev;
  if (!(have.load(std::memory_order_acquire) & bit)) {
    void* ptr = nullptr;
    KD_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return KD_ERR_LAUNCH;
    ptr_of_device[dev] = ptr;
    have.fetch_or(bit, std::memory_order_release);
  }
  void* const ptr = ptr_of_device[dev];
  q = Problem{};
  s = check_buffers(&pp, h_t, W_t, h_s, W_s, mask, loss, ptr, KD_STATIC_SCRATCH_BYTES, true, grad_h_s, grad_W_s, q, L);
  if (s != KD_OK) return s;
  q.per_token_loss = per_token_loss;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  s = run_forward(q, st);
  if (s != KD_OK) return s;
  return run_backward(&q, 1, st);
}

kd_status kd_loss_workspace_size_multi(const kd_loss_params* params, int n_teachers, const int64_t* H_t,
                                       size_t* bytes) {
  if (!bytes || !params || !H_t) return KD_ERR_NULL;
  if (n_teachers < 1 || n_teachers > 16) return KD_ERR_PARAM;
  bool repack_hv = false;
  kd_status s = multi_student_plan(params, n_teachers, H_t, repack_hv);
  if (s != KD_OK) return s;
  size_t base = 0;                       // teacher blocks lie side by side after the common part
  for (int k = 0; k < n_teachers; ++k) {
    kd_loss_params pk = *params;
    pk.H_t = H_t[k];
    if (pk.flags & KD_FLAG_TEACHER_FP8) pk.teacher_scale = 1.f;   // the size does not depend on the scales
    Problem q{};
    Layout L{};
    plan(&pk, q, L, true, base, repack_hv);
    base = L.total;
  }
  *bytes = base;
  return KD_OK;
}

kd_status kd_loss_fwd_bwd_multi(const kd_loss_params* params, int n_teachers, const void* const* h_t,
                                const void* const* W_t, const int64_t* H_t, const float* weights,
                                const float* teacher_scales,
                                const void* h_s, const void* W_s, const uint8_t* mask, float* loss,
                                float* per_token_loss, void* grad_h_s, void* grad_W_s, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  if (!params || !h_t || !W_t || !H_t || !weights) return KD_ERR_NULL;
  if (n_teachers < 1 || n_teachers > 16) return KD_ERR_PARAM;
  const bool fp8 = (params->flags & KD_FLAG_TEACHER_FP8) != 0;
  if (fp8 && !teacher_scales) return KD_ERR_NULL;
  // all checks for all teachers before the first launch
  Problem q[16];
  Layout L[16];
  bool repack_hv = false;
  {
    kd_status s = multi_student_plan(params, n_teachers, H_t, repack_hv);
    if (s != KD_OK) return s;
  }
  size_t base = 0;
  for (int k = 0; k < n_teachers; ++k) {
    if (!std::isfinite(weights[k])) return KD_ERR_PARAM;
    kd_loss_params pk = *params;
    pk.H_t = H_t[k];
    if (fp8) pk.teacher_scale = teacher_scales[k];
    q[k] = Problem{};
    kd_status s = check_buffers(&pk, h_t[k], W_t[k], h_s, W_s, mask, loss, workspace, workspace_bytes, true,
                                grad_h_s, grad_W_s, q[k], L[k], base, repack_hv);
    if (s != KD_OK) return s;
    // the backward pass and the student operands are laid out by teacher 0's plan: every teacher must agree
    if (L[k].common != L[0].common || L[k].dz != L[0].dz || L[k].h_sT != L[0].h_sT || L[k].gh32 != L[0].gh32 ||
        L[k].prep_h_s != L[0].prep_h_s || L[k].prep_W_s != L[0].prep_W_s || q[k].w_hv_inplace != q[0].w_hv_inplace ||
        q[k].prep_Ws != q[0].prep_Ws || q[k].prep_hs != q[0].prep_hs || q[k].V_c != q[0].V_c)
      return KD_ERR_UNSUPPORTED;
    base = L[k].total;
    q[k].per_token_loss = per_token_loss;
    q[k].out_weight *= weights[k];     // scales this teacher's loss and its share of dL/dz_s
    q[k].accumulate_loss = k > 0;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  for (int k = 0; k < n_teachers; ++k) {
    kd_status s = run_forward(q[k], st, k == 0);
    if (s != KD_OK) return s;
  }
  return run_backward(q, n_teachers, st);
}

kd_status kd_quantize_e4m3(const void* src, int32_t src_dtype, int64_t n, float scale, void* dst,
                           void* hip_stream) {
  if (!src || !dst) return KD_ERR_NULL;
  if (n < 1 || n > ((int64_t)1 << 40)) return KD_ERR_SHAPE;
  if (src_dtype != KD_BF16 && src_dtype != KD_F32) return KD_ERR_PARAM;
  if (!(scale > 0.f && scale < INFINITY)) return KD_ERR_PARAM;
  if (!aligned16(src) || !aligned16(dst)) return KD_ERR_ALIGN;
  KD_TRY(kd::launch_quantize_e4m3(src, src_dtype == KD_F32, n, 1.f / scale, dst, static_cast<hipStream_t>(hip_stream)));
  return KD_OK;
}

kd_status kd_probe_mfma_rate(const void* operands, int iters, float* sink, void* hip_stream) {
  if (!operands || !sink) return KD_ERR_NULL;
  if (iters < 1 || iters > (1 << 24)) return KD_ERR_PARAM;
  if (!aligned16(operands) || !aligned16(sink)) return KD_ERR_ALIGN;
  KD_TRY(kd::launch_mfma_probe(operands, iters, sink, g_clock_out, kd::kNumCU, static_cast<hipStream_t>(hip_stream)));
  return KD_OK;
}

kd_status kd_loss_profile_clock(void* two_int64_device) {
  if (reinterpret_cast<uintptr_t>(two_int64_device) & 7u) return KD_ERR_ALIGN;
  g_clock_out = static_cast<long long*>(two_int64_device);
  return KD_OK;
}

kd_status kd_loss_profile_hook(int which, void** events, int n_events) {
  if (which < 0) {
    g_hook = ProfileHook{};
    return KD_OK;
  }
  if (which > KD_PROF_GEMM_GRAD_H) return KD_ERR_PARAM;
  if (!events || n_events < 2) return KD_ERR_NULL;
  g_hook.which = which;
  g_hook.events = reinterpret_cast<hipEvent_t*>(events);
  g_hook.n_events = n_events;
  g_hook.used = 0;
  return KD_OK;
}

int kd_loss_profile_count(void) { return g_hook.used; }

const char* kd_build_info(void) { return kd::build_info(); }
int kd_build_ablation(void) { return kd::build_ablation(); }

const char* kd_status_string(kd_status status) {
  switch (status) {
    case KD_OK: return "ok";
    case KD_ERR_NULL: return "a required pointer is NULL";
    case KD_ERR_SHAPE: return "T, H_t, H_s or V out of range";
    case KD_ERR_ALIGN: return "pointer not 16-byte aligned or size not a multiple of 8";
    case KD_ERR_PARAM: return "invalid tau, beta, enum value or flag";
    case KD_ERR_WORKSPACE: return "workspace too small";
    case KD_ERR_UNSUPPORTED: return "valid request not implemented by this build";
    case KD_ERR_LAUNCH: return "HIP launch failed";
    case KD_ERR_TOO_LARGE: return "problem needs more scratch memory than the library's static array holds";
  }
  return "unknown status";
}

}  // extern "C"
