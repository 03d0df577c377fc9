// gfx950 kernels of libkdloss and their launchers.
//
// Pass structure (one call of kd_loss_fwd_bwd):
//   stats    : logit tiles (student then teacher) -> online max / sum-exp / cross term per token
//   combine  : merge partial statistics -> log-sum-exps, FKL / RKL row losses
//   rows     : (JSD, TVD, skewed KL, AKL) logit tiles again -> two row sums per token (RowTerm)
//   akl search : (AKL) teacher logit tiles only, a few times -> the teacher probability that splits head from tail
//   finalize : n = sum mask, loss, per-row gradient scale mask/(n tau)
//   per vocabulary chunk:
//     grad   : logit tiles again -> dL/dz_s tile in bf16, stored once as [T,Vc]
//     gemm   : grad_W_s[chunk] = dz^T . h_s     and     grad_h_s += dz . W_s[chunk]
//              (dz in the first and W_s in the second are contracted over their OUTER index:
//              they are read as they lie, through the k-major operand path of tile_loop)
//   gradh_finish : fp32 partial sums -> grad_h_s
// All logarithms inside the kernels are base 2: a = z * log2(e)/tau.
#include "kd_mfma.hpp"
#include "kd_launch.h"

#include <atomic>

// tile configurations (overridable for tuning experiments)
#ifndef KD_LOGIT_CFG
#define KD_LOGIT_CFG 2, 2, 4, 64, 3     // MI, NI, WN, BK, NST: 128 x 256 tile, 8 waves
#endif
#ifndef KD_GEMM_CFG
#define KD_GEMM_CFG 2, 2, 4, 64, 3      // 128 x 256 tile, 8 waves (the second wave per SIMD hides the
                                        // bursts of transposing LDS reads of the k-major operand)
#endif

// Ablation builds for measurements (never the product: RESULTS ARE WRONG when this is not 0).  They take one
// cost out of the logit kernels so that its share of the time and of the shader clock can be read off:
//   1  every workgroup loads the same head rows and the same token rows (all loads hit the L2: no traffic
//      behind it), everything else unchanged
//   2  the statistics epilogue (two exp2 per logit pair, running maxima) is replaced by a plain sum
//   3  both
#ifndef KD_ABLATE
#define KD_ABLATE 0
#endif

#if KD_LOOP_ABLATE
#error "KD_LOOP_ABLATE is for tile_loop_bench.hip only: the library's kernels must compute their products"
#endif

namespace kd {

typedef TileCfg<KD_LOGIT_CFG> LCfg;   // logit tiles: two accumulators per tile
typedef TileCfg<KD_GEMM_CFG> GCfg;    // backward products: one accumulator
constexpr int BK = LCfg::BK;
constexpr int NI = LCfg::NI;
static_assert(LCfg::BM == kTileM && BN == kTileN && GCfg::BM == kGemmTileM, "planner and kernels disagree");
constexpr int BM = LCfg::BM;
constexpr int MI = LCfg::MI;
typedef LCfg::Acc AccTile;
__device__ __forceinline__ int acc_m(int wm, int mt, int r, int lane) { return LCfg::acc_m(wm, mt, r, lane); }
__device__ __forceinline__ int acc_n(int wn, int nt, int lane) { return LCfg::acc_n(wn, nt, lane); }

// ------------------------------------------------------------------------------------------
// work maps
// ------------------------------------------------------------------------------------------

// Workgroups are dealt to the 8 XCDs round-robin by workgroup id.  Renumber so
// that consecutive logical ids sit on one XCD (and share its L2).
__device__ __forceinline__ int xcd_logical_id(int b, int G) {
  const int x = b % 8, q = G / 8, r = G % 8;       // XCD x holds q (+1 if x < r) of the G workgroups
  return x * q + (x < r ? x : r) + b / 8;
}

// Device-side plan, written by rowmap_kernel once the mask has been counted (the host never
// learns how many tokens are valid, so everything that depends on it is decided on the device).
enum { META_N_VALID = 0, META_N_TT = 1, META_N_SPLIT = 2, META_BA = 3, META_BB = 4, META_T_EFF = 5, META_WORDS = 8 };
__device__ __forceinline__ int meta_get(const int* meta, int i) { return uniform(meta[i]); }

// Index q over an (na x nb) grid walked in (ba x bb) blocks, a fastest inside a block.
__device__ __forceinline__ void block_decode(int q, int na, int ba, int bb, int& a, int& b) {
  const int per = ba * bb;
  const int blk = q / per, w = q - blk * per;
  const int nblk_a = na / ba;
  a = (blk % nblk_a) * ba + w % ba;
  b = (blk / nblk_a) * bb + w / ba;
}

struct LogitArgs {
  const bf16_t* W_s; const bf16_t* h_s; const bf16_t* W_t; const bf16_t* h_t;
  int T, V, H_s, H_t;  // H_*: contraction length and row stride of the (re-packed) operands
                       // (heads in [H][V] order: their row stride is V)
  const int* meta;     // device-side plan: valid tokens, token tiles, vocabulary splits, block shape
  int vt0, n_vt;       // vocabulary tiles [vt0, vt0 + n_vt) of BM rows handled by this launch
  int bb;              // grad kernel: block width of the work map along the vocabulary (bb | n_vt).
                       // An XCD's 32 workgroups cover 2 token tiles x 16 vocabulary tiles where the
                       // counts allow: measured 2-3 % faster than 4 x 8 for this kernel (1 x 32 and
                       // 8 x 4 are slower), while the statistics kernels do not care
  float c;             // log2(e) / tau
  float beta;
  float t_scale;       // fp8 teacher: z_t = t_scale * (product of the e4m3 codes); 1 otherwise
  int T_pad;
  float* partials;     // stats: [n_split*4][5][T_pad];  jsd: [n_split*4][2][T_pad]
  const f32x4* rowinfo;// [T_pad]: {lse2_t, lse2_s, mask/(n tau), row term}
  const float* akl;    // AKL only: [AKL_ROWS][T_pad] per-token values (see the AKL_* indices)
  bf16_t* dz;          // [T_pad][ldz]   chunk of dL/dz_s, vocabulary contiguous
  int ldz;
  int dz_accumulate;   // add to dz instead of overwriting it (further teachers of a multi-teacher call)
  long long* clock_out;// measurement aid (may be null): workgroup 0 of the statistics kernel stores the shader
                       // cycles and the 100 MHz ticks its tile loop took
};

// TF8: the teacher operands are e4m3 bytes (one byte per element, 128 elements per k-step).
// WHV: the heads are stored [H][V] (vocabulary contiguous), i.e. k-major for the logit products.
template <bool TF8, bool WHV>
__device__ __forceinline__ WorkItem logit_item(const LogitArgs& a, int vt, int tt) {
  WorkItem it;
  it.B0 = a.h_s + (int64_t)tt * BN * a.H_s;
  if (WHV) {
    it.A0 = a.W_s + vt * BM;
    it.A1 = a.W_t + vt * BM;
    it.B1 = a.h_t + (int64_t)tt * BN * a.H_t;
  } else if (TF8) {
    it.A0 = a.W_s + (int64_t)vt * BM * a.H_s;
    it.A1 = (const bf16_t*)((const char*)a.W_t + (int64_t)vt * BM * a.H_t);
    it.B1 = (const bf16_t*)((const char*)a.h_t + (int64_t)tt * BN * a.H_t);
  } else {
    it.A0 = a.W_s + (int64_t)vt * BM * a.H_s;
    it.A1 = a.W_t + (int64_t)vt * BM * a.H_t;
    it.B1 = a.h_t + (int64_t)tt * BN * a.H_t;
  }
#if KD_ABLATE & 1
  {   // same operand rows for every tile (the tile's coordinates below stay its own)
    it.B0 = a.h_s; it.B1 = a.h_t;
    it.A0 = a.W_s; it.A1 = a.W_t;
  }
#endif
  it.ka_rows = it.kb_rows = 1 << 30;       // hidden sizes are whole k-steps: no k-row is ever missing
  it.a_rows = min(BM, a.V - vt * BM);
  it.b_rows = min(BN, a.T - tt * BN);
  it.nk0 = a.H_s / BK;
  it.nk1 = a.H_t / (TF8 ? 2 * BK : BK);
  it.m0 = vt * BM;
  it.n0 = tt * BN;
  it.aux = 0;
  return it;
}

// One workgroup = one (token tile, vocabulary split); it walks the split's tiles in order.
template <bool TF8, bool WHV>
struct SplitWork {
  const LogitArgs& a;
  int tt, split, lo, cnt;
  __device__ SplitWork(const LogitArgs& a_) : a(a_) {
    const int n_tt = meta_get(a.meta, META_N_TT), n_split = meta_get(a.meta, META_N_SPLIT);
    const int active = n_tt * n_split;               // the grid is sized for the unmasked worst case
    tt = split = lo = cnt = 0;
    if ((int)blockIdx.x >= active) return;
    const int L = xcd_logical_id(blockIdx.x, active);
    block_decode(L, n_tt, meta_get(a.meta, META_BA), meta_get(a.meta, META_BB), tt, split);
    lo = (int)(((int64_t)split * a.n_vt) / n_split);
    const int hi = (int)(((int64_t)(split + 1) * a.n_vt) / n_split);
    cnt = hi - lo;
  }
  __device__ int n_items() const { return cnt; }
  __device__ WorkItem item(int i) const { return logit_item<TF8, WHV>(a, a.vt0 + lo + i, tt); }
};

// The same split of the work, teacher product only (one accumulator): the AKL threshold search.
template <bool WHV>
struct TeacherSplitWork {
  const LogitArgs& a;
  int tt, split, lo, cnt;
  __device__ TeacherSplitWork(const LogitArgs& a_) : a(a_) {
    const int n_tt = meta_get(a.meta, META_N_TT), n_split = meta_get(a.meta, META_N_SPLIT);
    const int active = n_tt * n_split;
    tt = split = lo = cnt = 0;
    if ((int)blockIdx.x >= active) return;
    const int L = xcd_logical_id(blockIdx.x, active);
    block_decode(L, n_tt, meta_get(a.meta, META_BA), meta_get(a.meta, META_BB), tt, split);
    lo = (int)(((int64_t)split * a.n_vt) / n_split);
    const int hi = (int)(((int64_t)(split + 1) * a.n_vt) / n_split);
    cnt = hi - lo;
  }
  __device__ int n_items() const { return cnt; }
  __device__ WorkItem item(int i) const {
    WorkItem it = logit_item<false, WHV>(a, a.vt0 + lo + i, tt);
    it.A0 = it.A1; it.B0 = it.B1;       // phase 0 is the teacher product
    it.nk0 = it.nk1;
    return it;
  }
};

// Persistent workgroups striding over the (token tile x vocabulary tile) grid of a chunk.
template <bool TF8, bool WHV>
struct ChunkWork {
  const LogitArgs& a;
  int L, G, n_tiles, n_tt, ba;
  __device__ ChunkWork(const LogitArgs& a_) : a(a_) {
    G = gridDim.x;
    L = xcd_logical_id(blockIdx.x, G);
    n_tt = meta_get(a.meta, META_N_TT);
    ba = 1;                                          // ba | n_tt, ba * bb <= 32: one block per XCD
    for (int d = 2; d * a.bb <= 32; ++d) if (n_tt % d == 0) ba = d;
    n_tiles = n_tt * a.n_vt;
  }
  __device__ int n_items() const { return L < n_tiles ? (n_tiles - L + G - 1) / G : 0; }
  __device__ WorkItem item(int i) const {
    int tt, vt;
    block_decode(i * G + L, n_tt, ba, a.bb, tt, vt);
    return logit_item<TF8, WHV>(a, a.vt0 + vt, tt);
  }
};

// ------------------------------------------------------------------------------------------
// epilogues of the logit tiles
// ------------------------------------------------------------------------------------------
constexpr float NEG_BIG = -1.0e30f;   // logit given to vocabulary rows beyond V: every exp of it is 0
// Running maxima start here, far below any real scaled logit and far above NEG_BIG * c (the host
// bounds tau so that c > 1e-9): a lane that has seen only masked rows keeps this maximum, so the
// exponent of a masked entry stays hugely negative instead of cancelling to a rounding residual.
constexpr float M_FLOOR = -1.0e20f;
constexpr float LN2 = 0.6931471805599453f;

// Adaptive KL: per-token values kept between its passes, [AKL_ROWS][T_pad] floats.
enum { AKL_FKL = 0, AKL_RKL = 1,   // the token's forward / reverse KL
       AKL_LO = 2, AKL_HI = 3,     // search interval of the head threshold (base-2 teacher log-probability):
                                   // mass{lt >= LO} > mu >= mass{lt >= HI}
       AKL_LTMAX = 4,              // the largest teacher log-probability of the token
       AKL_WR = 5,                 // weight of the reverse KL (the forward KL has 1 - that)
       AKL_ROWS = 6 };
constexpr int AKL_K = kAklThresholds;   // thresholds tried per search pass: each pass narrows the interval 17-fold
constexpr float AKL_TOP_EPS = 1.0e-4f;   // entries this close (base-2 log) to the token's largest one count as "the top entry"

__device__ __forceinline__ float fexp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float flog2(float x) { return __builtin_amdgcn_logf(x); }

// fp8 teacher: the accumulator holds the product of the e4m3 codes; bring it to logits.
__device__ __forceinline__ void scale_teacher(AccTile& accT, float ts) {
  if (ts == 1.f) return;
#pragma unroll
  for (int mt = 0; mt < MI; ++mt)
#pragma unroll
    for (int nt = 0; nt < NI; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) accT[mt][nt][r] *= ts;
}

// Rows of A beyond the vocabulary (last tile only) must not contribute: give them a
// huge negative logit in both accumulators (their exp is 0, their difference is 0).
__device__ __forceinline__ void mask_tail_rows(const WorkItem& it, AccTile& accS, AccTile& accT,
                                               int wm, int lane) {
  if (it.a_rows == BM) return;
#pragma unroll
  for (int mt = 0; mt < MI; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const bool ok = acc_m(wm, mt, r, lane) < it.a_rows;
#pragma unroll
      for (int nt = 0; nt < NI; ++nt) {
        accS[mt][nt][r] = ok ? accS[mt][nt][r] : NEG_BIG;
        accT[mt][nt][r] = ok ? accT[mt][nt][r] : NEG_BIG;
      }
    }
}

// Online log-sum-exp of both models plus the cross term of FKL / RKL.
//   FKL: X = sum_v 2^(a_t - m_t) (z_t - z_s)      RKL: X = sum_v 2^(a_s - m_s) (z_s - z_t)
template <int KIND>
struct StatsEpi {
  static constexpr int NV = KIND == 6 ? 6 : 5;     // values per token and part (AKL keeps both cross terms)
  float m_t[NI], S_t[NI], m_s[NI], S_s[NI], X[NI], X2[NI];
  float c, ts;
  int wm, wn, lane;
  __device__ StatsEpi(float c_, float ts_) : c(c_), ts(ts_) {
    lane = threadIdx.x & 63;
    wm = (threadIdx.x >> 6) & 1;
    wn = threadIdx.x >> 7;
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      m_t[nt] = M_FLOOR; m_s[nt] = M_FLOOR; S_t[nt] = 0.f; S_s[nt] = 0.f; X[nt] = 0.f; X2[nt] = 0.f;
    }
  }
  __device__ void begin_item(const WorkItem&) {}
  __device__ void end_item(const WorkItem& it, AccTile& accS, AccTile& accT) {
#if KD_ABLATE & 2
#pragma unroll
    for (int nt = 0; nt < NI; ++nt)
#pragma unroll
      for (int mt = 0; mt < MI; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) { S_t[nt] += accT[mt][nt][r]; S_s[nt] += accS[mt][nt][r]; }
    return;
#endif
    scale_teacher(accT, ts);
    mask_tail_rows(it, accS, accT, wm, lane);
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      float tmax = NEG_BIG, smax = NEG_BIG;
#pragma unroll
      for (int mt = 0; mt < MI; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          tmax = fmaxf(tmax, accT[mt][nt][r]);
          smax = fmaxf(smax, accS[mt][nt][r]);
        }
      const float nmt = fmaxf(m_t[nt], tmax * c);
      const float nms = fmaxf(m_s[nt], smax * c);
      const float sct = fexp2(m_t[nt] - nmt);
      const float scs = fexp2(m_s[nt] - nms);
      float st = S_t[nt] * sct, ss = S_s[nt] * scs;
      float x = X[nt] * ((KIND == 0 || KIND == 6) ? sct : scs);
      float x2 = X2[nt] * scs;
#pragma unroll
      for (int mt = 0; mt < MI; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float zt = accT[mt][nt][r], zs = accS[mt][nt][r];
          const float et = fexp2(fmaf(zt, c, -nmt));
          const float es = fexp2(fmaf(zs, c, -nms));
          st += et;
          ss += es;
          if (KIND == 0 || KIND == 6) x = fmaf(et, zt - zs, x);
          if (KIND == 1) x = fmaf(es, zs - zt, x);
          if (KIND == 6) x2 = fmaf(es, zs - zt, x2);
        }
      m_t[nt] = nmt; m_s[nt] = nms; S_t[nt] = st; S_s[nt] = ss; X[nt] = x; X2[nt] = x2;
    }
  }
  __device__ void write(const LogitArgs& a, int tt, int split) const {
    const int part = split * 4 + wm * 2 + (lane >> 5);
    float* p = a.partials + (int64_t)part * NV * a.T_pad;
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      const int t = tt * BN + acc_n(wn, nt, lane);
      p[0 * a.T_pad + t] = m_t[nt];
      p[1 * a.T_pad + t] = S_t[nt];
      p[2 * a.T_pad + t] = m_s[nt];
      p[3 * a.T_pad + t] = S_s[nt];
      p[4 * a.T_pad + t] = X[nt];
      if (KIND == 6) p[5 * a.T_pad + t] = X2[nt];
    }
  }
};

// Divergences whose row value needs both log-sum-exps first (JSD, TVD, skewed KL) share one
// scheme.  With D a function of the student probabilities and c = dD/dp_s, the gradient through the
// softmax is  dD/dz_s = p_s (c - R) / tau,  R = sum_v p_s c.  A row pass over the logit tiles
// accumulates two sums (a1, a2) per token, from which the row loss and R follow; the gradient pass
// evaluates c element by element.  lt, ls are base-2 log-probabilities, w is beta (JSD) or the skew
// weight alpha.
//   JSD       M = w p_t + (1-w) p_s    a1 = sum p_t (lt - lm)   a2 = sum p_s (ls - lm)
//             loss = ln2 (w a1 + (1-w) a2)     c = (1-w) ln2 (ls - lm)          R = (1-w) ln2 a2
//   TVD       d = p_s - p_t            a1 = sum |d|             a2 = sum p_s sign(d)
//             loss = a1 / 2                    c = sign(d) / 2                  R = a2 / 2
//   skew FKL  M = w p_t + (1-w) p_s    a1 = sum p_t (lt - lm)   a2 = sum p_s p_t / M
//             loss = ln2 a1                    c = -(1-w) p_t / M               R = -(1-w) a2
//   skew RKL  M = (1-w) p_t + w p_s    a1 = sum p_s (ls - lm)   a2 = sum p_s c
//             loss = ln2 a1                    c = ln2 (ls - lm) + 1 - w p_s / M   R = a2
template <int KIND>
struct RowTerm {
  // c for one element; also adds the element's contribution to (a1, a2) when ACC is set
  template <bool ACC>
  static __device__ __forceinline__ float eval(float lt, float ls, float w, float& a1, float& a2) {
    const float pt = fexp2(lt), ps = fexp2(ls);
    if (KIND == 3) {
      const float d = ps - pt;
      const float sg = (d > 0.f ? 1.f : 0.f) - (d < 0.f ? 1.f : 0.f);
      if (ACC) { a1 += fabsf(d); a2 = fmaf(ps, sg, a2); }
      return 0.5f * sg;
    }
    const float wt = (KIND == 5) ? 1.f - w : w;          // weight of p_t in the mixture
    // log M is taken relative to the larger of the two probabilities: with d = ls - lt and q = 2^-|d| <= 1,
    //   p_t >= p_s:  M / p_t = wt + (1-wt) q      p_t < p_s:  M / p_s = wt q + (1-wt)
    // so the logarithm's argument lies in [min(wt, 1-wt), 1]: no large logarithms are subtracted from one
    // another (the hardware log of M itself, of size log2 V, is half an ulp short on average, which
    // showed as a bias of 3e-7 in small losses), and nothing degenerates where p_t and p_s underflow.
    const float d = ls - lt;
    const bool t_big = d <= 0.f;
    const float q = fexp2(t_big ? d : -d);
    const float mix = t_big ? fmaf(1.f - wt, q, wt) : fmaf(wt, q, 1.f - wt);
    const float lmix = flog2(mix);
    const float lt_lm = t_big ? -lmix : -d - lmix;       // lt - lm
    const float ls_lm = t_big ? d - lmix : -lmix;        // ls - lm
    const float inv = __builtin_amdgcn_rcpf(mix);
    if (KIND == 2) {
      if (ACC) { a1 = fmaf(pt, lt_lm, a1); a2 = fmaf(ps, ls_lm, a2); }
      return (1.f - w) * LN2 * ls_lm;
    }
    if (KIND == 4) {
      const float r = t_big ? inv : q * inv;             // p_t / M
      if (ACC) { a1 = fmaf(pt, lt_lm, a1); a2 = fmaf(ps, r, a2); }
      return -(1.f - w) * r;
    }
    const float r = t_big ? q * inv : inv;               // p_s / M
    const float cc = fmaf(LN2, ls_lm, 1.f - w * r);
    if (ACC) { a1 = fmaf(ps, ls_lm, a1); a2 = fmaf(ps, cc, a2); }
    return cc;
  }
};

// AKL (KIND 6) uses the same pass for its gaps:  a1 = sum over the head of |p_t - p_s|,  a2 = the same over
// the tail, the head being the entries whose teacher log-probability reaches the token's threshold.
template <int KIND>
struct RowsEpi {
  float A1[NI], A2[NI], Lt[NI], Ls[NI], Thr[NI];
  float c, w, ts;
  int wm, wn, lane;
  __device__ RowsEpi(const LogitArgs& a, int tt) : c(a.c), w(a.beta), ts(a.t_scale) {
    lane = threadIdx.x & 63;
    wm = (threadIdx.x >> 6) & 1;
    wn = threadIdx.x >> 7;
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      const int t = tt * BN + acc_n(wn, nt, lane);
      const f32x4 ri = a.rowinfo[t];
      Lt[nt] = ri[0]; Ls[nt] = ri[1]; A1[nt] = 0.f; A2[nt] = 0.f;
      Thr[nt] = 0.f;
      if (KIND == 6)    // the top entry is head whatever its mass
        Thr[nt] = fminf(a.akl[AKL_HI * a.T_pad + t], a.akl[AKL_LTMAX * a.T_pad + t] - AKL_TOP_EPS);
    }
  }
  __device__ void begin_item(const WorkItem&) {}
  __device__ void end_item(const WorkItem& it, AccTile& accS, AccTile& accT) {
    scale_teacher(accT, ts);
    mask_tail_rows(it, accS, accT, wm, lane);
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      float a1 = A1[nt], a2 = A2[nt];
#pragma unroll
      for (int mt = 0; mt < MI; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float lt = fmaf(accT[mt][nt][r], c, -Lt[nt]);
          const float ls = fmaf(accS[mt][nt][r], c, -Ls[nt]);
          if constexpr (KIND == 6) {
            const float gap = fabsf(fexp2(lt) - fexp2(ls));
            const bool head = lt >= Thr[nt];
            a1 += head ? gap : 0.f;
            a2 += head ? 0.f : gap;
          } else {
            (void)RowTerm<KIND>::template eval<true>(lt, ls, w, a1, a2);
          }
        }
      A1[nt] = a1; A2[nt] = a2;
    }
  }
  __device__ void write(const LogitArgs& a, int tt, int split) const {
    const int part = split * 4 + wm * 2 + (lane >> 5);
    float* p = a.partials + (int64_t)part * 2 * a.T_pad;
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      const int t = tt * BN + acc_n(wn, nt, lane);
      p[0 * a.T_pad + t] = A1[nt];
      p[1 * a.T_pad + t] = A2[nt];
    }
  }
};

// dL/dz_s tile.  rowinfo = {lse2_t, lse2_s, s = mask/(n tau), R}
//   FKL: dz = s (p_s - p_t)
//   RKL: dz = s p_s (ln2 (l_s - l_t) - R),   R = row loss
//   JSD, TVD, skewed KL: dz = s p_s (c - R)  (RowTerm above)
//   AKL: dz = s (w_f (p_s - p_t) + w_r p_s (ln2 (l_s - l_t) - RKL)) = s (p_s (w_r ln2 (l_s - l_t) + R) - w_f p_t),
//        R = w_f - w_r RKL, the weights being constants for the gradient
template <int KIND>
struct GradEpi {
  const LogitArgs& a;
  float Lt[NI], Ls[NI], sc[NI], R[NI], Wr[NI];
  int wm, wn, lane;
  __device__ GradEpi(const LogitArgs& a_) : a(a_) {
    lane = threadIdx.x & 63;
    wm = (threadIdx.x >> 6) & 1;
    wn = threadIdx.x >> 7;
  }
  __device__ void begin_item(const WorkItem& it) {
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      const f32x4 ri = a.rowinfo[it.n0 + acc_n(wn, nt, lane)];
      Lt[nt] = ri[0]; Ls[nt] = ri[1]; sc[nt] = ri[2]; R[nt] = ri[3];
      Wr[nt] = 0.f;
      if (KIND == 6) Wr[nt] = a.akl[AKL_WR * a.T_pad + it.n0 + acc_n(wn, nt, lane)];
    }
  }
  __device__ void end_item(const WorkItem& it, AccTile& accS, AccTile& accT) {
    scale_teacher(accT, a.t_scale);
    const float c = a.c, w = a.beta;
    const int mloc0 = it.m0 - a.vt0 * BM;      // vocabulary offset inside the chunk
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      const int n = it.n0 + acc_n(wn, nt, lane);
      const float s = sc[nt];
#pragma unroll
      for (int mt = 0; mt < MI; ++mt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int m = acc_m(wm, mt, 4 * q, lane);
          const bool ok = m < it.a_rows;
          bf16x4* const dst = (bf16x4*)(a.dz + (int64_t)n * a.ldz + mloc0 + m);
          bf16x4 o;
          if (a.dz_accumulate) o = *dst;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float lt = fmaf(accT[mt][nt][4 * q + i], c, -Lt[nt]);
            const float ls = fmaf(accS[mt][nt][4 * q + i], c, -Ls[nt]);
            const float ps = fexp2(ls);
            float g;
            if (KIND == 0) {
              g = ps - fexp2(lt);
            } else if (KIND == 1) {
              g = ps * fmaf(LN2, ls - lt, -R[nt]);
            } else if (KIND == 6) {
              g = fmaf(ps, fmaf(Wr[nt] * LN2, ls - lt, R[nt]), -(1.f - Wr[nt]) * fexp2(lt));
            } else {
              float u1, u2;
              g = ps * (RowTerm<KIND>::template eval<false>(lt, ls, w, u1, u2) - R[nt]);
            }
            const float d = ok ? s * g : 0.f;
            o[i] = (bf16_t)(a.dz_accumulate ? (float)o[i] + d : d);
          }
          *dst = o;
        }
    }
  }
};

// ------------------------------------------------------------------------------------------
// logit kernels
// ------------------------------------------------------------------------------------------
#define KD_LOGIT_KERNEL __global__ __launch_bounds__(LCfg::NT)
#define KD_GEMM_KERNEL __global__ __launch_bounds__(GCfg::NT)

template <int KIND, bool TF8, bool WHV>
KD_LOGIT_KERNEL void stats_kernel(const LogitArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  SplitWork<TF8, WHV> work(a);
  StatsEpi<KIND> epi(a.c, a.t_scale);
  long long c0 = 0, r0 = 0;
  if (a.clock_out) { c0 = clock64(); r0 = wall_clock64(); }     // measurement aid, off unless asked for
  tile_loop<2, LCfg, WHV ? 1 : 0, TF8>(work, epi, WHV ? a.V : a.H_s, WHV ? a.V : a.H_t, a.H_s, a.H_t, smem);
  if (a.clock_out && blockIdx.x == 0 && threadIdx.x == 0) {
    a.clock_out[0] = clock64() - c0;
    a.clock_out[1] = wall_clock64() - r0;
  }
  if (work.cnt > 0) epi.write(a, work.tt, work.split);
}

template <int KIND, bool TF8, bool WHV>
KD_LOGIT_KERNEL void rows_kernel(const LogitArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  SplitWork<TF8, WHV> work(a);
  RowsEpi<KIND> epi(a, work.tt);
  tile_loop<2, LCfg, WHV ? 1 : 0, TF8>(work, epi, WHV ? a.V : a.H_s, WHV ? a.V : a.H_t, a.H_s, a.H_t, smem);
  if (work.cnt > 0) epi.write(a, work.tt, work.split);
}

// AKL threshold search, one pass: for AKL_K thresholds spread evenly inside the token's current interval
// (LO, HI), the teacher mass of the entries at or above each threshold.
struct SearchEpi {
  float Lt[NI], th0[NI], step[NI];
  float mass[NI][AKL_K];
  float c;
  int wm, wn, lane;
  __device__ SearchEpi(const LogitArgs& a, int tt) : c(a.c) {
    lane = threadIdx.x & 63;
    wm = (threadIdx.x >> 6) & 1;
    wn = threadIdx.x >> 7;
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      const int t = tt * BN + acc_n(wn, nt, lane);
      Lt[nt] = a.rowinfo[t][0];
      const float lo = a.akl[AKL_LO * a.T_pad + t], hi = a.akl[AKL_HI * a.T_pad + t];
      step[nt] = (hi - lo) * (1.f / (AKL_K + 1));
      th0[nt] = lo + step[nt];
#pragma unroll
      for (int k = 0; k < AKL_K; ++k) mass[nt][k] = 0.f;
    }
  }
  __device__ void begin_item(const WorkItem&) {}
  __device__ void end_item(const WorkItem& it, AccTile& accT, AccTile&) {
#pragma unroll
    for (int nt = 0; nt < NI; ++nt)
#pragma unroll
      for (int mt = 0; mt < MI; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const bool ok = acc_m(wm, mt, r, lane) < it.a_rows;      // rows beyond the vocabulary hold nothing
          const float lt = ok ? fmaf(accT[mt][nt][r], c, -Lt[nt]) : NEG_BIG;
          const float p = fexp2(lt);
#pragma unroll
          for (int k = 0; k < AKL_K; ++k) mass[nt][k] += (lt >= fmaf((float)k, step[nt], th0[nt])) ? p : 0.f;
        }
  }
  __device__ void write(const LogitArgs& a, int tt, int split) const {
    const int part = split * 4 + wm * 2 + (lane >> 5);
    float* p = a.partials + (int64_t)part * AKL_K * a.T_pad;
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      const int t = tt * BN + acc_n(wn, nt, lane);
#pragma unroll
      for (int k = 0; k < AKL_K; ++k) p[k * a.T_pad + t] = mass[nt][k];
    }
  }
};

template <bool WHV>
KD_LOGIT_KERNEL void akl_search_kernel(const LogitArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  TeacherSplitWork<WHV> work(a);
  SearchEpi epi(a, work.tt);
  tile_loop<1, LCfg, WHV ? 1 : 0, false>(work, epi, WHV ? a.V : a.H_t, WHV ? a.V : a.H_t, a.H_t, a.H_t, smem);
  if (work.cnt > 0) epi.write(a, work.tt, work.split);
}

template <int KIND, bool TF8, bool WHV>
KD_LOGIT_KERNEL void grad_kernel(const LogitArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  ChunkWork<TF8, WHV> work(a);
  GradEpi<KIND> epi(a);
  tile_loop<2, LCfg, WHV ? 1 : 0, TF8>(work, epi, WHV ? a.V : a.H_s, WHV ? a.V : a.H_t, a.H_s, a.H_t, smem);
}

// ------------------------------------------------------------------------------------------
// plain products for the backward pass:  out[n][m] (+)= sum_k A[m][k] B[n][k]
// ------------------------------------------------------------------------------------------
struct GemmArgs {
  const bf16_t* A; const bf16_t* B;
  int lda, ldb;
  int M, N;            // valid rows of A / of B
  int K;               // contraction length, a multiple of 64
  int n_ksplit;        // split-K parts; part s writes out + s * out_split_stride
  int ksteps;          // k-steps per part
  void* out; int64_t ldo; int64_t out_split_stride;   // in elements
  int out_f32;         // 1: float, 0: bf16
  int accumulate;      // 1: out += D
  int n_mt, n_nt;
  int ba, bb;          // block shape of the work map (ba | n_mt, bb | n_nt)
  const int* meta;     // device-side plan (may be null when neither flag below is set)
  int n_from_meta;     // N = number of valid tokens (rows of the compacted B operand)
  int k_from_meta;     // K = valid tokens rounded up to whole token tiles
  int k_rows;          // k-major operand: k-rows that exist in memory (rows beyond are clamped)
};

// KM: which operand is stored k-major (0: none, 1: A[k][m], 2: B[k][n]); the others are K-contiguous.
template <int KM>
struct GemmWork {
  const GemmArgs& a;
  int L, G, n_tiles, N, K, n_nt, bb;
  __device__ GemmWork(const GemmArgs& a_) : a(a_) {
    G = gridDim.x;
    L = xcd_logical_id(blockIdx.x, G);
    N = a.N; K = a.K; n_nt = a.n_nt; bb = a.bb;
    if (a.n_from_meta) {
      N = meta_get(a.meta, META_N_VALID);
      n_nt = (N + BN - 1) / BN;
      bb = n_nt % 4 == 0 ? 4 : (n_nt % 3 == 0 ? 3 : (n_nt % 2 == 0 ? 2 : 1));
    }
    if (a.k_from_meta) K = meta_get(a.meta, META_T_EFF);
    n_tiles = a.n_mt * n_nt * a.n_ksplit;
  }
  __device__ int n_items() const { return L < n_tiles ? (n_tiles - L + G - 1) / G : 0; }
  __device__ WorkItem item(int i) const {
    const int q = i * G + L;
    const int per_split = a.n_mt * n_nt;
    const int ks = q / per_split;
    int mt, nt;
    block_decode(q - ks * per_split, a.n_mt, a.ba, bb, mt, nt);
    const int k0 = ks * a.ksteps * GCfg::BK;
    WorkItem it;
    it.A0 = it.A1 = (KM & 1) ? a.A + (int64_t)k0 * a.lda + mt * GCfg::BM : a.A + (int64_t)mt * GCfg::BM * a.lda + k0;
    it.B0 = it.B1 = (KM & 2) ? a.B + (int64_t)k0 * a.ldb + nt * BN : a.B + (int64_t)nt * BN * a.ldb + k0;
    it.ka_rows = it.kb_rows = a.k_rows - k0;
    it.a_rows = min(GCfg::BM, a.M - mt * GCfg::BM);
    it.b_rows = min(BN, N - nt * BN);
    it.nk0 = it.nk1 = a.k_from_meta ? K / GCfg::BK : min(a.ksteps, K / GCfg::BK - ks * a.ksteps);
    it.m0 = mt * GCfg::BM;
    it.n0 = nt * BN;
    it.aux = ks;
    return it;
  }
};

struct StoreEpi {
  const GemmArgs& a;
  int wm, wn, lane;
  __device__ StoreEpi(const GemmArgs& a_) : a(a_) {
    lane = threadIdx.x & 63;
    wm = (threadIdx.x >> 6) & 1;
    wn = threadIdx.x >> 7;
  }
  __device__ void begin_item(const WorkItem&) {}
  __device__ void end_item(const WorkItem& it, GCfg::Acc& acc, GCfg::Acc&) {
#pragma unroll
    for (int nt = 0; nt < GCfg::NI; ++nt) {
      const int nl = GCfg::acc_n(wn, nt, lane);
      if (nl >= it.b_rows) continue;
      const int64_t row = (int64_t)(it.n0 + nl) * a.ldo + (int64_t)it.aux * a.out_split_stride;
#pragma unroll
      for (int mt = 0; mt < GCfg::MI; ++mt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int ml = GCfg::acc_m(wm, mt, 4 * q, lane);
          if (ml >= it.a_rows) continue;
          f32x4 v = {acc[mt][nt][4 * q], acc[mt][nt][4 * q + 1], acc[mt][nt][4 * q + 2], acc[mt][nt][4 * q + 3]};
          if (a.out_f32) {
            f32x4* p = (f32x4*)((float*)a.out + row + it.m0 + ml);
            if (a.accumulate) v += *p;
            *p = v;
          } else {
            bf16x4* p = (bf16x4*)((bf16_t*)a.out + row + it.m0 + ml);
            if (a.accumulate) {
              const bf16x4 old = *p;
#pragma unroll
              for (int i = 0; i < 4; ++i) v[i] += (float)old[i];
            }
            bf16x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = (bf16_t)v[i];
            *p = o;
          }
        }
    }
  }
};

template <int KM>
KD_GEMM_KERNEL void gemm_kernel(const GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  GemmWork<KM> work(a);
  StoreEpi epi(a);
  tile_loop<1, GCfg, KM>(work, epi, a.lda, a.lda, a.ldb, a.ldb, smem);
}

// ------------------------------------------------------------------------------------------
// small kernels
// ------------------------------------------------------------------------------------------

// One workgroup.  Compacts the valid tokens (mask != 0; all of them when mask is null) to the front:
// rowmap[j] = index of the j-th valid token, inv[t] = its compacted index or -1, and writes the
// device-side plan that depends on how many there are.  Every later kernel works on the compacted
// token axis, so masked tokens cost nothing.
__global__ void rowmap_kernel(const uint8_t* mask, int T, int T_pad, int n_split_max, int n_cu,
                              int* rowmap, int* inv, int* meta) {
  __shared__ int s_scan[1024];
  __shared__ int s_running;
  const int tid = threadIdx.x;
  if (tid == 0) s_running = 0;
  __syncthreads();
  for (int base = 0; base < T; base += 1024) {
    const int t = base + tid;
    const int on = (t < T && (mask == nullptr || mask[t] != 0)) ? 1 : 0;
    s_scan[tid] = on;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {          // inclusive scan
      const int v = tid >= d ? s_scan[tid - d] : 0;
      __syncthreads();
      s_scan[tid] += v;
      __syncthreads();
    }
    const int run = s_running;
    if (t < T) {
      const int j = run + s_scan[tid] - on;
      if (on) rowmap[j] = t;
      inv[t] = on ? j : -1;
    }
    __syncthreads();
    if (tid == 1023) s_running = run + s_scan[1023];
    __syncthreads();
  }
  const int n = s_running;
  const int last = n > 0 ? rowmap[n - 1] : 0;
  __syncthreads();
  for (int j = n + tid; j < T_pad; j += 1024) rowmap[j] = last;   // never dereferenced for results
  if (tid == 0) {
    int n_tt = (n + BN - 1) / BN;
    if (n_tt < 1) n_tt = 1;
    int n_split = n_cu / n_tt;                     // as many splits as keep one workgroup per CU
    if (n_split < 8) n_split = 8;
    if (n_split > n_split_max) n_split = n_split_max;
    int ba = 1, bb = 1;
    for (int d = 2; d <= 4; ++d) if (n_tt % d == 0) ba = d;
    for (int d = 2; d <= 8; ++d) if (n_split % d == 0) bb = d;
    meta[META_N_VALID] = n;
    meta[META_N_TT] = n_tt;
    meta[META_N_SPLIT] = n_split;
    meta[META_BA] = ba;
    meta[META_BB] = bb;
    meta[META_T_EFF] = n_tt * BN;
  }
}

// Merge the partial statistics of one (compacted) token; write log-sum-exps and, for FKL / RKL, the
// row loss.
__global__ void combine_kernel(const float* partials, const int* meta, int T_pad, int kind, float c,
                               f32x4* rowinfo, float* row_loss, float* akl) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T_pad) return;
  const int n_valid = meta[META_N_VALID], n_parts = 4 * meta[META_N_SPLIT];
  const int nv = kind == 6 ? 6 : 5;
  if (t >= n_valid) {   // padding rows: probabilities evaluate to 0, gradient scale 0
    rowinfo[t] = f32x4{1.0e30f, 1.0e30f, 0.f, 0.f};
    row_loss[t] = 0.f;
    if (kind == 6)
      for (int i = 0; i < AKL_ROWS; ++i) akl[i * T_pad + t] = 0.f;
    return;
  }
  float Mt = M_FLOOR, Ms = M_FLOOR;
  for (int p = 0; p < n_parts; ++p) {
    const float* q = partials + (int64_t)p * nv * T_pad + t;
    Mt = fmaxf(Mt, q[0]);
    Ms = fmaxf(Ms, q[2 * T_pad]);
  }
  float St = 0.f, Ss = 0.f, X = 0.f, X2 = 0.f;
  for (int p = 0; p < n_parts; ++p) {
    const float* q = partials + (int64_t)p * nv * T_pad + t;
    const float wt = fexp2(q[0] - Mt), ws = fexp2(q[2 * T_pad] - Ms);
    St = fmaf(q[1 * T_pad], wt, St);
    Ss = fmaf(q[3 * T_pad], ws, Ss);
    X = fmaf(q[4 * T_pad], (kind == 0 || kind == 6) ? wt : ws, X);
    if (kind == 6) X2 = fmaf(q[5 * T_pad], ws, X2);
  }
  // The row loss is a difference of quantities of size log2 V, far larger than itself when the two
  // distributions are close: this last step is done in double (one thread per token, so it costs nothing).
  const double Ltd = (double)Mt + log2((double)St), Lsd = (double)Ms + log2((double)Ss);
  double lossd = 0.0;
  if (kind == 0) lossd = (double)c * X / St - Ltd + Lsd;   // kinds >= 2: filled in by combine_rows_kernel
  if (kind == 1) lossd = (double)c * X / Ss - Lsd + Ltd;
  const float loss = (float)(0.6931471805599453 * lossd);
  rowinfo[t] = f32x4{(float)Ltd, (float)Lsd, 0.f, loss};
  row_loss[t] = loss;
  if (kind == 6) {      // both KLs, and the first search interval: from 2^-40 of the largest teacher probability
    const double fkl = (double)c * X / St - Ltd + Lsd, rkl = (double)c * X2 / Ss - Lsd + Ltd;
    const float ltmax = (float)((double)Mt - Ltd);
    akl[AKL_FKL * T_pad + t] = (float)(0.6931471805599453 * fkl);
    akl[AKL_RKL * T_pad + t] = (float)(0.6931471805599453 * rkl);
    akl[AKL_LO * T_pad + t] = ltmax - 40.f;
    akl[AKL_HI * T_pad + t] = ltmax + 1.0e-3f;         // above every entry: mass 0
    akl[AKL_LTMAX * T_pad + t] = ltmax;
    akl[AKL_WR * T_pad + t] = 0.f;
  }
}

// AKL: merge one search pass.  mass_k = teacher mass at or above threshold k (decreasing in k); the new
// interval is the pair of neighbouring thresholds between which the mass drops to mu or below.
__global__ void akl_search_combine_kernel(const float* partials, const int* meta, int T_pad, float mu, float* akl) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int n_valid = meta[META_N_VALID], n_parts = 4 * meta[META_N_SPLIT];
  if (t >= n_valid) return;
  const float lo = akl[AKL_LO * T_pad + t], hi = akl[AKL_HI * T_pad + t];
  const float step = (hi - lo) * (1.f / (AKL_K + 1)), th0 = lo + step;
  float new_lo = lo, new_hi = hi;
  bool found = false;
  for (int k = 0; k < AKL_K; ++k) {
    float m = 0.f;
    for (int p = 0; p < n_parts; ++p) m += partials[((int64_t)p * AKL_K + k) * T_pad + t];
    const float th = fmaf((float)k, step, th0);     // the very expression the search kernel compares with
    if (!found) {
      if (m <= mu) { new_hi = th; found = true; }
      else new_lo = th;
    }
  }
  akl[AKL_LO * T_pad + t] = new_lo;
  akl[AKL_HI * T_pad + t] = new_hi;
}

// AKL: gaps -> weights, row loss and the row term of the gradient (see GradEpi).
__global__ void akl_weights_kernel(const float* partials, const int* meta, int T_pad, f32x4* rowinfo,
                                   float* row_loss, float* akl) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int n_valid = meta[META_N_VALID], n_parts = 4 * meta[META_N_SPLIT];
  if (t >= n_valid) return;
  float gh = 0.f, gt = 0.f;
  for (int p = 0; p < n_parts; ++p) {
    const float* q = partials + (int64_t)p * 2 * T_pad + t;
    gh += q[0];
    gt += q[T_pad];
  }
  const float tot = gh + gt;
  const float wr = tot > 0.f ? gt / tot : 0.5f, wf = 1.f - wr;
  const float fkl = akl[AKL_FKL * T_pad + t], rkl = akl[AKL_RKL * T_pad + t];
  f32x4 ri = rowinfo[t];
  ri[3] = wf - wr * rkl;
  rowinfo[t] = ri;
  row_loss[t] = wf * fkl + wr * rkl;
  akl[AKL_WR * T_pad + t] = wr;
}

// JSD / TVD / skewed KL: merge the row sums into the row loss and R (see RowTerm).
__global__ void combine_rows_kernel(const float* partials, const int* meta, int T_pad, int kind, float w,
                                    f32x4* rowinfo, float* row_loss) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int n_valid = meta[META_N_VALID], n_parts = 4 * meta[META_N_SPLIT];
  if (t >= n_valid) return;
  float A1 = 0.f, A2 = 0.f;
  for (int p = 0; p < n_parts; ++p) {
    const float* q = partials + (int64_t)p * 2 * T_pad + t;
    A1 += q[0];
    A2 += q[T_pad];
  }
  float loss, R;
  if (kind == 2) { loss = LN2 * (w * A1 + (1.f - w) * A2); R = (1.f - w) * LN2 * A2; }
  else if (kind == 3) { loss = 0.5f * A1; R = 0.5f * A2; }
  else if (kind == 4) { loss = LN2 * A1; R = -(1.f - w) * A2; }
  else { loss = LN2 * A1; R = A2; }
  f32x4 ri = rowinfo[t];
  ri[3] = R;
  rowinfo[t] = ri;
  row_loss[t] = loss;
}

// One workgroup: loss = sum of the valid rows' losses / n (fixed-order fp64 tree), per-row gradient
// scale 1 / (n tau), and the caller's per-token losses (0 for masked tokens).
// `weight` scales what leaves the call (teacher weight, optional tau^2); with `accumulate` the loss
// outputs are added to (further teachers of a multi-teacher call).
__global__ void finalize_kernel(const int* meta, const int* inv, const float* row_loss, int T, float tau,
                                float weight, int accumulate, f32x4* rowinfo, float* loss_out,
                                float* per_token_out) {
  __shared__ double s_sum[1024];
  const int tid = threadIdx.x;
  const int n = meta[META_N_VALID];
  double acc = 0.0;
  for (int j = tid; j < n; j += 1024) acc += (double)row_loss[j];
  s_sum[tid] = acc;
  __syncthreads();
  for (int s = 512; s > 0; s >>= 1) {
    if (tid < s) s_sum[tid] += s_sum[tid + s];
    __syncthreads();
  }
  if (tid == 0) {
    const float l = n > 0 ? weight * (float)(s_sum[0] / (double)n) : 0.f;
    *loss_out = accumulate ? *loss_out + l : l;
  }
  const float scale = n > 0 ? weight / ((float)n * tau) : 0.f;
  for (int j = tid; j < n; j += 1024) rowinfo[j][2] = scale;
  if (per_token_out)
    for (int t = tid; t < T; t += 1024) {
      const int j = inv[t];
      const float l = j >= 0 ? weight * row_loss[j] : 0.f;
      per_token_out[t] = accumulate ? per_token_out[t] + l : l;
    }
}

// dst[c][r] = src[r][c] for r < R, zero for R <= r < R_pad;  c < C.  64 x 64 tiles through LDS.
template <class E>
__global__ void transpose_kernel(const E* src, int64_t ld_src, int R, int C, E* dst, int64_t ld_dst, int R_pad) {
  __shared__ E tile[64][66];
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    tile[i][tx] = (r < R && c < C) ? src[(int64_t)r * ld_src + c] : E(0);
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (c < C && r < R_pad) dst[(int64_t)c * ld_dst + r] = tile[tx][i];
  }
}

// Re-pack one operand as bf16 [R][K]: plain copy (bf16 source) or the high / low bf16 parts of an
// fp32 source laid side by side along K, zero-padded up to K.
//   split_mode 1 (heads):         [hi | hi | lo]
//   split_mode 2 (hidden states): [hi | lo | hi]
// so that sum_k A'[m][k] B'[n][k] = hi.hi + hi.lo + lo.hi.
// With a row map, destination row j takes source row rowmap[j] for j < n_valid and is zero beyond:
// the compacted copy of the hidden states.
// With src_transposed the source is stored [H][R] (a head kept as [H][V]): element (r, c) lies at c * R + r.
// The strided reads make this the slow way in; it only serves [H][V] heads that must be re-packed anyway.
__global__ void prepare_kernel(const void* src, int src_f32, int R, int H, bf16_t* dst, int K, int split_mode,
                               const int* rowmap, const int* meta, int src_transposed) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)R * K) return;
  int r = (int)(i / K);
  const int c = (int)(i % K);
  bf16_t v = (bf16_t)0.f;
  bool live = true;
  if (rowmap) {
    live = r < meta[META_N_VALID];
    r = rowmap[r];
  }
  const int64_t sr = src_transposed ? 1 : H, sc = src_transposed ? R : 1;    // source strides of (r, c)
  if (!live) {
  } else if (!src_f32) {
    if (c < H) v = ((const bf16_t*)src)[r * sr + c * sc];
  } else if (c < 3 * H) {
    const int part = c / H, col = c - part * H;
    const float x = ((const float*)src)[r * sr + col * sc];
    const bf16_t hi = (bf16_t)x;
    const bool want_lo = (split_mode == 1 && part == 2) || (split_mode == 2 && part == 1);
    v = want_lo ? (bf16_t)(x - (float)hi) : hi;
  }
  dst[i] = v;
}

// The common case of the above, 16 bytes per thread: bf16 (or byte) rows that only have to be gathered
// (K == H, H a multiple of 8).  Row j of dst is row rowmap[j] of src for j < n_valid, zero beyond.
__global__ void gather_rows_kernel(const u32x4* src, u32x4* dst, int R, int chunks_per_row, const int* rowmap,
                                   const int* meta) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)R * chunks_per_row) return;
  const int j = (int)(i / chunks_per_row), c = (int)(i % chunks_per_row);
  u32x4 v = {0u, 0u, 0u, 0u};
  if (j < meta[META_N_VALID]) v = src[(int64_t)rowmap[j] * chunks_per_row + c];
  dst[i] = v;
}

// Measurement aid: what the matrix pipe sustains with nothing else going on.  Same occupancy as the
// logit kernels (one workgroup of 8 waves per CU, forced by the LDS request), 8 independent 32x32x16
// accumulators per wave, operands taken from the caller's buffer (the shader clock under MFMA load
// depends on the operand values, so they should look like real data).
__global__ __launch_bounds__(512) void mfma_probe_kernel(const bf16x8* operands, int iters, float* sink,
                                                         long long* clock_out) {
  const long long c0 = clock64(), r0 = wall_clock64();
  const int lane_id = (blockIdx.x * 512 + threadIdx.x) & 2047;      // 2048 x 4 x 16 B = 128 KiB of operands
  bf16x8 a0 = operands[lane_id * 4 + 0], a1 = operands[lane_id * 4 + 1];
  bf16x8 b0 = operands[lane_id * 4 + 2], b1 = operands[lane_id * 4 + 3];
  f32x16 c[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
    c[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, c[0], 0, 0, 0);
    c[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, c[1], 0, 0, 0);
    c[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, c[2], 0, 0, 0);
    c[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, c[3], 0, 0, 0);
    c[4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0, a0, c[4], 0, 0, 0);
    c[5] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1, a0, c[5], 0, 0, 0);
    c[6] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0, a1, c[6], 0, 0, 0);
    c[7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1, a1, c[7], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c[i][r];
  sink[blockIdx.x * 512 + threadIdx.x] = s;
  if (clock_out && blockIdx.x == 0 && threadIdx.x == 0) {
    clock_out[0] = clock64() - c0;
    clock_out[1] = wall_clock64() - r0;
  }
}

// OCP e4m3 (4 exponent bits, bias 7, 3 mantissa bits, no infinities, 0x7f = NaN, largest 448):
// round to nearest even, magnitudes beyond 448 saturate to 448.
__device__ __forceinline__ uint32_t f32_to_e4m3(float x) {
  const uint32_t u = __float_as_uint(x);
  const uint32_t sign = (u >> 24) & 0x80u;
  const float a = fabsf(x);
  if (!(a == a)) return sign | 0x7fu;
  if (a >= 448.f) return sign | 0x7eu;
  if (a < 0.015625f) return sign | (uint32_t)__builtin_rintf(a * 512.f);   // steps of 2^-9; 8 = smallest normal
  const uint32_t ua = u & 0x7fffffffu;
  const uint32_t m = ua & 0x7fffffu, rem = m & 0xfffffu;
  uint32_t code = (((ua >> 23) - 120u) << 3) | (m >> 20);                   // exponent re-biased 127 -> 7
  if (rem > 0x80000u || (rem == 0x80000u && (code & 1u))) ++code;           // a carry moves into the exponent
  return sign | code;
}

// dst[i] = e4m3(src[i] * inv_scale), 8 values per thread
__global__ void quantize_e4m3_kernel(const void* src, int src_f32, int64_t n, float inv_scale, uint8_t* dst) {
  const int64_t i0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (i0 >= n) return;
  uint32_t w[2] = {0u, 0u};
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int64_t i = i0 + k;
    float x = 0.f;
    if (i < n) x = src_f32 ? ((const float*)src)[i] : (float)((const bf16_t*)src)[i];
    w[k >> 2] |= f32_to_e4m3(x * inv_scale) << (8 * (k & 3));
  }
  if (i0 + 8 <= n) {
    *(uint2*)(dst + i0) = make_uint2(w[0], w[1]);
  } else {
    for (int k = 0; i0 + k < n; ++k) dst[i0 + k] = (uint8_t)(w[k >> 2] >> (8 * (k & 3)));
  }
}

// grad_h_s row t = sum over split-K parts of the fp32 partial sums of its compacted row (zero for a
// masked token), converted to the output dtype.
__global__ void gradh_finish_kernel(const float* parts, int n_parts, int T, int H, const int* inv,
                                    int out_f32, void* out) {
  const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  const int64_t n = (int64_t)T * H;
  if (i >= n) return;
  const int t = (int)(i / H), h = (int)(i % H);
  const int j = inv[t];
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (j >= 0) {
    const float* src = parts + (int64_t)j * H + h;
    v = *(const f32x4*)src;
    for (int p = 1; p < n_parts; ++p) v += *(const f32x4*)(src + (int64_t)p * n);
  }
  if (out_f32) {
    *(f32x4*)((float*)out + i) = v;
  } else {
    bf16x4 o;
#pragma unroll
    for (int k = 0; k < 4; ++k) o[k] = (bf16_t)v[k];
    *(bf16x4*)((bf16_t*)out + i) = o;
  }
}

// ------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------
static int largest_divisor_le(int n, int cap) {
  for (int d = cap; d > 1; --d)
    if (n % d == 0) return d;
  return 1;
}

// Launch of a kernel that needs more dynamic LDS than the default limit.  The limit is a property of
// the kernel on a device: it is raised once per kernel and device (one flag word per instantiation,
// one bit per device), not on every launch.
template <auto Kern>
static hipError_t launch_big(int grid, int threads, int smem_bytes, hipStream_t st, const void* args_ptr) {
  static std::atomic<uint64_t> attr_done{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (!(attr_done.load(std::memory_order_acquire) & bit)) {
    e = hipFuncSetAttribute((const void*)Kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes);
    if (e != hipSuccess) return e;
    attr_done.fetch_or(bit, std::memory_order_release);
  }
  void* params[] = {const_cast<void*>(args_ptr)};
  return hipLaunchKernel((const void*)Kern, dim3(grid), dim3(threads), params, smem_bytes, st);
}

static LogitArgs make_logit_args(const Problem& p) {
  LogitArgs a{};
  a.W_s = (const bf16_t*)p.W_s; a.h_s = (const bf16_t*)p.h_s;
  a.W_t = (const bf16_t*)p.W_t; a.h_t = (const bf16_t*)p.h_t;
  a.T = p.T; a.V = p.V; a.H_s = p.K_s; a.H_t = p.K_t;   // contraction lengths = row strides
  a.meta = p.meta;
  a.c = 1.4426950408889634f / p.tau;
  a.beta = p.beta;
  a.t_scale = p.t_fp8 ? p.t_scale : 1.f;
  a.T_pad = p.T_pad;
  a.rowinfo = (const f32x4*)p.rowinfo;
  a.akl = p.akl;
  return a;
}

hipError_t launch_stats(const Problem& p, hipStream_t st) {
  LogitArgs a = make_logit_args(p);
  a.vt0 = 0; a.n_vt = p.n_vt;
  a.partials = p.partials;
  a.clock_out = p.clock_out;
  const int grid = p.n_tt * p.n_split;      // worst case; workgroups beyond the device-side plan exit
#define KD_STATS(K) (p.t_fp8 ? launch_big<stats_kernel<K, true, false>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a) \
                     : p.w_hv_inplace ? launch_big<stats_kernel<K, false, true>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a) \
                              : launch_big<stats_kernel<K, false, false>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a))
  switch (p.kind) {
    case 0: return KD_STATS(0);
    case 1: return KD_STATS(1);
    case 6: return KD_STATS(6);    // both cross terms (AKL)
    default: return KD_STATS(2);   // log-sum-exps only
  }
#undef KD_STATS
}

hipError_t launch_rows(const Problem& p, hipStream_t st) {
  LogitArgs a = make_logit_args(p);
  a.vt0 = 0; a.n_vt = p.n_vt;
  a.partials = p.partials;
  const int grid = p.n_tt * p.n_split;
#define KD_ROWS(K) (p.t_fp8 ? launch_big<rows_kernel<K, true, false>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a) \
                    : p.w_hv_inplace ? launch_big<rows_kernel<K, false, true>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a) \
                             : launch_big<rows_kernel<K, false, false>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a))
  switch (p.kind) {
    case 2: return KD_ROWS(2);
    case 3: return KD_ROWS(3);
    case 4: return KD_ROWS(4);
    case 6: return KD_ROWS(6);
    default: return KD_ROWS(5);
  }
#undef KD_ROWS
}

// AKL: one pass of the threshold search (teacher logit tiles only) and its merge.
hipError_t launch_akl_search(const Problem& p, hipStream_t st) {
  LogitArgs a = make_logit_args(p);
  a.vt0 = 0; a.n_vt = p.n_vt;
  a.partials = p.partials;
  const int grid = p.n_tt * p.n_split;
  hipError_t e = p.w_hv_inplace ? launch_big<akl_search_kernel<true>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a)
                                : launch_big<akl_search_kernel<false>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(akl_search_combine_kernel, dim3((p.T + 255) / 256), dim3(256), 0, st, p.partials, p.meta,
                     p.T_pad, p.beta, p.akl);
  return hipGetLastError();
}

hipError_t launch_akl_weights(const Problem& p, hipStream_t st) {
  hipLaunchKernelGGL(akl_weights_kernel, dim3((p.T + 255) / 256), dim3(256), 0, st, p.partials, p.meta, p.T_pad,
                     (f32x4*)p.rowinfo, p.row_loss, p.akl);
  return hipGetLastError();
}

hipError_t launch_rowmap(const Problem& p, hipStream_t st) {
  hipLaunchKernelGGL(rowmap_kernel, dim3(1), dim3(1024), 0, st, p.mask, p.T, p.T_pad, p.n_split, p.n_cu, p.rowmap,
                     p.inv, p.meta);
  return hipGetLastError();
}

hipError_t launch_combine(const Problem& p, hipStream_t st) {
  hipLaunchKernelGGL(combine_kernel, dim3((p.T_pad + 255) / 256), dim3(256), 0, st, p.partials, p.meta, p.T_pad,
                     p.kind, 1.4426950408889634f / p.tau, (f32x4*)p.rowinfo, p.row_loss, p.akl);
  return hipGetLastError();
}

hipError_t launch_combine_rows(const Problem& p, hipStream_t st) {
  hipLaunchKernelGGL(combine_rows_kernel, dim3((p.T + 255) / 256), dim3(256), 0, st, p.partials, p.meta, p.T_pad,
                     p.kind, p.beta, (f32x4*)p.rowinfo, p.row_loss);
  return hipGetLastError();
}

hipError_t launch_finalize(const Problem& p, hipStream_t st) {
  hipLaunchKernelGGL(finalize_kernel, dim3(1), dim3(1024), 0, st, p.meta, p.inv, p.row_loss, p.T, p.tau,
                     p.out_weight, p.accumulate_loss, (f32x4*)p.rowinfo, p.loss, p.per_token_loss);
  return hipGetLastError();
}

hipError_t launch_grad_chunk(const Problem& p, int v0, int width, bool accumulate, hipStream_t st) {
  LogitArgs a = make_logit_args(p);
  a.dz_accumulate = accumulate ? 1 : 0;
  a.vt0 = v0 / BM;
  a.n_vt = (width + BM - 1) / BM;
  a.bb = largest_divisor_le(a.n_vt, 16);
  a.dz = (bf16_t*)p.dz; a.ldz = p.V_c;
  const int tiles = p.n_tt * a.n_vt;
  int grid = tiles < p.n_cu ? tiles : p.n_cu;
#define KD_GRAD(K) (p.t_fp8 ? launch_big<grad_kernel<K, true, false>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a) \
                    : p.w_hv_inplace ? launch_big<grad_kernel<K, false, true>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a) \
                             : launch_big<grad_kernel<K, false, false>>(grid, LCfg::NT, LCfg::SMEM_BYTES, st, &a))
  switch (p.kind) {
    case 0: return KD_GRAD(0);
    case 1: return KD_GRAD(1);
    case 2: return KD_GRAD(2);
    case 3: return KD_GRAD(3);
    case 4: return KD_GRAD(4);
    case 6: return KD_GRAD(6);
    default: return KD_GRAD(5);
  }
#undef KD_GRAD
}

hipError_t launch_transpose(const void* src, int64_t ld_src, int R, int C, void* dst, int64_t ld_dst, int R_pad,
                            int elem_bytes, hipStream_t st) {
  dim3 grid((R_pad + 63) / 64, (C + 63) / 64);
  if (elem_bytes == 1)
    hipLaunchKernelGGL(transpose_kernel<uint8_t>, grid, dim3(256), 0, st, (const uint8_t*)src, ld_src, R, C,
                       (uint8_t*)dst, ld_dst, R_pad);
  else
    hipLaunchKernelGGL(transpose_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)src, ld_src, R, C,
                       (bf16_t*)dst, ld_dst, R_pad);
  return hipGetLastError();
}

hipError_t launch_gemm(const GemmDesc& d, int n_cu, hipStream_t st) {
  GemmArgs a{};
  a.A = (const bf16_t*)d.A; a.B = (const bf16_t*)d.B;
  a.lda = d.lda; a.ldb = d.ldb; a.M = d.M; a.N = d.N; a.K = d.K;
  const int ksteps_total = d.K / GCfg::BK;
  a.ksteps = d.k_per_split > 0 ? d.k_per_split / GCfg::BK : ksteps_total;
  a.n_ksplit = (ksteps_total + a.ksteps - 1) / a.ksteps;     // every part has at least one k-step
  a.out = d.out; a.ldo = d.ldo; a.out_split_stride = d.out_split_stride;
  a.out_f32 = d.out_f32; a.accumulate = d.accumulate;
  a.n_mt = (d.M + GCfg::BM - 1) / GCfg::BM;
  a.n_nt = (d.N + BN - 1) / BN;
  a.ba = largest_divisor_le(a.n_mt, 8);
  a.bb = largest_divisor_le(a.n_nt, 4);
  a.meta = d.meta; a.n_from_meta = d.n_from_meta; a.k_from_meta = d.k_from_meta;
  a.k_rows = d.k_rows;
  const int tiles = a.n_mt * a.n_nt * a.n_ksplit;       // worst case (no token masked)
  const int grid = tiles < n_cu ? tiles : n_cu;
  if (d.k_major == 0) return launch_big<gemm_kernel<0>>(grid, GCfg::NT, GCfg::SMEM_BYTES, st, &a);
  if (d.k_major == 1) return launch_big<gemm_kernel<1>>(grid, GCfg::NT, GCfg::SMEM_BYTES, st, &a);
  if (d.k_major == 2) return launch_big<gemm_kernel<2>>(grid, GCfg::NT, GCfg::SMEM_BYTES, st, &a);
  return hipErrorInvalidValue;
}

hipError_t launch_prepare(const void* src, int src_f32, int R, int H, void* dst, int K, int split_mode,
                          const int* rowmap, const int* meta, int src_transposed, hipStream_t st) {
  const int64_t n = (int64_t)R * K;
  if (!src_f32 && !src_transposed && K == H && H % 8 == 0 && rowmap) {
    const int64_t chunks = n / 8;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st,
                       (const u32x4*)src, (u32x4*)dst, R, H / 8, rowmap, meta);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(prepare_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src, src_f32, R, H,
                     (bf16_t*)dst, K, split_mode, rowmap, meta, src_transposed);
  return hipGetLastError();
}

hipError_t launch_mfma_probe(const void* operands, int iters, float* sink, long long* clock_out, int n_cu,
                             hipStream_t st) {
  struct { const bf16x8* o; int it; float* s; long long* c; } a{(const bf16x8*)operands, iters, sink, clock_out};
  hipError_t e = hipFuncSetAttribute((const void*)mfma_probe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     LCfg::SMEM_BYTES);
  if (e != hipSuccess) return e;
  void* params[] = {&a.o, &a.it, &a.s, &a.c};
  return hipLaunchKernel((const void*)mfma_probe_kernel, dim3(n_cu), dim3(512), params, LCfg::SMEM_BYTES, st);
}

hipError_t launch_quantize_e4m3(const void* src, int src_f32, int64_t n, float inv_scale, void* dst, hipStream_t st) {
  const int64_t threads = (n + 7) / 8;
  hipLaunchKernelGGL(quantize_e4m3_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, src, src_f32, n,
                     inv_scale, (uint8_t*)dst);
  return hipGetLastError();
}

#define KD_STR2(...) #__VA_ARGS__
#define KD_STR(...) KD_STR2(__VA_ARGS__)
const char* build_info() {
  return "logit tile cfg (MI,NI,WN,BK,NST) = " KD_STR(KD_LOGIT_CFG) "; product tile cfg = " KD_STR(KD_GEMM_CFG)
         "; ablation = " KD_STR(KD_ABLATE);
}
int build_ablation() { return KD_ABLATE; }

hipError_t launch_gradh_finish(const Problem& p, hipStream_t st) {
  const int64_t n = (int64_t)p.T * p.H_s;
  const int64_t threads = (n + 3) / 4;
  hipLaunchKernelGGL(gradh_finish_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, p.gh32,
                     p.n_ksplit_h, p.T, p.H_s, p.inv, p.grad_f32, p.grad_h_s);
  return hipGetLastError();
}

}  // namespace kd
