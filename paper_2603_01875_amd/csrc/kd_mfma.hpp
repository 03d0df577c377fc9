// Device-side building blocks for the MFMA kernels of libkdloss (gfx950).
//
// Every contraction on the hot path (teacher logits, student logits, and the
// two backward products; paper Sec. 3.1-3.2) has the form
//     D[m][n] = sum_k A[m][k] * B[n][k].
// An operand is normally stored K-contiguous ("row m of A" is a contiguous run
// of K bf16 values); the backward products also take one operand stored the
// other way round (k-major, see tile_loop).  One workgroup owns a BM (M) x 256
// (N) tile, its waves arranged 2 (M) x WN (N), each wave owning MI x NI MFMA
// 32x32x16 blocks.  The M axis is the register axis of the MFMA result (a lane
// holds 4 consecutive m for one n), the N axis the lane axis.  For the logit
// tiles M = vocabulary and N = tokens, so the per-token reductions over the
// vocabulary are in-lane and need no cross-lane traffic inside the vocabulary
// loop.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Loop ablations for measurements with tile_loop_bench.hip only (the library is never built with them: the
// products come out wrong).  Bit 1: no global->LDS loads after the first k-steps; bit 2: no LDS fragment reads
// after the first; bit 4: no workgroup barrier.  Each takes one consumer of time and energy out of the loop.
#ifndef KD_LOOP_ABLATE
#define KD_LOOP_ABLATE 0
#endif

namespace kd {

typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int BN = 256;          // tile rows of B (MFMA N axis)

// Tile shape and pipeline depth.  A workgroup is 2 (M) x WN (N) waves; a wave owns MI x NI
// MFMA blocks of 32 x 32, so the tile has BM = 64 MI rows of A and BN = 32 NI WN = 256
// rows of B.  A k-step covers BK elements (32 or 64); NST LDS stages of one k-step each.
// WN = 2 (4 waves, one per SIMD, up to 512 registers each) suits one big accumulator;
// WN = 4 (8 waves, two per SIMD, 256 registers each) gives every SIMD a second
// instruction stream: a wave can keep only one ds_read_b128 per 32 cycles in flight, and
// the second wave also covers the other one's barrier and memory waits.
//
// LDS tile layout: row r occupies ROWB = 2 BK bytes; its CH = BK/8 16-byte chunks are
// permuted by XOR with a few row bits so that 16 lanes reading the same logical chunk of
// 16 consecutive rows hit 16 distinct 16-byte bank groups (conflict-free ds_read_b128),
// while the direct loads still write each wave's 1 KiB linearly.
template <int MI_, int NI_, int WN_, int BK_, int NST_>
struct TileCfg {
  static constexpr int MI = MI_;
  static constexpr int NI = NI_;
  static constexpr int WN = WN_;
  static constexpr int NT = 128 * WN_;                     // threads per workgroup
  static_assert(32 * NI_ * WN_ == BN, "tile rows of B");
  static constexpr int BK = BK_;
  static constexpr int NST = NST_;
  static constexpr int KS = BK_ / 16;                      // MFMA sub-steps per k-step
  static constexpr int BM = 64 * MI_;
  static constexpr int ROWB = BK_ * 2;
  static constexpr int CH = BK_ / 8;
  static constexpr int SW_SHIFT = BK_ == 64 ? 1 : 2;       // swizzle = (row >> SW_SHIFT) & (CH - 1)
  static constexpr int ROWS_PER_LOAD = NT / CH;      // tile rows covered by one load instruction
  static constexpr int A_LOADS = BM / ROWS_PER_LOAD;       // 16-byte loads per thread per k-step
  static constexpr int B_LOADS = BN / ROWS_PER_LOAD;
  static constexpr int LOADS = A_LOADS + B_LOADS;
  static constexpr int LOADS_PER_SUB = (LOADS + KS - 1) / KS;
  static constexpr int LOADS_BEFORE_BARRIER = (KS - 1) * LOADS_PER_SUB < LOADS ? (KS - 1) * LOADS_PER_SUB : LOADS;
  static constexpr int A_STAGE_BYTES = BM * ROWB;
  static constexpr int B_STAGE_BYTES = BN * ROWB;
  static constexpr int STAGE_BYTES = A_STAGE_BYTES + B_STAGE_BYTES;
  static constexpr int SMEM_BYTES = NST_ * STAGE_BYTES;
  // vector-memory operations that may still be pending when k-step g+1 has to be in LDS:
  // whole k-steps g+2 .. g+NST-2 and the part of k-step g+NST-1 issued before the barrier
  static constexpr int WAIT_STEADY = (NST_ - 3) * LOADS + LOADS_BEFORE_BARRIER;
  static constexpr int WAIT_PROLOGUE = (NST_ - 2) * LOADS;
  static_assert(BK_ == 32 || BK_ == 64, "k-step");
  static_assert(NST_ >= 3, "the stage being refilled is the one released one k-step earlier");
  static_assert(SMEM_BYTES <= 160 * 1024, "LDS of a gfx950 CU");
  static_assert(WAIT_STEADY < 64 && WAIT_PROLOGUE < 64, "vmcnt is a 6-bit counter");
  typedef f32x16 Acc[MI_][NI];
  // Coordinates of accumulator element (mt, nt, r) of this lane inside the tile.
  static __device__ __forceinline__ int acc_m(int wm, int mt, int r, int lane) {
    return wm * (32 * MI_) + mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
  }
  static __device__ __forceinline__ int acc_n(int wn, int nt, int lane) {
    return wn * (32 * NI_) + nt * 32 + (lane & 31);
  }
  static __device__ __forceinline__ void zero(Acc& acc) {
#pragma unroll
    for (int i = 0; i < MI_; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  }
};

// One unit of work for a persistent workgroup: a BM x 256 tile whose value is
// built in NPHASE accumulators (phase p contracts A[p] with B[p] over K[p]).
// (Scalar fields, no arrays: the struct must stay in scalar registers.)
struct WorkItem {
  const bf16_t *A0, *A1;   // first row of the tile in A (phase 0 / 1)
  const bf16_t *B0, *B1;   // first row of the tile in B
  int a_rows;              // valid rows of A in this tile (1..BM); rows beyond are clamped
  int b_rows;              // valid rows of B in this tile (1..BN)
  int ka_rows, kb_rows;    // k-major operands only: k-rows that exist from the item's k origin on
  int nk0, nk1;            // k-steps of BK elements per phase (>= 1 for phases in use)
  int m0, n0;              // tile origin, passed through to the epilogue
  int aux;                 // free for the work map (e.g. split-K index)
};

// Values that are the same in every lane but that the compiler cannot prove so.
__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }
template <class T>
__device__ __forceinline__ const T* uniform(const T* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const T*)(((uint64_t)hi << 32) | lo);
}

// Persistent tile loop with a continuous software pipeline.
//
// Work:  int n_items() const;  WorkItem item(int i) const;   (wave-uniform)
// Epi:   void begin_item(const WorkItem&)            called before the first k-step of an item
//        void end_item(const WorkItem&, Acc& acc0, Acc& acc1)
//                                                    called after the last k-step of an item
// ld*[p] are the same for every item of a launch; the k-step counts may differ per item.
//
// Pipeline: NST LDS stages filled by direct global->LDS loads (16 bytes per lane, no
// staging registers).  While k-step g is multiplied, the loads of k-step g+NST-1 are
// issued a few at a time between its MFMAs (a wave issues in order, so a burst of loads
// would starve the matrix pipe), into the stage that k-step g-1 released.  One barrier per
// k-step, placed before the last group of MFMAs so that the first fragments of k-step g+1
// are read in their shadow.  The stream of k-steps does not drain between phases or
// between items: the operands of the next tile are in flight while the epilogue runs.
//
// Synchronisation: every k-step issues exactly LOADS direct loads per thread (past the end
// of its work a workgroup re-issues its last loads as dummies so that this holds to the
// end) and vector-memory loads complete in order, so "at most WAIT_STEADY operations
// outstanding" implies that k-step g+1 has landed.  Other vector-memory traffic of the
// thread (epilogue loads and stores) only adds to the counter, which makes the wait
// stricter, never weaker.
typedef __attribute__((address_space(3))) void lds_void_t;

// sched_group_barrier masks
constexpr int SG_MFMA = 0x008, SG_VMEM = 0x010, SG_DSREAD = 0x100;

//
// k-major operands (KM bit 0: A, bit 1: B).  An operand may instead be stored with the
// contraction index outermost: element (row r, k) at P[k * ld + r], P pointing at (k origin,
// first row of the tile).  Its LDS tile is then [BK][R] (R = BM or BN rows, contiguous), the
// 16-byte chunks of a k-row permuted by XOR with 4 (k mod 4), and a fragment is fetched by
// two transposing reads (ds_read_b64_tr_b16): in every group of 16 lanes, lane i receives as
// element j the (i mod 4)-th of the four values addressed by lane i/4 + 4j, so lane i
// addresses k-row i/4 (+4 for the second read), rows 4 (i mod 4) .. +3 of its group's 16.
// The four k-rows that half a wave reads at once then fall into four different 64-byte
// bank groups.  Chunks past the valid rows and k-rows past ka_rows / kb_rows are clamped to
// the last valid one (the other operand must be zero there).
//
// The transposing reads are written as inline assembly with hand-placed waits: issued through
// the compiler's builtin, every one of them is preceded by a wait for ALL outstanding direct
// loads (the compiler cannot tell that they target another LDS stage), which serialises the
// pipeline.  A k-major fragment therefore lives in two register pairs that the hardware fills
// asynchronously; km_wait() ties them to an "s_waitcnt lgkmcnt(0)" placed at the top of the
// sub-step that consumes them (their reads were issued one sub-step earlier), and only the
// values that leave km_wait() are ever used.
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;

struct KmFrag { s16x4 lo, hi; };
template <bool KMAJOR> struct FragT { typedef bf16x8 type; };
template <> struct FragT<true> { typedef KmFrag type; };

__device__ __forceinline__ bf16x8 frag_op(const bf16x8& f) { return f; }
__device__ __forceinline__ bf16x8 frag_op(const KmFrag& f) {
  const s16x8 v = __builtin_shufflevector(f.lo, f.hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}
// k-rows k and k+4 of one fragment: OFF = byte offset of k-row k from addr, ROWB4 = 4 k-rows
template <int OFF, int ROWB4>
__device__ __forceinline__ void km_read(KmFrag& f, uint32_t addr) {
  static_assert(OFF >= 0 && OFF + ROWB4 < 65536, "ds offset field");
  asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
               : "=&v"(f.lo), "=&v"(f.hi)
               : "v"(addr), "n"(OFF), "n"(OFF + ROWB4));
}
template <int N>
__device__ __forceinline__ void km_wait(KmFrag (&f)[N]) {
  static_assert(N >= 1 && N <= 4, "fragments per wave and operand");
  if constexpr (N == 1)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi));
  else if constexpr (N == 2)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi));
  else if constexpr (N == 3)
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi), "+v"(f[2].lo), "+v"(f[2].hi));
  else
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi), "+v"(f[2].lo), "+v"(f[2].hi),
                   "+v"(f[3].lo), "+v"(f[3].hi));
}
template <int N>
__device__ __forceinline__ void km_wait(bf16x8 (&)[N]) {}

template <int V> struct IntC { static constexpr int value = V; };
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(IntC<I>{});
    static_for<I + 1, N>(f);
  }
}

//
// fp8 second phase (P1F8).  The operands of phase 1 may be OCP e4m3 bytes instead of bf16: a
// k-step then covers 128 elements (the same 128 bytes per tile row, so loads, LDS layout and
// synchronisation are unchanged) and is multiplied by 2 x MI x NI MFMAs 32x32x64 (f8f6f4,
// unit scales), each lane holding 32 consecutive bytes of its row per operand.  Both
// operands use the same byte-to-lane map, so the order of k inside an instruction does not
// matter.  ld*1 are then in bytes (= elements).
typedef int i32x8 __attribute__((ext_vector_type(8)));

template <int NPHASE, class Cfg, int KM = 0, bool P1F8 = false, class Work, class Epi>
__device__ __forceinline__ void tile_loop(const Work& work, Epi& epi,
                                          const int lda0, const int lda1, const int ldb0, const int ldb1,
                                          char* smem) {
  constexpr int MI = Cfg::MI, NI = Cfg::NI, NST = Cfg::NST, KS = Cfg::KS, CH = Cfg::CH;
  constexpr int A_LOADS = Cfg::A_LOADS, LOADS = Cfg::LOADS, LPS = Cfg::LOADS_PER_SUB;
  constexpr int A_STAGE_BYTES = Cfg::A_STAGE_BYTES, STAGE_BYTES = Cfg::STAGE_BYTES;
  constexpr int ROWB = Cfg::ROWB;
  constexpr bool AKM = (KM & 1) != 0, BKM = (KM & 2) != 0;
  constexpr int BK = Cfg::BK;
  constexpr int CPR_A = Cfg::BM / 8, CPR_B = BN / 8;                 // chunks per k-row
  constexpr int KPL_A = Cfg::NT / CPR_A, KPL_B = Cfg::NT / CPR_B;    // k-rows per load instruction
  static_assert(KM == 0 || (KPL_A % 4 == 0 && KPL_B % 4 == 0 && BK % 16 == 0), "k-major swizzle");
  static_assert(!P1F8 || (KM == 0 && NPHASE == 2 && BK == 64 && Cfg::LOADS_BEFORE_BARRIER == LOADS),
                "fp8 phase: 128-byte rows, every load of a k-step issued before its barrier");
  typedef typename Cfg::Acc Acc;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;

  const int n_items = work.n_items();
  if (n_items == 0) return;

  // ---- load cursor ------------------------------------------------------------------
  // Load j of lane (wave w, lane l) fills the 16-byte LDS slot j*NT + w*64 + l of the
  // stage (A region first, then B): tile row j*ROWS_PER_LOAD + tid/CH, physical chunk
  // tid%CH.  The chunk it fetches from global memory is the logical one that the XOR
  // layout keeps in that slot.
  const int lrow = tid / CH;
  const int lchunk = (tid % CH) ^ ((lrow >> Cfg::SW_SHIFT) & (CH - 1));
  int l_item = 0, l_phase = 0, l_k = 0, l_nk;
  bool more = true;
  WorkItem li = work.item(0);
  const char *l_pa, *l_pb;      // uniform: tile base + k offset, in bytes
  int64_t l_step_a = ROWB, l_step_b = ROWB;   // bytes from one k-step to the next
  uint32_t loff[LOADS];         // per lane: byte offset of its 16 bytes inside the k-slab
  const int kma_row = tid / CPR_A, kma_c = (tid % CPR_A) ^ (4 * (kma_row & 3));
  const int kmb_row = tid / CPR_B, kmb_c = (tid % CPR_B) ^ (4 * (kmb_row & 3));
  // offsets of the k-major operands for the k-step that starts k_done elements into the phase
  auto km_offsets = [&](int k_done) {
    if (AKM) {
      const uint32_t la = (uint32_t)(l_phase ? lda1 : lda0);
      const int clim = (li.a_rows + 7) / 8 - 1, rem = li.ka_rows - k_done - 1;
      const int c = kma_c < clim ? kma_c : clim;
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j) {
        int kr = kma_row + KPL_A * j;
        kr = kr < rem ? kr : rem;
        kr = kr > 0 ? kr : 0;
        loff[j] = ((uint32_t)kr * la + c * 8) * 2;
      }
    }
    if (BKM) {
      const uint32_t lb = (uint32_t)(l_phase ? ldb1 : ldb0);
      const int clim = (li.b_rows + 7) / 8 - 1, rem = li.kb_rows - k_done - 1;
      const int c = kmb_c < clim ? kmb_c : clim;
#pragma unroll
      for (int j = 0; j < Cfg::B_LOADS; ++j) {
        int kr = kmb_row + KPL_B * j;
        kr = kr < rem ? kr : rem;
        kr = kr > 0 ? kr : 0;
        loff[A_LOADS + j] = ((uint32_t)kr * lb + c * 8) * 2;
      }
    }
  };
  auto set_cursor = [&]() {
    const uint32_t la = (uint32_t)(l_phase ? lda1 : lda0), lb = (uint32_t)(l_phase ? ldb1 : ldb0);
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const bool isA = j < A_LOADS;
      if (isA ? AKM : BKM) continue;
      int r = lrow + Cfg::ROWS_PER_LOAD * (isA ? j : j - A_LOADS);
      const int lim = isA ? li.a_rows : li.b_rows;
      r = r < lim ? r : lim - 1;
      const uint32_t es = (P1F8 && l_phase) ? 1 : 2;       // bytes per element
      loff[j] = (uint32_t)r * (isA ? la : lb) * es + lchunk * 16;
    }
    if (KM) km_offsets(0);
    if (AKM) l_step_a = (int64_t)BK * 2 * la;
    if (BKM) l_step_b = (int64_t)BK * 2 * lb;
    l_pa = (const char*)uniform(l_phase ? li.A1 : li.A0);
    l_pb = (const char*)uniform(l_phase ? li.B1 : li.B0);
    l_nk = l_phase ? li.nk1 : li.nk0;
  };
  set_cursor();

  // loads [j0, j1) of the k-step under the cursor, into LDS stage `stage`
  bool in_main_loop = false;     // (only read by the loop ablations)
  auto issue_loads = [&](int stage, int j0, int j1) {
    if ((KD_LOOP_ABLATE & 1) && in_main_loop && (l_item > 0 || l_k > 5)) return;   // every stage holds data by then
    char* sbase = smem + stage * STAGE_BYTES + wave * 1024;
#pragma unroll
    for (int j = j0; j < j1; ++j)
      __builtin_amdgcn_global_load_lds((const void*)((j < A_LOADS ? l_pa : l_pb) + loff[j]),
                                       (lds_void_t*)(sbase + j * (Cfg::NT * 16)), 16, 0, 0);
  };
  auto advance = [&]() {
    l_pa += AKM ? l_step_a : ROWB;
    l_pb += BKM ? l_step_b : ROWB;
    if (KM && l_k + 1 < l_nk) {
      // the k-step now under the cursor runs past the last k-row that exists: clamp its rows
      const int k_end = (l_k + 2) * BK;
      if ((AKM && k_end > li.ka_rows) || (BKM && k_end > li.kb_rows)) km_offsets((l_k + 1) * BK);
    }
    if (++l_k == l_nk) {
      l_k = 0;
      if (NPHASE > 1 && l_phase == 0) {
        l_phase = 1;
      } else {
        l_phase = 0;
        ++l_item;
        if (l_item < n_items) li = work.item(l_item);
        else more = false;
      }
      if (more) {
        set_cursor();
      } else {
        // past the end: keep re-reading the last k-step (valid memory, data unused) so that
        // every k-step of the loop issues the same number of loads
        l_item = n_items - 1;
        l_phase = NPHASE - 1;
        l_k = l_nk - 1;
        l_pa -= AKM ? l_step_a : ROWB;
        l_pb -= BKM ? l_step_b : ROWB;
      }
    }
  };

  // ---- fragment read offsets ----------------------------------------------------------
  // A fragment (mt, ks): row = wm*32*MI + mt*32 + (lane & 31), chunk = 2 ks + (lane >> 5)
  const int frow = lane & 31;
  const int fsw = (frow >> Cfg::SW_SHIFT) & (CH - 1);
  int fk[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) fk[ks] = ((2 * ks + (lane >> 5)) ^ fsw) << 4;
  const int a_base = (wm * 32 * MI + frow) * ROWB;
  const int b_base = A_STAGE_BYTES + (wn * 32 * NI + frow) * ROWB;
  // fp8 fragment (sub-step s of 64 bytes, lane half hb): chunks 4 s + 2 hb and the next one
  int fk8[2][2];
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int j = 0; j < 2; ++j) fk8[sb][j] = ((4 * sb + 2 * (lane >> 5) + j) ^ fsw) << 4;

  // k-major fragments: byte offset of the lane's first transposing read of sub-step 0
  int kma_f[MI], kmb_f[NI];
  {
    const int g = lane >> 4, r = lane & 15;
    const int sw = 4 * (r >> 2), low = 2 * (g & 1) + ((r & 3) >> 1), kr = 8 * (g >> 1) + (r >> 2);
#pragma unroll
    for (int mt = 0; mt < MI; ++mt)
      kma_f[mt] = kr * (2 * Cfg::BM) + ((((wm * 32 * MI + mt * 32) / 8) ^ sw) + low) * 16 + (r & 1) * 8;
#pragma unroll
    for (int nt = 0; nt < NI; ++nt)
      kmb_f[nt] = A_STAGE_BYTES + kr * (2 * BN) + ((((wn * 32 * NI + nt * 32) / 8) ^ sw) + low) * 16 + (r & 1) * 8;
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void_t*)smem;   // LDS byte address of stage 0
  typedef typename FragT<AKM>::type AFrag;
  typedef typename FragT<BKM>::type BFrag;

  Acc acc0, acc1;
  Cfg::zero(acc0);
  if (NPHASE > 1) Cfg::zero(acc1);

  int stage = 0;            // LDS stage of the k-step being consumed
  int fill = NST - 1;       // LDS stage being refilled (released by the previous k-step)

  auto read_frags = [&](int st, auto ks_c, AFrag (&af)[MI], BFrag (&bfr)[NI]) {
    constexpr int ks = decltype(ks_c)::value;
    if ((KD_LOOP_ABLATE & 2) && in_main_loop) return;
    const char* base = smem + st * STAGE_BYTES;
    const uint32_t lbase = lds0 + st * STAGE_BYTES;
#pragma unroll
    for (int mt = 0; mt < MI; ++mt) {
      if constexpr (AKM) km_read<ks * 16 * (2 * Cfg::BM), 4 * (2 * Cfg::BM)>(af[mt], lbase + kma_f[mt]);
      else af[mt] = *(const bf16x8*)(base + a_base + mt * 32 * ROWB + fk[ks]);
    }
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      if constexpr (BKM) km_read<ks * 16 * (2 * BN), 4 * (2 * BN)>(bfr[nt], lbase + kmb_f[nt]);
      else bfr[nt] = *(const bf16x8*)(base + b_base + nt * 32 * ROWB + fk[ks]);
    }
  };
  auto read_frags8 = [&](int st, auto s_c, i32x8 (&af)[MI], i32x8 (&bfr)[NI]) {
    constexpr int sb = decltype(s_c)::value;
    const char* base = smem + st * STAGE_BYTES;
#pragma unroll
    for (int mt = 0; mt < MI; ++mt) {
      const u32x4 lo = *(const u32x4*)(base + a_base + mt * 32 * ROWB + fk8[sb][0]);
      const u32x4 hi = *(const u32x4*)(base + a_base + mt * 32 * ROWB + fk8[sb][1]);
      af[mt] = __builtin_bit_cast(i32x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) {
      const u32x4 lo = *(const u32x4*)(base + b_base + nt * 32 * ROWB + fk8[sb][0]);
      const u32x4 hi = *(const u32x4*)(base + b_base + nt * 32 * ROWB + fk8[sb][1]);
      bfr[nt] = __builtin_bit_cast(i32x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };
  auto mma8 = [&](Acc& acc, const i32x8 (&af)[MI], const i32x8 (&bfr)[NI]) {
#pragma unroll
    for (int mt = 0; mt < MI; ++mt)
#pragma unroll
      for (int nt = 0; nt < NI; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(af[mt], bfr[nt], acc[mt][nt], 0, 0, 0, 0, 0, 0);
  };
  // one fp8 sub-step: per MFMA (64 cycles) a share of the fragment reads and of the loads
  auto schedule_substep8 = [&](auto n_ds_c, auto n_vm_c) {
    constexpr int n_mfma = MI * NI, n_ds = decltype(n_ds_c)::value, n_vm = decltype(n_vm_c)::value;
    constexpr int ds_per = (n_ds + n_mfma - 1) / n_mfma, vm_per = (n_vm + n_mfma - 1) / n_mfma;
#pragma unroll
    for (int i = 0; i < n_mfma; ++i) {
      __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
      if (ds_per > 0) __builtin_amdgcn_sched_group_barrier(SG_DSREAD, ds_per, 0);
      if (vm_per > 0) __builtin_amdgcn_sched_group_barrier(SG_VMEM, vm_per, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // waits for the k-major fragments about to be multiplied (no-op for K-contiguous operands,
  // whose reads the compiler tracks itself)
  auto wait_frags = [&](AFrag (&af)[MI], BFrag (&bfr)[NI]) {
    km_wait(af);
    km_wait(bfr);
  };
  auto mma = [&](Acc& acc, const AFrag (&af)[MI], const BFrag (&bfr)[NI]) {
#pragma unroll
    for (int mt = 0; mt < MI; ++mt)
#pragma unroll
      for (int nt = 0; nt < NI; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_op(af[mt]), frag_op(bfr[nt]), acc[mt][nt], 0, 0, 0);
  };
  // Order inside one sub-step: fragment reads first (two per MFMA), then one load per MFMA.
  auto schedule_substep = [&]() {
    constexpr int n_mfma = MI * NI, n_ds = (AKM ? 0 : MI) + (BKM ? 0 : NI);   // reads the scheduler sees
    constexpr int ds_slots = (n_ds + 1) / 2 < n_mfma ? (n_ds + 1) / 2 : n_mfma - 1;
    constexpr int vm_slots = n_mfma - ds_slots < LPS ? n_mfma - ds_slots : (LPS > 0 ? LPS : 1);
    constexpr int vm_per = (LPS + vm_slots - 1) / vm_slots;
#pragma unroll
    for (int i = 0; i < ds_slots; ++i) {
      __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
      __builtin_amdgcn_sched_group_barrier(SG_DSREAD, (n_ds + ds_slots - 1) / ds_slots, 0);
    }
#pragma unroll
    for (int i = 0; i < vm_slots; ++i) {
      __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
      __builtin_amdgcn_sched_group_barrier(SG_VMEM, vm_per, 0);
    }
    if (n_mfma - ds_slots - vm_slots > 0)
      __builtin_amdgcn_sched_group_barrier(SG_MFMA, n_mfma - ds_slots - vm_slots, 0);
    __builtin_amdgcn_sched_barrier(0);
  };

  // Fragments of sub-step 0 of the k-step about to be consumed; kept across k-steps.
  AFrag fa0[MI];
  BFrag fb0[NI];
  i32x8 ga0[MI], gb0[NI];   // the same for an fp8 k-step

  // One fp8 k-step (two sub-steps of 64 bytes).  On entry ga0/gb0 hold sub-step 0; on exit the
  // first fragments of the next k-step are on their way, fp8 ones if NEXT8, else bf16 ones.
  auto kstep8 = [&](Acc& acc, auto next8_c) {
    constexpr bool NEXT8 = decltype(next8_c)::value != 0;
    i32x8 ga1[MI], gb1[NI];
    const int next = stage == NST - 1 ? 0 : stage + 1;
    read_frags8(stage, IntC<1>{}, ga1, gb1);
    issue_loads(fill, 0, LOADS);
    mma8(acc, ga0, gb0);
    schedule_substep8(IntC<2 * (MI + NI)>{}, IntC<LOADS>{});
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(Cfg::WAIT_STEADY) : "memory");
    if constexpr (NEXT8) read_frags8(next, IntC<0>{}, ga0, gb0);
    else read_frags(next, IntC<0>{}, fa0, fb0);
    mma8(acc, ga1, gb1);
    schedule_substep8(IntC<(NEXT8 ? 2 : 1) * (MI + NI)>{}, IntC<0>{});
    advance();
    fill = stage;
    stage = next;
  };

  // One k-step.  On entry fa0/fb0 hold sub-step 0.
  auto kstep = [&](Acc& acc, auto next8_c) {
    constexpr bool NEXT8 = decltype(next8_c)::value != 0;
    AFrag fa1[MI];
    BFrag fb1[NI];
    const int next = stage == NST - 1 ? 0 : stage + 1;
    static_for<0, KS - 1>([&](auto ks_c) {
      constexpr int ks = decltype(ks_c)::value;
      // even sub-steps multiply (fa0, fb0) and fetch into (fa1, fb1); odd ones the reverse
      if constexpr (ks % 2 == 0) {
        wait_frags(fa0, fb0);
        read_frags(stage, IntC<ks + 1>{}, fa1, fb1);
        issue_loads(fill, ks * LPS < LOADS ? ks * LPS : LOADS, (ks + 1) * LPS < LOADS ? (ks + 1) * LPS : LOADS);
        mma(acc, fa0, fb0);
      } else {
        wait_frags(fa1, fb1);
        read_frags(stage, IntC<ks + 1>{}, fa0, fb0);
        issue_loads(fill, ks * LPS < LOADS ? ks * LPS : LOADS, (ks + 1) * LPS < LOADS ? (ks + 1) * LPS : LOADS);
        mma(acc, fa1, fb1);
      }
      schedule_substep();
    });
    // k-step g+1 must have landed; after the barrier nobody reads stage `stage` any more
    if (KD_LOOP_ABLATE & 4) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(Cfg::WAIT_STEADY) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(Cfg::WAIT_STEADY) : "memory");
    // last sub-step (KS-1, odd): multiplies (fa1, fb1), fetches sub-step 0 of the next k-step
    wait_frags(fa1, fb1);
    issue_loads(fill, Cfg::LOADS_BEFORE_BARRIER, LOADS);
    if constexpr (NEXT8) read_frags8(next, IntC<0>{}, ga0, gb0);
    else read_frags(next, IntC<0>{}, fa0, fb0);
    mma(acc, fa1, fb1);
    schedule_substep();
    advance();
    fill = stage;
    stage = next;
  };

  // ---- prologue: NST-1 k-steps in flight, first fragments read -------------------------------
#pragma unroll
  for (int i = 0; i < NST - 1; ++i) {
    issue_loads(i, 0, LOADS);
    advance();
  }
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(Cfg::WAIT_PROLOGUE) : "memory");
  read_frags(0, IntC<0>{}, fa0, fb0);
  in_main_loop = true;

  for (int c_item = 0; c_item < n_items; ++c_item) {
    const WorkItem ci = work.item(c_item);
    epi.begin_item(ci);
    if constexpr (P1F8) {
      for (int k = 1; k < ci.nk0; ++k) kstep(acc0, IntC<0>{});
      kstep(acc0, IntC<1>{});
      for (int k = 1; k < ci.nk1; ++k) kstep8(acc1, IntC<1>{});
      kstep8(acc1, IntC<0>{});
    } else {
      for (int k = 0; k < ci.nk0; ++k) kstep(acc0, IntC<0>{});
      if (NPHASE > 1)
        for (int k = 0; k < ci.nk1; ++k) kstep(acc1, IntC<0>{});
    }
    epi.end_item(ci, acc0, acc1);
    Cfg::zero(acc0);
    if (NPHASE > 1) Cfg::zero(acc1);
  }
  // the loads issued past the end still target this workgroup's LDS: let them land
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

}  // namespace kd
