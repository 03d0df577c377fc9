// Device-side building blocks for the bf16 MFMA kernels of libkdloss (gfx950).
//
// Every contraction on the hot path (teacher logits, student logits, and the
// two backward products; paper Sec. 3.1-3.2) is brought to one form:
//     D[m][n] = sum_k A[m][k] * B[n][k]
// with both operands stored K-contiguous ("row m of A" and "row n of B" are
// contiguous runs of K bf16 values).  One workgroup of 256 threads (4 waves,
// 2 x 2) owns a 128 (M) x 256 (N) tile; each wave owns 64 x 128 of it as
// 2 x 4 MFMA 32x32x16 blocks.  The M axis is the register axis of the MFMA
// result (a lane holds 4 consecutive m for one n), the N axis the lane axis.
// For the logit tiles M = vocabulary and N = tokens, so the per-token
// reductions over the vocabulary are in-lane and need no cross-lane traffic
// inside the vocabulary loop.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kd {

typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int BM = 128;          // tile rows of A (MFMA M axis)
constexpr int BN = 256;          // tile rows of B (MFMA N axis)
constexpr int BK = 64;           // k-step, in elements (128 bytes per tile row)
constexpr int NTHREADS = 256;
constexpr int MI = 2;            // 32-row MFMA blocks per wave along M
constexpr int NI = 4;            // 32-row MFMA blocks per wave along N
constexpr int A_LOADS = BM * BK / 8 / NTHREADS;   // 16-byte loads per thread per k-step (4)
constexpr int B_LOADS = BN * BK / 8 / NTHREADS;   // (8)
constexpr int A_STAGE_BYTES = BM * BK * 2;
constexpr int B_STAGE_BYTES = BN * BK * 2;
constexpr int STAGE_BYTES = A_STAGE_BYTES + B_STAGE_BYTES;
constexpr int NSTAGE = 3;
constexpr int SMEM_BYTES = NSTAGE * STAGE_BYTES;   // 144 KiB of the 160 KiB LDS

typedef f32x16 AccTile[MI][NI];

// One unit of work for a persistent workgroup: a 128 x 256 tile whose value is
// built in NPHASE accumulators (phase p contracts A[p] with B[p] over K[p]).
// (Scalar fields, no arrays: the struct must stay in scalar registers.)
struct WorkItem {
  const bf16_t *A0, *A1;   // first row of the tile in A (phase 0 / 1)
  const bf16_t *B0, *B1;   // first row of the tile in B
  int a_rows;              // valid rows of A in this tile (1..BM); rows beyond are clamped
  int b_rows;              // valid rows of B in this tile (1..BN)
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

// LDS tile layout: row r occupies bytes [128 r, 128 r + 128); its eight 16-byte
// chunks are permuted by XOR with ((r >> 1) & 7) so that 16 lanes reading the
// same chunk index of 16 consecutive rows hit 16 distinct 16-byte bank groups.
__device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * (BK * 2) + ((chunk ^ ((row >> 1) & 7)) << 4);
}

__device__ __forceinline__ void zero_acc(AccTile& acc) {
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
}

// Coordinates of accumulator element (mt, nt, r) of this lane inside the tile.
__device__ __forceinline__ int acc_m(int wm, int mt, int r, int lane) {
  return wm * 64 + mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}
__device__ __forceinline__ int acc_n(int wn, int nt, int lane) {
  return wn * 128 + nt * 32 + (lane & 31);
}

// Persistent tile loop with a continuous software pipeline.
//
// Work:  int n_items() const;  WorkItem item(int i) const;   (wave-uniform)
// Epi:   void begin_item(const WorkItem&)            called before the first k-step of an item
//        void end_item(const WorkItem&, AccTile& acc0, AccTile& acc1)
//                                                    called after the last k-step of an item
// ld*[p] are the same for every item of a launch; the k-step counts may differ per item.
//
// Pipeline: three LDS stages filled by direct global->LDS loads (16 bytes per
// lane, no staging registers).  The loads of k-step g+3 are issued near the
// end of k-step g, into the stage it has just finished reading; one barrier
// per k-step.  The stream of k-steps does
// not drain between phases or between items, so the operands of the next tile
// are already in flight while the epilogue of the current one runs.
//
// Synchronisation: each thread issues exactly LOADS_PER_STEP direct loads per
// k-step (the last three k-steps of a workgroup re-issue the final loads as
// dummies so that this holds to the end) and vector-memory loads complete in
// order, so "at most LOADS_PER_STEP operations outstanding" implies that
// everything older than the youngest k-step has landed.  Other vector-memory traffic of the thread (epilogue
// loads and stores) only adds to the counter, which makes the wait stricter,
// never weaker.
constexpr int LOADS_PER_STEP = A_LOADS + B_LOADS;
static_assert(LOADS_PER_STEP == 12, "s_waitcnt immediates below assume 12 loads per k-step");

typedef __attribute__((address_space(3))) void lds_void_t;

// sched_group_barrier masks
constexpr int SG_MFMA = 0x008, SG_VMEM = 0x010, SG_DSREAD = 0x100;

template <int NPHASE, class Work, class Epi>
__device__ __forceinline__ void tile_loop(const Work& work, Epi& epi,
                                          const int lda0, const int lda1, const int ldb0, const int ldb1,
                                          char* smem) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int wm = wave & 1, wn = wave >> 1;

  const int n_items = work.n_items();
  if (n_items == 0) return;

  // ---- load cursor ------------------------------------------------------------------
  // Lane (wave w, lane l) of load j fills the 16-byte LDS slot j*256 + w*64 + l of the A
  // (or B) region: tile row j*32 + tid/8, physical chunk tid%8.  The chunk it fetches from
  // global memory is the logical one that the XOR layout keeps in that slot.
  const int lrow = tid >> 3;
  const int lchunk = (tid & 7) ^ ((tid >> 4) & 7);
  int l_item = 0, l_phase = 0, l_k = 0, l_nk;
  bool more = true;
  WorkItem li = work.item(0);
  const char *l_pa, *l_pb;                  // uniform: tile base + k offset, in bytes
  uint32_t aoff[A_LOADS], boff[B_LOADS];    // per lane: byte offset of its 16 bytes inside the k-slab
  auto set_cursor = [&]() {
    const uint32_t la = (uint32_t)(l_phase ? lda1 : lda0), lb = (uint32_t)(l_phase ? ldb1 : ldb0);
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
      int r = lrow + 32 * j;
      r = r < li.a_rows ? r : li.a_rows - 1;
      aoff[j] = ((uint32_t)r * la + lchunk * 8) * 2;
    }
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
      int r = lrow + 32 * j;
      r = r < li.b_rows ? r : li.b_rows - 1;
      boff[j] = ((uint32_t)r * lb + lchunk * 8) * 2;
    }
    l_pa = (const char*)uniform(l_phase ? li.A1 : li.A0);
    l_pb = (const char*)uniform(l_phase ? li.B1 : li.B0);
    l_nk = l_phase ? li.nk1 : li.nk0;
  };
  set_cursor();

  auto issue_loads = [&](int stage) {
    char* sbase = smem + stage * STAGE_BYTES + wave * 1024;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j)
      __builtin_amdgcn_global_load_lds((const void*)(l_pa + aoff[j]), (lds_void_t*)(sbase + j * 4096), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j)
      __builtin_amdgcn_global_load_lds((const void*)(l_pb + boff[j]),
                                       (lds_void_t*)(sbase + A_STAGE_BYTES + j * 4096), 16, 0, 0);
  };
  auto advance = [&]() {
    l_pa += BK * 2;
    l_pb += BK * 2;
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
        l_pa -= BK * 2;
        l_pb -= BK * 2;
      }
    }
  };

  // ---- fragment read offsets ----------------------------------------------------------
  // A fragment (mt, ks): row = wm*64 + mt*32 + (lane & 31), chunk = 2 ks + (lane >> 5)
  const int frow = lane & 31;
  const int fsw = (frow >> 1) & 7;
  int fk[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) fk[ks] = ((2 * ks + (lane >> 5)) ^ fsw) << 4;
  const int a_base = (wm * 64 + frow) * (BK * 2);
  const int b_base = A_STAGE_BYTES + (wn * 128 + frow) * (BK * 2);

  AccTile acc0, acc1;
  zero_acc(acc0);
  if (NPHASE > 1) zero_acc(acc1);

  int stage = 0;       // LDS stage of the k-step being consumed

  auto read_frags = [&](int st, int ks, bf16x8 (&af)[MI], bf16x8 (&bfr)[NI]) {
    const char* base = smem + st * STAGE_BYTES;
#pragma unroll
    for (int mt = 0; mt < MI; ++mt) af[mt] = *(const bf16x8*)(base + a_base + mt * 32 * BK * 2 + fk[ks]);
#pragma unroll
    for (int nt = 0; nt < NI; ++nt) bfr[nt] = *(const bf16x8*)(base + b_base + nt * 32 * BK * 2 + fk[ks]);
  };
  auto mma = [&](AccTile& acc, const bf16x8 (&af)[MI], const bf16x8 (&bfr)[NI]) {
#pragma unroll
    for (int mt = 0; mt < MI; ++mt)
#pragma unroll
      for (int nt = 0; nt < NI; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mt], bfr[nt], acc[mt][nt], 0, 0, 0);
  };

  // Fragments of sub-step 0 of the k-step about to be consumed; kept across k-steps.
  bf16x8 fa0[MI], fb0[NI];

  // One k-step.  On entry fa0/fb0 hold sub-step 0.  The barrier sits before the last group
  // of MFMAs: after it the stage just read is refilled with the k-step three ahead and the
  // first fragments of the next k-step are read, all in the shadow of that last group.
  auto kstep = [&](AccTile& acc) {
    bf16x8 fa1[MI], fb1[NI];
    const int next = stage == 2 ? 0 : stage + 1;
    read_frags(stage, 1, fa1, fb1);
    mma(acc, fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(stage, 2, fa0, fb0);
    mma(acc, fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(stage, 3, fa1, fb1);
    mma(acc, fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    // k-steps g, g+1, g+2 are in flight; at most the 12 loads of g+2 may still be pending
    asm volatile("s_waitcnt vmcnt(12) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    issue_loads(stage);
    read_frags(next, 0, fa0, fb0);
    mma(acc, fa1, fb1);
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
      __builtin_amdgcn_sched_group_barrier(SG_DSREAD, 2, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
      __builtin_amdgcn_sched_group_barrier(SG_VMEM, 3, 0);
    }
    __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
    __builtin_amdgcn_sched_barrier(0);
    advance();
    stage = next;
  };

  // ---- prologue: three k-steps in flight, first fragments read ------------------------------
  issue_loads(0);
  advance();
  issue_loads(1);
  advance();
  issue_loads(2);
  advance();
  asm volatile("s_waitcnt vmcnt(24)\n\ts_barrier" ::: "memory");
  read_frags(0, 0, fa0, fb0);

  for (int c_item = 0; c_item < n_items; ++c_item) {
    const WorkItem ci = work.item(c_item);
    epi.begin_item(ci);
    for (int k = 0; k < ci.nk0; ++k) kstep(acc0);
    if (NPHASE > 1)
      for (int k = 0; k < ci.nk1; ++k) kstep(acc1);
    epi.end_item(ci, acc0, acc1);
    zero_acc(acc0);
    if (NPHASE > 1) zero_acc(acc1);
  }
  // the loads issued past the end still target this workgroup's LDS: let them land
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

}  // namespace kd
