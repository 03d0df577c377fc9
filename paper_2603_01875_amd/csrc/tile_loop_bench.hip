// Measurement aid, not part of the library: the rate of the tile loop of kd_mfma.hpp on a plain product
// D[m][n] = sum_k A[m][k] B[n][k] with ONE accumulator and no epilogue work, for a tile configuration chosen
// at compile time.  It answers "what would another tile shape buy": the logit kernels of the library keep two
// accumulators per tile and are therefore held to 128 x 256 tiles.
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -DCFG="4,2,4,32,4" tile_loop_bench.hip -o tile_loop_bench_256x256 && ./tile_loop_bench_256x256 153600 4096 4096
//
// CFG = MI, NI, WN, BK, NST (see TileCfg): tile = 64 MI x 256, 2 x WN waves, NST stages of BK elements.
// -DKD_LOOP_ABLATE=n (bit 1: no global->LDS loads, 2: no LDS fragment reads, 4: no barrier; see kd_mfma.hpp)
// takes one consumer out of the loop: what is left runs that much faster.
// Operands are N(0,1) and N(0,0.02^2) values rounded to bf16, drawn on the device (the shader clock the chip
// holds under MFMA load depends on the operand values).  The result is reduced to one number per lane and stored
// only if it matches a value it cannot have: nothing is written, nothing is checked here.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#include "kd_mfma.hpp"

#ifndef CFG
#define CFG 2, 2, 4, 64, 3
#endif
#define STR2(...) #__VA_ARGS__
#define STR(...) STR2(__VA_ARGS__)

using namespace kd;
typedef TileCfg<CFG> Cfg;

struct Args { const bf16_t* A; const bf16_t* B; float* out; long long* clocks; int K, n_mt, n_nt; };

// 8 x 4 blocks of tiles per XCD (the map of the library's backward products)
struct Work {
  const Args& a; int L, G, n_tiles;
  __device__ Work(const Args& a_) : a(a_) {
    G = gridDim.x;
    L = (G % 8 == 0) ? (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8 : blockIdx.x;
    n_tiles = a.n_mt * a.n_nt;
  }
  __device__ int n_items() const { return L < n_tiles ? (n_tiles - L + G - 1) / G : 0; }
  __device__ WorkItem item(int i) const {
    const int q = i * G + L, blk = q / 32, w = q % 32, nblk = a.n_mt / 8;
    const int mt = (blk % nblk) * 8 + w % 8, nt = (blk / nblk) * 4 + w / 8;
    WorkItem it;
    it.A0 = it.A1 = a.A + (int64_t)mt * Cfg::BM * a.K;
    it.B0 = it.B1 = a.B + (int64_t)nt * BN * a.K;
    it.a_rows = Cfg::BM; it.b_rows = BN;
    it.ka_rows = it.kb_rows = 1 << 30;
    it.nk0 = it.nk1 = a.K / Cfg::BK;
    it.m0 = mt * Cfg::BM; it.n0 = nt * BN; it.aux = 0;
    return it;
  }
};

struct SumEpi {
  const Args& a;
  __device__ SumEpi(const Args& a_) : a(a_) {}
  __device__ void begin_item(const WorkItem&) {}
  __device__ void end_item(const WorkItem&, Cfg::Acc& acc, Cfg::Acc&) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < Cfg::MI; ++i)
#pragma unroll
      for (int j = 0; j < Cfg::NI; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][j][r];
    if (s == 123.456f) a.out[threadIdx.x] = s;
  }
};

__global__ __launch_bounds__(Cfg::NT, 1) void product_kernel(const Args a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  Work w(a);
  SumEpi e(a);
  const long long c0 = clock64(), r0 = wall_clock64();
  tile_loop<1, Cfg>(w, e, a.K, a.K, a.K, a.K, smem);
  if (blockIdx.x == 0 && threadIdx.x == 0) {     // shader cycles and 100 MHz ticks of workgroup 0's loop
    a.clocks[0] = clock64() - c0;
    a.clocks[1] = wall_clock64() - r0;
  }
}

// x[i] = bf16(std * N(0,1)), from a counter-based hash and the Box-Muller transform
__global__ void fill_normal(bf16_t* x, size_t n, float std, uint32_t seed) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint32_t h = (uint32_t)i * 2654435761u ^ seed;
  h ^= h >> 16; h *= 0x7feb352du; h ^= h >> 15; h *= 0x846ca68bu; h ^= h >> 16;
  uint32_t g = h * 747796405u + 2891336453u;
  g ^= g >> 16; g *= 0x7feb352du; g ^= g >> 15;
  const float u1 = ((h >> 8) + 1) * (1.f / 16777217.f), u2 = (g >> 8) * (1.f / 16777216.f);
  x[i] = (bf16_t)(std * sqrtf(-2.f * logf(u1)) * cosf(6.2831853f * u2));
}

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

int main(int argc, char** argv) {
  const int M = argc > 1 ? atoi(argv[1]) : 153600, N = argc > 2 ? atoi(argv[2]) : 4096, K = argc > 3 ? atoi(argv[3]) : 4096;
  if (M <= 0 || N <= 0 || K <= 0 || M % (8 * Cfg::BM) || N % (4 * BN) || K % Cfg::BK) {
    printf("need M %% %d == 0, N %% %d == 0, K %% %d == 0\n", 8 * Cfg::BM, 4 * BN, Cfg::BK);
    return 2;
  }
  bf16_t *A, *B;
  float* out;
  long long* clocks;
  const size_t na = (size_t)M * K, nb = (size_t)N * K;
  HIP_OK(hipMalloc(&A, na * 2)); HIP_OK(hipMalloc(&B, nb * 2)); HIP_OK(hipMalloc(&out, 4096));
  HIP_OK(hipMalloc(&clocks, 16));
  hipLaunchKernelGGL(fill_normal, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, 0, A, na, 0.02f, 1u);
  hipLaunchKernelGGL(fill_normal, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, 0, B, nb, 1.0f, 2u);
  HIP_OK(hipDeviceSynchronize());
  Args a{A, B, out, clocks, K, M / Cfg::BM, N / BN};
  HIP_OK(hipFuncSetAttribute((const void*)product_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::SMEM_BYTES));
  hipEvent_t e0, e1;
  HIP_OK(hipEventCreate(&e0)); HIP_OK(hipEventCreate(&e1));
  for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(product_kernel, dim3(256), dim3(Cfg::NT), Cfg::SMEM_BYTES, 0, a);
  HIP_OK(hipDeviceSynchronize());
  const int reps = 10;
  HIP_OK(hipEventRecord(e0));
  for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(product_kernel, dim3(256), dim3(Cfg::NT), Cfg::SMEM_BYTES, 0, a);
  HIP_OK(hipEventRecord(e1));
  HIP_OK(hipEventSynchronize(e1));
  HIP_OK(hipGetLastError());
  float ms = 0.f;
  HIP_OK(hipEventElapsedTime(&ms, e0, e1));
  ms /= reps;
  long long hc[2] = {0, 1};
  HIP_OK(hipMemcpy(hc, clocks, 16, hipMemcpyDeviceToHost));
  const double ghz = (double)hc[0] / (double)hc[1] * 0.1;
  const double tflops = 2.0 * M * N * K / ms / 1e9;
  printf("loop ablation %d, tile cfg (MI,NI,WN,BK,NST) = %s: tile %d x %d, %d waves, %d KB LDS | M=%d N=%d K=%d: %.3f ms, %.0f TFLOP/s, shader clock %.2f GHz, MFMA busy %.2f\n",
         KD_LOOP_ABLATE, STR(CFG), Cfg::BM, BN, Cfg::NT / 64, Cfg::SMEM_BYTES / 1024, M, N, K, ms, tflops, ghz,
         tflops / (1024 * 1024 * ghz * 1e9 / 1e12));
  return 0;
}
