// Stand-alone probe, not part of libwildcat: how fast one, two and four wavefronts per SIMD of a gfx950 compute unit
// issue vector, transcendental, scalar and MFMA instructions, alone and in fixed mixes (no memory traffic).  The
// WtdAttn kernel's instruction budget per MFMA is derived from these figures.  Every loop is a fixed number of
// iterations over registers; the only memory written is one clock count per wave.
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops paper_2602_10056_amd/csrc/probe_issue_rates.hip -o probe_issue_rates
// Output per line: s_memtime ticks (core clocks) per unit of ONE wave, and wall time per unit over the launch.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)

template <int MODE, int NT = 256>
__global__ __launch_bounds__(NT, 1) void k(unsigned long long *clk, float *sink, int iters) {
  float x[8];
  for (int i = 0; i < 8; ++i) x[i] = 0.001f * (threadIdx.x + i);
  floatx16 acc[4] = {};
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(0.01f * i); b[i] = (__bf16)(0.02f * i); }
  const unsigned long long t0 = __builtin_amdgcn_s_memtime();
  for (int it = 0; it < iters; ++it) {
    if (MODE == 0) {            // 8 exp
#pragma unroll
      for (int i = 0; i < 8; ++i) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
    } else if (MODE == 1) {     // 8 fma
#pragma unroll
      for (int i = 0; i < 8; ++i) asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[i]));
    } else if (MODE == 2) {     // 4 mfma
#pragma unroll
      for (int i = 0; i < 4; ++i) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[i]) : "v"(a), "v"(b));
    } else if (MODE == 3) {     // 4 x (mfma + 6 fma)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[i]) : "v"(a), "v"(b));
#pragma unroll
        for (int j = 0; j < 6; ++j) asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[j]));
      }
    } else if (MODE == 4) {     // 4 x (mfma + 1 exp + 2 fma)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[i]) : "v"(a), "v"(b));
        asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
        asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[4]));
        asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[5]));
      }
    } else if (MODE == 5) {     // 4 x (mfma + 2 exp + 3 fma)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[i]) : "v"(a), "v"(b));
        asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
        asm volatile("v_exp_f32 %0, %0" : "+v"(x[i + 4]));
        asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[(i + 1) % 4]));
        asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[(i + 2) % 4]));
        asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[(i + 3) % 4]));
      }
    } else if (MODE == 6) {     // 8 s_nop 0 (scalar issue cost)
#pragma unroll
      for (int i = 0; i < 8; ++i) asm volatile("s_nop 0");
    } else if (MODE == 7) {     // 4 x (mfma + 7 s_nop)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[i]) : "v"(a), "v"(b));
#pragma unroll
        for (int j = 0; j < 7; ++j) asm volatile("s_nop 0");
      }
    } else if (MODE == 8) {     // 8 cvt_pkrtz
#pragma unroll
      for (int i = 0; i < 8; ++i) asm volatile("v_cvt_pkrtz_f16_f32 %0, %0, %0" : "+v"(x[i]));
    } else if (MODE == 9) {     // 8 max3
#pragma unroll
      for (int i = 0; i < 8; ++i) asm volatile("v_max3_f32 %0, %0, %0, %0" : "+v"(x[i]));
    }
  }
  const unsigned long long t1 = __builtin_amdgcn_s_memtime();
  float s = 0;
  for (int i = 0; i < 8; ++i) s += x[i];
  for (int i = 0; i < 4; ++i) s += acc[i][0] + acc[i][7];
  if (threadIdx.x % 64 == 0 && threadIdx.x < 256) clk[blockIdx.x * 4 + threadIdx.x / 64] = t1 - t0;
  if (s == 12345.678f) sink[0] = s;
}

template <int MODE, int NT = 256>
int run(const char *name, int per_iter_units, unsigned long long *dclk, float *dsink, int grid) {
  const int iters = 20000;
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  hipLaunchKernelGGL((k<MODE, NT>), dim3(grid), dim3(NT), 0, 0, dclk, dsink, 100);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  hipLaunchKernelGGL((k<MODE, NT>), dim3(grid), dim3(NT), 0, 0, dclk, dsink, iters);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  std::vector<unsigned long long> h(grid * 4);
  CK(hipMemcpy(h.data(), dclk, sizeof(unsigned long long) * grid * 4, hipMemcpyDeviceToHost));
  double mean = 0; for (auto v : h) mean += (double)v; mean /= h.size();
  printf("%-28s grid %4d: %8.2f s_memtime ticks per unit, %8.3f ns per unit (wall), %6.3f ms\n", name, grid,
         mean / iters / per_iter_units, ms * 1e6 / iters / per_iter_units, ms);
  return 0;
}

int main() {
  unsigned long long *dclk; float *dsink;
  CK(hipMalloc(&dclk, sizeof(unsigned long long) * 1024 * 4)); CK(hipMalloc(&dsink, 4));
  printf("--- two waves per SIMD (512 threads); ticks are per unit of ONE wave ---\n");
  if (run<1, 512>("2w: v_fma_f32", 8, dclk, dsink, 256)) return 1;
  if (run<0, 512>("2w: v_exp_f32", 8, dclk, dsink, 256)) return 1;
  if (run<2, 512>("2w: mfma", 4, dclk, dsink, 256)) return 1;
  if (run<3, 512>("2w: mfma + 6 fma", 4, dclk, dsink, 256)) return 1;
  if (run<5, 512>("2w: mfma + 2 exp + 3 fma", 4, dclk, dsink, 256)) return 1;
  if (run<7, 512>("2w: mfma + 7 s_nop", 4, dclk, dsink, 256)) return 1;
  printf("--- four waves per SIMD (1024 threads) ---\n");
  if (run<1, 1024>("4w: v_fma_f32", 8, dclk, dsink, 256)) return 1;
  if (run<0, 1024>("4w: v_exp_f32", 8, dclk, dsink, 256)) return 1;
  if (run<3, 1024>("4w: mfma + 6 fma", 4, dclk, dsink, 256)) return 1;
  if (run<5, 1024>("4w: mfma + 2 exp + 3 fma", 4, dclk, dsink, 256)) return 1;
  for (int grid : {256}) {
    if (run<0>("v_exp_f32", 8, dclk, dsink, grid)) return 1;
    if (run<1>("v_fma_f32", 8, dclk, dsink, grid)) return 1;
    if (run<8>("v_cvt_pkrtz", 8, dclk, dsink, grid)) return 1;
    if (run<9>("v_max3_f32", 8, dclk, dsink, grid)) return 1;
    if (run<6>("s_nop 0", 8, dclk, dsink, grid)) return 1;
    if (run<2>("mfma 32x32x16 bf16", 4, dclk, dsink, grid)) return 1;
    if (run<3>("mfma + 6 fma", 4, dclk, dsink, grid)) return 1;
    if (run<7>("mfma + 7 s_nop", 4, dclk, dsink, grid)) return 1;
    if (run<4>("mfma + exp + 2 fma", 4, dclk, dsink, grid)) return 1;
    if (run<5>("mfma + 2 exp + 3 fma", 4, dclk, dsink, grid)) return 1;
  }
  return 0;
}
