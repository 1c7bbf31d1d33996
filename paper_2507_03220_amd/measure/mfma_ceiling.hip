// Stand-alone measurement, not part of the library: sustained bf16 MFMA rate of the whole chip
// with N(0,1) operand data held in registers (no memory traffic at all).  On a power-limited
// part this, not the nominal peak, is what a GEMM's matrix pipes can reach.
// Build: python -m paper_2507_03220_amd.build --ceiling   Run: paper_2507_03220_amd/mfma_ceiling
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <vector>
#include <random>
#include <cstring>
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1;}}while(0)

__global__ void __launch_bounds__(512) mfma_rand(const bf16x8* __restrict__ src, float* out, int iters, unsigned long long* clk) {
  unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  floatx16 acc[8];
  for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8 a[4], b[2];
  for (int i = 0; i < 4; ++i) a[i] = src[(blockIdx.x * 6 + i) * 512 + threadIdx.x];
  for (int i = 0; i < 2; ++i) b[i] = src[(blockIdx.x * 6 + 4 + i) * 512 + threadIdx.x];
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i * 2 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i * 2 + j], 0, 0, 0);
    // rotate operands so successive MFMAs see different data
    bf16x8 t = a[0]; a[0] = a[1]; a[1] = a[2]; a[2] = a[3]; a[3] = t;
  }
  float s = 0; for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
  unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0) { clk[blockIdx.x * 2] = c1 - c0; clk[blockIdx.x * 2 + 1] = r1 - r0; }
}

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
// the same flops through v_mfma_f32_16x16x32_bf16: 32 independent 16x16 accumulators per wavefront
__global__ void __launch_bounds__(512) mfma_rand16(const bf16x8* __restrict__ src, float* out, int iters, unsigned long long* clk) {
  unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  floatx4 acc[32];
  for (int i = 0; i < 32; ++i) for (int r = 0; r < 4; ++r) acc[i][r] = 0.f;
  bf16x8 a[8], b[4];
  for (int i = 0; i < 8; ++i) a[i] = src[(blockIdx.x * 6 + (i % 4)) * 512 + (threadIdx.x + 37 * (i / 4)) % 512];
  for (int i = 0; i < 4; ++i) b[i] = src[(blockIdx.x * 6 + 4 + (i % 2)) * 512 + (threadIdx.x + 91 * (i / 2)) % 512];
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i * 4 + j], 0, 0, 0);
    bf16x8 t = a[0];
#pragma unroll
    for (int i = 0; i < 7; ++i) a[i] = a[i + 1];
    a[7] = t;
  }
  float s = 0; for (int i = 0; i < 32; ++i) for (int r = 0; r < 4; ++r) s += acc[i][r];
  unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0) { clk[blockIdx.x * 2] = c1 - c0; clk[blockIdx.x * 2 + 1] = r1 - r0; }
}

int main(int argc, char** argv) {
  const bool constant = argc > 1 && !strcmp(argv[1], "--constant");   // all operands 1.0: few toggling bits
  const size_t n = 256 * 6 * 512 * 8;
  std::vector<uint16_t> h(n);
  std::mt19937 g(1); std::normal_distribution<float> nd(0.f, 1.f);
  for (auto& v : h) { float f = constant ? 1.f : nd(g); uint32_t u; memcpy(&u, &f, 4); v = (uint16_t)(u >> 16); }
  void* d; CK(hipMalloc(&d, n * 2)); CK(hipMemcpy(d, h.data(), n * 2, hipMemcpyHostToDevice));
  float* out; CK(hipMalloc(&out, 4 << 20)); unsigned long long* clk; CK(hipMalloc(&clk, 4096)); unsigned long long hc[512];
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms;
  for (int iters : {20000, 100000, 400000}) {
    CK(hipEventRecord(e0)); mfma_rand<<<256, 512>>>((const bf16x8*)d, out, iters, clk); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    double fl = 256.0 * 8 * iters * 8 * 32768.0;
    CK(hipMemcpy(hc, clk, 4096, hipMemcpyDeviceToHost));
    double cyc = 0, rt = 0; for (int i = 0; i < 256; ++i) { cyc += (double)hc[2 * i]; rt += (double)hc[2 * i + 1]; }
    printf("v_mfma_f32_32x32x16_bf16, %s operands in registers, 256 workgroups x 8 wavefronts, %.1f ms: %.1f TFLOP/s (%.1f%% of the 2500 TFLOP/s nominal peak); cycle counter / 100 MHz real-time counter = %.0f MHz\n",
           constant ? "constant" : "N(0,1)", ms, fl / ms / 1e9, fl / ms / 1e9 / 25.0, cyc / rt * 100.0);
  }
  // per iteration and wavefront: 32 x 16384 flops, the same as 16 of the 32x32x16 instructions
  for (int iters : {100000, 400000}) {
    CK(hipEventRecord(e0)); mfma_rand16<<<256, 512>>>((const bf16x8*)d, out, iters / 2, clk); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    double fl = 256.0 * 8 * (iters / 2) * 32 * 16384.0;
    CK(hipMemcpy(hc, clk, 4096, hipMemcpyDeviceToHost));
    double cyc = 0, rt = 0; for (int i = 0; i < 256; ++i) { cyc += (double)hc[2 * i]; rt += (double)hc[2 * i + 1]; }
    printf("v_mfma_f32_16x16x32_bf16, %s operands in registers, 256 workgroups x 8 wavefronts, %.1f ms: %.1f TFLOP/s (%.1f%% of the 2500 TFLOP/s nominal peak); cycle counter / 100 MHz real-time counter = %.0f MHz\n",
           constant ? "constant" : "N(0,1)", ms, fl / ms / 1e9, fl / ms / 1e9 / 25.0, cyc / rt * 100.0);
  }
  return 0;
}
