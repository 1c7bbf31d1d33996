// Stand-alone measurement, not part of the library: rate at which direct global->LDS loads
// (global_load_lds_dwordx4) bring operand tiles from L2 into LDS, by request size.  The L2 serves
// one request per channel and clock whatever its size, so a K-contiguous operand fetched as 64-byte
// row pieces costs twice the L2 cycles of whole 128-byte lines; this is why the GEMM main loop
// works on 64-k stages.
// Build: python -m paper_2507_03220_amd.build --l2-probe   Run: paper_2507_03220_amd/l2_lds_probe
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <vector>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1;}}while(0)
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;
typedef unsigned short bf16;

template <int BK, int INFL, int PAIR, int WALK>
__global__ void __launch_bounds__(256) dtl(const bf16* __restrict__ A, const bf16* __restrict__ B, int M, int N, int K,
                                           int nmt, int nnt, int group_m, unsigned* sink) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int total = nmt * nnt, per_xcd = (total + 7) >> 3;
  const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lin >= total || (int)(blockIdx.x >> 3) >= per_xcd) return;
  int tm, tn;
  if (WALK == 0) {
    const int width = group_m * nnt, first_m = (lin / width) * group_m, gsz = min(nmt - first_m, group_m);
    tm = first_m + (lin % width) % gsz; tn = (lin % width) / gsz;
  } else {
    // chip-level super-tiles of 16x16 tiles; XCD x owns the 8x4 block (x&1, x>>1) of each
    const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3, r = k >> 5, q = k & 31;
    const int sn = nnt / 16, sr = r / sn, sc = r % sn;
    tm = sr * 16 + (xcd & 1) * 8 + (q & 7); tn = sc * 16 + (xcd >> 1) * 4 + (q >> 3);
    if (WALK == 2) { tm = sr * 16 + (xcd & 1) * 8 + (q >> 2); tn = sc * 16 + (xcd >> 1) * 4 + (q & 3); }
    if (tm >= nmt || tn >= nnt) return;
  }
  const int m0 = tm * 256, n0 = tn * 256;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int RPI = 1024 / (BK * 2), LPR = BK * 2 / 16, AI = 256 / RPI / 4;
  constexpr int STAGE = 512 * BK * 2, NS = 131072 / STAGE;
  unsigned a_off[AI], b_off[AI];
#pragma unroll
  for (int j = 0; j < AI; ++j) {
    const int row = (wave * AI + j) * RPI + lane / LPR;
    a_off[j] = (unsigned)row * (unsigned)K + (lane % LPR) * 8;
    b_off[j] = a_off[j];
  }
  const bf16* at = A + (size_t)m0 * K;
  const bf16* bt = B + (size_t)n0 * K;
  const int KS = K / BK;
  if (PAIR == 0) {
    for (int s = 0; s < KS; ++s) {
      unsigned char* sa = smem + (s % NS) * STAGE;
      unsigned char* sb = sa + STAGE / 2;
#pragma unroll
      for (int j = 0; j < AI; ++j)
        __builtin_amdgcn_global_load_lds((glb_void_t*)(at + a_off[j]), (lds_void_t*)(sa + (wave * AI + j) * 1024), 16, 0, 0);
#pragma unroll
      for (int j = 0; j < AI; ++j)
        __builtin_amdgcn_global_load_lds((glb_void_t*)(bt + b_off[j]), (lds_void_t*)(sb + (wave * AI + j) * 1024), 16, 0, 0);
      at += BK; bt += BK;
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(INFL));
    }
  } else {
    // two 32-k stages at a time: both 64-byte halves of each line requested back to back
    for (int s = 0; s < KS; s += 2) {
      unsigned char* sa0 = smem + (s % NS) * STAGE;
      unsigned char* sa1 = smem + ((s + 1) % NS) * STAGE;
#pragma unroll
      for (int j = 0; j < AI; ++j) {
        __builtin_amdgcn_global_load_lds((glb_void_t*)(at + a_off[j]), (lds_void_t*)(sa0 + (wave * AI + j) * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((glb_void_t*)(at + a_off[j] + BK), (lds_void_t*)(sa1 + (wave * AI + j) * 1024), 16, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < AI; ++j) {
        __builtin_amdgcn_global_load_lds((glb_void_t*)(bt + b_off[j]), (lds_void_t*)(sa0 + STAGE / 2 + (wave * AI + j) * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((glb_void_t*)(bt + b_off[j] + BK), (lds_void_t*)(sa1 + STAGE / 2 + (wave * AI + j) * 1024), 16, 0, 0);
      }
      at += 2 * BK; bt += 2 * BK;
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(INFL));
    }
  }
  asm volatile("s_waitcnt vmcnt(0)");
  __syncthreads();
  if (threadIdx.x == 0) sink[lin] = *(unsigned*)(smem + 4 * (lin & 1023));
}

// every workgroup streams the same L2-resident tile pair (rows 0..255 of A and B, K2 k), `reps` times
template <int BK, int INFL>
__global__ void __launch_bounds__(256) dtl_res(const bf16* __restrict__ A, const bf16* __restrict__ B, int K, int K2, int reps, unsigned* sink) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int RPI = 1024 / (BK * 2), LPR = BK * 2 / 16, AI = 256 / RPI / 4;
  constexpr int STAGE = 512 * BK * 2, NS = 131072 / STAGE;
  unsigned a_off[AI];
#pragma unroll
  for (int j = 0; j < AI; ++j) a_off[j] = (unsigned)((wave * AI + j) * RPI + lane / LPR) * (unsigned)K + (lane % LPR) * 8;
  const int KS = K2 / BK;
  for (int r = 0; r < reps; ++r) {
    const bf16* at = A; const bf16* bt = B;
    for (int s = 0; s < KS; ++s) {
      unsigned char* sa = smem + (s % NS) * STAGE;
      unsigned char* sb = sa + STAGE / 2;
#pragma unroll
      for (int j = 0; j < AI; ++j)
        __builtin_amdgcn_global_load_lds((glb_void_t*)(at + a_off[j]), (lds_void_t*)(sa + (wave * AI + j) * 1024), 16, 0, 0);
#pragma unroll
      for (int j = 0; j < AI; ++j)
        __builtin_amdgcn_global_load_lds((glb_void_t*)(bt + a_off[j]), (lds_void_t*)(sb + (wave * AI + j) * 1024), 16, 0, 0);
      at += BK; bt += BK;
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(INFL));
    }
  }
  asm volatile("s_waitcnt vmcnt(0)");
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = *(unsigned*)(smem + 4 * (blockIdx.x & 1023));
}

template <int BK, int INFL>
int run_res(const char* name, const bf16* A, const bf16* B, int K, int K2, int wgs, unsigned* sink) {
  auto kern = dtl_res<BK, INFL>;
  CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  const int reps = 40; float best = 1e9f;
  for (int it = 0; it < 3; ++it) {
    CK(hipEventRecord(e0));
    kern<<<wgs, 256, 131072>>>(A, B, K, K2, reps, sink);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1)); if (it > 0 && ms < best) best = ms;
  }
  CK(hipGetLastError());
  const double bytes = (double)wgs * reps * (K2 / 32) * 32768.0;
  printf("%-36s %4d workgroups %7.3f ms  %6.2f TB/s  %.1f B/clk/CU at 2.4 GHz\n", name, wgs, best, bytes / best / 1e9, bytes / best / 1e-3 / wgs / 2.4e9);
  return 0;
}

template <int BK, int INFL, int PAIR, int WALK>
int run(const char* name, const bf16* A, const bf16* B, int M, int N, int K, unsigned* sink) {
  auto kern = dtl<BK, INFL, PAIR, WALK>;
  CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
  const int nmt = M / 256, nnt = N / 256, total = nmt * nnt, per = (total + 7) / 8;
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float best = 1e9f;
  for (int it = 0; it < 4; ++it) {
    CK(hipEventRecord(e0));
    kern<<<per * 8, 256, 131072>>>(A, B, M, N, K, nmt, nnt, 8, sink);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1)); if (it > 0 && ms < best) best = ms;
  }
  CK(hipGetLastError());
  const double bytes = (double)total * (double)(K / 32) * 32768.0;
  printf("%-44s %7.3f ms  %6.2f TB/s into LDS  (%.1f B/clk/CU at 2.4 GHz; per tile %.1f us)\n", name, best, bytes / best / 1e9,
         bytes / best / 1e-3 / 256 / 2.4e9, best * 1e3 / ((total + 255) / 256));
  return 0;
}

int main() {
  const int M = 20480, N = 36864, K = 4608;
  bf16 *A, *B; unsigned* sink;
  CK(hipMalloc(&A, (size_t)M * K * 2)); CK(hipMalloc(&B, (size_t)N * K * 2)); CK(hipMalloc(&sink, 1 << 20));
  CK(hipMemset(A, 0x3c, (size_t)M * K * 2)); CK(hipMemset(B, 0x3c, (size_t)N * K * 2));
  printf("-- the GEMM's own tile walk over X [20480][4608] and W [36864][4608], loads only\n");
  if (run<32, 24, 0, 0>("64-byte row pieces (32-k stages)", A, B, M, N, K, sink)) return 1;
  if (run<64, 16, 0, 0>("whole 128-byte lines (64-k stages)", A, B, M, N, K, sink)) return 1;
  if (run<32, 16, 1, 0>("64-byte pieces, both halves of a line back to back", A, B, M, N, K, sink)) return 1;
  if (run<64, 16, 0, 1>("whole lines, chip-level 16x16 super-tiles", A, B, M, N, K, sink)) return 1;
  printf("-- every workgroup streams the same L2-resident 1.2 MB, by number of workgroups (one per CU)\n");
  for (int wgs : {8, 64, 256}) {
    if (run_res<32, 24>("64-byte row pieces", A, B, K, 1152, wgs, sink)) return 1;
    if (run_res<64, 16>("whole 128-byte lines", A, B, K, 1152, wgs, sink)) return 1;
  }
  return 0;
}
