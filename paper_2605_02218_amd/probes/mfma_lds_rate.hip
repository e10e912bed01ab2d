// Stand-alone probe (not part of the library):
//   hipcc --offload-arch=gfx950 -O3 paper_2605_02218_amd/probes/mfma_lds_rate.hip -o /tmp/mfma_lds_rate && /tmp/mfma_lds_rate
// MFMA + LDS fragment reads with the GEMM's instruction mix (8 ds_read_b128 per 16 MFMA 32x32x16 bf16):
// effect of operand data (constant vs random bits) and of occupancy (1 or 2 workgroups per CU).
// All LDS offsets are < 64 KB; no global traffic besides the final store.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s line %d\n", hipGetErrorString(e), __LINE__); return 1;}}while(0)
template <bool LDS>
__global__ __launch_bounds__(256) void k(float* out, int iters, int random) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // first 64 KB used
  for (int i = threadIdx.x; i < 65536 / 4; i += 256) {
    unsigned h = (unsigned)i * 2654435761u; h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12;
    // two bf16 in [-2, 2): sign random, exponent 0x3f/0x40 region, mantissa random
    unsigned lo = 0x3f00u | (h & 0x80ffu), hi = 0x3f00u | ((h >> 16) & 0x80ffu);
    ((unsigned*)lds)[i] = random ? (lo | (hi << 16)) : 0x3f803f80u;
  }
  __syncthreads();
  f32x16 acc[16];
  for (int a = 0; a < 16; ++a) for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;
  const int lane = threadIdx.x & 63;
  u32x4 fa = *(const u32x4*)(lds + lane * 16);
  bf16x8 A = __builtin_bit_cast(bf16x8, fa), B = A;
  for (int it = 0; it < iters; ++it) {
    bf16x8 af[4], bf[4];
    for (int i = 0; i < 4; ++i) {
      if (LDS) {
        int r = i * 32 + (lane & 31), c = ((it & 3) * 2 + (lane >> 5));
        u32x4 t = *(const u32x4*)(lds + r * 128 + ((c ^ (r & 7)) << 4));
        u32x4 u = *(const u32x4*)(lds + 32768 + r * 128 + ((c ^ (r & 7)) << 4));
        af[i] = __builtin_bit_cast(bf16x8, t); bf[i] = __builtin_bit_cast(bf16x8, u);
      } else { af[i] = A; bf[i] = B; }
    }
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j)
      acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i * 4 + j], 0, 0, 0);
  }
  float s = 0; for (int a = 0; a < 16; ++a) for (int v = 0; v < 16; ++v) s += acc[a][v];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}
template <bool LDS> int run(const char* name, int random, size_t ldsbytes) {
  float* out; CK(hipMalloc(&out, 2048 * 256 * 4));
  int iters = 4096;
  CK(hipFuncSetAttribute((const void*)k<LDS>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  k<LDS><<<2048, 256, ldsbytes>>>(out, 16, random); CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0)); k<LDS><<<2048, 256, ldsbytes>>>(out, iters, random); CK(hipEventRecord(e1)); CK(hipDeviceSynchronize());
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  double flops = 2048.0 * 4 * iters * 16 * 32768.0;
  printf("%-64s %8.3f ms  %8.1f TFLOP/s\n", name, ms, flops / ms / 1e9);
  CK(hipFree(out));
  return 0;
}
int main() {
  run<false>("mfma only, constant operands, 2 WG/CU", 0, 65536);
  run<false>("mfma only, random operands, 2 WG/CU", 1, 65536);
  run<false>("mfma only, random operands, 1 WG/CU", 1, 131072);
  run<true>("mfma + ds_read (8 per 16), constant operands, 2 WG/CU", 0, 65536);
  run<true>("mfma + ds_read (8 per 16), random operands, 2 WG/CU", 1, 65536);
  run<true>("mfma + ds_read (8 per 16), constant operands, 1 WG/CU", 0, 131072);
  run<true>("mfma + ds_read (8 per 16), random operands, 1 WG/CU", 1, 131072);
  return 0;
}
