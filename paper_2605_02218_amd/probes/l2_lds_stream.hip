// Stand-alone probe (not part of the library):
//   hipcc --offload-arch=gfx950 -O3 paper_2605_02218_amd/probes/l2_lds_stream.hip -o /tmp/l2_lds_stream && /tmp/l2_lds_stream
// L2 -> LDS streaming rate of global_load_lds (16 B per lane) by row-segment width.
// Every address is base + (offset & (bytes-1)): in bounds by construction.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

// SEG = bytes of one row segment covered by consecutive lanes (64 or 128); pitch = row pitch in bytes
template <int SEG>
__global__ __launch_bounds__(256) void stream_kernel(const unsigned char* base, unsigned long mask, long pitch, int iters, int rows_per_wg, float* sink) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // 4 x 32 KB
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int LPR = SEG / 16;            // lanes per row
  constexpr int RPI = 64 / LPR;            // rows per instruction
  // a WG walks over `rows_per_wg` rows starting at its own row block, along k
  const long row0 = (long)blockIdx.x * rows_per_wg;
  for (int it = 0; it < iters; ++it) {
    unsigned char* st = smem + (it & 3) * 32768 + wave * 8192;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const long row = row0 + ((wave * 8 + j) * RPI + lane / LPR) % rows_per_wg;
      const unsigned long off = ((unsigned long)(row * pitch + (long)it * SEG + (lane % LPR) * 16)) & mask & ~15ul;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + off),
                                       (__attribute__((address_space(3))) void*)(st + j * 1024), 16, 0, 0);
    }
    if ((it & 3) == 3) { __builtin_amdgcn_s_waitcnt(0x0078); }   // keep ~1 stage in flight
  }
  __builtin_amdgcn_s_waitcnt(0x0070);
  __syncthreads();
  if (threadIdx.x == 0 && sink) sink[blockIdx.x] = ((float*)smem)[0];
}

int main() {
  const unsigned long bytes = 1ul << 30;   // 1 GiB buffer
  unsigned char* buf; float* sink;
  CHECK(hipMalloc(&buf, bytes)); CHECK(hipMemset(buf, 1, bytes)); CHECK(hipMalloc(&sink, 4096 * 4));
  hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  CHECK(hipFuncSetAttribute((const void*)stream_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
  CHECK(hipFuncSetAttribute((const void*)stream_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
  const long pitch = 8192;   // K = 4096 bf16
  for (int fp = 0; fp < 2; ++fp) {
    // footprint: small (all WGs share 256 rows x 8 KB = 2 MB -> L2 hits) or large (each WG own rows -> HBM/MALL)
    const unsigned long mask = fp == 0 ? (1ul << 21) - 1 : bytes - 1;
    for (int seg = 64; seg <= 128; seg *= 2) {
      const int wgs = 256, rows = 256;
      const int iters = seg == 64 ? 4096 : 2048;     // same bytes: 32 KB per iteration either way
      for (int rep = 0; rep < 2; ++rep) {
        CHECK(hipEventRecord(e0));
        if (seg == 64) hipLaunchKernelGGL(stream_kernel<64>, dim3(wgs), dim3(256), 131072, 0, buf, mask, pitch, iters, rows, sink);
        else hipLaunchKernelGGL(stream_kernel<128>, dim3(wgs), dim3(256), 131072, 0, buf, mask, pitch, iters, rows, sink);
        CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
        float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
        const double gb = (double)wgs * iters * 32768 / 1e9;
        if (rep) printf("footprint %s  segment %3d B  %.3f ms  %.2f TB/s\n", fp == 0 ? "2 MB (L2)" : "1 GB      ", seg, ms, gb / ms);
      }
    }
  }
  return 0;
}
