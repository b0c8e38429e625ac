// LDS read throughput of the access patterns of the attention kernels (no matrix work): cycles per wave-level instruction per SIMD.
// Build and run:  hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops lds_patterns.hip -o lds_patterns && ./lds_patterns
#include <hip/hip_runtime.h>
#include <cstdio>
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
// PAT 0: ds_read_b128 contiguous (lane * 16).  1: row per lane (l32 * 256), chunk 2 ks + hf, swizzled.  2: same without swizzle.
// 3: ds_read_b64_tr_b16, swizzled tile.  4: same without swizzle.  5: bias strip pattern (4 copies 176 entries apart).
// 6: ds_read_b64 (plain) contiguous.  7: ds_read_b128 row per lane with a 272-byte padded row (no swizzle)
template <int PAT>
__global__ __launch_bounds__(512) void k(float* out, int iters) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  for (int i = threadIdx.x; i < 16384; i += blockDim.x) ((float*)lds)[i] = i;
  __syncthreads();
  const int lane = threadIdx.x & 63, hf = lane >> 5, l32 = lane & 31, grp16 = lane >> 4, i16 = lane & 15;
  const int base = (int)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  const int zl = 4 * (l32 & 3) + ((l32 >> 2) & 3);
  int addr[8];
  for (int i = 0; i < 8; ++i) {
    if (PAT == 0) addr[i] = base + lane * 16 + i * 1024;
    else if (PAT == 1) addr[i] = base + l32 * 256 + ((((2 * i + hf) ^ zl) & 15) << 4);
    else if (PAT == 2) addr[i] = base + l32 * 256 + ((2 * i + hf) << 4);
    else if (PAT == 3 || PAT == 4) {
      const int vchunk = 2 * (grp16 & 1) + ((i16 & 3) >> 1), vbyte = 8 * (i16 & 1);
      const int row = 4 * hf + (i16 >> 2) + 8 * (i & 1), ob = i >> 1;
      const int z = PAT == 3 ? 4 * (row & 3) + ((row >> 2) & 3) : 0;
      addr[i] = base + row * 256 + ((((4 * ob + vchunk) ^ z) & 15) << 4) + vbyte;
    } else if (PAT == 5) {
      const int s0 = 127 - l32 + 4 * hf;
      addr[i] = base + 4 * ((s0 & 3) * 176 + (s0 & ~3)) + 32 * (i & 3);
    } else if (PAT == 6) addr[i] = base + lane * 8 + i * 512;
    else addr[i] = base + l32 * 272 + ((2 * i + hf) << 4);
    asm volatile("" : "+v"(addr[i]));
  }
  f32x4 acc[8] = {};
  const long long t0 = clock64(); const unsigned long long r0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (PAT == 3 || PAT == 4) { s16x4 t; asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(t) : "v"(addr[i])); asm volatile("" :: "v"(t)); }
      else if (PAT == 6) { s16x4 t; asm volatile("ds_read_b64 %0, %1" : "=v"(t) : "v"(addr[i])); asm volatile("" :: "v"(t)); }
      else asm volatile("ds_read_b128 %0, %1" : "=v"(acc[i]) : "v"(addr[i]));
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  const long long t1 = clock64(); const unsigned long long r1 = wall_clock64();
  float s = 0; for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][3];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { ((long long*)(out + 256 * 1024))[0] = t1 - t0; ((long long*)(out + 256 * 1024))[1] = (long long)(r1 - r0); }
}
static float* g_d;
template <int PAT> void run(int wps, const char* tag) {
  const int iters = 20000;
  hipFuncSetAttribute((const void*)k<PAT>, hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024);
  hipLaunchKernelGGL((k<PAT>), dim3(256), dim3(256 * wps), 100 * 1024, 0, g_d, 100);
  hipDeviceSynchronize();
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  hipEventRecord(e0);
  hipLaunchKernelGGL((k<PAT>), dim3(256), dim3(256 * wps), 100 * 1024, 0, g_d, iters);
  hipEventRecord(e1); hipDeviceSynchronize();
  float ms; hipEventElapsedTime(&ms, e0, e1);
  long long tt[2]; hipMemcpy(tt, g_d + 256 * 1024, 16, hipMemcpyDeviceToHost);
  const double ghz = tt[0] / (tt[1] * 10.0);
  const double n = (double)wps * iters * 8;
  printf("wps=%d %-52s: %6.2f ns = %5.1f cycles per instruction per SIMD (%.2f GHz)\n", wps, tag, ms * 1e6 / n, ms * 1e6 / n * ghz, ghz);
}
int main() {
  hipMalloc(&g_d, 256 * 1024 * 4 + 64);
  for (int wps = 1; wps <= 2; ++wps) {
    run<0>(wps, "ds_read_b128 contiguous");
    run<1>(wps, "ds_read_b128 row per lane, swizzled (K fragments)");
    run<2>(wps, "ds_read_b128 row per lane, no swizzle");
    run<7>(wps, "ds_read_b128 row per lane, 272-byte rows");
    run<3>(wps, "ds_read_b64_tr_b16 swizzled (V fragments)");
    run<4>(wps, "ds_read_b64_tr_b16 no swizzle");
    run<5>(wps, "ds_read_b128 bias strip");
    run<6>(wps, "ds_read_b64 contiguous");
  }
  return 0;
}
