// Same-wave instruction mixes around v_mfma_f32_32x32x16_bf16: what one tile of the attention loop issues, added component
// by component, at 1 to 4 waves per SIMD.  Prints time and shader clock (s_memtime against the 100 MHz wall clock), so cycles
// per matrix-instruction slot and the matrix pipe's share of them.  All operands are constants: the chip draws less power
// than under real data and holds a higher clock than the attention kernels get.
// Build and run:  hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops tile_loop_mix.hip -o tile_loop_mix && ./tile_loop_mix
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define MFMA(ACC) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(ACC) : "v"(a), "v"(b))
#define FMA(X) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(X) : "v"(c1), "v"(c2))
#define EXP(X) asm volatile("v_exp_f32 %0, %0" : "+v"(X))
#define RCP(X) asm volatile("v_rcp_f32 %0, %0" : "+v"(X))
#define CVT(X, Y) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(X) : "v"(Y))

// flags
enum { F_WAIT = 512, F_T = 1, F_P = 2, F_CVT = 4, F_LDS = 8, F_TR = 16, F_DMA = 32, F_BAR = 64, F_XOR = 128, F_SALU = 256 };

// one "tile" = 16 slots; per slot: 1 matrix instruction, NT transcendental + NP plain VALU (alternating), every 2nd slot a cvt,
// NL ds_read_b128 per 4 slots... all independent of each other; barrier and a wait for the DMA once per tile.
template <int FL, int NT, int NP, int NS = 0>
__global__ __launch_bounds__(512) void k(float* out, const float* gsrc, int tiles, float c1, float c2) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  for (int i = threadIdx.x; i < 8192; i += blockDim.x) ((float*)lds)[i] = i;   // 32 KB read area; 16 KB behind it receive the loads
  __syncthreads();
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x + i); b[i] = (__bf16)(float)(i); }
  f32x16 acc[4];
  for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  float v[8];
  for (int i = 0; i < 8; ++i) v[i] = threadIdx.x * 0.001f + i;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lds0 = (int)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  int lp = lds0 + lane * 16;                                            // conflict-free 16-byte reads
  // transpose reads: 16 lanes cover 4 rows x 64 B of a 256-byte-row tile, swizzled so that rows fall on different banks
  const int i16 = lane & 15, grp = lane >> 4;
  int tp = lds0 + ((grp * 4 + (i16 >> 2)) * 256 + (((i16 & 3) * 8) ^ ((i16 >> 2) << 6)));
  int xr = lane * 4;
  i32x4 rs = {(int)(uint32_t)(uintptr_t)gsrc, (int)((uint64_t)(uintptr_t)gsrc >> 32), 1 << 20, 0x00020000};
  uint32_t voff = lane * 16 + wave * 1024 + blockIdx.x % 64 * 8192;
  f32x4 l[4] = {};
  s16x4 tr[4] = {};
  int sreg[4] = {tiles, tiles + 1, tiles + 2, tiles + 3};
  const long long t0 = clock64(); const unsigned long long r0 = wall_clock64();
  for (int it = 0; it < tiles; ++it) {
#pragma unroll
    for (int sl = 0; sl < 16; ++sl) {
      MFMA(acc[sl & 3]);
      if constexpr (FL & F_T) { EXP(v[0]); if (NT > 1) RCP(v[1]); if (NT > 2) EXP(v[2]); if (NT > 3) RCP(v[3]); }
      if constexpr (FL & F_P) { FMA(v[4]); if (NP > 1) FMA(v[5]); if (NP > 2) FMA(v[6]); if (NP > 3) FMA(v[7]); if (NP > 4) FMA(v[4]); if (NP > 5) FMA(v[5]); if (NP > 6) FMA(v[6]); if (NP > 7) FMA(v[7]); }
      if constexpr (FL & F_CVT) { if (sl & 1) CVT(v[6], v[7]); }
      if constexpr (FL & F_XOR) { asm volatile("v_xor_b32 %0, %0, %1" : "+v"(xr) : "v"(lane)); }
      if constexpr (FL & F_LDS) {                                     // 12 b128 per tile
        if ((sl & 3) != 3) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(l[sl & 3]) : "v"(lp), "n"((sl & 7) * 1024));
      }
      if constexpr (FL & F_TR) {                                      // 16 transpose reads per tile
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(tr[sl & 3]) : "v"(tp), "n"((sl & 7) * 4096));
      }
      if constexpr (FL & F_DMA) {                                     // 8 loads straight to LDS per tile
        if (sl & 1) {
          const uint32_t dst = (uint32_t)lds0 + 32768u + (wave * 2 + ((sl >> 1) & 1)) * 1024u;
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" :: "s"(dst), "v"(voff), "s"(rs) : "memory", "m0");
        }
      }
      if constexpr (FL & F_SALU) {
#pragma unroll
        for (int q = 0; q < NS; ++q) asm volatile("s_add_u32 %0, %0, 3" : "+s"(sreg[q & 3]) :: "scc");
      }
      if constexpr (FL & F_WAIT) {
#pragma unroll
        for (int q = 0; q < NS; ++q) asm volatile("s_nop 0");
      }
    }
    if constexpr ((FL & F_LDS) || (FL & F_TR)) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if constexpr (FL & F_BAR) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  const long long t1 = clock64(); const unsigned long long r1 = wall_clock64();
  float sum = 0; for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) sum += acc[j][i];
  for (int i = 0; i < 8; ++i) sum += v[i];
  for (int i = 0; i < 4; ++i) sum += l[i][0] + l[i][3] + tr[i][0];
  out[blockIdx.x * blockDim.x + threadIdx.x] = sum + xr + sreg[0] + sreg[1] + sreg[2] + sreg[3];
  if (threadIdx.x == 0 && blockIdx.x == 0) { ((long long*)(out + 256 * 1024))[0] = t1 - t0; ((long long*)(out + 256 * 1024))[1] = (long long)(r1 - r0); }
}
static float* g_d; static float* g_src;
template <int FL, int NT, int NP, int NS = 0> void run(int wps, int wgs, const char* tag) {
  const int tiles = 4000;
  const int lds_bytes = wgs == 1 ? 140 * 1024 : (wgs == 2 ? 76 * 1024 : 50 * 1024);   // forces `wgs` workgroups per compute unit
  const int threads = 256 * wps / wgs;
  hipFuncSetAttribute((const void*)k<FL, NT, NP, NS>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  hipLaunchKernelGGL((k<FL, NT, NP, NS>), dim3(256 * wgs), dim3(threads), lds_bytes, 0, g_d, g_src, 100, 1.0001f, 0.5f);
  hipDeviceSynchronize();
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  hipEventRecord(e0);
  hipLaunchKernelGGL((k<FL, NT, NP, NS>), dim3(256 * wgs), dim3(threads), lds_bytes, 0, g_d, g_src, tiles, 1.0001f, 0.5f);
  hipEventRecord(e1); hipDeviceSynchronize();
  float ms; hipEventElapsedTime(&ms, e0, e1);
  long long tt[2]; hipMemcpy(tt, g_d + 256 * 1024, 16, hipMemcpyDeviceToHost);
  const double ghz = tt[0] / (tt[1] * 10.0);
  const double slots = (double)wps * tiles * 16;
  printf("wps=%d wgs=%d %-44s : %7.3f ms %6.2f ns/slot %5.2f GHz %6.1f cyc/slot  matrix-pipe %4.1f %%\n", wps, wgs, tag, ms, ms * 1e6 / slots, ghz,
         ms * 1e6 / slots * ghz, 100.0 * 32.0 / (ms * 1e6 / slots * ghz));
  fflush(stdout);
}
int main() {
  hipMalloc(&g_d, 256 * 1024 * 4 + 64); hipMalloc(&g_src, 1 << 20); hipMemset(g_src, 0, 1 << 20);
  const int cfgs[4][2] = {{1, 1}, {2, 2}, {3, 3}, {4, 2}};
  for (int cfg = 0; cfg < 4; ++cfg) {
    const int wps = cfgs[cfg][0], wgs = cfgs[cfg][1];
    printf("---- %d waves per SIMD in %d workgroups per compute unit\n", wps, wgs);
    run<0, 0, 0>(wps, wgs, "matrix instructions only");
    run<F_T | F_P, 2, 2>(wps, wgs, "+ SiLU (exp, fma, rcp, fma)");
    run<F_T | F_P | F_CVT, 2, 2>(wps, wgs, "+ SiLU + cvt/2");
    run<F_T | F_P | F_CVT | F_LDS, 2, 2>(wps, wgs, "+ SiLU + cvt/2 + 12 ds_read_b128");
    run<F_T | F_P | F_CVT | F_LDS | F_TR, 2, 2>(wps, wgs, "+ SiLU + cvt/2 + LDS reads (b128, tr)");
    run<F_T | F_P | F_CVT | F_LDS | F_TR | F_DMA, 2, 2>(wps, wgs, "+ ... + 8 loads to LDS");
    run<F_T | F_P | F_CVT | F_LDS | F_TR | F_DMA | F_BAR, 2, 2>(wps, wgs, "forward mix (... + wait + barrier per tile)");
    run<F_T | F_P | F_CVT | F_SALU, 2, 2, 2>(wps, wgs, "SiLU + cvt/2 + 2 salu per slot");
    run<F_T | F_P | F_CVT | F_SALU, 2, 2, 4>(wps, wgs, "SiLU + cvt/2 + 4 salu per slot");
    run<F_T | F_P | F_CVT | F_WAIT, 2, 2, 4>(wps, wgs, "SiLU + cvt/2 + 4 s_nop per slot");
    run<F_T | F_P | F_CVT | F_LDS | F_TR | F_DMA | F_BAR | F_SALU, 2, 2, 4>(wps, wgs, "forward mix + 4 salu per slot");
  }
  return 0;
}
