// Issue-rate microbenchmark: v_mfma_f32_32x32x16_bf16 against vector / transcendental / LDS / scalar instructions, in the same
// wave (mode 0) and in different waves of one SIMD (mode 1), at 1 to 4 waves per SIMD.
// Build and run:  hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops issue_rates.hip -o issue_rates && ./issue_rates
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define MFMA(ACC) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(ACC) : "v"(a), "v"(b))
#define FMA(X) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(X) : "v"(c1), "v"(c2))
#define MUL(X) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(X) : "v"(c1))
#define EXP(X) asm volatile("v_exp_f32 %0, %0" : "+v"(X))
#define RCP(X) asm volatile("v_rcp_f32 %0, %0" : "+v"(X))
#define CVT(X, Y) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(X) : "v"(Y))
#define XOR(X) asm volatile("v_xor_b32 %0, %0, %1" : "+v"(X) : "v"(c1))
#define SAL(X) asm volatile("s_add_u32 %0, %0, 3" : "+s"(X))
#define LDS128(X, P) asm volatile("ds_read_b128 %0, %1" : "=v"(X) : "v"(P))
#define LDSTR(X, P) asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(X) : "v"(P))

// KIND of the filler: 0 fma, 1 exp, 2 rcp, 3 mul, 4 cvt_pk, 5 xor, 6 salu, 7 lds128, 8 ldstr, 9 silu mix (exp,fma,rcp,mul)
template <int KIND, int I>
__device__ __forceinline__ void filler(float (&v)[8], float c1, float c2, int& s, f32x4 (&l)[4], int lp) {
  float& x = v[I % 8];
  if constexpr (KIND == 0) FMA(x);
  else if constexpr (KIND == 1) EXP(x);
  else if constexpr (KIND == 2) RCP(x);
  else if constexpr (KIND == 3) MUL(x);
  else if constexpr (KIND == 4) CVT(x, v[(I + 1) % 8]);
  else if constexpr (KIND == 5) XOR(x);
  else if constexpr (KIND == 6) SAL(s);
  else if constexpr (KIND == 7) { LDS128(l[I % 4], lp); }
  else if constexpr (KIND == 8) { typedef short s4 __attribute__((ext_vector_type(4))); s4 t; LDSTR(t, lp); asm volatile("" :: "v"(t)); }
  else if constexpr (KIND == 9) {
    if constexpr (I % 4 == 0) EXP(x); else if constexpr (I % 4 == 1) FMA(x); else if constexpr (I % 4 == 2) RCP(x); else MUL(x);
  }
}
template <int KIND, int N, int I = 0>
__device__ __forceinline__ void fillers(float (&v)[8], float c1, float c2, int& s, f32x4 (&l)[4], int lp) {
  if constexpr (I < N) { filler<KIND, I>(v, c1, c2, s, l, lp); fillers<KIND, N, I + 1>(v, c1, c2, s, l, lp); }
}

// MODE 0: every wave runs (MFMA + NV fillers) x 4 per iteration.
// MODE 1: waves with (wave / 4) even run MFMA only; odd ones run fillers only (4*NV per iteration); needs >= 2 waves per SIMD.
// NM: matrix instructions per slot (0 = fillers only)
template <int KIND, int NV, int NM, int MODE>
__global__ __launch_bounds__(1024) void k(float* out, int iters, float c1, float c2) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  for (int i = threadIdx.x; i < 16384; i += blockDim.x) lds[i] = i;
  __syncthreads();
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x + i); b[i] = (__bf16)(float)(i); }
  f32x16 acc[4];
  for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  float v[8];
  for (int i = 0; i < 8; ++i) v[i] = threadIdx.x * 0.001f + i;
  int s = __builtin_amdgcn_readfirstlane(iters);
  f32x4 l[4] = {};
  const int lane = threadIdx.x & 63;
  int lp = (int)(uintptr_t)(__attribute__((address_space(3))) void*)lds + lane * 16 + (threadIdx.x >> 6) * 1024;
  if (KIND == 8) lp = (int)(uintptr_t)(__attribute__((address_space(3))) void*)lds + (lane >> 2) * 256 + (lane & 3) * 8 + (threadIdx.x >> 6) * 4096;
  const int wave = threadIdx.x >> 6;
  const bool do_m = MODE == 0 || ((wave >> 2) & 1) == 0;
  const bool do_v = MODE == 0 || ((wave >> 2) & 1) == 1;
  const long long t0 = clock64(); const unsigned long long r0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
    if (MODE == 0) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if constexpr (NM >= 1) MFMA(acc[j]);
        if constexpr (NM >= 2) MFMA(acc[(j + 2) & 3]);
        fillers<KIND, NV>(v, c1, c2, s, l, lp);
      }
    } else if (do_m) {
#pragma unroll
      for (int j = 0; j < 4; ++j) MFMA(acc[j]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) fillers<KIND, NV>(v, c1, c2, s, l, lp);
    }
  }
  asm volatile("s_waitcnt lgkmcnt(0)");
  const long long t1 = clock64(); const unsigned long long r1 = wall_clock64();
  float sum = 0; for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) sum += acc[j][i];
  for (int i = 0; i < 8; ++i) sum += v[i];
  for (int i = 0; i < 4; ++i) sum += l[i][0] + l[i][3];
  out[blockIdx.x * blockDim.x + threadIdx.x] = sum + s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { ((long long*)(out + 256 * 1024))[0] = t1 - t0; ((long long*)(out + 256 * 1024))[1] = (long long)(r1 - r0); }
}
static float* g_d;
static const char* kname[] = {"fma", "exp", "rcp", "mul", "cvt_pk_bf16", "xor", "salu", "ds_read_b128", "ds_read_tr", "silu-mix"};
template <int KIND, int NV, int NM, int MODE> void run(int wps) {
  const int iters = 20000;
  hipFuncSetAttribute((const void*)k<KIND, NV, NM, MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024);
  hipLaunchKernelGGL((k<KIND, NV, NM, MODE>), dim3(256), dim3(256 * wps), 100 * 1024, 0, g_d, 500, 1.0001f, 0.5f);
  hipDeviceSynchronize();
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  hipEventRecord(e0);
  hipLaunchKernelGGL((k<KIND, NV, NM, MODE>), dim3(256), dim3(256 * wps), 100 * 1024, 0, g_d, iters, 1.0001f, 0.5f);
  hipEventRecord(e1); hipDeviceSynchronize();
  float ms; hipEventElapsedTime(&ms, e0, e1);
  // slots executed per SIMD: MODE 0: wps waves x iters x 4; MODE 1: the matrix waves (wps/2) x iters x 4 (the filler waves run beside them)
  const double slots = (MODE == 0 ? wps : wps / 2) * (double)iters * 4;
  long long tt[2]; hipMemcpy(tt, g_d + 256 * 1024, 16, hipMemcpyDeviceToHost);
  printf("mode=%d wps=%d %-13s NM=%d NV=%2d : %8.3f ms  %7.2f ns per slot per SIMD   memtime %lld ticks, realtime %lld ticks (x10 ns = %.3f ms), memtime/ns %.3f\n", MODE, wps, kname[KIND], NM, NV, ms, ms * 1e6 / slots, tt[0], tt[1], tt[1] * 1e-5, tt[0] / (tt[1] * 10.0));
  fflush(stdout);
}
template <int KIND> void sweep(int wps) {
  run<KIND, 1, 1, 0>(wps); run<KIND, 2, 1, 0>(wps); run<KIND, 4, 1, 0>(wps); run<KIND, 6, 1, 0>(wps); run<KIND, 8, 1, 0>(wps);
  run<KIND, 12, 1, 0>(wps); run<KIND, 16, 1, 0>(wps);
}
int main() {
  hipMalloc(&g_d, 256 * 1024 * 4 + 64);
  for (int wps = 1; wps <= 4; ++wps) {
    printf("---- %d waves per SIMD\n", wps);
    run<0, 0, 1, 0>(wps);                      // matrix only
    run<0, 8, 0, 0>(wps); run<1, 8, 0, 0>(wps); run<2, 8, 0, 0>(wps); run<4, 8, 0, 0>(wps); run<5, 8, 0, 0>(wps);   // fillers only
    run<7, 8, 0, 0>(wps); run<8, 8, 0, 0>(wps); run<9, 8, 0, 0>(wps);
    sweep<0>(wps); sweep<1>(wps); sweep<9>(wps);   // one matrix instruction + NV fillers per slot, same wave
    if (wps % 2 == 0) {                            // matrix instructions and fillers in different waves of one SIMD
      run<0, 4, 1, 1>(wps); run<0, 8, 1, 1>(wps); run<0, 16, 1, 1>(wps);
      run<9, 4, 1, 1>(wps); run<9, 8, 1, 1>(wps); run<9, 16, 1, 1>(wps);
    }
  }
  return 0;
}
