// Micro-benchmark behind the instruction-mix figures quoted in the design notes: what one wavefront per SIMD loses when
// vector work is interleaved with matrix instructions.  Not part of the library; build and run by hand:
//   hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops mfma_valu_mix.hip -o mfma_valu_mix && ./mfma_valu_mix
// Per iteration: 16 MFMA (32x32x16 bf16), each followed by NV vector instructions of a given kind.
//   ACC: 0 = accumulators in VGPRs, 1 = in AGPRs.   KIND: 0 v_fma, 1 v_exp, 2 v_accvgpr_read (of a second AGPR tile), 3 v_cvt_pk_bf16
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

template <int ACC, int NV, int KIND, int DEP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1))) void k(float* out, int iters, float seed) {
  f32x16 acc[4], other;
  for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  for (int i = 0; i < 16; ++i) other[i] = seed * i;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)seed; b[e] = (__bf16)1.0f; }
  float v[16];
  for (int i = 0; i < 16; ++i) v[i] = seed * i + threadIdx.x;
  asm volatile("" : "+a"(other));
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      // DEP = 1: every MFMA continues the chain of the previous one (same accumulator)
      f32x16& c = acc[DEP ? 0 : (m & 3)];
      if (ACC == 1) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
      else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int r = (m * NV + j) & 15;
        if (KIND == 0) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(v[r]) : "v"(seed));
        else if (KIND == 1) asm volatile("v_exp_f32 %0, %0" : "+v"(v[r]));
        else if (KIND == 2) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v[r]) : "a"(other[r]));
        else asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(v[r]) : "v"(seed));
      }
    }
  }
  float s = 0;
  for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) s += acc[j][i];
  for (int i = 0; i < 16; ++i) s += v[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int ACC, int NV, int KIND, int DEP>
void run() {
  float* out; CHECK(hipMalloc(&out, 256 * 256 * 4));
  hipEvent_t a, b; CHECK(hipEventCreate(&a)); CHECK(hipEventCreate(&b));
  const int iters = 4000;
  hipLaunchKernelGGL((k<ACC, NV, KIND, DEP>), dim3(256), dim3(256), 0, 0, out, 10, 1.0f);
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(a));
  hipLaunchKernelGGL((k<ACC, NV, KIND, DEP>), dim3(256), dim3(256), 0, 0, out, iters, 1.0f);
  CHECK(hipEventRecord(b)); CHECK(hipEventSynchronize(b));
  float ms; CHECK(hipEventElapsedTime(&ms, a, b));
  const char* kinds[] = {"fma", "exp", "accread", "cvt_pk"};
  printf("acc in %s, %s chain, %d x %-7s per MFMA: %6.1f ns per 16 MFMA  (%.1f ns per MFMA)\n", ACC ? "AGPR" : "VGPR", DEP ? "one " : "four", NV, kinds[KIND],
         ms * 1e6 / iters, ms * 1e6 / iters / 16);
  fflush(stdout);
  CHECK(hipFree(out));
}

int main() {
  run<0, 0, 0, 0>(); run<1, 0, 0, 0>(); run<1, 0, 0, 1>();
  run<0, 4, 0, 0>(); run<1, 4, 0, 0>();
  run<0, 6, 0, 0>(); run<1, 6, 0, 0>(); run<1, 6, 0, 1>();
  run<0, 8, 0, 0>(); run<1, 8, 0, 0>();
  run<1, 2, 1, 0>(); run<1, 4, 1, 0>();
  run<1, 2, 2, 0>(); run<1, 4, 2, 0>(); run<1, 6, 2, 0>();
  run<1, 4, 3, 0>(); run<0, 4, 3, 0>();
  return 0;
}
