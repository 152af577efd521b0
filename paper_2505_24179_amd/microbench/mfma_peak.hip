// Rate the matrix pipes sustain with nothing else in the loop.
//
// Not part of the library: a standalone probe behind the "sustained" column the kernels' MFMA fractions are
// compared with.  2048 workgroups of 4 waves, each wave issuing four independent accumulator chains of one
// MFMA type for 4000 iterations, timed with HIP events.
//
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops mfma_peak.hip -o mfma_peak
#include <hip/hip_runtime.h>

#include <cstdio>

#define CK(x)                                                                        \
  do {                                                                               \
    hipError_t e_ = (x);                                                             \
    if (e_ != hipSuccess) {                                                          \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);          \
      return 1;                                                                      \
    }                                                                                \
  } while (0)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;

enum { kBf16 = 0, kFp6, kFp8, kFp4, kInt8 };

template <int MODE>
__global__ __launch_bounds__(256) void probe(float* out, int iters) {
  f32x16 acc[4];
  i32x16 iacc[4];
  for (int t = 0; t < 4; ++t)
    for (int r = 0; r < 16; ++r) { acc[t][r] = 0; iacc[t][r] = 0; }
  bf16x8 a, b;
  i32x8 a8, b8;
  i32x4 a4, b4;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x & 3); b[e] = (__bf16)1.0f; a8[e] = threadIdx.x; b8[e] = 0x08080808; }
  for (int e = 0; e < 4; ++e) { a4[e] = threadIdx.x; b4[e] = 0x01010101; }
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (MODE == kBf16) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
      if (MODE == kFp6) acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[t], 2, 2, 0, 0, 0, 0);      // E2M3
      if (MODE == kFp8) acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[t], 0, 0, 0, 0, 0, 0);
      if (MODE == kFp4) acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[t], 4, 4, 0, 0, 0, 0);
      if (MODE == kInt8) iacc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a4, b4, iacc[t], 0, 0, 0);
    }
  }
  float s = 0;
  for (int t = 0; t < 4; ++t)
    for (int r = 0; r < 16; ++r) s += acc[t][r] + iacc[t][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

template <int MODE>
int run(const char* name, double flop_per_mfma) {
  float* out;
  CK(hipMalloc(&out, 4096 * 256 * 4));
  const int iters = 4000, blocks = 2048;
  probe<MODE><<<blocks, 256>>>(out, 10);
  CK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  CK(hipEventRecord(e0));
  probe<MODE><<<blocks, 256>>>(out, iters);
  CK(hipEventRecord(e1));
  CK(hipEventSynchronize(e1));
  float ms;
  CK(hipEventElapsedTime(&ms, e0, e1));
  const double flops = (double)blocks * 4 * iters * 4 * flop_per_mfma;
  printf("%-22s %8.2f ms  %8.1f TFLOP/s\n", name, ms, flops / ms / 1e9);
  CK(hipFree(out));
  return 0;
}

int main() {
  return run<kBf16>("bf16 32x32x16", 2.0 * 32 * 32 * 16) || run<kFp6>("fp6 e2m3 32x32x64", 2.0 * 32 * 32 * 64) ||
         run<kFp8>("fp8 32x32x64", 2.0 * 32 * 32 * 64) || run<kFp4>("fp4 32x32x64", 2.0 * 32 * 32 * 64) ||
         run<kInt8>("i8 32x32x32", 2.0 * 32 * 32 * 32);
}
