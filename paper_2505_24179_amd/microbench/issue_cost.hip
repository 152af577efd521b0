// What one wave of gfx950 pays per instruction, and how much of it hides behind its own MFMAs.
//
// Not part of the library: a standalone probe behind the issue-cost table the attention kernels are priced
// with.  Workgroups of 256 threads; the dynamic LDS request decides how many fit a CU, i.e. how many waves
// share a SIMD (1, 2 or 4).  Every wave runs the same unrolled body on registers only.
//   * 128 independent VALU instructions of one kind per iteration;
//   * two v_mfma_f32_32x32x16_bf16 (or two FP6 v_mfma_scale_f32_32x32x64_f8f6f4) on two accumulators, each
//     followed by n fp32 FMAs that depend on neither.
// Prints SIMD cycles per instruction (all waves of the SIMD counted) at a nominal 2.4 GHz.
//
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops issue_cost.hip -o issue_cost
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

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) int i32x8;

enum { kFma = 0, kExp2, kCvtPk, kDot2, kMax3, kSwap32, kMfma = 10, kMfma6 = 40 };      // kMfma(6) + n: MFMA followed by n FMAs

template <int MODE>
__global__ __launch_bounds__(256) void probe(float* out, int iters, float seed) {
  extern __shared__ float occupancy_pad[];
  if (seed == 12345.f) occupancy_pad[threadIdx.x] = seed;
  float x[16];
  for (int i = 0; i < 16; ++i) x[i] = seed + threadIdx.x * 1e-3f + i;
  f32x16 acc0 = {0}, acc1 = {0};
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(seed + i); b[i] = (__bf16)(seed * 0.5f + i); }
  bf16x2 ones;
  ones[0] = (__bf16)1.0f; ones[1] = (__bf16)1.0f;
  i32x8 a6, b6;
  for (int i = 0; i < 8; ++i) { a6[i] = i < 6 ? (int)threadIdx.x * 0x01010101 : 0; b6[i] = i < 6 ? 0x08080808 : 0; }
  for (int it = 0; it < iters; ++it) {
    if (MODE >= kMfma6) {
      acc0 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a6, b6, acc0, 2, 2, 0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < MODE - kMfma6; ++i) x[i] = __builtin_fmaf(x[i], 0.999f, 0.001f);
      acc1 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a6, b6, acc1, 2, 2, 0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < MODE - kMfma6; ++i) x[i] = __builtin_fmaf(x[i], 0.998f, 0.002f);
      continue;
    }
    if (MODE >= kMfma) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc0, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < MODE - kMfma; ++i) x[i] = __builtin_fmaf(x[i], 0.999f, 0.001f);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc1, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < MODE - kMfma; ++i) x[i] = __builtin_fmaf(x[i], 0.998f, 0.002f);
      continue;
    }
#pragma unroll
    for (int rep = 0; rep < 8; ++rep)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        if (MODE == kFma) { x[i] = __builtin_fmaf(x[i], 0.999f, 0.001f); x[i + 1] = __builtin_fmaf(x[i + 1], 0.999f, 0.001f); }
        if (MODE == kExp2) { x[i] = __builtin_amdgcn_exp2f(x[i]); x[i + 1] = __builtin_amdgcn_exp2f(x[i + 1]); }
        if (MODE == kCvtPk) {
          bf16x2 pk;
          pk[0] = (__bf16)x[i]; pk[1] = (__bf16)x[i + 1];
          x[i] = __builtin_bit_cast(float, pk);
        }
        if (MODE == kDot2) x[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, x[i + 1]), ones, x[i], false);
        if (MODE == kMax3) x[i] = fmaxf(fmaxf(x[i], x[i + 1]), seed);
        if (MODE == kSwap32) x[i] = __shfl_xor(x[i], 32, 64);
      }
  }
  float s = 0.f;
  for (int i = 0; i < 16; ++i) s += x[i] + acc0[i] + acc1[i];
  out[(blockIdx.x & 255) * 256 + threadIdx.x] = s;
}

template <int MODE>
int run(const char* name, double counted, int waves_per_simd) {
  float* out;
  CK(hipMalloc(&out, 256 * 256 * 4));
  const int iters = MODE < kMfma ? 25000 : 200000, rounds = 4;
  const int lds = (waves_per_simd == 1 ? 100 : waves_per_simd == 2 ? 60 : 36) * 1024;
  CK(hipFuncSetAttribute((const void*)probe<MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024));
  probe<MODE><<<256, 256, lds>>>(out, 10, 0.5f);
  CK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  CK(hipEventRecord(e0));
  probe<MODE><<<256 * rounds * waves_per_simd, 256, lds>>>(out, iters, 0.5f);
  CK(hipEventRecord(e1));
  CK(hipEventSynchronize(e1));
  float ms;
  CK(hipEventElapsedTime(&ms, e0, e1));
  const double cycles = ms * 1e6 / ((double)iters * rounds) * 2.4;      // per iteration of all waves of a SIMD
  printf("%d wave(s)/SIMD  %-22s %7.2f SIMD cycles per instruction of one wave, %6.2f per instruction issued\n",
         waves_per_simd, name, cycles / counted, cycles / counted / waves_per_simd);
  CK(hipFree(out));
  return 0;
}

int main() {
  for (int w = 1; w <= 4; w *= 2) {
    if (run<kFma>("v_fma_f32", 128, w) || run<kExp2>("v_exp_f32", 128, w) || run<kCvtPk>("v_cvt_pk_bf16_f32", 64, w) ||
        run<kDot2>("v_dot2c_f32_bf16", 64, w) || run<kMax3>("v_max3_f32", 64, w) || run<kSwap32>("lane ^ 32 exchange", 64, w))
      return 1;
    if (run<kMfma>("mfma", 2, w) || run<kMfma + 2>("mfma + 2 fma", 2, w) || run<kMfma + 4>("mfma + 4 fma", 2, w) ||
        run<kMfma + 6>("mfma + 6 fma", 2, w) || run<kMfma + 8>("mfma + 8 fma", 2, w) || run<kMfma + 12>("mfma + 12 fma", 2, w))
      return 1;
    if (run<kMfma6>("fp6 mfma", 2, w) || run<kMfma6 + 2>("fp6 mfma + 2 fma", 2, w) || run<kMfma6 + 4>("fp6 mfma + 4 fma", 2, w) ||
        run<kMfma6 + 6>("fp6 mfma + 6 fma", 2, w) || run<kMfma6 + 8>("fp6 mfma + 8 fma", 2, w) ||
        run<kMfma6 + 12>("fp6 mfma + 12 fma", 2, w))
      return 1;
  }
  return 0;
}
