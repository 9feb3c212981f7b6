// Register-resident MFMA loop on gfx950: the rate the matrix cores sustain when nothing but
// v_mfma_f32_32x32x16_{bf16,f16} is issued (no LDS, no memory traffic), with the accumulator blocking of
// the Newton-Schulz GEMM (8 waves per CU, 4 x 2 accumulators of 32 x 32 per wave) and with others.
// Operands are all ones, or random values of full range: the switching activity of the operands changes the
// power drawn and with it the clock the part sustains, so both figures are the practical ceilings that the
// GEMM kernels' TFLOP/s are to be read against, next to the nominal 2.5 PFLOP/s.
//
//   mfma_peak [milliseconds per measurement, default 200]
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define CK(x)                                                                        \
  do {                                                                               \
    hipError_t e_ = (x);                                                             \
    if (e_ != hipSuccess) {                                                          \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      exit(1);                                                                       \
    }                                                                                \
  } while (0)

template <int NT, int FM, int FN, bool HALF>
__global__ void __launch_bounds__(NT) mfma_loop(const bf16x8* __restrict__ src, float* __restrict__ sink, int iters) {
  bf16x8 fa[FM], fb[FN];
  for (int i = 0; i < FM; ++i) fa[i] = src[(threadIdx.x + 64 * i) & 1023];
  for (int j = 0; j < FN; ++j) fb[j] = src[(threadIdx.x + 64 * (j + 8)) & 1023];
  f32x16 acc[FM][FN];
  for (int i = 0; i < FM; ++i)
    for (int j = 0; j < FN; ++j)
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        if (HALF)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, fb[j]),
                                                             __builtin_bit_cast(f16x8, fa[i]), acc[i][j], 0, 0, 0);
        else
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
      }
  }
  float s = 0.f;
  for (int i = 0; i < FM; ++i)
    for (int j = 0; j < FN; ++j)
      for (int v = 0; v < 16; ++v) s += acc[i][j][v];
  sink[blockIdx.x * NT + threadIdx.x] = s;
}

template <int NT, int FM, int FN, bool HALF>
static void measure(const char* name, const bf16x8* src, int blocks, double target_ms) {
  float* sink;
  CK(hipMalloc(&sink, (size_t)blocks * NT * 4));
  hipEvent_t a, b;
  CK(hipEventCreate(&a));
  CK(hipEventCreate(&b));
  int iters = 2000;
  float ms = 0.f;
  for (int rep = 0; rep < 3; ++rep) {  // the last repetition runs for about target_ms at the clock reached by then
    CK(hipEventRecord(a, 0));
    hipLaunchKernelGGL((mfma_loop<NT, FM, FN, HALF>), dim3(blocks), dim3(NT), 0, 0, src, sink, iters);
    CK(hipEventRecord(b, 0));
    CK(hipDeviceSynchronize());
    CK(hipEventElapsedTime(&ms, a, b));
    if (rep < 2) iters = (int)(iters * target_ms / (ms > 0.01f ? ms : 0.01f));
    if (iters < 100) iters = 100;
  }
  const double flop = (double)blocks * (NT / 64) * iters * FM * FN * 2.0 * 32 * 32 * 16;
  printf("  %-40s %8.2f ms  %8.1f TFLOP/s  (%.3f of 2500)\n", name, ms, flop / ms / 1e9, flop / ms / 1e9 / 2500.0);
  CK(hipEventDestroy(a));
  CK(hipEventDestroy(b));
  CK(hipFree(sink));
}

int main(int argc, char** argv) {
  const double target_ms = argc > 1 ? atof(argv[1]) : 200.0;
  int dev = 0, n_cu = 256;
  CK(hipGetDevice(&dev));
  CK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  unsigned short* h = (unsigned short*)malloc(1024 * 16);
  bf16x8* d;
  CK(hipMalloc(&d, 1024 * 16));
  printf("register-resident v_mfma_f32_32x32x16 loop, one workgroup per CU (%d CUs), about %.0f ms per line\n", n_cu, target_ms);
  for (int mode = 0; mode < 3; ++mode) {
    srand(1);
    for (int i = 0; i < 8192; ++i) {
      const unsigned r = (unsigned)rand();
      if (mode == 0) h[i] = 0x3f80;  // bf16 1.0 (as f16 bits: 1.875)
      else if (mode == 1) h[i] = (unsigned short)(0x3c00 + (r & 0x3ff) + (((r >> 10) & 1) << 15));  // +-[0.0078, 0.031) bf16; +-[1, 2) f16
      else h[i] = (unsigned short)((r & 0x7fff) % 0x4000 + 0x2000 + (((r >> 16) & 1) << 15));  // exponents spread, all bits toggling
    }
    CK(hipMemcpy(d, h, 1024 * 16, hipMemcpyHostToDevice));
    printf("operands: %s\n", mode == 0 ? "constant" : mode == 1 ? "random mantissa and sign, one exponent" : "random sign, exponent and mantissa");
    measure<512, 4, 2, false>("bf16, 8 waves/CU, 4x2 acc (GEMM's shape)", d, n_cu, target_ms);
    measure<512, 4, 2, true>("f16,  8 waves/CU, 4x2 acc (GEMM's shape)", d, n_cu, target_ms);
    measure<256, 4, 4, false>("bf16, 4 waves/CU, 4x4 acc", d, n_cu, target_ms);
    measure<1024, 2, 2, false>("bf16, 16 waves/CU, 2x2 acc", d, n_cu, target_ms);
  }
  free(h);
  CK(hipFree(d));
  return 0;
}
