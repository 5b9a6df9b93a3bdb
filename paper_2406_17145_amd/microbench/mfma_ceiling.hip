// What the matrix cores of this chip sustain when nothing but the MFMA instruction itself is in the way, and
// how many ordinary vector instructions fit into an MFMA's shadow.  A stand-alone program (not part of the
// library): it backs the ceilings that the kernel notes quote.
//
// Every wave runs v_mfma_f32_32x32x16_bf16 back to back on four independent accumulators from operands that
// stay in registers (no LDS, no memory), optionally with K vector instructions (integer add, fused multiply-add
// or exponential) behind each MFMA.  Two operand fills: small integers (few bits toggle) and random values in
// (-1, 1) (what the workloads' activations and weights look like to the multipliers).
//
//   usage: mfma_ceiling            prints one line per case: operands, waves per SIMD, K, duration, TFLOP/s
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

enum { FILL_SMALL = 0, FILL_RANDOM = 1 };
enum { OP_ADD = 0, OP_EXP = 1, OP_FMA = 2 };

template <int K, int OP, int FILL>
__global__ __launch_bounds__(256) void k_mfma_loop(float *out, int iters) {
  f32x16 acc[4];
  for (int j = 0; j < 4; ++j)
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
  bf16x8 a, b;
  uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  for (int e = 0; e < 8; ++e) {
    if (FILL == FILL_SMALL) {
      a[e] = (__bf16)(float)((threadIdx.x + e) & 3);
      b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 3);
    } else {
      h = h * 1664525u + 1013904223u;
      a[e] = (__bf16)(((int)(h >> 8) & 0xffff) * (1.0f / 32768.0f) - 1.0f);
      h = h * 1664525u + 1013904223u;
      b[e] = (__bf16)(((int)(h >> 8) & 0xffff) * (1.0f / 32768.0f) - 1.0f);
    }
  }
  uint32_t x[8];
  float y[8];
  for (int e = 0; e < 8; ++e) {
    x[e] = threadIdx.x + e;
    y[e] = 0.001f * (threadIdx.x + e);
  }
  const uint32_t one = 1 + (threadIdx.x >> 10);      // not a compile-time constant
  const float fone = 1.0f + (threadIdx.x >> 10);
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
#pragma unroll
      for (int k = 0; k < K; ++k) {
        if (OP == OP_ADD) asm volatile("v_add_u32 %0, %0, %1" : "+v"(x[k % 8]) : "v"(one));
        else if (OP == OP_EXP) asm volatile("v_exp_f32 %0, %0" : "+v"(y[k % 8]));
        else asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(y[k % 8]) : "v"(fone));
      }
    }
  }
  float s = 0.0f;
  for (int j = 0; j < 4; ++j)
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  for (int e = 0; e < 8; ++e) s += (float)x[e] + y[e];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

static bool ok(hipError_t e, const char *what) {
  if (e == hipSuccess) return true;
  fprintf(stderr, "mfma_ceiling: %s: %s\n", what, hipGetErrorString(e));
  return false;
}

// workgroups of four waves (one per SIMD); waves_per_simd of them on each of the 256 compute units
template <int K, int OP, int FILL>
static int run(float *out, int waves_per_simd, int iters) {
  static const char *op_name[] = {"v_add_u32", "v_exp_f32", "v_fma_f32"};
  hipEvent_t e0, e1;
  if (!ok(hipEventCreate(&e0), "event") || !ok(hipEventCreate(&e1), "event")) return 1;
  const dim3 grid(256 * waves_per_simd), block(256);
  hipLaunchKernelGGL((k_mfma_loop<K, OP, FILL>), grid, block, 0, 0, out, iters);     // warm-up
  if (!ok(hipDeviceSynchronize(), "warm-up launch")) return 1;
  if (!ok(hipEventRecord(e0), "record")) return 1;
  hipLaunchKernelGGL((k_mfma_loop<K, OP, FILL>), grid, block, 0, 0, out, iters);
  if (!ok(hipEventRecord(e1), "record") || !ok(hipEventSynchronize(e1), "timed launch")) return 1;
  float ms = 0.0f;
  if (!ok(hipEventElapsedTime(&ms, e0, e1), "elapsed")) return 1;
  const double mfmas_per_simd = (double)iters * 4 * waves_per_simd;
  const double tflops = 2.0 * 32 * 32 * 16 * mfmas_per_simd * 1024 / (ms * 1e-3) / 1e12;
  printf("%-15s %d waves/SIMD  %2d x %-9s per MFMA  %7.3f ms  %6.0f TFLOP/s  %5.2f ns per MFMA and SIMD\n",
         FILL == FILL_SMALL ? "small integers" : "random (-1, 1)", waves_per_simd, K, K ? op_name[OP] : "-", ms, tflops,
         ms * 1e6 / mfmas_per_simd);
  fflush(stdout);
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  return 0;
}

int main() {
  float *out = nullptr;
  if (!ok(hipMalloc(&out, (size_t)256 * 4 * 256 * sizeof(float)), "hipMalloc")) return 1;
  int bad = 0;
  const int n = 20000;
  for (int w : {2, 4}) {
    bad += run<0, OP_ADD, FILL_SMALL>(out, w, n);
    bad += run<0, OP_ADD, FILL_SMALL>(out, w, 10 * n);
    bad += run<0, OP_ADD, FILL_RANDOM>(out, w, n);
    bad += run<0, OP_ADD, FILL_RANDOM>(out, w, 10 * n);
  }
  // the shadow of an MFMA: vector instructions behind each one (two waves per SIMD, small-integer operands so that
  // the clock does not move)
  bad += run<2, OP_ADD, FILL_SMALL>(out, 2, n);
  bad += run<4, OP_ADD, FILL_SMALL>(out, 2, n);
  bad += run<6, OP_ADD, FILL_SMALL>(out, 2, n);
  bad += run<8, OP_ADD, FILL_SMALL>(out, 2, n);
  bad += run<12, OP_ADD, FILL_SMALL>(out, 2, n);
  bad += run<6, OP_FMA, FILL_SMALL>(out, 2, n);
  bad += run<8, OP_FMA, FILL_SMALL>(out, 2, n);
  bad += run<1, OP_EXP, FILL_SMALL>(out, 2, n);
  bad += run<2, OP_EXP, FILL_SMALL>(out, 2, n);
  bad += run<4, OP_EXP, FILL_SMALL>(out, 2, n);
  hipFree(out);
  return bad ? 1 : 0;
}
