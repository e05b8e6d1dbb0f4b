// What MFMA rate does this chip sustain with nothing else going on?  256 blocks, one or two waves per
// SIMD, random bf16 operands held in registers, eight (32x32x16) or thirty-two (16x16x32) independent
// accumulators per wave, back-to-back MFMAs.  Variants: accumulators in VGPRs or AGPRs, a barrier every so
// many MFMAs, an s_nop after each MFMA.  Prints TFLOP/s per variant; context for the roofline of the
// grouped-FFN kernel (the 2.5 PFLOP/s datasheet figure assumes a clock the chip does not hold under load).
//
// build: python -m paper_2603_06350_amd.build   (writes mfma_rate.exe beside this file)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

#define CHECK(x)                                                                  \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                \
      std::exit(1);                                                               \
    }                                                                             \
  } while (0)

// BAR: barrier every BAR groups of MFMAs (0 = never).  AG: accumulators in AGPRs.
// SHAPE 0: v_mfma_f32_32x32x16_bf16, 8 per group.  SHAPE 1: v_mfma_f32_16x16x32_bf16, 16 per group
// (the same flops).  NOP: s_nop 3 after each 32x32x16 MFMA.
template <int BAR, int AG, int SHAPE, int NOP>
__global__ __launch_bounds__(512) void mfma_loop(const uint4* __restrict__ src, float* __restrict__ out,
                                                 int iters) {
  const int tid = blockIdx.x * blockDim.x + threadIdx.x;
  bf16x8 x0, x1, w0, w1, w2, w3;
  {
    uint4 v = src[(tid * 6 + 0) & 65535]; x0 = __builtin_bit_cast(bf16x8, v);
    v = src[(tid * 6 + 1) & 65535]; x1 = __builtin_bit_cast(bf16x8, v);
    v = src[(tid * 6 + 2) & 65535]; w0 = __builtin_bit_cast(bf16x8, v);
    v = src[(tid * 6 + 3) & 65535]; w1 = __builtin_bit_cast(bf16x8, v);
    v = src[(tid * 6 + 4) & 65535]; w2 = __builtin_bit_cast(bf16x8, v);
    v = src[(tid * 6 + 5) & 65535]; w3 = __builtin_bit_cast(bf16x8, v);
  }
  float r = 0;
  if (SHAPE == 0) {
    f32x16 acc[8];
    for (int a = 0; a < 8; ++a)
      for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;
#define MF(A, W, X)                                                                              \
  do {                                                                                           \
    if (AG) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(A) : "v"(W), "v"(X));  \
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(A) : "v"(W), "v"(X));     \
    if (NOP) asm volatile("s_nop 3");                                                            \
  } while (0)
    for (int it = 0; it < iters; ++it) {
      if (BAR && (it % BAR) == 0) __builtin_amdgcn_s_barrier();
      MF(acc[0], w0, x0); MF(acc[1], w1, x0); MF(acc[2], w2, x0); MF(acc[3], w3, x0);
      MF(acc[4], w0, x1); MF(acc[5], w1, x1); MF(acc[6], w2, x1); MF(acc[7], w3, x1);
    }
#undef MF
    asm volatile("s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15");   // asm MFMAs: let the results retire
    for (int a = 0; a < 8; ++a) r += acc[a][0] + acc[a][7];
  } else {
    f32x4 acc[32];
    for (int a = 0; a < 32; ++a)
      for (int v = 0; v < 4; ++v) acc[a][v] = 0.f;
#define MG(A, W, X)                                                                              \
  do {                                                                                           \
    if (AG) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(A) : "v"(W), "v"(X));  \
    else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(A) : "v"(W), "v"(X));     \
  } while (0)
    for (int it = 0; it < iters; ++it) {
      if (BAR && (it % BAR) == 0) __builtin_amdgcn_s_barrier();
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        MG(acc[q * 16 + 0], w0, x0); MG(acc[q * 16 + 1], w1, x0); MG(acc[q * 16 + 2], w2, x0);
        MG(acc[q * 16 + 3], w3, x0); MG(acc[q * 16 + 4], w0, x1); MG(acc[q * 16 + 5], w1, x1);
        MG(acc[q * 16 + 6], w2, x1); MG(acc[q * 16 + 7], w3, x1);
      }
    }
#undef MG
    asm volatile("s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15");
    for (int a = 0; a < 32; ++a) r += acc[a][0] + acc[a][3];
  }
  out[tid] = r;
}

static uint4* g_src;
static float* g_out;

template <int BAR, int AG, int SHAPE, int NOP>
static void run(const char* name, int threads) {
  const int blocks = 256, iters = 20000;
  mfma_loop<BAR, AG, SHAPE, NOP><<<blocks, threads>>>(g_src, g_out, 200);
  CHECK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  CHECK(hipEventRecord(e0));
  mfma_loop<BAR, AG, SHAPE, NOP><<<blocks, threads>>>(g_src, g_out, iters);
  CHECK(hipEventRecord(e1));
  CHECK(hipDeviceSynchronize());
  float ms;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  const double flops = static_cast<double>(blocks) * (threads / 64) * iters * 8 * 32768.0;
  std::printf("%-46s waves/SIMD=%d: %.3f ms %.0f TFLOP/s\n", name, threads / 256, ms,
              flops / (ms * 1e-3) / 1e12);
  std::fflush(stdout);
}

int main() {
  // bf16 values in +-[0.5, 1): sums of random signs stay far from overflow
  uint32_t* h = static_cast<uint32_t*>(std::malloc(65536 * 16));
  std::srand(1);
  for (int i = 0; i < 65536 * 4; ++i) {
    const uint32_t lo = 0x3f00 + (std::rand() & 0xff) + ((std::rand() & 1) << 15);
    const uint32_t hi = 0x3f00 + (std::rand() & 0xff) + ((std::rand() & 1) << 15);
    h[i] = lo | (hi << 16);
  }
  CHECK(hipMalloc(&g_src, 65536 * 16));
  CHECK(hipMemcpy(g_src, h, 65536 * 16, hipMemcpyHostToDevice));
  CHECK(hipMalloc(&g_out, 256 * 512 * 4));
  run<0, 0, 0, 0>("32x32x16 vgpr acc, no barrier", 256);
  run<0, 0, 0, 0>("32x32x16 vgpr acc, no barrier", 512);
  run<4, 0, 0, 0>("32x32x16 vgpr acc, barrier per 32 mfma", 512);
  run<0, 1, 0, 0>("32x32x16 agpr acc, no barrier", 256);
  run<0, 1, 0, 0>("32x32x16 agpr acc, no barrier", 512);
  run<0, 0, 0, 1>("32x32x16 vgpr acc, s_nop 3 after each", 512);
  run<0, 0, 1, 0>("16x16x32 vgpr acc, no barrier", 256);
  run<0, 0, 1, 0>("16x16x32 vgpr acc, no barrier", 512);
  run<4, 0, 1, 0>("16x16x32 vgpr acc, barrier per 64 mfma", 512);
  run<0, 1, 1, 0>("16x16x32 agpr acc, no barrier", 256);
  return 0;
}
