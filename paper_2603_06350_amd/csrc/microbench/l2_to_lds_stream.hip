// How fast can the CUs pull the grouped-FFN up-projection's operand tiles through the L2 into LDS if they
// do nothing else?  Same tile shape (256 activation rows + 128 W1 rows + 128 W3 rows, 64 K-elements per
// stage = 64 KiB), same per-lane addressing, same XCD-aware tile order as the FFN kernel at the Mixtral
// shape (d = 4096, F = 14336, 8 experts x 4 m-tiles x 112 n-tiles), but no MFMA and no LDS reads, and with
// DEPTH stages of loads in flight (LDS slots alias: nobody reads the data).  Prints the aggregate L2->LDS
// rate per depth, for the flat-address and the buffer form of the direct-to-LDS load.
//
// build: python -m paper_2603_06350_amd.build   (writes l2_to_lds_stream.exe beside this file)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                  \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                \
      std::exit(1);                                                               \
    }                                                                             \
  } while (0)

constexpr int K = 4096, F = 14336, E = 8, MT = 4, NT = F / 128, ROWB = 128, KT = K * 2 / ROWB;

template <int DEPTH, bool BUF>
__global__ __launch_bounds__(512) void stream(const unsigned char* x, const unsigned char* w1,
                                              const unsigned char* w3, uint32_t* out) {
  extern __shared__ __align__(1024) unsigned char lds[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  constexpr int total = E * NT * MT;
  const int per = total / 8;                         // contiguous range of the tile list per XCD
  const int vid = (blockIdx.x % 8) * per + blockIdx.x / 8;
  const int e = vid / (NT * MT), rem = vid % (NT * MT), n = rem / MT, m = rem % MT;
  const unsigned char* base[3];
  base[0] = x + static_cast<size_t>(e * MT + m) * 256 * K * 2;
  base[1] = w1 + (static_cast<size_t>(e) * F + n * 128) * K * 2;
  base[2] = w3 + (static_cast<size_t>(e) * F + n * 128) * K * 2;
  uint32_t soff[8];                                  // 8 loads per wave per stage, 8 rows x 128 B each
  for (int i = 0; i < 8; ++i) {
    const int g = i * 8 + wave;
    const int row = (g * 8 + (lane >> 3)) & (i < 4 ? 255 : 127);
    soff[i] = row * K * 2 + (((lane & 7) ^ (row & 7)) * 16);
  }
  __amdgpu_buffer_rsrc_t rs[3];
  for (int j = 0; j < 3; ++j)
    rs[j] = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(base[j]), 0, 0x7FFFFFFF, 0x00020000);
  auto issue = [&](int kt) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int g = i * 8 + wave;
      const int j = i < 4 ? 0 : (i < 6 ? 1 : 2);
      auto dst = (__attribute__((address_space(3))) void*)(lds + (kt & 1) * 65536 + g * 1024);
      if (BUF)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs[j], dst, 16, static_cast<int>(soff[i]), kt * ROWB, 0, 0);
      else
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(base[j] + static_cast<size_t>(kt) * ROWB + soff[i]),
            dst, 16, 0, 0);
    }
  };
  for (int s = 0; s < DEPTH; ++s) issue(s);
  for (int kt = 0; kt < KT; ++kt) {
    if (kt + DEPTH < KT) {
      // the oldest stage has landed when at most (DEPTH - 1) stages' loads are outstanding
      if (DEPTH == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (DEPTH == 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      if (DEPTH == 3) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
      if (DEPTH == 4) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      issue(kt + DEPTH);
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
    }
  }
  out[blockIdx.x * 512 + threadIdx.x] = lds[threadIdx.x];
}

template <int DEPTH, bool BUF>
static void run(const unsigned char* x, const unsigned char* w1, const unsigned char* w3, uint32_t* out) {
  CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(stream<DEPTH, BUF>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
  const int grid = E * NT * MT;
  stream<DEPTH, BUF><<<grid, 512, 131072>>>(x, w1, w3, out);
  CHECK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  CHECK(hipEventRecord(e0));
  for (int r = 0; r < 5; ++r) stream<DEPTH, BUF><<<grid, 512, 131072>>>(x, w1, w3, out);
  CHECK(hipEventRecord(e1));
  CHECK(hipDeviceSynchronize());
  float ms;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  ms /= 5;
  const double bytes = static_cast<double>(grid) * KT * 65536;
  std::printf("%d stage(s) in flight, %s: %.3f ms  %.2f TB/s L2->LDS (%.1f B/clk/CU at 2.4 GHz)\n", DEPTH,
              BUF ? "buffer_load ... lds" : "global_load_lds   ", ms, bytes / (ms * 1e-3) / 1e12,
              bytes / 256 / (ms * 1e-3) / 2.4e9);
  std::fflush(stdout);
}

int main() {
  unsigned char *x, *w1, *w3;
  uint32_t* out;
  const size_t xb = static_cast<size_t>(E) * MT * 256 * K * 2, wb = static_cast<size_t>(E) * F * K * 2;
  CHECK(hipMalloc(&x, xb));
  CHECK(hipMalloc(&w1, wb));
  CHECK(hipMalloc(&w3, wb));
  CHECK(hipMemset(x, 1, xb));
  CHECK(hipMemset(w1, 1, wb));
  CHECK(hipMemset(w3, 1, wb));
  CHECK(hipMalloc(&out, static_cast<size_t>(E) * NT * MT * 512 * 4));
  run<1, false>(x, w1, w3, out);
  run<2, false>(x, w1, w3, out);
  run<3, false>(x, w1, w3, out);
  run<1, true>(x, w1, w3, out);
  run<2, true>(x, w1, w3, out);
  run<3, true>(x, w1, w3, out);
  run<4, true>(x, w1, w3, out);
  return 0;
}
