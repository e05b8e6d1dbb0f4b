// How fast can the chip read HBM if it does nothing else?  Context for the decode-shaped layer, whose
// grouped FFN is bound by streaming every expert weight once.
//   * contiguous: every block reads its own contiguous share of a 4 GiB buffer, 16 B per lane, eight
//     loads in flight per lane;
//   * tile rows: the small-tile FFN kernel's weight stream: a block walks 256 rows x 128 B per stage
//     at a row pitch of 8 KiB (one 256-row weight tile with d = 4096), 64 stages per tile, with 2 or 4
//     stages of loads in flight;
//   * packed: the same bytes if each stage of a tile were contiguous (what re-tiling the weights would
//     give).
// Prints the rate of each.  Nothing is written except one word per launch that the compiler cannot
// prove unwritten.
//
// build: python -m paper_2603_06350_amd.build   (writes hbm_read_stream.exe beside this file)
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

constexpr int UNR = 8;
__global__ __launch_bounds__(256) void read_contiguous(const uint4* __restrict__ p, size_t n, uint32_t* out) {
  const size_t per = n / gridDim.x;
  const uint4* q = p + static_cast<size_t>(blockIdx.x) * per;
  uint32_t acc = 0;
  for (size_t i = threadIdx.x; i + (UNR - 1) * 256 < per; i += UNR * 256) {
    uint4 v[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) v[u] = q[i + u * 256];
#pragma unroll
    for (int u = 0; u < UNR; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x12345678u) out[0] = acc;
}

constexpr int TILE_ROWS = 256, STAGE_BYTES = TILE_ROWS * 128, STAGES = 64;
constexpr size_t PITCH = 8192;
template <bool PACKED, int DEPTH>
__global__ __launch_bounds__(512) void read_tiles(const unsigned char* __restrict__ w, uint32_t* out) {
  const size_t base = static_cast<size_t>(blockIdx.x) * TILE_ROWS * PITCH;
  const int tid = threadIdx.x;
  uint32_t acc = 0;
  for (int s0 = 0; s0 < STAGES; s0 += DEPTH) {
    uint4 v[DEPTH][4];
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int s = s0 + dd;
        const size_t off = PACKED ? base + static_cast<size_t>(s) * STAGE_BYTES + i * 8192 + tid * 16
                                  : base + static_cast<size_t>(tid / 8 + 64 * i) * PITCH +
                                        static_cast<size_t>(s) * 128 + (tid % 8) * 16;
        v[dd][i] = *reinterpret_cast<const uint4*>(w + off);
      }
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc ^= v[dd][i].x ^ v[dd][i].y ^ v[dd][i].z ^ v[dd][i].w;
  }
  if (acc == 0x12345678u) out[0] = acc;
}

int main() {
  const int tiles = 2048;                                        // 2048 tiles x 256 rows x 8 KiB = 4 GiB
  const size_t bytes = static_cast<size_t>(tiles) * TILE_ROWS * PITCH;
  unsigned char* p = nullptr;
  uint32_t* out = nullptr;
  CHECK(hipMalloc(&p, bytes));
  CHECK(hipMalloc(&out, 4));
  CHECK(hipMemset(p, 1, bytes));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  auto run = [&](const char* name, auto launch) {
    for (int i = 0; i < 2; ++i) launch();
    CHECK(hipEventRecord(e0, 0));
    for (int i = 0; i < 5; ++i) launch();
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    std::printf("%-44s %.3f ms  %.2f TB/s\n", name, ms / 5, bytes / (ms / 5 * 1e-3) / 1e12);
  };
  run("contiguous, 4096 blocks x 256 threads", [&] {
    hipLaunchKernelGGL(read_contiguous, dim3(4096), dim3(256), 0, 0, reinterpret_cast<const uint4*>(p), bytes / 16, out);
  });
  run("tile rows (8 KiB pitch), 2 stages in flight", [&] {
    hipLaunchKernelGGL((read_tiles<false, 2>), dim3(tiles), dim3(512), 0, 0, p, out);
  });
  run("tile rows (8 KiB pitch), 4 stages in flight", [&] {
    hipLaunchKernelGGL((read_tiles<false, 4>), dim3(tiles), dim3(512), 0, 0, p, out);
  });
  run("packed stages, 2 stages in flight", [&] {
    hipLaunchKernelGGL((read_tiles<true, 2>), dim3(tiles), dim3(512), 0, 0, p, out);
  });
  run("packed stages, 4 stages in flight", [&] {
    hipLaunchKernelGGL((read_tiles<true, 4>), dim3(tiles), dim3(512), 0, 0, p, out);
  });
  CHECK(hipDeviceSynchronize());
  return 0;
}
