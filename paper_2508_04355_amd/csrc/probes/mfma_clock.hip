// Probe behind the choice of MFMA shape in gemm_bf16_kernels.hip: what the chip sustains on a
// loop of nothing but independent bf16 MFMAs on register operands (one workgroup of four
// wavefronts per compute unit, no memory traffic in the loop), for the two shapes that deliver
// 1024 flop per cycle and SIMD.  Prints TFLOP/s over a few seconds of launches back to back;
// with the MFMA pipes ~99 % busy that is the clock: GHz = TFLOP/s / (256 CUs x 4096 flop).
//   usage: mfma_clock [shape 32|16] [seconds] [sigma_b]
#include <hip/hip_runtime.h>
#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// per wavefront and iteration: a 128 x 128 block of accumulators advanced by k = 32
// (32: 2 x 16 MFMA 32x32x16;  16: 64 MFMA 16x16x32)
template <int SHAPE>
__global__ __launch_bounds__(256, 1) void burn(const bf16x8* src, float* out, int iters) {
  const int tid = threadIdx.x;
  float total = 0.f;
  if (SHAPE == 32) {
    bf16x8 a[2][4], b[2][4];
    for (int s = 0; s < 2; ++s)
      for (int i = 0; i < 4; ++i) { a[s][i] = src[(s * 8 + i) * 256 + tid]; b[s][i] = src[(s * 8 + 4 + i) * 256 + tid]; }
    f32x16 acc[4][4];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(a[s][i]), "v"(b[s][j]));
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 4; ++j) for (int v = 0; v < 16; ++v) total += acc[i][j][v];
  } else {
    bf16x8 a[8], b[8];
    for (int i = 0; i < 8; ++i) { a[i] = src[i * 256 + tid]; b[i] = src[(8 + i) * 256 + tid]; }
    f32x4 acc[8][8];
    for (int i = 0; i < 8; ++i) for (int j = 0; j < 8; ++j) for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
          asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(a[i]), "v"(b[j]));
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    for (int i = 0; i < 8; ++i) for (int j = 0; j < 8; ++j) for (int v = 0; v < 4; ++v) total += acc[i][j][v];
  }
  out[blockIdx.x * 256 + tid] = total;
}

static uint16_t bf16_of(float x) { uint32_t u; memcpy(&u, &x, 4); u += 0x7fff + ((u >> 16) & 1); return (uint16_t)(u >> 16); }

int main(int argc, char** argv) {
  const int shape = argc > 1 ? atoi(argv[1]) : 16;
  const double seconds = argc > 2 ? atof(argv[2]) : 2.0;
  const float sigma_b = argc > 3 ? (float)atof(argv[3]) : 0.02f;
  if (shape != 16 && shape != 32) { fprintf(stderr, "shape must be 16 or 32\n"); return 2; }
  const int nvec = 16 * 256;             // 16 fragments per lane: A-type (sigma 1) and B-type (sigma_b)
  std::vector<uint16_t> h((size_t)nvec * 8);
  srand(1);
  for (int v = 0; v < nvec; ++v) {
    const int f = v / 256;
    const bool isb = shape == 32 ? (f % 8) >= 4 : f >= 8;
    for (int e = 0; e < 8; ++e) {
      float s = 0.f;
      for (int q = 0; q < 12; ++q) s += rand() / (float)RAND_MAX;      // ~ N(0, 1)
      h[(size_t)v * 8 + e] = bf16_of((s - 6.f) * (isb ? sigma_b : 1.f));
    }
  }
  bf16x8* d = nullptr; float* out = nullptr;
  if (hipMalloc(&d, h.size() * 2) != hipSuccess || hipMalloc(&out, 256 * 256 * 4) != hipSuccess) return 1;
  if (hipMemcpy(d, h.data(), h.size() * 2, hipMemcpyHostToDevice) != hipSuccess) return 1;
  const int iters = 4000;
  const double flop_per_launch = 256.0 * 4 * iters * (2.0 * 128 * 128 * 32);
  auto launch = [&]() {
    if (shape == 32) hipLaunchKernelGGL(burn<32>, dim3(256), dim3(256), 0, 0, d, out, iters);
    else hipLaunchKernelGGL(burn<16>, dim3(256), dim3(256), 0, 0, d, out, iters);
  };
  launch();
  if (hipDeviceSynchronize() != hipSuccess) return 1;
  const auto t0 = std::chrono::steady_clock::now();
  double elapsed = 0;
  int n = 0;
  while (elapsed < seconds) {
    const auto a = std::chrono::steady_clock::now();
    for (int r = 0; r < 10; ++r) launch();
    if (hipDeviceSynchronize() != hipSuccess) { printf("launch failed\n"); return 1; }
    const auto b = std::chrono::steady_clock::now();
    const double dt = std::chrono::duration<double>(b - a).count();
    elapsed = std::chrono::duration<double>(b - t0).count();
    if (++n % 5 == 0)
      printf("MFMA %s  t=%.2f s  %.1f TFLOP/s  (%.3f GHz at full pipes)\n", shape == 32 ? "32x32x16" : "16x16x32", elapsed,
             10 * flop_per_launch / dt / 1e12, 10 * flop_per_launch / dt / (256.0 * 4096) / 1e9);
  }
  (void)hipFree(d); (void)hipFree(out);
  return 0;
}
