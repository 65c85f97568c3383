// Probe behind the instruction plan of the main loop in gemm_bf16_kernels.hip: what other
// instructions cost behind back-to-back independent MFMA 16x16x32 (16 cycles each) when a SIMD
// holds one wavefront.  Prints cycles per MFMA (shader clock counter) with NS scalar, NV vector
// and NL LDS-read instructions, or NW s_waitcnt, behind every MFMA.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

template <int NS, int NV, int NL, int NW>
__global__ __launch_bounds__(256, 1) void probe(const bf16x8* src, float* out, unsigned long long* cyc, int iters) {
  __shared__ __attribute__((aligned(16))) char lds[65536];
  const int tid = threadIdx.x;
  for (int o = tid; o < 65536 / 16; o += 256) reinterpret_cast<i32x4*>(lds)[o] = i32x4{o, o, o, o};
  __syncthreads();
  bf16x8 a[8], b[8];
  for (int i = 0; i < 8; ++i) { a[i] = src[i * 256 + tid]; b[i] = src[(8 + i) * 256 + tid]; }
  f32x4 acc[8][8];
  for (int i = 0; i < 8; ++i) for (int j = 0; j < 8; ++j) for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
  int sa = 1, sb = 0, sc = 0, va = tid;
  i32x4 lv = {0, 0, 0, 0};
  const unsigned lp = (unsigned)(size_t)(lds + (tid & 63) * 16);
  const unsigned long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(a[i]), "v"(b[j]));
#pragma unroll
        for (int x = 0; x < NS; ++x) {      // independent of each other
          if (x & 1) asm volatile("s_add_u32 %0, %1, 3" : "=s"(sb) : "s"(sa) : "scc");
          else       asm volatile("s_add_u32 %0, %1, 5" : "=s"(sc) : "s"(sa) : "scc");
        }
#pragma unroll
        for (int x = 0; x < NV; ++x) asm volatile("v_add_u32 %0, 3, %0" : "+v"(va));
#pragma unroll
        for (int x = 0; x < NL; ++x) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(lv) : "v"(lp), "n"((i * 8 + j) * 1024 % 49152));
#pragma unroll
        for (int x = 0; x < NW; ++x) asm volatile("s_waitcnt lgkmcnt(15)" ::: "memory");
      }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  const unsigned long long t1 = __builtin_readcyclecounter();
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  float total = (float)(sa + sb + sc + va + lv[0]);
  for (int i = 0; i < 8; ++i) for (int j = 0; j < 8; ++j) for (int v = 0; v < 4; ++v) total += acc[i][j][v];
  out[blockIdx.x * 256 + tid] = total;
  if (tid == 0) cyc[blockIdx.x] = t1 - t0;
}

template <int NS, int NV, int NL, int NW>
static void run(const bf16x8* d, float* out, unsigned long long* cyc) {
  const int iters = 2000;
  for (int rep = 0; rep < 3; ++rep) hipLaunchKernelGGL((probe<NS, NV, NL, NW>), dim3(256), dim3(256), 0, 0, d, out, cyc, iters);
  std::vector<unsigned long long> h(256);
  if (hipMemcpy(h.data(), cyc, 256 * 8, hipMemcpyDeviceToHost) != hipSuccess) { printf("failed\n"); return; }
  double s = 0;
  for (auto x : h) s += (double)x;
  printf("behind every MFMA: %d scalar, %d vector, %d LDS read, %d s_waitcnt  ->  %.2f cycles per MFMA\n", NS, NV, NL, NW,
         s / 256 / iters / 64);
}

int main() {
  std::vector<unsigned short> h(16 * 256 * 8);
  srand(1);
  for (auto& x : h) x = (unsigned short)(0x3f00 + (rand() & 0xff));
  bf16x8* d = nullptr; float* out = nullptr; unsigned long long* cyc = nullptr;
  if (hipMalloc(&d, h.size() * 2) != hipSuccess || hipMalloc(&out, 256 * 256 * 4) != hipSuccess ||
      hipMalloc(&cyc, 256 * 8) != hipSuccess) return 1;
  if (hipMemcpy(d, h.data(), h.size() * 2, hipMemcpyHostToDevice) != hipSuccess) return 1;
  run<0, 0, 0, 0>(d, out, cyc);
  run<1, 0, 0, 0>(d, out, cyc);
  run<2, 0, 0, 0>(d, out, cyc);
  run<3, 0, 0, 0>(d, out, cyc);
  run<0, 1, 0, 0>(d, out, cyc);
  run<0, 2, 0, 0>(d, out, cyc);
  run<0, 0, 1, 0>(d, out, cyc);
  run<0, 0, 2, 0>(d, out, cyc);
  run<1, 0, 1, 0>(d, out, cyc);
  run<2, 0, 1, 0>(d, out, cyc);
  run<0, 1, 1, 0>(d, out, cyc);
  run<0, 0, 0, 2>(d, out, cyc);
  run<0, 0, 1, 1>(d, out, cyc);
  (void)hipFree(d); (void)hipFree(out); (void)hipFree(cyc);
  return 0;
}
