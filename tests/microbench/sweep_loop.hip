// Stand-alone loop with the instruction mix of the scoring kernel's sweeps (Sec. 4.2.2, Eq. Al: one 32x32x128
// product of bf16 fragments = 8 MFMAs, then per logit one multiply, one exp2 and one add), on every SIMD of the
// chip, with nothing else going on: no key loads, no exchange between workgroups, no barriers.  It gives the
// rate at which the vector and matrix pipes can turn products into exponentials, i.e. the floor of two exact
// fp32 softmax sweeps, and the shader clock the chip sustains under that load.
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         tests/microbench/sweep_loop.hip -o /tmp/sweep_loop && /tmp/sweep_loop
//
// Variants: sweep 1 mix (plain) and sweep 2 mix (a ninth MFMA per product that adds the normaliser, Q fragments
// re-read from LDS for every second product); one or two waves per SIMD (256 or 512 workgroups of 4 waves);
// operand bits all zero or random (the clock under load depends on how many bits toggle).
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8 as_frag(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }
#define PIN2(a, b) asm volatile("" : "+v"(a), "+v"(b))
#define MF(A, B, C) __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B, C, 0, 0, 0)

template <int SWEEP2>
__global__ __launch_bounds__(256, 2) void loop_kernel(const u32x4* __restrict__ src, float* out, int iters, float a,
                                                      long long* clk) {
  __shared__ u32x4 qs[128 * 17];
  __shared__ unsigned long long cfr[128];
  const long long c0 = clock64(), w0 = wall_clock64();
  const int lane = threadIdx.x & 63, l32 = lane & 31, hf = lane >> 5;
  for (int e = threadIdx.x; e < 128 * 17; e += 256) qs[e] = src[e % 2048];
  if (threadIdx.x < 128) cfr[threadIdx.x] = 0x00003F803F803F80ull;
  __syncthreads();
  bf16x8 fa[8], fb[32];  // one row tile of Q, four key tiles: what a wave of the scoring kernel holds
  const u32x4* ql = qs + l32 * 17 + hf;
#pragma unroll
  for (int i = 0; i < 8; ++i) fa[i] = as_frag(ql[2 * i]);
#pragma unroll
  for (int i = 0; i < 32; ++i) fb[i] = as_frag(src[(8 + i) * 64 + lane]);
  const u32x4 ones_u = (hf == 0) ? u32x4{0x3F803F80u, 0x00003F80u, 0u, 0u} : u32x4{0u, 0u, 0u, 0u};
  const bf16x8 ones = as_frag(ones_u);
  const unsigned long long* cl = cfr + l32;
  f32x16 zero16;
  for (int v = 0; v < 16; ++v) zero16[v] = 0.f;
  f32x16 accA = zero16, accB = zero16;
  float s0 = 0.f, s1 = 0.f;
  bf16x8 bfr = as_frag(u32x4{0u, 0u, 0u, 0u});
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {  // four products per iteration, the two accumulators swapping roles
      const int rtn = (2 * it + (p >> 1) + 1) & 3;
      f32x16& outp = (p & 1) ? accA : accB;
      const f32x16& fin = (p & 1) ? accB : accA;
      if (SWEEP2) {
        outp = MF(bfr, ones, zero16);
        if ((p & 1) == 0) {
          const unsigned long long w = cl[32 * rtn];
          bfr = as_frag(u32x4{(unsigned)w, (unsigned)(w >> 32), 0u, 0u});
        }
      } else {
        outp = zero16;
      }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        outp = MF(fa[ks], fb[p * 8 + ks], outp);
        if (SWEEP2 && (p & 1) == 0) fa[ks] = as_frag(ql[32 * rtn * 17 + 2 * ks]);
        const float x0 = fin[2 * ks] * a, x1 = fin[2 * ks + 1] * a;
        const float e0 = __builtin_amdgcn_exp2f(x0), e1 = __builtin_amdgcn_exp2f(x1);
        s0 += e0;
        s1 += e1;
        PIN2(s0, s1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  float t = s0 + s1;
  for (int v = 0; v < 16; ++v) t += accA[v] + accB[v];
  out[blockIdx.x * 256 + threadIdx.x] = t;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clk[0] = clock64() - c0;
    clk[1] = wall_clock64() - w0;
  }
}

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

template <int SWEEP2>
static int run(int pattern, int waves_per_simd, const u32x4* src, float* out, long long* clk) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const int iters = 1000, blocks = 256 * waves_per_simd;
  hipLaunchKernelGGL((loop_kernel<SWEEP2>), dim3(blocks), dim3(256), 0, 0, src, out, iters, -0.01f, clk);  // warm-up
  CK(hipEventRecord(e0));
  hipLaunchKernelGGL((loop_kernel<SWEEP2>), dim3(blocks), dim3(256), 0, 0, src, out, iters, -0.01f, clk);
  CK(hipEventRecord(e1));
  CK(hipEventSynchronize(e1));
  float ms;
  CK(hipEventElapsedTime(&ms, e0, e1));
  long long h[2];
  CK(hipMemcpy(h, clk, 16, hipMemcpyDeviceToHost));
  // a SIMD finishes 4 * waves_per_simd products per iteration
  const double ns = ms * 1e6 / iters / 4 / waves_per_simd, mhz = (double)h[0] / h[1] * 100.0;
  printf("operands %-6s %s mix, %d wave(s) per SIMD: %6.1f ns per product and SIMD = %4.0f clk at %4.0f MHz; "
         "2 x 1048576 products (32 layers of the 32k workload) over 1024 SIMDs: %.3f ms\n",
         pattern ? "random" : "zero", SWEEP2 ? "sweep-2" : "sweep-1", waves_per_simd, ns, ns * mhz * 1e-3, mhz,
         ns * 2048 * 1e-6);
  return 0;
}

int main() {
  float* out;
  long long* clk;
  u32x4* src;
  const size_t n = 2048 + 40 * 64;
  unsigned* h = (unsigned*)malloc(n * 16);
  CK(hipMalloc(&src, n * 16));
  CK(hipMalloc(&out, 4096 * 256 * 4));
  CK(hipMalloc(&clk, 16));
  srand(1);
  for (int pattern = 0; pattern < 2; ++pattern) {
    for (size_t i = 0; i < n * 4; ++i)  // random: bf16 pairs of moderate magnitude and random sign
      h[i] = pattern == 0 ? 0u : (unsigned)(rand() & 0x3fff3fff) | (rand() & 1 ? 0x80000000u : 0u) | (rand() & 1 ? 0x8000u : 0u);
    CK(hipMemcpy(src, h, n * 16, hipMemcpyHostToDevice));
    for (int wps = 1; wps <= 2; ++wps) {
      if (run<0>(pattern, wps, src, out, clk)) return 1;
      if (run<1>(pattern, wps, src, out, clk)) return 1;
    }
  }
  return 0;
}
