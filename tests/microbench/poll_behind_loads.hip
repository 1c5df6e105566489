// Does a small load of one workgroup wait behind the outstanding bulk loads of ANOTHER workgroup of the same
// compute unit?  The scoring kernel's exchange polls single words (agent-scope relaxed loads) while the other
// workgroup of its compute unit requests the 128 KB of its next keys; this measures the round trip of such a poll
//   (a) on an idle chip,
//   (b) while the second workgroup of the SAME compute units streams from HBM in bursts of 32 x 16 bytes per lane,
//   (c) while the same number of workgroups stream on OTHER compute units only (same load on the memory system,
//       none on the poller's compute unit),
//   (d) as (b) with smaller bursts (8 and 2 loads per lane between waits): if a poll only queued at the entrance
//       of the memory pipeline behind the requests of a burst, short bursts would let it through; if loads return
//       in the order in which the compute unit issued them, it still waits for the data of the burst before it.
// 512 workgroups of 256 threads with 80 KB of LDS each, so exactly two share a compute unit (blockIdx % 8 is the
// XCD and an XCD gives every compute unit one workgroup before any gets a second one).
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         tests/microbench/poll_behind_loads.hip -o /tmp/poll_behind_loads && /tmp/poll_behind_loads
//
// Every loop has a fixed trip count or a bounded one; nothing here can hang.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <algorithm>
#include <vector>
typedef unsigned long long u64;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u64 get(const u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// role of a workgroup: 0 leaves at once, 1 polls, 2 streams
__host__ __device__ __forceinline__ int role_of(int mode, int set, int cu) {
  const bool even = (cu & 1) == 0;
  if (mode == 0) return (set == 0 && even) ? 1 : 0;
  if (mode == 1) return even ? (set == 0 ? 1 : 2) : 0;           // streamers share the pollers' compute units
  return (set == 0 && even) ? 1 : ((set == 1 && !even) ? 2 : 0);  // streamers on the other compute units
}

template <int NB>
__global__ __launch_bounds__(256) void poll_kernel(int mode, const u64* words, int iters, long long* rt_out,
                                                   const char* bg, size_t bg_bytes, int max_reps, unsigned* sink,
                                                   int* stop, int* pollers_left) {
  extern __shared__ char lds_pad[];  // only there to limit residency to two workgroups per compute unit
  const int kk = blockIdx.x >> 3, set = kk >> 5, cu = kk & 31;
  const int role = role_of(mode, set, cu);
  if (role == 0) return;
  if (threadIdx.x == 0) lds_pad[0] = 0;
  if (role == 1) {
    if (threadIdx.x >= 64) return;
    // dependent polls of one word: the next address depends on the value just read (always 0)
    const u64* p = words + (blockIdx.x & 255) * 16;
    u64 v = 0;
    const long long t0 = wall_clock64();
    for (int i = 0; i < iters; ++i) v += get(p + v);
    const long long t1 = wall_clock64();
    if (threadIdx.x == 0) {
      rt_out[blockIdx.x] = t1 - t0 + (long long)v;
      if (__hip_atomic_fetch_add(pollers_left, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 1)
        __hip_atomic_store(stop, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return;
  }
  // streamer: bursts of 32 loads of 16 bytes per lane, one 256-byte row per lane pair (the key-load pattern of the
  // scoring kernel), the workgroup's 128 KB per burst taken from a region of its own
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  unsigned acc = 0;
  const size_t nburst = bg_bytes / (128 * 1024);
  for (int rep = 0; rep < max_reps; ++rep) {
    const size_t burst = ((size_t)rep * 512 + blockIdx.x) % nburst;
    const char* base = bg + burst * (128 * 1024) + (size_t)wave * (32 * 1024);
    // NB loads per lane are requested together; the wave waits for them before it requests the next NB
#pragma unroll
    for (int i0 = 0; i0 < 32; i0 += NB) {
      u32x4 v[NB];
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int t = (i0 + i) >> 3, ks = (i0 + i) & 7;
        v[i] = *reinterpret_cast<const u32x4*>(base + (size_t)(32 * t + l32) * 256 + 16 * hf + 32 * ks);
      }
#pragma unroll
      for (int i = 0; i < NB; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
      asm volatile("" : "+v"(acc));
    }
    if (__hip_atomic_load(stop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
  }
  if (acc == 0x12345678u) *sink = acc;
}

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

int main() {
  const int G = 512, iters = 400;
  const size_t lds = 80 * 1024;
  CK(hipFuncSetAttribute(reinterpret_cast<const void*>(poll_kernel<32>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  CK(hipFuncSetAttribute(reinterpret_cast<const void*>(poll_kernel<8>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  CK(hipFuncSetAttribute(reinterpret_cast<const void*>(poll_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  u64* words; CK(hipMalloc(&words, 256 * 16 * 8)); CK(hipMemset(words, 0, 256 * 16 * 8));
  long long* rt; CK(hipMalloc(&rt, G * 8));
  int* flags; CK(hipMalloc(&flags, 8));
  unsigned* sink; CK(hipMalloc(&sink, 4));
  const size_t bg_bytes = (size_t)4 << 30;
  char* bg; CK(hipMalloc(&bg, bg_bytes)); CK(hipMemset(bg, 1, bg_bytes));
  const char* names[5] = {"idle chip", "streamers on the pollers' compute units", "streamers on other compute units",
                          "... on the pollers' units, 8 loads per burst", "... on the pollers' units, 2 loads per burst"};
  for (int rep = 0; rep < 2; ++rep)
    for (int cs = 0; cs < 5; ++cs) {
      const int mode = cs < 3 ? cs : 1;
      int npoll = 0;
      for (int b = 0; b < G; ++b) npoll += role_of(mode, (b >> 3) >> 5, (b >> 3) & 31) == 1;
      const int init[2] = {0, npoll};
      CK(hipMemcpy(flags, init, 8, hipMemcpyHostToDevice));
      CK(hipMemset(rt, 0, G * 8));
      CK(hipDeviceSynchronize());
      hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
      CK(hipEventRecord(e0));
      if (cs < 3) poll_kernel<32><<<G, 256, lds>>>(mode, words, iters, rt, bg, bg_bytes, 20000, sink, flags, flags + 1);
      else if (cs == 3) poll_kernel<8><<<G, 256, lds>>>(mode, words, iters, rt, bg, bg_bytes, 20000, sink, flags, flags + 1);
      else poll_kernel<2><<<G, 256, lds>>>(mode, words, iters, rt, bg, bg_bytes, 20000, sink, flags, flags + 1);
      CK(hipEventRecord(e1));
      CK(hipDeviceSynchronize());
      float ms = 0; CK(hipEventElapsedTime(&ms, e0, e1));
      std::vector<long long> h(G);
      CK(hipMemcpy(h.data(), rt, G * 8, hipMemcpyDeviceToHost));
      std::vector<double> us;
      for (int b = 0; b < G; ++b) if (h[b] > 0) us.push_back(h[b] * 0.01 / iters);
      std::sort(us.begin(), us.end());
      double mean = 0; for (double x : us) mean += x; mean /= us.size();
      printf("%-42s: %3zu pollers, poll round trip mean %.3f us, median %.3f, slowest poller %.3f  (kernel %.2f ms)\n",
             names[cs], us.size(), mean, us[us.size() / 2], us.back(), ms);
    }
  return 0;
}
