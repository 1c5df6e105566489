// Which XCD does workgroup i of a 512-workgroup launch run on, and how long does a word take from one workgroup
// to another: agent-scope relaxed store on one side, agent-scope relaxed load in a spin loop on the other (what
// the scoring kernel's exchange of softmax statistics uses), between workgroups of the same XCD and of different
// XCDs, on an idle chip and beside a streaming read by all other workgroups.
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         tests/microbench/xcd_latency.hip -o /tmp/xcd_latency && /tmp/xcd_latency
//
// Every wait is bounded by a probe count; nothing here can hang.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>
typedef unsigned long long u64;

__global__ void where_kernel(int* xcc, int* hwid) {
  if (threadIdx.x == 0) {
    xcc[blockIdx.x] = __builtin_amdgcn_s_getreg((3 << 11) | 20);   // HW_REG_XCC_ID, bits 0..3
    hwid[blockIdx.x] = __builtin_amdgcn_s_getreg((31 << 11) | 4);  // HW_REG_HW_ID
  }
  // stay a while so that every workgroup of the grid is resident at once
  const long long t0 = wall_clock64();
  while (wall_clock64() - t0 < 2000) __builtin_amdgcn_s_sleep(8);
}

__device__ __forceinline__ void put(u64* p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ u64 get(u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Workgroups A and B bounce a counter: A writes 2i+1 to ab, B answers 2i+2 on ba.  Everybody else streams `bg`
// (or leaves at once if bg is null).  Every wait is bounded by `limit` probes.
__global__ __launch_bounds__(256) void ping_kernel(u64* ab, u64* ba, int A, int B, int iters, int limit, long long* out,
                                                   const uint4* bg, size_t bg_n, unsigned* sink, int* stop) {
  const int b = blockIdx.x;
  if (b != A && b != B) {
    if (!bg) return;
    unsigned acc = 0;
    for (int rep = 0; rep < 64; ++rep) {
      for (size_t i = (size_t)b * 256 + threadIdx.x; i < bg_n; i += (size_t)gridDim.x * 256) {
        const uint4 v = bg[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
      }
      if (__hip_atomic_load(stop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
    }
    if (acc == 0x12345678u) *sink = acc;
    return;
  }
  if (threadIdx.x != 0) return;
  const long long t0 = wall_clock64();
  int fails = 0;
  for (int i = 0; i < iters; ++i) {
    if (b == A) {
      put(ab, (u64)(2 * i + 1));
      int n = 0;
      while (get(ba) != (u64)(2 * i + 2) && ++n < limit) {}
      fails += n >= limit;
    } else {
      int n = 0;
      while (get(ab) != (u64)(2 * i + 1) && ++n < limit) {}
      fails += n >= limit;
      put(ba, (u64)(2 * i + 2));
    }
    if (fails) break;
  }
  out[b == A ? 0 : 1] = wall_clock64() - t0;
  out[2 + (b == A ? 0 : 1)] = fails;
  if (b == A) __hip_atomic_store(stop, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

int main() {
  const int G = 512;
  int *xcc, *hwid;
  CK(hipMalloc(&xcc, G * 4)); CK(hipMalloc(&hwid, G * 4));
  where_kernel<<<G, 256>>>(xcc, hwid);
  CK(hipDeviceSynchronize());
  std::vector<int> hx(G), hh(G);
  CK(hipMemcpy(hx.data(), xcc, G * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(hh.data(), hwid, G * 4, hipMemcpyDeviceToHost));
  int mism = 0;
  for (int i = 0; i < G; ++i) mism += (hx[i] & 15) != (i & 7);
  printf("xcc id of workgroups 0..15:");
  for (int i = 0; i < 16; ++i) printf(" %d", hx[i] & 15);
  printf("\nworkgroups whose XCC id != blockIdx %% 8: %d of %d\n", mism, G);
  printf("hw_id of workgroups 0,8,16,256,264: %08x %08x %08x %08x %08x\n", hh[0], hh[8], hh[16], hh[256], hh[264]);

  u64* words;
  CK(hipMalloc(&words, 4096));
  long long* out; CK(hipMalloc(&out, 64));
  int* stop; CK(hipMalloc(&stop, 4));
  unsigned* sink; CK(hipMalloc(&sink, 4));
  const size_t bg_bytes = (size_t)1 << 30;
  uint4* bg; CK(hipMalloc(&bg, bg_bytes));
  CK(hipMemset(bg, 1, bg_bytes));
  const int iters = 2000, limit = 200000;
  for (int load = 0; load < 2; ++load)
    for (int pair = 0; pair < 3; ++pair) {
      // partner of workgroup 0: same XCD, other compute unit / other XCD / same XCD, second workgroup of a compute unit
      const int A = 0, B = pair == 0 ? 8 : (pair == 1 ? 1 : 264);
      CK(hipMemset(words, 0, 4096)); CK(hipMemset(out, 0, 64)); CK(hipMemset(stop, 0, 4));
      CK(hipDeviceSynchronize());
      ping_kernel<<<G, 256>>>(words, words + 64, A, B, iters, limit, out, load ? bg : nullptr, bg_bytes / 16, sink, stop);
      CK(hipDeviceSynchronize());
      long long h[4];
      CK(hipMemcpy(h, out, 32, hipMemcpyDeviceToHost));
      printf("%s, workgroups (0,%3d): round trip %.3f us, one way %.3f us  (waits given up: %lld %lld)\n",
             load ? "beside a streaming read" : "idle chip             ", B, h[0] * 0.01 / iters, h[0] * 0.005 / iters, h[2], h[3]);
    }
  return 0;
}
