// Group mean, 1-D pooling and per-head top-k selection (Sec. 4.2.2: "a pooling layer", "the top k^l
// tokens with the highest scores are selected"; the alpha instruction tokens are always kept).
//
// One 1024-thread workgroup per (sequence, KV head):
//   A. pooled[i] = pool_w-wide max / average of (1/G) * sum over row blocks of raw[i], prefix only;
//   B. radix select on the fp32 bit patterns (scores are >= 0, so unsigned order = numeric order):
//      three digit levels (12 + 10 + 10 bits), each a histogram of the keys that match the digits
//      found so far, followed by a suffix scan that locates the digit holding the kk-th largest key;
//      the result is the exact threshold T, and how many keys equal to T must be taken;
//   C. one ordered sweep emits the positions with key > T, and the lowest-position keys == T, in
//      ascending position order, followed by the window positions.
// All counters are integers and the sweep is ordered, so the result does not depend on scheduling.
#include "pkv_internal.h"

namespace pkv {
namespace {

constexpr int NT = kSelectThreads;
constexpr int NW = NT / 64;
constexpr int TS = 4096;  // pooling tile (outputs per iteration)
constexpr int HIST = 4096;

// Inclusive scan over the workgroup, thread order.  `scratch` holds NW entries.
template <typename T>
__device__ __forceinline__ T block_inclusive_scan(T v, T* scratch, T* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    T u = __shfl_up(v, o);
    if (lane >= o) v += u;
  }
  __syncthreads();  // scratch may still be read from a previous use
  if (lane == 63) scratch[wave] = v;
  __syncthreads();
  T base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const T s = scratch[w];
    if (w < wave) base += s;
    tot += s;
  }
  if (total) *total = tot;
  return v + base;
}

__global__ __launch_bounds__(NT) void pool_select_kernel(const SelectArgs a) {
  __shared__ float tilebuf[TS + 2 * 32];
  __shared__ uint32_t hist[HIST];
  __shared__ unsigned long long scan64[NW];
  __shared__ uint32_t scan32[NW];
  __shared__ uint32_t sel_bin, sel_above;

  const int tid = threadIdx.x;
  const int bg = blockIdx.x;
  const int b = bg / a.Hkv;
  const int g = bg - b * a.Hkv;
  int n = a.N;
  if (a.seq_lens) {
    n = a.seq_lens[b];
    n = n < 0 ? 0 : (n > a.N ? a.N : n);
  }
  const int count = a.k_l < n ? a.k_l : n;
  if (g == 0 && tid == 0) a.count_out[b] = count;
  int32_t* idx = a.idx_out + (size_t)bg * a.k_cap;

  if (a.k_l >= n) {  // keep everything
    for (int j = tid; j < a.k_cap; j += NT) idx[j] = j < n ? j : -1;
    return;
  }
  const int npre = n - a.alpha;
  const int kk = a.k_l - a.alpha;  // prefix tokens to select; kk < npre
  float* pooled = a.pooled + (size_t)bg * a.N;

  // ---- A. group mean + pooling, tile by tile through LDS ----
  const int r = (a.pool == PKV_POOL_NONE) ? 0 : (a.pool_w - 1) / 2;
  const bool is_max = a.pool == PKV_POOL_MAX;
  const float inv_w = 1.0f / (float)a.pool_w;
  const size_t rb_stride = (size_t)a.B * a.Hkv * a.N;
  const float* raw = a.raw + (size_t)bg * a.N;
  for (int t0 = 0; t0 < npre; t0 += TS) {
    for (int e = tid; e < TS + 2 * r; e += NT) {
      const int i = t0 - r + e;
      float v = is_max ? -INFINITY : 0.f;
      if (i >= 0 && i < npre) {
        float s = 0.f;
        for (int q = 0; q < a.nrb; ++q) s += raw[q * rb_stride + i];
        v = s * a.inv_G;
      }
      tilebuf[e] = v;
    }
    __syncthreads();
    for (int e = tid; e < TS; e += NT) {
      const int i = t0 + e;
      if (i < npre) {
        float v;
        if (r == 0) {
          v = tilebuf[e];
        } else if (is_max) {
          v = tilebuf[e];
          for (int u = 1; u <= 2 * r; ++u) v = fmaxf(v, tilebuf[e + u]);
        } else {
          v = 0.f;
          for (int u = 0; u <= 2 * r; ++u) v += tilebuf[e + u];
          v *= inv_w;
        }
        pooled[i] = v;
      }
    }
    __syncthreads();
  }

  if (kk > 0) {
    // ---- B. radix select of the kk-th largest key ----
    const uint32_t* keys = reinterpret_cast<const uint32_t*>(pooled);
    uint32_t prefix = 0, prefix_mask = 0;
    uint32_t remaining = (uint32_t)kk;
    const int shifts[3] = {20, 10, 0};
    const int bits[3] = {12, 10, 10};
    for (int lvl = 0; lvl < 3; ++lvl) {
      const int shift = shifts[lvl];
      const uint32_t dmask = (1u << bits[lvl]) - 1u;
      for (int e = tid; e < HIST; e += NT) hist[e] = 0;
      __syncthreads();
      for (int i = tid; i < npre; i += NT) {
        const uint32_t key = keys[i];
        if ((key & prefix_mask) == prefix) atomicAdd(&hist[(key >> shift) & dmask], 1u);
      }
      __syncthreads();
      // thread t owns bins [4t, 4t+4); suffix sum over higher threads
      const int nbin = 1 << bits[lvl];
      uint32_t h[4], local = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int bin = 4 * tid + q;
        h[q] = bin < nbin ? hist[bin] : 0u;
        local += h[q];
      }
      uint32_t total;
      const uint32_t incl = block_inclusive_scan<uint32_t>(local, scan32, &total);
      uint32_t above = total - incl;  // keys in bins owned by higher threads
#pragma unroll
      for (int q = 3; q >= 0; --q) {
        if (above < remaining && above + h[q] >= remaining) {
          sel_bin = (uint32_t)(4 * tid + q);
          sel_above = above;
        }
        above += h[q];
      }
      __syncthreads();
      prefix |= sel_bin << shift;
      prefix_mask |= dmask << shift;
      remaining -= sel_above;
      __syncthreads();
    }
    const uint32_t T = prefix;          // bit pattern of the kk-th largest pooled score
    const uint32_t need_eq = remaining; // keys equal to T to take, lowest positions first (>= 1)

    // ---- C. ordered emission ----
    const int seg = (npre + NT - 1) / NT;
    const int s0 = min(tid * seg, npre), s1 = min(s0 + seg, npre);
    uint32_t cgt = 0, ceq = 0;
    for (int i = s0; i < s1; ++i) {
      const uint32_t key = keys[i];
      cgt += key > T;
      ceq += key == T;
    }
    const unsigned long long packed = ((unsigned long long)cgt << 32) | ceq;
    const unsigned long long incl = block_inclusive_scan<unsigned long long>(packed, scan64, nullptr);
    uint32_t gt_before = (uint32_t)(incl >> 32) - cgt;
    uint32_t eq_before = (uint32_t)(incl & 0xffffffffu) - ceq;
    for (int i = s0; i < s1; ++i) {
      const uint32_t key = keys[i];
      if (key > T) {
        idx[gt_before + min(eq_before, need_eq)] = i;
        ++gt_before;
      } else if (key == T) {
        if (eq_before < need_eq) idx[gt_before + eq_before] = i;
        ++eq_before;
      }
    }
  }
  for (int t = tid; t < a.alpha; t += NT) idx[kk + t] = npre + t;
}

}  // namespace

hipError_t launch_pool_select(const SelectArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(pool_select_kernel, dim3(a.B * a.Hkv), dim3(NT), 0, s, a);
  return hipGetLastError();
}

}  // namespace pkv
