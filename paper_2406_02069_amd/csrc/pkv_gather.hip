// Eviction by gather (appendix "Details of Proposed Method"): the kept K and V rows are copied, bit
// for bit and in ascending position order, into a new compact cache; the old cache is left untouched.
// Rotary phases are therefore exactly those of the original positions (appendix on rotary embeddings).
//
// A row is 2*d bytes (128 or 256); d/8 neighbouring lanes move one row with 16-byte accesses, so both
// the read of a kept row and the write of the compact row are fully coalesced.  All layers of a call
// are served by one launch (grid.z = layer).  This is the only place where V is touched.
//
// Paged output (appendix "PyramidKV Implementation at vLLM": one block table per layer, since every layer keeps a
// different number of tokens): kept row j of head g goes to page table[b][j / P], head g, slot j % P of the
// layer's pool [num_pages][Hkv][P][d]; nothing else in the pool is written.
#include "pkv_internal.h"

namespace pkv {
namespace {

template <int D>
__global__ __launch_bounds__(256) void gather_batch_kernel(const GatherBatchArgs a) {
  constexpr int LPR = D / 8;  // lanes per row
  const GatherLayer& ly = a.layer[blockIdx.z];
  const int bg = blockIdx.y;
  const int b = bg / a.Hkv;
  const int g = bg - b * a.Hkv;
  const int t = blockIdx.x * 256 + threadIdx.x;
  const int j = t / LPR, seg = t - j * LPR;
  if (j >= ly.k_cap) return;
  gather_row_segment(a, ly, b, g, j, seg);
}

// Plain streaming read (bandwidth probe): every lane folds its 16-byte words into a checksum.
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ p, size_t n16, uint32_t* sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * 256 * 4;
  for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i < n16; i += stride) {
    uint4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = (i + 256 * k < n16) ? p[i + 256 * k] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int k = 0; k < 4; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
  }
  if (acc == 0x9E3779B9u) *sink = acc;
}

}  // namespace

hipError_t launch_probe_read(const void* buf, size_t bytes, uint32_t* sink, hipStream_t s) {
  hipLaunchKernelGGL(probe_read_kernel, dim3(256 * 8), dim3(256), 0, s, static_cast<const uint4*>(buf), bytes / 16, sink);
  return hipGetLastError();
}

hipError_t launch_gather_batch(const GatherBatchArgs& a, hipStream_t s) {
  const int lpr = a.d / 8;
  dim3 grid(((size_t)a.k_cap_max * lpr + 255) / 256, a.B * a.Hkv, a.L), block(256);
  if (a.d == 128)
    hipLaunchKernelGGL(gather_batch_kernel<128>, grid, block, 0, s, a);
  else if (a.d == 64)
    hipLaunchKernelGGL(gather_batch_kernel<64>, grid, block, 0, s, a);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace pkv
