// Eviction by gather (appendix "Details of Proposed Method"): the kept K and V rows are copied, bit
// for bit and in ascending position order, into a new compact cache; the old cache is left untouched.
// Rotary phases are therefore exactly those of the original positions (appendix on rotary embeddings).
//
// A row is 2*d bytes (128 or 256); d/8 neighbouring lanes move one row with 16-byte accesses, so both
// the read of a kept row and the write of the compact row are fully coalesced.  This is the only
// place where V is touched.
#include "pkv_internal.h"

namespace pkv {
namespace {

template <int D>
__global__ __launch_bounds__(256) void gather_kernel(const GatherArgs a) {
  constexpr int LPR = D / 8;  // lanes per row
  const int bg = blockIdx.y;
  const int b = bg / a.Hkv;
  const int g = bg - b * a.Hkv;
  const int t = blockIdx.x * 256 + threadIdx.x;
  const int j = t / LPR, seg = t - j * LPR;
  if (j >= a.k_cap) return;
  const int src = a.idx[(size_t)bg * a.k_cap + j];
  uint4 kv = make_uint4(0, 0, 0, 0), vv = kv;
  if (src >= 0) {
    const size_t off = (size_t)b * a.kv_sb + (size_t)g * a.kv_sh + (size_t)src * a.kv_st + seg * 8;
    kv = *reinterpret_cast<const uint4*>(a.K + off);
    vv = *reinterpret_cast<const uint4*>(a.V + off);
  }
  const size_t o = (size_t)b * a.o_sb + (size_t)g * a.o_sh + (size_t)j * a.o_st + seg * 8;
  *reinterpret_cast<uint4*>(a.K_out + o) = kv;
  *reinterpret_cast<uint4*>(a.V_out + o) = vv;
}

}  // namespace

hipError_t launch_gather(const GatherArgs& a, hipStream_t s) {
  const int lpr = a.d / 8;
  dim3 grid(((size_t)a.k_cap * lpr + 255) / 256, a.B * a.Hkv), block(256);
  if (a.d == 128)
    hipLaunchKernelGGL(gather_kernel<128>, grid, block, 0, s, a);
  else if (a.d == 64)
    hipLaunchKernelGGL(gather_kernel<64>, grid, block, 0, s, a);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace pkv
