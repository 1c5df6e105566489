// The step after the compression path: one decoding query per sequence attends over the compacted cache of a
// layer (Sec. 3: after compression the model attends over K_s, V_s only).  The kept rows were copied bit for bit,
// so they carry the rotary phases of their original positions and nothing is re-rotated here (appendix on rotary
// embeddings); the cache is ragged (count_b rows per sequence) and may be paged with the layer's own block table
// (appendix "PyramidKV Implementation at vLLM").
//
// Work split: (sequence, KV head) x S key ranges, one 512-thread workgroup each; the G <= 8 query heads of a KV head
// share every key and value row.  S is chosen on the host so that a small batch still fills the chip; with S > 1
// the workgroups leave un-normalised partial results (reference exponent, sum, weighted values) in a workspace and
// a second small kernel merges them, with S = 1 the first kernel writes the result itself.
//   A. logits: the G queries, padded to a 32-row tile, are the A operand of v_mfma_f32_32x32x16_bf16; every wave
//      takes 32-key tiles, loaded from memory straight into the B-operand layout (one row per lane pair), the
//      next tile while the current one is multiplied.  The useful rows of the product are elements 0..3 of both
//      wave halves.  Logits go to LDS (log2 domain).
//   B. per head: maximum and sum over the range's keys; 2^(x - max) stored in place.
//   C. values: a lane moves 16 bytes of a value row per load (a wave: 4 rows at d = 128), eight loads in flight;
//      every lane keeps G x 8 partial outputs, added up over the lanes that share columns and then over the
//      waves through LDS, in a fixed order.
// HBM-bound: every kept K and V row is read once (2 x count x d x 2 bytes per head), the rest stays on chip.
#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ bf16x8 as_frag(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

constexpr int kMaxSplits = 16;     // key ranges per (sequence, KV head), at most
constexpr int kTabEntries = 1026;  // block-table entries of a key range kept in LDS (pages of 4 slots or more)

// Row j of (sequence b, head g) of a cache, or null if its page number is out of range.  tab: the block-table
// entries from page index q0 on (LDS), or null: read from the table in memory.
template <int D>
__device__ __forceinline__ const uint16_t* cache_row(const DecodeArgs& a, const uint16_t* base, int b, int g, int j,
                                                     const int* tab, int q0) {
  if (a.page_size > 0) {
    const int q = j / a.page_size, slot = j - q * a.page_size;
    const int pg = tab ? tab[q - q0] : a.table[(size_t)b * a.max_pages + q];
    if ((uint32_t)pg >= (uint32_t)a.num_pages) return nullptr;
    return base + (((size_t)pg * a.Hkv + g) * a.page_size + slot) * D;
  }
  return base + (size_t)b * a.c_sb + (size_t)g * a.c_sh + (size_t)j * a.c_st;
}

// Key range sp of (sequence b, KV head g) of one layer's cache.
// FINAL: S == 1, the result is written here; else partial results go to the workspace.
template <int D, bool FINAL>
__device__ __forceinline__ void decode_range(const DecodeArgs& a, int sp, int g, int b, float* dsm) {
  constexpr int KS = D / 16, SEG = D / 8, PITCH = SEG + 1;
  // dsm: [8][chunk] logits / weights | [32 * PITCH] Q tile (16-byte slots) | [4][8][D] partial outputs | [8][2]
  // (max, sum) | [kTabEntries] block-table entries of this key range
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int cnt = a.count[b];
  cnt = cnt < 0 ? 0 : (cnt > a.k_cap ? a.k_cap : cnt);
  const int j_lo = sp * a.chunk;
  const int nloc = max(min(cnt - j_lo, a.chunk), 0);  // keys of this workgroup: j_lo .. j_lo + nloc - 1
  float* s_p = dsm;
  u32x4* s_q = reinterpret_cast<u32x4*>(dsm + 8 * a.chunk);
  float* s_o = reinterpret_cast<float*>(s_q + 32 * PITCH);
  float* s_mz = s_o + 4 * 8 * D;
  int* s_tab = reinterpret_cast<int*>(s_mz + 16);
  const size_t unit = (size_t)b * a.Hkv + g;
  float* out = a.out + ((size_t)b * a.Hq + (size_t)g * a.G) * D;
  float* part_o = a.part_o + (unit * a.S + sp) * 8 * D;
  float* part_mz = a.part_mz + (unit * a.S + sp) * 16;
  if (nloc == 0) {  // nothing here: a neutral partial result, or (FINAL) zero rows and lse = -inf
    if (FINAL) {
      for (int e = tid; e < a.G * D; e += kThreads) out[e] = 0.f;
      if (a.lse && tid < a.G) a.lse[(size_t)b * a.Hq + g * a.G + tid] = -INFINITY;
    } else {
      for (int e = tid; e < a.G * D; e += kThreads) part_o[e] = 0.f;
      if (tid < a.G) {
        part_mz[2 * tid] = -INFINITY;
        part_mz[2 * tid + 1] = 0.f;
      }
    }
    return;
  }
  // paged cache: this range's block-table entries once into LDS, so that a row's address costs one memory access
  const int* tab = nullptr;
  int q0 = 0;
  if (a.page_size >= 4) {  // (at most chunk / 4 + 2 entries then)
    q0 = j_lo / a.page_size;
    const int n_ent = (j_lo + nloc - 1) / a.page_size - q0 + 1;
    for (int e = tid; e < n_ent; e += kThreads) s_tab[e] = a.table[(size_t)b * a.max_pages + q0 + e];
    tab = s_tab;
  }
  // ---- Q tile: rows 0..G-1 the group's queries, the rest zero ----
  for (int e = tid; e < 32 * SEG; e += kThreads) {
    const int r = e / SEG, seg = e - r * SEG;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (r < a.G) v = *reinterpret_cast<const u32x4*>(a.q + ((size_t)b * a.Hq + (size_t)g * a.G + r) * D + seg * 8);
    s_q[r * PITCH + seg] = v;
  }
  __syncthreads();
  // ---- A. logits ----
  const int l32 = lane & 31, hf = lane >> 5;
  const int ntiles = (nloc + 31) / 32;
  if (wave < ntiles) {
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = as_frag(s_q[l32 * PITCH + 2 * ks + hf]);
    // fragments of local key tile t (keys at or beyond the range's end: its last row, masked below)
    auto load_tile = [&](int t, bf16x8 (&kf)[KS], bool& ok) {
      const int key = t * 32 + l32;
      const uint16_t* row = cache_row<D>(a, a.K, b, g, j_lo + min(key, nloc - 1), tab, q0);
      ok = key < nloc && row != nullptr;
      if (row == nullptr) row = a.K;  // a bad page number: some readable row, masked
      const char* rp = reinterpret_cast<const char*>(row) + 16 * hf;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[ks] = as_frag(*reinterpret_cast<const u32x4*>(rp + 32 * ks));
    };
    bf16x8 kf[KS], kn[KS];
    bool ok = false, okn = false;
    load_tile(wave, kf, ok);
    for (int t = wave; t < ntiles; t += kWaves) {
      const bool more = t + kWaves < ntiles;
      if (more) load_tile(t + kWaves, kn, okn);
      f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[ks], kf[ks], acc, 0, 0, 0);
      // element v (0..3) of this lane: query row v + 4 * hf, local key t * 32 + l32
#pragma unroll
      for (int v = 0; v < 4; ++v) s_p[(v + 4 * hf) * a.chunk + t * 32 + l32] = ok ? acc[v] * a.scale_log2 : -INFINITY;
      if (more) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[ks] = kn[ks];
        ok = okn;
      }
    }
  }
  __syncthreads();
  // ---- B. per head: maximum, weights 2^(x - max) in place, their sum ----
  for (int h = wave; h < a.G; h += kWaves) {
    float* p = s_p + h * a.chunk;
    float m = -INFINITY;
    for (int j = lane; j < nloc; j += 64) m = fmaxf(m, p[j]);
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
    const float ms = (m == -INFINITY) ? 0.f : m;  // every page number bad: all rows masked
    float z = 0.f;
    for (int j = lane; j < nloc; j += 64) {
      const float e = __builtin_amdgcn_exp2f(p[j] - ms);
      p[j] = e;
      z += e;
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) z += __shfl_xor(z, s);
    if (lane == 0) {
      s_mz[2 * h] = m;
      s_mz[2 * h + 1] = z;
    }
  }
  __syncthreads();
  // ---- C. values: o[h][c] = sum_j w[h][j] V[j][c] ----
  // A lane moves 16 bytes (8 columns) of a value row per load, so a wave covers RPW rows per load and has UN of
  // those in flight; every lane keeps G x 8 partial outputs for its columns and its share of the rows.
  constexpr int LPR = D / 8;     // lanes per row
  constexpr int RPW = 64 / LPR;  // rows per wave and load
  constexpr int UN = 8;
  const int sub = lane / LPR, col = lane - sub * LPR;
  float o[8][8];
#pragma unroll
  for (int h = 0; h < 8; ++h)
#pragma unroll
    for (int c = 0; c < 8; ++c) o[h][c] = 0.f;
  for (int r0 = wave * RPW; r0 < nloc; r0 += UN * kWaves * RPW) {
    u32x4 w[UN];
    int rr[UN];
#pragma unroll
    for (int i = 0; i < UN; ++i) {
      const int r = r0 + i * kWaves * RPW + sub;
      rr[i] = r < nloc ? r : -1;
      const uint16_t* row = cache_row<D>(a, a.V, b, g, j_lo + min(r, nloc - 1), tab, q0);
      if (row == nullptr) {  // a bad page number: the row counts as absent (its weight is zero as well)
        row = a.V;
        rr[i] = -1;
      }
      w[i] = *reinterpret_cast<const u32x4*>(row + 8 * col);
    }
#pragma unroll
    for (int i = 0; i < UN; ++i) {
      const bool have = rr[i] >= 0;
      if (!have) w[i] = u32x4{0u, 0u, 0u, 0u};  // whatever was read there must not reach the sums
      float v[8];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        v[2 * c] = __uint_as_float(w[i][c] << 16);
        v[2 * c + 1] = __uint_as_float(w[i][c] & 0xFFFF0000u);
      }
      const int rc = have ? rr[i] : 0;
#pragma unroll
      for (int h = 0; h < 8; ++h) {
        if (h < a.G) {
          const float p = have ? s_p[h * a.chunk + rc] : 0.f;
#pragma unroll
          for (int c = 0; c < 8; ++c) o[h][c] = __builtin_fmaf(p, v[c], o[h][c]);
        }
      }
    }
  }
  // over the RPW row shares of a wave (lanes LPR apart hold the same columns), in a fixed order
#pragma unroll
  for (int h = 0; h < 8; ++h) {
    if (h < a.G) {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
#pragma unroll
        for (int sft = 32; sft >= LPR; sft >>= 1) o[h][c] += __shfl_xor(o[h][c], sft);
      }
    }
  }
  // over the waves: waves 0..3 store, then waves 4..7 add to slot (wave & 3)
  for (int r = 0; r < kWaves / 4; ++r) {
    if ((wave >> 2) == r && sub == 0) {
#pragma unroll
      for (int h = 0; h < 8; ++h) {
        if (h < a.G) {
#pragma unroll
          for (int c = 0; c < 8; ++c) {
            float* dst = &s_o[((wave & 3) * 8 + h) * D + 8 * col + c];
            *dst = (r == 0 ? 0.f : *dst) + o[h][c];
          }
        }
      }
    }
    __syncthreads();
  }
  for (int e = tid; e < a.G * D; e += kThreads) {
    const int h = e / D, c = e - h * D;
    const float x = s_o[(0 * 8 + h) * D + c] + s_o[(1 * 8 + h) * D + c] + s_o[(2 * 8 + h) * D + c] + s_o[(3 * 8 + h) * D + c];
    if (FINAL) {
      const float z = s_mz[2 * h + 1];
      out[e] = z > 0.f ? x / z : 0.f;
    } else {
      part_o[e] = x;
    }
  }
  if (tid < a.G) {
    const float m = s_mz[2 * tid], z = s_mz[2 * tid + 1];
    if (FINAL) {
      if (a.lse) a.lse[(size_t)b * a.Hq + g * a.G + tid] = z > 0.f ? (m + __builtin_amdgcn_logf(z)) * 0.69314718055994530942f : -INFINITY;
    } else {
      part_mz[2 * tid] = m;
      part_mz[2 * tid + 1] = z;
    }
  }
}

template <int D, bool FINAL>
__global__ __launch_bounds__(kThreads) void decode_partial_kernel(const DecodeArgs a) {
  extern __shared__ float dsm[];
  decode_range<D, FINAL>(a, blockIdx.x, blockIdx.y, blockIdx.z, dsm);
}

// Merge of the S partial results of a (sequence, KV head): common reference exponent, sums, weighted values.
template <int D>
__device__ __forceinline__ void decode_merge(const DecodeArgs& a, int g, int b) {
  const size_t unit = (size_t)b * a.Hkv + g;
  const float* part_o = a.part_o + unit * a.S * 8 * D;
  const float* part_mz = a.part_mz + unit * a.S * 16;
  float* out = a.out + ((size_t)b * a.Hq + (size_t)g * a.G) * D;
  for (int e = threadIdx.x; e < a.G * D; e += 256) {
    const int h = e / D;
    // all loads first (S <= kMaxSplits, so the loops unroll): one memory round trip instead of one per range
    float pm[kMaxSplits], pz[kMaxSplits], px[kMaxSplits];
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) {
      const bool have = s < a.S;
      pm[s] = have ? part_mz[s * 16 + 2 * h] : -INFINITY;
      pz[s] = have ? part_mz[s * 16 + 2 * h + 1] : 0.f;
      px[s] = have ? part_o[(size_t)s * 8 * D + e] : 0.f;
    }
    float M = -INFINITY;
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) M = fmaxf(M, pm[s]);
    const float Ms = (M == -INFINITY) ? 0.f : M;
    float z = 0.f, x = 0.f;
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s) {
      const float f = __builtin_amdgcn_exp2f(pm[s] - Ms);
      z += pz[s] * f;
      x += px[s] * f;
    }
    out[e] = z > 0.f ? x / z : 0.f;
    if (a.lse && e == h * D)
      a.lse[(size_t)b * a.Hq + g * a.G + h] = z > 0.f ? (M + __builtin_amdgcn_logf(z)) * 0.69314718055994530942f : -INFINITY;
  }
}

template <int D>
__global__ __launch_bounds__(256) void decode_merge_kernel(const DecodeArgs a) {
  decode_merge<D>(a, blockIdx.x, blockIdx.y);
}

// ---- all layers of a decoding step in one launch ----
// The layers' caches are small at batch 1 (a few hundred rows each under a pyramidal budget), and a launch per layer
// costs more than the rows it reads; here workgroup w of the grid finds its layer from the table's running workgroup
// counts and works on one key range of one (sequence, KV head) of it, exactly as above.
__device__ __forceinline__ DecodeArgs layer_args(const DecodeBatchArgs& a, int l) {
  const DecodeLayer& ly = a.layer[l];
  DecodeArgs d;
  d.q = ly.q; d.K = ly.K; d.V = ly.V; d.table = ly.table; d.count = ly.count; d.out = ly.out; d.lse = ly.lse;
  d.part_o = a.part_o + (size_t)ly.part0 * 8 * a.d;
  d.part_mz = a.part_mz + (size_t)ly.part0 * 16;
  d.B = a.B; d.Hq = a.Hq; d.Hkv = a.Hkv; d.G = a.G; d.d = a.d; d.k_cap = ly.k_cap;
  d.page_size = a.page_size; d.num_pages = ly.num_pages; d.max_pages = ly.max_pages;
  d.S = ly.S; d.chunk = ly.chunk;
  d.c_sb = ly.c_sb; d.c_sh = ly.c_sh; d.c_st = ly.c_st;
  d.scale_log2 = a.scale_log2;
  return d;
}

template <int D>
__global__ __launch_bounds__(kThreads) void decode_partial_layers_kernel(const DecodeBatchArgs a) {
  extern __shared__ float dsm[];
  const int w = blockIdx.x;
  int l = 0;
  while (l + 1 < a.L && w >= a.layer[l + 1].wg0) ++l;  // (wave-uniform: scalar loads from the argument table)
  const DecodeArgs d = layer_args(a, l);
  const int rel = w - a.layer[l].wg0;          // [b][g][sp]
  const int sp = rel % d.S, bg = rel / d.S;
  const int g = bg % a.Hkv, b = bg / a.Hkv;
  if (d.S == 1) decode_range<D, true>(d, sp, g, b, dsm);
  else decode_range<D, false>(d, sp, g, b, dsm);
}

template <int D>
__global__ __launch_bounds__(256) void decode_merge_layers_kernel(const DecodeBatchArgs a) {
  const int l = blockIdx.z;
  if (a.layer[l].S == 1) return;  // that layer's ranges wrote the result themselves
  const DecodeArgs d = layer_args(a, l);
  decode_merge<D>(d, blockIdx.x, blockIdx.y);
}

size_t lds_bytes(int d, int chunk) {
  return (size_t)8 * chunk * sizeof(float) + (size_t)32 * (d / 8 + 1) * 16 + (size_t)4 * 8 * d * sizeof(float) + 64 +
         kTabEntries * sizeof(int);
}

template <int D>
hipError_t launch(const DecodeArgs& a, hipStream_t s) {
  const size_t lds = lds_bytes(D, a.chunk);
  static size_t granted_all[kMaxDevices][2];  // per device: the limit set so far for each of the two kernels
  const int dev = current_device_slot();
  if (dev < 0) return hipErrorInvalidDevice;
  size_t* granted = granted_all[dev];
  const int fin = a.S == 1 ? 1 : 0;
  if (lds > granted[fin]) {  // raise the dynamic LDS limit when a larger cache comes along (no allocation)
    const void* f = fin ? reinterpret_cast<const void*>(decode_partial_kernel<D, true>)
                        : reinterpret_cast<const void*>(decode_partial_kernel<D, false>);
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    granted[fin] = lds;
  }
  const dim3 grid(a.S, a.Hkv, a.B);
  if (fin) {
    hipLaunchKernelGGL((decode_partial_kernel<D, true>), grid, dim3(kThreads), lds, s, a);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((decode_partial_kernel<D, false>), grid, dim3(kThreads), lds, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(decode_merge_kernel<D>, dim3(a.Hkv, a.B), dim3(256), 0, s, a);
  return hipGetLastError();
}

template <int D>
hipError_t launch_layers(const DecodeBatchArgs& a, int total_wgs, int max_chunk, bool any_split, hipStream_t s) {
  const size_t lds = lds_bytes(D, max_chunk);
  static size_t granted_all[kMaxDevices];
  const int dev = current_device_slot();
  if (dev < 0) return hipErrorInvalidDevice;
  if (lds > granted_all[dev]) {  // raise the dynamic LDS limit when a larger range comes along (no allocation)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_partial_layers_kernel<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    granted_all[dev] = lds;
  }
  hipLaunchKernelGGL(decode_partial_layers_kernel<D>, dim3(total_wgs), dim3(kThreads), lds, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !any_split) return e;
  hipLaunchKernelGGL(decode_merge_layers_kernel<D>, dim3(a.Hkv, a.B, a.L), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

// Key ranges per (sequence, KV head): enough workgroups to fill the chip, at least 128 keys each.
int decode_splits(int B, int Hkv, int k_cap) {
  int S = (512 + B * Hkv - 1) / (B * Hkv);
  if (S > kMaxSplits) S = kMaxSplits;
  const int by_len = k_cap / 128;
  if (S > by_len) S = by_len;
  return S < 1 ? 1 : S;
}

// All layers in one launch: keys per range so that the layers together give about 512 workgroups, between 256 and
// 1024 keys (multiple of 32); a layer's cache is cut into at most 16 ranges of that size.  (Measured on caches of
// 0.02 to 2 GB per step: 256 to 1024 workgroups are equally fast, more are slower (the merge grows); caches that fit
// one range per head skip the merge launch, which is a third of the time of a small step.)
int decode_layers_chunk(int64_t rows_total) {
  int64_t c = (rows_total + 511) / 512;
  c = c < 256 ? 256 : (c > 1024 ? 1024 : c);
  return (int)((c + 31) / 32 * 32);
}
int decode_layers_splits(int k_cap, int chunk_target, int* chunk) {
  int S = (k_cap + chunk_target - 1) / chunk_target;
  S = S < 1 ? 1 : (S > kMaxSplits ? kMaxSplits : S);
  *chunk = ((k_cap + S - 1) / S + 31) / 32 * 32;
  return S;
}

hipError_t launch_decode_attention_layers(const DecodeBatchArgs& a, int total_wgs, int max_chunk, bool any_split,
                                          hipStream_t s) {
  if (a.d == 128) return launch_layers<128>(a, total_wgs, max_chunk, any_split, s);
  if (a.d == 64) return launch_layers<64>(a, total_wgs, max_chunk, any_split, s);
  return hipErrorInvalidValue;
}

hipError_t launch_decode_attention(const DecodeArgs& a, hipStream_t s) {
  if (a.d == 128) return launch<128>(a, s);
  if (a.d == 64) return launch<64>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace pkv
