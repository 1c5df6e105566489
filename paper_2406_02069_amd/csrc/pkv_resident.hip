// Register-resident window scoring (Sec. 4.2.2, Eq. Al and Eq. att_score) for MI355X: K is read from
// HBM exactly once.
//
// The score of a key needs the softmax normaliser of every window query, which is known only after
// all keys of the head have been seen; so the product Q K^T has to be formed twice (statistics, then
// normalised scores).  Re-reading K for the second sweep costs as much as the first (the 4 MB L2 per
// XCD cannot hold a head, and the memory-side cache is no faster than HBM), so K stays on chip
// between the sweeps instead: persistent 256-thread workgroups, two per compute unit, each hold 512
// keys as MFMA operand fragments in their vector registers (4 waves x 4 tiles x 32 keys; 512
// workgroups x 512 keys = 8 KV heads x 32768 keys, a whole Llama-3-8B layer at 32k context).
//
// A "task" is (unit = layer x sequence x KV head, 512-key part).  Tasks are handed out in rounds of
// up to 512 (one per workgroup); a unit never straddles a round.  Per round a workgroup
//   1. loads its keys: coalesced 16-byte global loads -> wave-private swizzled LDS tile -> fragments;
//   2. sweep 1: for every 32-row tile of Q (staged in LDS, used as the second MFMA operand) and every
//      resident key tile, logits -> running (max, sum exp2) per query row; the 4 waves are merged in
//      LDS and the per-part statistics written to global memory;
//   3. unit barrier: an agent-scope counter per unit; when all parts of the unit have arrived every
//      workgroup of the unit folds the parts into the per-row normaliser c_r = max + log2(sum);
//   4. sweep 2: same products from the same registers, s_i = sum_r exp2(kappa q_r.k_i - c_r), written
//      once per key (already divided by the group size).
// Products are 16x16x32 MFMAs (4 accumulator registers each): the matrix work of the next 16x16
// product is issued in between the exponentials of the current one, so the MFMA and the vector pipes
// run side by side inside a wave, and the register budget (128 for K, 32 for Q) leaves room for it.
// With blockIdx -> XCD round-robin placement the parts of a unit sit on one XCD whenever 64 is a
// multiple of the parts per unit, so the barrier traffic stays in that XCD's L2.
//
// Every wait is bounded: a workgroup that spins too long raises the error word and carries on, so the
// grid always drains.  The launch uses exactly 512 workgroups, two per compute unit (register- and
// LDS-limited), which the host checks against the device before choosing this path.
#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// 16 bytes as a native vector (HIP's uint4 class keeps such values out of registers when staged in arrays)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kTilesPerWave = 4;
constexpr int kRowBlock = 128;
constexpr long long kSpinLimit = 1ll << 22;
constexpr long long kGoSpinLimit = 1ll << 16;  // start-up stagger only: giving up early is harmless

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
#define PKV_MFMA16(A, B, C) __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, B, C, 0, 0, 0)
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ bf16x8 as_frag(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

template <int SEG>
__device__ __forceinline__ int lds_slot(int row, int seg) {
  const int swz = (SEG == 16) ? (row & 15) : ((row >> 1) & 7);
  return row * SEG + (seg ^ swz);
}

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ void merge_stats(float& m, float& z, float m2, float z2) {
  const float M = fmaxf(m, m2);
  const float Ms = (M == -INFINITY) ? 0.f : M;
  z = z * fast_exp2(m - Ms) + z2 * fast_exp2(m2 - Ms);
  m = M;
}

// One 32-key tile as loaded from global memory: NLD wave-wide 16-byte loads (row-major, coalesced).
template <int NLD>
struct RawTile {
  u32x4 v[NLD];
};

template <int SEG>
__device__ __forceinline__ RawTile<SEG / 2> load_raw_tile(const uint16_t* Kbase, int64_t kv_st, int row0, int n,
                                                           bool whole, int lane) {
  constexpr int NLD = SEG / 2, RPL = 64 / SEG;  // RPL rows per wave-wide load
  const int lrow = lane / SEG, lseg = lane - lrow * SEG;
  RawTile<NLD> r;
  if (whole) {  // wave-uniform row pointer + one per-lane offset
    const uint32_t loff = (uint32_t)lrow * (uint32_t)kv_st + (uint32_t)lseg * 8u;
#pragma unroll
    for (int i = 0; i < NLD; ++i)
      r.v[i] = *reinterpret_cast<const u32x4*>(Kbase + (size_t)(row0 + RPL * i) * kv_st + loff);
  } else {  // clamp: rows at or beyond n are never read
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int key = min(row0 + RPL * i + lrow, n - 1);
      r.v[i] = *reinterpret_cast<const u32x4*>(Kbase + (size_t)key * kv_st + lseg * 8);
    }
  }
  return r;
}

// Row-major tile -> wave-private swizzled LDS tile -> 16x16x32 MFMA operand fragments of this lane:
// fragment [ns * KS + ks] holds, for key 16*ns + (lane & 15), the 8 elements at 32*ks + 8*(lane >> 4).
template <int SEG>
__device__ __forceinline__ void raw_to_frags(const RawTile<SEG / 2>& r, u32x4* tile, int lane, bf16x8 (&kf)[SEG / 2]) {
  constexpr int NLD = SEG / 2, KS = SEG / 4;
  const int l16 = lane & 15, kq = lane >> 4;
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int e = i * 64 + lane;
    const int row = e / SEG, seg = e - row * SEG;
    tile[lds_slot<SEG>(row, seg)] = r.v[i];
  }
  wave_lds_fence();
#pragma unroll
  for (int ns = 0; ns < 2; ++ns)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kf[ns * KS + ks] = as_frag(tile[lds_slot<SEG>(16 * ns + l16, 4 * ks + kq)]);
  wave_lds_fence();
}

template <int D>
__global__ __launch_bounds__(kThreads, 2) void score_resident_kernel(const ResidentArgs a) {
  constexpr int KS = D / 32;   // 16x16x32 MFMA k-steps per dot product
  constexpr int SEG = D / 8;   // 16-byte segments per row
  constexpr int NLD = SEG / 2; // wave-wide global loads per 32-key tile
  constexpr int NF = 2 * KS;   // fragments per 32-row / 32-key tile
  constexpr int TILE_U4 = 32 * SEG;
  constexpr int NSUB = kTilesPerWave * 4;  // 16x16 products per 32-row tile of Q
  __shared__ u32x4 kstage[kWaves * TILE_U4];     // one landing tile per wave
  __shared__ u32x4 qs[kRowBlock * SEG];          // current 128-row block of Q
  __shared__ float2 red[kWaves][kRowBlock];
  __shared__ float cst[kResidentMaxRows];
  __shared__ int qoff[kRowBlock];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps addressing in scalar registers
  const int l16 = lane & 15;
  const int kq = lane >> 4;
  const f32x4 kZero4 = {0.f, 0.f, 0.f, 0.f};

  // Two sets of 256 workgroups.  With round-robin placement (block -> XCD blockIdx % 8, then one block
  // per CU before a CU gets its second) the two workgroups of a CU belong to different sets.  Inside a
  // set the workgroups of one XCD take consecutive tasks.  Set 1 starts half a round late (below), so
  // that on every CU one workgroup streams keys or waits at a unit barrier while the other computes.
  const int kk_ = blockIdx.x >> 3;
  const int set = kk_ / (kResidentGrid / 16);
  const int pos = set * (kResidentGrid / 2) + (blockIdx.x & 7) * (kResidentGrid / 16) + kk_ % (kResidentGrid / 16);
  const int BH = a.B * a.Hkv;
  u32x4* tile = kstage + wave * TILE_U4;

#ifdef PKV_RES_TIMING
  long long tstamp[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#define PKV_T(i) tstamp[i] += wall_clock64()
#define PKV_TN(i) tstamp[i] -= wall_clock64()
#else
#define PKV_T(i)
#define PKV_TN(i)
#endif
  bool first = true;
  if (set == 1 && tid == 0) {  // bounded wait for the first set-0 workgroup to finish its first sweep
    long long spins = 0;
    while (__hip_atomic_load(a.go, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0 && ++spins < kGoSpinLimit)
      __builtin_amdgcn_s_sleep(8);
  }
  __syncthreads();
  for (int round = 0; round < a.nrounds; ++round) {
    if (pos >= a.UPR * a.TPU) break;  // idle in every round
    const int u = round * a.UPR + pos / a.TPU;
    const int part_id = pos % a.TPU;
    if (u >= a.U) break;
    const int l = u / BH;
    const int bg = u - l * BH;
    const int b = bg / a.Hkv;
    const int g = bg - b * a.Hkv;
    int n = a.N;
    if (a.seq_lens) {
      n = a.seq_lens[b];
      n = n < 0 ? 0 : (n > a.N ? a.N : n);
    }
    if (a.layer[l].k_l >= n) continue;  // whole sequence kept: no scores needed (uniform over the unit)
    const int key0 = part_id * kResidentKeys;
    if (key0 >= n) continue;            // no keys here; this part is not counted below
    const int nparts = (n + kResidentKeys - 1) / kResidentKeys;
    const int npre = n - a.alpha;
    const int wkey0 = key0 + wave * (kTilesPerWave * 32);
    const uint16_t* Qbase = a.layer[l].Q + (size_t)b * a.q_sb + (size_t)(g * a.G) * a.q_sh;
    const uint16_t* Kbase = a.layer[l].K + (size_t)b * a.kv_sb + (size_t)g * a.kv_sh;

    // Stage a 128-row block of Q in LDS.  qoff[row] = element offset of the row (-1: padding row).
    auto stage_q = [&](int rb) {
      if (tid < kRowBlock) {
        const int r = rb * kRowBlock + tid;
        int off = -1;
        if (r < a.R) {
          const int hh = r / a.alpha, t = r - hh * a.alpha;
          off = (int)(hh * a.q_sh + t * a.q_st);
        }
        qoff[tid] = off;
      }
      __syncthreads();
#pragma unroll 1
      for (int e = tid; e < kRowBlock * SEG; e += kThreads) {
        const int row = e / SEG, seg = e - row * SEG;
        const int off = qoff[row];
        u32x4 v = u32x4{0u, 0u, 0u, 0u};
        if (off >= 0) v = *reinterpret_cast<const u32x4*>(Qbase + off + seg * 8);
        qs[lds_slot<SEG>(row, seg)] = v;
      }
    };

    // ---- 1. keys -> registers ----
    PKV_TN(0);
    bf16x8 kf[kTilesPerWave][NF];
    {
      // Two tiles of global loads (and the Q block) are in flight while an earlier tile goes through LDS.
      const bool whole = wkey0 + kTilesPerWave * 32 <= n;
      RawTile<NLD> ra = load_raw_tile<SEG>(Kbase, a.kv_st, wkey0, n, whole, lane);
      RawTile<NLD> rb = load_raw_tile<SEG>(Kbase, a.kv_st, wkey0 + 32, n, whole, lane);
      stage_q(0);
      raw_to_frags<SEG>(ra, tile, lane, kf[0]);
      ra = load_raw_tile<SEG>(Kbase, a.kv_st, wkey0 + 64, n, whole, lane);
      raw_to_frags<SEG>(rb, tile, lane, kf[1]);
      rb = load_raw_tile<SEG>(Kbase, a.kv_st, wkey0 + 96, n, whole, lane);
      raw_to_frags<SEG>(ra, tile, lane, kf[2]);
      raw_to_frags<SEG>(rb, tile, lane, kf[3]);
    }
    PKV_T(0);
    PKV_TN(1);

    // ---- 2. sweep 1: per-row statistics over this workgroup's keys ----
    // Sub-product i = (t, ns, ms) of a 32-row tile: keys 32t+16ns.., query rows 16ms..; the product's
    // rows are keys (lane holds keys 4*kq..+3 of the sub-tile), its columns query rows (lane & 15).
    float2* part = a.part + ((size_t)u * a.TPU + part_id) * a.Rpad;
    for (int rb = 0; rb < a.nrb; ++rb) {
      if (rb > 0) stage_q(rb);
      __syncthreads();
      const int rows_here = min(kRowBlock, a.R - rb * kRowBlock);
      const int nrt = (rows_here + 31) / 32;
      bf16x8 qf[NF];
#pragma unroll
      for (int ms = 0; ms < 2; ++ms)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ms * KS + ks] = as_frag(qs[lds_slot<SEG>(16 * ms + l16, 4 * ks + kq)]);
      f32x4 acc_cur = kZero4, acc_nxt;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc_cur = PKV_MFMA16(kf[0][ks], qf[ks], acc_cur);
#pragma unroll 1
      for (int rt = 0; rt < nrt; ++rt) {
        const int rt_next = (rt + 1 < nrt) ? rt + 1 : 0;  // after the last tile one unused product is issued
        // Running statistics of this lane's two query rows over this lane's keys, relative to a reference
        // exponent sm that is only raised when a product would overflow it (the common case costs one
        // fma, one exp2 and one add per logit).
        float sm[2] = {-INFINITY, -INFINITY}, sz[2] = {0.f, 0.f};
        int limit[2];
#pragma unroll
        for (int ms = 0; ms < 2; ++ms) {
          const int r = rb * kRowBlock + 32 * rt + 16 * ms + l16;
          limit[ms] = (r < a.R) ? npre + (r % a.alpha) : -1;  // last key this query sees (causal)
        }
#pragma unroll
        for (int i = 0; i < NSUB; ++i) {
          const int t = i >> 2, ns = (i >> 1) & 1, ms = i & 1;
          const int j = (i + 1) % NSUB, tj = j >> 2, nsj = (j >> 1) & 1, msj = j & 1;
          const int sub_base = wkey0 + 32 * t + 16 * ns;
          if (sub_base + 16 > npre) {  // touches the window or the end of the sequence
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (sub_base + 4 * kq + v > limit[ms]) acc_cur[v] = -INFINITY;
          }
          if (i >= NSUB - 2) {  // the Q fragments of this half tile are free: fetch the next row tile's
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
              qf[(i & 1) * KS + ks] = as_frag(qs[lds_slot<SEG>(32 * rt_next + 16 * (i & 1) + l16, 4 * ks + kq)]);
          }
          acc_nxt = kZero4;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) acc_nxt = PKV_MFMA16(kf[tj][nsj * KS + ks], qf[msj * KS + ks], acc_nxt);
          const float nref = -sm[ms];
          float e0 = fast_exp2(__builtin_fmaf(acc_cur[0], a.kappa, nref));
          float e1 = fast_exp2(__builtin_fmaf(acc_cur[1], a.kappa, nref));
          float e2 = fast_exp2(__builtin_fmaf(acc_cur[2], a.kappa, nref));
          float e3 = fast_exp2(__builtin_fmaf(acc_cur[3], a.kappa, nref));
          float sum = (e0 + e1) + (e2 + e3);
          if (__any(!(sum <= 0x1p60f))) {
            // first product, masked product, or a logit far above the reference: exact update
            const float tm = fmaxf(fmaxf(acc_cur[0], acc_cur[1]), fmaxf(acc_cur[2], acc_cur[3]));
            const float mn = fmaxf(sm[ms], tm * a.kappa);
            const float mz = (mn == -INFINITY) ? 0.f : mn;
            sum = 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) sum += fast_exp2(__builtin_fmaf(acc_cur[v], a.kappa, -mz));
            sz[ms] = sz[ms] * fast_exp2(sm[ms] - mz) + sum;
            sm[ms] = mn;
          } else {
            sz[ms] += sum;
          }
          acc_cur = acc_nxt;
        }
#pragma unroll
        for (int ms = 0; ms < 2; ++ms) {
          // the 4 lanes with equal (lane & 15) hold the same query row over different keys
          float m2 = __shfl_xor(sm[ms], 16), z2 = __shfl_xor(sz[ms], 16);
          merge_stats(sm[ms], sz[ms], m2, z2);
          m2 = __shfl_xor(sm[ms], 32), z2 = __shfl_xor(sz[ms], 32);
          merge_stats(sm[ms], sz[ms], m2, z2);
          if (kq == 0) red[wave][32 * rt + 16 * ms + l16] = make_float2(sm[ms], sz[ms]);
        }
      }
      __syncthreads();
      if (tid < rows_here) {
        float m = red[0][tid].x, z = red[0][tid].y;
#pragma unroll
        for (int w = 1; w < kWaves; ++w) merge_stats(m, z, red[w][tid].x, red[w][tid].y);
        // device-scope store: written through, so that other XCDs see it without an L2 write-back
        const unsigned long long bits = ((unsigned long long)__float_as_uint(z) << 32) | __float_as_uint(m);
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(part + rb * kRowBlock + tid), bits, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      }
      __syncthreads();  // also waits for the stores above to be acknowledged
    }

    PKV_T(1);
    PKV_TN(2);
    // ---- 3. unit barrier, then fold the parts into the per-row normaliser ----
    // (the statistics were written through and acknowledged before the workgroup barrier that ends
    // sweep 1, so the arrival counter needs no cache write-back of its own)
    if (tid == 0) {
      if (first && set == 0) __hip_atomic_store(a.go, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(&a.cnt[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      long long spins = 0;
      while (__hip_atomic_load(&a.cnt[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < nparts) {
        __builtin_amdgcn_s_sleep(2);
        if (++spins > kSpinLimit) {
          __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
      }
    }
    __syncthreads();
    PKV_T(2);
    PKV_TN(3);
    {
      // The statistics were written by other workgroups: read them with device-scope atomic loads, which
      // cannot be served from a stale line, instead of invalidating caches.
      // NQ threads per row, each folds every NQ-th part (8 independent loads in flight), then they meet in LDS
      constexpr int NQ = kThreads / kRowBlock;
      const int q = tid >> 7, rl = tid & 127;
      for (int r0 = 0; r0 < a.Rpad; r0 += kRowBlock) {
        const int r = r0 + rl;
        float m = -INFINITY, z = 0.f;
        if (r < a.R) {
          for (int p0 = q; p0 < nparts; p0 += 8 * NQ) {
            float2 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const int p = p0 + NQ * k;
              v[k] = make_float2(-INFINITY, 0.f);
              if (p < nparts) {
                const unsigned long long bits = __hip_atomic_load(
                    reinterpret_cast<const unsigned long long*>(a.part + ((size_t)u * a.TPU + p) * a.Rpad + r),
                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                v[k] = make_float2(__uint_as_float((uint32_t)bits), __uint_as_float((uint32_t)(bits >> 32)));
              }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) merge_stats(m, z, v[k].x, v[k].y);
          }
        }
        red[q][rl] = make_float2(m, z);
        __syncthreads();
        if (q == 0) {
#pragma unroll
          for (int k = 1; k < NQ; ++k) merge_stats(m, z, red[k][rl].x, red[k][rl].y);
          // stored as -c_r/kappa (see sweep 2); padding rows get -inf and contribute exp2(-inf) = 0
          cst[r] = (r < a.R) ? -(m + fast_log2(z)) * a.inv_kappa : -INFINITY;
        }
        __syncthreads();
      }
    }

    PKV_T(3);
    PKV_TN(4);
    // ---- 4. sweep 2: normalised probabilities summed over the query rows ----
    // Here the product's rows are query rows (lane holds rows 4*kq..+3 of the sub-tile) and its columns
    // keys (lane & 15).  cst[] holds -c_r/kappa and is the initial accumulator of each product, so the
    // product comes out as (q.k - c_r/kappa) and one multiply + exp2 per logit remain.
    float e[kTilesPerWave][2];
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) e[t][0] = e[t][1] = 0.f;
    for (int rb = 0; rb < a.nrb; ++rb) {
      if (a.nrb > 1) {
        stage_q(rb);
        __syncthreads();
      }
      const int rows_here = min(kRowBlock, a.R - rb * kRowBlock);
      const int nrt = (rows_here + 31) / 32;
      bf16x8 qf[NF];
      f32x4 cinit[2];
#pragma unroll
      for (int ms = 0; ms < 2; ++ms) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ms * KS + ks] = as_frag(qs[lds_slot<SEG>(16 * ms + l16, 4 * ks + kq)]);
        cinit[ms] = *reinterpret_cast<const f32x4*>(&cst[rb * kRowBlock + 16 * ms + 4 * kq]);
      }
      f32x4 acc_cur = cinit[0], acc_nxt;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc_cur = PKV_MFMA16(qf[ks], kf[0][ks], acc_cur);
#pragma unroll 1
      for (int rt = 0; rt < nrt; ++rt) {
        const int rt_next = (rt + 1 < nrt) ? rt + 1 : 0;
#pragma unroll
        for (int i = 0; i < NSUB; ++i) {
          const int t = i >> 2, ns = (i >> 1) & 1;
          const int j = (i + 1) % NSUB, tj = j >> 2, nsj = (j >> 1) & 1, msj = j & 1;
          if (i >= NSUB - 2) {  // this half tile's Q fragments and normalisers are free: fetch the next row tile's
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
              qf[(i & 1) * KS + ks] = as_frag(qs[lds_slot<SEG>(32 * rt_next + 16 * (i & 1) + l16, 4 * ks + kq)]);
            cinit[i & 1] = *reinterpret_cast<const f32x4*>(&cst[rb * kRowBlock + 32 * rt_next + 16 * (i & 1) + 4 * kq]);
          }
          acc_nxt = cinit[msj];
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) acc_nxt = PKV_MFMA16(qf[msj * KS + ks], kf[tj][nsj * KS + ks], acc_nxt);
          const float e0 = fast_exp2(acc_cur[0] * a.kappa), e1 = fast_exp2(acc_cur[1] * a.kappa);
          const float e2 = fast_exp2(acc_cur[2] * a.kappa), e3 = fast_exp2(acc_cur[3] * a.kappa);
          e[t][ns] += (e0 + e1) + (e2 + e3);
          acc_cur = acc_nxt;
        }
      }
      if (a.nrb > 1) __syncthreads();
    }
    float* raw = a.raw + (size_t)u * a.N;
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t)
#pragma unroll
      for (int ns = 0; ns < 2; ++ns) {
        float tot = e[t][ns];
        tot += __shfl_xor(tot, 16);
        tot += __shfl_xor(tot, 32);
        const int key = wkey0 + 32 * t + 16 * ns + l16;
        if (kq == 0 && key < npre) raw[key] = tot * a.inv_G;
      }
    __syncthreads();  // cst / qs / red are reused by the next round
    first = false;
    PKV_T(4);
  }
  // a set-0 workgroup that never reached a barrier must not leave set 1 waiting
  if (set == 0 && tid == 0) __hip_atomic_store(a.go, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#ifdef PKV_RES_TIMING
  if (tid == 0 && a.dbg)
    for (int i = 0; i < 8; ++i) a.dbg[blockIdx.x * 8 + i] = tstamp[i];
#endif
}

__global__ void zero_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

}  // namespace

hipError_t launch_score_resident(const ResidentArgs& a, hipStream_t s) {
  // the counters (and the error and go words behind them) must start at zero
  const int nz = a.U + 2;
  hipLaunchKernelGGL(zero_kernel, dim3((nz + 255) / 256), dim3(256), 0, s, a.cnt, nz);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.d == 128)
    hipLaunchKernelGGL(score_resident_kernel<128>, dim3(kResidentGrid), dim3(kThreads), 0, s, a);
  else if (a.d == 64)
    hipLaunchKernelGGL(score_resident_kernel<64>, dim3(kResidentGrid), dim3(kThreads), 0, s, a);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace pkv
