// Group mean, 1-D pooling and per-head top-k selection (Sec. 4.2.2: pooling of the window scores, then
// the k^l - alpha highest-scoring prefix tokens per head; the alpha instruction tokens are always kept).
//
// One 1024-thread workgroup per unit (layer x sequence x KV head); all layers of a call run in one
// launch.
//   A. pooled[i] = pool_w-wide max / average of the un-pooled scores, prefix only.  When the prefix fits in
//      LDS (<= 32768 keys) all loads are issued at once, the scores are pooled out of LDS into registers
//      (32 positions per thread, each wave owning a contiguous range of 2048 positions) and stay there; longer
//      prefixes go through LDS in tiles of 16384 positions (all loads of a tile in flight at once) and keep their
//      keys in the pooled array in global memory.  The
//      fp32 bit patterns are the selection keys (scores are >= 0, so unsigned order = numeric order).
//   B. the kk-th largest key T.  Keys in registers: binary search on T, one bit per round from the top; a
//      round counts the keys >= the candidate (per lane, then per wave through ballots, then 16 wave counts
//      through LDS: one barrier, no atomics).  As soon as at most 512 keys still agree with the decided
//      bits, those keys move to a list and one wave decides the remaining bits on its own.
//      Keys in global memory: radix select with LDS histograms, digits of up to 11 bits below the leading bits
//      that all keys share (read off the largest and the smallest key).
//   C. ordered emission: every wave owns a contiguous range of positions; ballots give each kept key
//      its rank, so positions with key > T, and the lowest positions with key == T, come out in
//      ascending order, followed by the window positions.
// All counters are integers and the emission is ordered, so the result does not depend on scheduling.
#include <type_traits>

#include "pkv_internal.h"

namespace pkv {
namespace {

constexpr int NT = kSelectThreads;
constexpr int NW = NT / 64;
constexpr int TL = 16384;          // pooling tile of long prefixes (outputs per iteration)
constexpr int HIST = 2048;         // bins of the widest digit
constexpr int kLdsKeys = 32768;    // prefix lengths up to this keep their keys in LDS

// Workgroup barrier that orders LDS traffic only.  A full __syncthreads() carries fences over global memory too,
// and the waits the compiler builds for them cover the global loads still in flight: a memory round trip per use,
// where only LDS contents change hands.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Largest of a value over the 64 lanes of a wave, valid in lane 63.  Data-parallel-primitive row operations (no LDS
// traffic): running maximum within each row of 16 lanes by shifts of 1, 2, 4, 8 (lanes without a source take 0),
// then the last lane of row 0 / row 2 is handed to row 1 / row 3, and lane 31 to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_max_lane63(uint32_t v) {
#define PKV_DPP_MAX(ctrl, rows) v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, rows, 0xF, false))
  PKV_DPP_MAX(0x111, 0xF);  // row_shr:1
  PKV_DPP_MAX(0x112, 0xF);  // row_shr:2
  PKV_DPP_MAX(0x114, 0xF);  // row_shr:4
  PKV_DPP_MAX(0x118, 0xF);  // row_shr:8
  PKV_DPP_MAX(0x142, 0xA);  // row_bcast:15 into rows 1 and 3
  PKV_DPP_MAX(0x143, 0xC);  // row_bcast:31 into rows 2 and 3
#undef PKV_DPP_MAX
  return v;
}

// Inclusive scan over the workgroup, thread order.  `scratch` holds NW entries.
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, uint32_t* scratch, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t u = __shfl_up(v, o);
    if (lane >= o) v += u;
  }
  __syncthreads();  // scratch may still be read from a previous use
  if (lane == 63) scratch[wave] = v;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const uint32_t s = scratch[w];
    if (w < wave) base += s;
    tot += s;
  }
  *total = tot;
  return v + base;
}


// PERT (prefix in LDS only): positions per thread, 1024 * PERT >= npre.  A short prefix is spread over all waves
// (8 or 16 positions per thread) instead of filling the first few waves with 32 positions per thread and leaving
// the others without keys: the rounds of the threshold search cost what the busiest wave needs.
template <bool LDSKEYS, int PERT>
__device__ __forceinline__ void select_unit(const float* raw, int nrb, size_t rb_stride, float inv_G, float* pooled,
                                            bool write_pooled, int32_t* idx, int npre, int kk, int alpha, int pool,
                                            int pool_w, uint32_t* lkeys, uint32_t* hist,
                                            uint32_t* scan32, uint32_t* sel) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const uint32_t* gkeys = reinterpret_cast<const uint32_t*>(pooled);

  // ---- A. group mean + pooling ----
  constexpr int PER = PERT;            // positions per thread when the prefix lives in LDS
  constexpr int CW = 64 * PER;         // ... and per wave: wave w owns positions [w * CW, (w + 1) * CW)
  uint32_t rkeys[PER];                 // pooled keys of positions wave * CW + 64 * j + lane (0: no such position)
  const int r = (pool == PKV_POOL_NONE) ? 0 : (pool_w - 1) / 2;
  const bool is_max = pool == PKV_POOL_MAX;
  const float inv_w = 1.0f / (float)pool_w;
  const int pos0 = wave * CW + lane;   // the thread's first position; the others follow in steps of 64
  // number of the thread's positions that exist (position pos0 + 64 * j exists iff j < nval): one register instead
  // of 32 position registers kept alive for the comparisons
  const int nval = min(max((npre - pos0 + 63) >> 6, 0), PER);
  uint32_t gmax = 0u, gmin = 0xFFFFFFFFu;  // long prefixes: largest and smallest key this thread has produced
  // long prefixes: largest key of every group of 64 positions, in LDS behind the pooling tile (if they fit)
  constexpr int kGrpOff = 16512, kGrpCap = kLdsKeys - kGrpOff;
  static_assert(kGrpOff >= TL + 2 * (kMaxPoolW / 2), "group maxima lie behind the tile");
  uint32_t* grp = lkeys + kGrpOff;
  const int ngrp = (npre + 63) >> 6;
  const bool use_grp = !LDSKEYS && ngrp <= kGrpCap;
  // fn(gi) for every group gi of [g_lo, g_hi), ascending, whose largest key is at least `bound`: 64 groups are
  // tested at a time, one per lane, and the wave then walks the set bits (all arguments wave-uniform)
  auto for_groups_at_least = [&](int g_lo, int g_hi, uint32_t bound, auto fn) {
    for (int g0 = g_lo; g0 < g_hi; g0 += 64) {
      const int gl = g0 + lane;
      unsigned long long m = __ballot(gl < g_hi && grp[gl] >= bound);
      while (m) {
        const int bsel = __ffsll((long long)m) - 1;
        m &= m - 1;
        fn(g0 + bsel);
      }
    }
  };
  if (LDSKEYS) {
    // The whole prefix fits in LDS: every load of the un-pooled scores is in flight at once (one memory round
    // trip), then each thread pools its positions out of LDS; the pooled values stay in registers, already in
    // the order in which positions are emitted later (each wave owns a contiguous range).
    float* lsc = reinterpret_cast<float*>(lkeys);
    float v[PER];
    if (nrb == 1) {
      const float* rp = raw + pos0;
#pragma unroll
      for (int j = 0; j < PER; ++j) v[j] = (j < nval) ? rp[64 * j] : 0.f;
    } else {
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        const int i = pos0 + 64 * j;
        float sacc = 0.f;
        if (i < npre)
          for (int q = 0; q < nrb; ++q) sacc += raw[q * rb_stride + i];
        v[j] = sacc;
      }
    }
    {
      float* lp = lsc + pos0;
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        v[j] *= inv_G;
        if (j < nval) lp[64 * j] = v[j];
      }
    }
    __syncthreads();
    // window of half-width R around position i, summed (or maximised) in ascending position order.  A group of
    // 64 positions whose windows lie inside the prefix reads with constant offsets and no predicates.
    auto pool_fixed = [&](auto RR, auto MX) {
      constexpr int R = decltype(RR)::value;
      constexpr bool mx = decltype(MX)::value;
      const float* lp = lsc + pos0;
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        const int g0 = wave * CW + 64 * j;  // first position of the group (wave-uniform)
        float acc;
        if (g0 - R >= 0 && g0 + 63 + R < npre) {
          acc = lp[64 * j - R];
#pragma unroll
          for (int u = -R + 1; u <= R; ++u) acc = mx ? fmaxf(acc, lp[64 * j + u]) : acc + lp[64 * j + u];
          v[j] = mx ? acc : acc * inv_w;
        } else if (g0 < npre) {
          const int i = g0 + lane;
          acc = mx ? -INFINITY : 0.f;
#pragma unroll
          for (int u = -R; u <= R; ++u) {
            const int p = i + u;
            const bool ok = p >= 0 && p < npre;
            const float x = lsc[ok ? p : 0];
            if (mx) acc = ok ? fmaxf(acc, x) : acc;
            else acc += ok ? x : 0.f;
          }
          if (j < nval) v[j] = mx ? acc : acc * inv_w;
        }
      }
    };
    using std::integral_constant;
    if (r >= 1 && r <= 3) {
      if (is_max) {
        if (r == 1) pool_fixed(integral_constant<int, 1>{}, std::true_type{});
        else if (r == 2) pool_fixed(integral_constant<int, 2>{}, std::true_type{});
        else pool_fixed(integral_constant<int, 3>{}, std::true_type{});
      } else {
        if (r == 1) pool_fixed(integral_constant<int, 1>{}, std::false_type{});
        else if (r == 2) pool_fixed(integral_constant<int, 2>{}, std::false_type{});
        else pool_fixed(integral_constant<int, 3>{}, std::false_type{});
      }
    }
    else if (r > 3) {
      for (int j = 0; j < PER; ++j) {
        const int i = pos0 + 64 * j;
        if (i < npre) {
          const int lo = max(i - r, 0), hi = min(i + r, npre - 1);
          float acc = is_max ? -INFINITY : 0.f;
          for (int u = lo; u <= hi; ++u) acc = is_max ? fmaxf(acc, lsc[u]) : acc + lsc[u];
          v[j] = is_max ? acc : acc * inv_w;
        }
      }
    }
    if (write_pooled) {
      float* pp = pooled + pos0;
#pragma unroll
      for (int j = 0; j < PER; ++j)
        if (j < nval) pp[64 * j] = v[j];
    }
#pragma unroll
    for (int j = 0; j < PER; ++j) rkeys[j] = (j < nval) ? __float_as_uint(v[j]) : 0u;
  } else {
    // Long prefix: tiles of TL outputs go through LDS, every load of a tile in flight at once; the pooled values
    // are the keys, kept in global memory.  On the way the largest and the smallest key are noted, and the largest
    // key of every group of 64 consecutive positions (kept in LDS behind the tile): later passes skip the groups
    // that cannot hold a key they look for, which is nearly all of them.
    float* lsc = reinterpret_cast<float*>(lkeys);
    constexpr int PT = TL / NT;  // outputs per thread and tile; one more load covers the 2 r halo positions
    static_assert(TL + 2 * (kMaxPoolW / 2) <= (PT + 1) * NT && TL + 2 * (kMaxPoolW / 2) <= kLdsKeys, "tile fits");
    float v[PT + 1];
    // the tile's scores (with the halo of r positions on both sides) into registers
    auto request_tile = [&](int t0) {
#pragma unroll
      for (int j = 0; j <= PT; ++j) {
        const int e = tid + NT * j, i = t0 - r + e;
        v[j] = 0.f;
        if (e < TL + 2 * r && i >= 0 && i < npre) v[j] = raw[i];
      }
      if (nrb > 1) {  // (kept apart: a loop of unknown length behind every load would make each wait for its own)
#pragma unroll
        for (int j = 0; j <= PT; ++j) {
          const int e = tid + NT * j, i = t0 - r + e;
          if (e < TL + 2 * r && i >= 0 && i < npre)
            for (int q = 1; q < nrb; ++q) v[j] += raw[q * rb_stride + i];
        }
      }
    };
    request_tile(0);
    for (int t0 = 0; t0 < npre; t0 += TL) {
      uint32_t wmax[PT];
#pragma unroll
      for (int j = 0; j <= PT; ++j) {
        const int e = tid + NT * j, i = t0 - r + e;
        if (e < TL + 2 * r) lsc[e] = (i >= 0 && i < npre) ? v[j] * inv_G : (is_max ? -INFINITY : 0.f);
      }
      lds_barrier();
      if (t0 + TL < npre) request_tile(t0 + TL);  // travels while this tile is pooled
      // window of 2 RR + 1 tile entries from the output's own slot on, in ascending position order; RR < 0: the
      // half-width is known at run time only.  (A compile-time width lets the LDS reads of all outputs of a thread
      // go out together instead of one dependent chain after the other.)
      auto pool_tile = [&](auto RR) {
        constexpr int R = decltype(RR)::value;
        const int w2 = R >= 0 ? 2 * R : 2 * r;
        constexpr int HB = 8;  // outputs worked on together (register budget)
#pragma unroll
        for (int j0 = 0; j0 < PT; j0 += HB) {
          float acc[HB];
#pragma unroll
          for (int j = 0; j < HB; ++j) acc[j] = lsc[tid + NT * (j0 + j)];
          if (R >= 0) {
#pragma unroll
            for (int u = 1; u <= (R >= 0 ? 2 * R : 0); ++u)
#pragma unroll
              for (int j = 0; j < HB; ++j) {
                const float x = lsc[tid + NT * (j0 + j) + u];
                acc[j] = is_max ? fmaxf(acc[j], x) : acc[j] + x;
              }
          } else {
            for (int u = 1; u <= w2; ++u)
#pragma unroll
              for (int j = 0; j < HB; ++j) {
                const float x = lsc[tid + NT * (j0 + j) + u];
                acc[j] = is_max ? fmaxf(acc[j], x) : acc[j] + x;
              }
          }
#pragma unroll
          for (int j = 0; j < HB; ++j) {
            const int i = t0 + tid + NT * (j0 + j);
            wmax[j0 + j] = 0u;
            if (i < npre) {
              const float y = (!is_max && w2 > 0) ? acc[j] * inv_w : acc[j];
              pooled[i] = y;
              wmax[j0 + j] = __float_as_uint(y);
              gmax = max(gmax, wmax[j0 + j]);
              gmin = min(gmin, wmax[j0 + j]);
            }
          }
        }
      };
      using std::integral_constant;
      if (r == 0) pool_tile(integral_constant<int, 0>{});
      else if (r == 1) pool_tile(integral_constant<int, 1>{});
      else if (r == 2) pool_tile(integral_constant<int, 2>{});
      else if (r == 3) pool_tile(integral_constant<int, 3>{});
      else pool_tile(integral_constant<int, -1>{});
      if (use_grp) {  // the 64 lanes of a wave hold 64 consecutive positions
#pragma unroll
        for (int j = 0; j < PT; ++j) {
          const uint32_t m = wave_max_lane63(wmax[j]);
          const int gi = (t0 + NT * j) / 64 + wave;
          if (lane == 63 && gi < ngrp) grp[gi] = m;
        }
      }
      lds_barrier();  // (the tile is rewritten next; the pooled values are read only after the loop)
    }
    __syncthreads();  // the keys in global memory and the group maxima are complete
  }

  if (kk > 0) {
    // ---- B. the kk-th largest key ----
    uint32_t prefix = 0;
    uint32_t remaining = (uint32_t)kk;
    if (LDSKEYS) {
      // Keys sit in registers: binary search for the largest T with count(key >= T) >= kk, one bit per round
      // from the top.  Per round every wave counts its keys (ballots and scalar pop-counts: no LDS atomics,
      // nothing that depends on timing) and the 16 wave counts meet in LDS: one barrier per bit.  All 32 bits are searched although scores are >= 0: whatever bit patterns the scores
      // hold (NaN, negative zero), exactly kk positions are selected.  Positions that do not exist carry key 0
      // and are never counted (T >= 1 in every comparison).
      //
      // Bookkeeping that comes for free: U = number of keys that still agree with the decided bits (the only
      // ones whose comparison is open), G = number of keys above all of them.  Once U is at most 512
      // the open keys are moved to a list in LDS and a single wave decides the remaining bits on its own.
      uint32_t U = (uint32_t)npre, G = 0;
      uint32_t* list = lkeys;  // the un-pooled scores are no longer needed
      int bit = 31;
      {
        // The leading bits that all keys share (sign, the top of the exponent: scores span a few binades) are T's
        // leading bits as well (count(key >= that prefix) = npre >= kk, and nothing lies above it): they are
        // read off the largest and the smallest key instead of being searched, one round of counting each.
        uint32_t kmax = 0u, kmin = 0xFFFFFFFFu;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
          if (j < nval) {
            kmax = max(kmax, rkeys[j]);
            kmin = min(kmin, rkeys[j]);
          }
        }
#pragma unroll
        for (int sft = 32; sft > 0; sft >>= 1) {
          kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, sft));
          kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, sft));
        }
        if (lane == 0) {
          scan32[wave] = kmax;
          scan32[NW + wave] = kmin;
        }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          kmax = max(kmax, scan32[w]);
          kmin = min(kmin, scan32[NW + w]);
        }
        __syncthreads();  // the slots are reused by the rounds below
        const uint32_t diff = kmax ^ kmin;
        if (diff == 0u) {  // all keys equal: T is that key
          prefix = kmax;
          bit = -1;
        } else {
          bit = 31 - __clz((int)diff);                      // the first bit in which keys differ
          prefix = (bit == 31) ? 0u : (kmax >> (bit + 1)) << (bit + 1);
        }
      }
      // rounds over all keys, until few enough are open
      constexpr int kList = 512;  // open keys that the finishing wave can hold (8 per lane)
      for (; bit >= 0 && U > (uint32_t)kList; --bit) {
        const uint32_t cand = prefix | (1u << bit);
        uint32_t wcount = 0;  // ballot + scalar pop-count per key: the scalar unit counts while the vector unit compares
#pragma unroll
        for (int j = 0; j < PER; ++j) wcount += __popcll(__ballot(rkeys[j] >= cand));
        uint32_t* slot = scan32 + ((bit & 1) ? NW : 0);  // two sets of per-wave slots: one barrier per bit
        if (lane == 0) slot[wave] = wcount;
        __syncthreads();
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) c += slot[w];
        if (c >= (uint32_t)kk) {
          prefix = cand;
          U = c - G;
        } else {
          U -= c - G;
          G = c;
        }
      }
      if (bit >= 0) {
        // the open keys (existing positions whose bits above `bit` equal the prefix's) move to a list in LDS ...
        uint32_t my = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
          const bool open = j < nval && (bit == 31 || (rkeys[j] >> (bit + 1)) == (prefix >> (bit + 1)));
          my += open ? 1u : 0u;
        }
        uint32_t total;
        uint32_t off = block_inclusive_scan(my, hist, &total) - my;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
          const bool open = j < nval && (bit == 31 || (rkeys[j] >> (bit + 1)) == (prefix >> (bit + 1)));
          if (open) list[off++] = rkeys[j];
        }
        __syncthreads();
        // ... and one wave finishes the search on them alone: 8 keys per lane, no barrier between the rounds
        if (wave == 0) {
          constexpr int LK = kList / 64;
          uint32_t lk[LK];
#pragma unroll
          for (int i = 0; i < LK; ++i) lk[i] = (uint32_t)(lane + 64 * i) < total ? list[lane + 64 * i] : 0u;
          for (; bit >= 0; --bit) {
            const uint32_t cand = prefix | (1u << bit);
            uint32_t cnt = 0;
#pragma unroll
            for (int i = 0; i < LK; ++i) cnt += (lk[i] >= cand) ? 1u : 0u;
            uint32_t c = G;  // keys above every key of the list
#pragma unroll
            for (int b = 0; b < 4; ++b) c += (uint32_t)__popcll(__ballot((cnt >> b) & 1u)) << b;  // cnt <= 8
            if (c >= (uint32_t)kk) prefix = cand;
          }
          if (lane == 0) sel[0] = prefix;
        }
        __syncthreads();
        prefix = sel[0];
      }
    } else {
      // Keys in global memory: radix select.  The leading bits that all keys share are T's as well and are read off
      // the largest and the smallest key; below them digits of up to 11 bits, most significant first, each with an
      // LDS histogram over the keys that agree with the digits decided so far.  (Starting at the first bit in which
      // keys differ also spreads the first digit over many bins: scores span a few binades, and a digit made of
      // sign and exponent bits would send nearly every key to the same few counters.)  Every thread has its 16
      // loads of a round in flight before it counts.
#pragma unroll
      for (int sft = 32; sft > 0; sft >>= 1) {
        gmax = max(gmax, (uint32_t)__shfl_xor((int)gmax, sft));
        gmin = min(gmin, (uint32_t)__shfl_xor((int)gmin, sft));
      }
      if (lane == 0) {
        scan32[wave] = gmax;
        scan32[NW + wave] = gmin;
      }
      __syncthreads();
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        gmax = max(gmax, scan32[w]);
        gmin = min(gmin, scan32[NW + w]);
      }
      __syncthreads();
      const uint32_t diff = gmax ^ gmin;
      int top = (diff == 0u) ? 0 : 32 - __clz((int)diff);  // undecided low bits
      prefix = (top >= 32) ? 0u : (gmax >> top) << top;
      constexpr int NB = 16;  // keys per thread and round
      bool first_level = true;
      while (top > 0) {
        const int nb = min(11, top), shift = top - nb;
        const uint32_t dmask = (1u << nb) - 1u;
        for (int e = tid; e < HIST; e += NT) hist[e] = 0;
        __syncthreads();
        if (use_grp && !first_level) {
          // an open key is at least `prefix` (its decided bits, zeros below): only groups whose largest key reaches
          // that can hold one
          const int gw = (ngrp + NW - 1) / NW;  // groups per wave
          for_groups_at_least(wave * gw, min(wave * gw + gw, ngrp), prefix, [&](int gi) {
            const int i = 64 * gi + lane;
            const uint32_t key = i < npre ? gkeys[i] : 0u;
            if (i < npre && (key >> top) == (prefix >> top)) atomicAdd(&hist[(key >> shift) & dmask], 1u);
          });
        } else {
          for (int i0 = 0; i0 < npre; i0 += NB * NT) {
            uint32_t key[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j) {
              const int i = i0 + tid + NT * j;
              key[j] = i < npre ? gkeys[i] : 0u;
            }
#pragma unroll
            for (int j = 0; j < NB; ++j) {
              const int i = i0 + tid + NT * j;
              const bool open = top >= 32 || (key[j] >> top) == (prefix >> top);
              if (i < npre && open) atomicAdd(&hist[(key[j] >> shift) & dmask], 1u);
            }
          }
        }
        first_level = false;
        __syncthreads();
        // thread t owns bins 2t, 2t+1; suffix sums over the bins owned by higher threads
        const uint32_t h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
        uint32_t total;
        const uint32_t incl = block_inclusive_scan(h0 + h1, scan32, &total);
        uint32_t above = total - incl;
        if (above < remaining && above + h1 >= remaining) {
          sel[0] = (uint32_t)(2 * tid + 1);
          sel[1] = above;
        }
        above += h1;
        if (above < remaining && above + h0 >= remaining) {
          sel[0] = (uint32_t)(2 * tid);
          sel[1] = above;
        }
        __syncthreads();
        prefix |= sel[0] << shift;
        remaining -= sel[1];
        top = shift;
        __syncthreads();
      }
    }
    const uint32_t T = prefix;           // bit pattern of the kk-th largest pooled score

    // ---- C. ordered emission ----
    if (LDSKEYS) {
      // keys equal to T to take (lowest positions first) = kk - count(key > T); the counts per wave also give
      // every wave the rank at which its range starts
      uint32_t ngt = 0, neq = 0;  // per lane, at most 32 each
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        const bool ok = j < nval;
        ngt += (ok && rkeys[j] > T) ? 1u : 0u;
        neq += (ok && rkeys[j] == T) ? 1u : 0u;
      }
      uint32_t cgt = 0, ceq = 0;
#pragma unroll
      for (int b = 0; b < 6; ++b) {
        cgt += (uint32_t)__popcll(__ballot((ngt >> b) & 1u)) << b;
        ceq += (uint32_t)__popcll(__ballot((neq >> b) & 1u)) << b;
      }
      if (lane == 0) {
        hist[wave] = cgt;
        hist[NW + wave] = ceq;
      }
      __syncthreads();
      uint32_t gt_before = 0, eq_before = 0, gt_total = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const uint32_t g = hist[w], q = hist[NW + w];
        gt_total += g;
        if (w < wave) {
          gt_before += g;
          eq_before += q;
        }
      }
      const uint32_t need_eq = (uint32_t)kk - gt_total;  // >= 1
      const unsigned long long lt_mask = (1ull << lane) - 1ull;
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        const bool ok = j < nval;
        const bool gt = ok && rkeys[j] > T, eq = ok && rkeys[j] == T;
        const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
        if ((bgt | beq) == 0) continue;  // nothing kept among these 64 positions (the usual case)
        const uint32_t gtb = gt_before + __popcll(bgt & lt_mask);
        const uint32_t eqb = eq_before + __popcll(beq & lt_mask);
        const int i = pos0 + 64 * j;
        if (gt) idx[gtb + min(eqb, need_eq)] = i;
        if (eq && eqb < need_eq) idx[gtb + eqb] = i;
        gt_before += __popcll(bgt);
        eq_before += __popcll(beq);
      }
    } else {
      // every wave owns a contiguous range of positions; two passes over its keys (count, then emit).  With the
      // group maxima at hand only the groups that hold a key >= T are read; else eight groups of 64 positions per
      // round with their loads in flight together.
      constexpr int NE = 8;
      const int cw = ((npre + NW - 1) / NW + 63) & ~63;  // positions per wave, multiple of 64
      const int w0 = min(wave * cw, npre), w1 = min(w0 + cw, npre);
      uint32_t cgt = 0, ceq = 0;
      if (use_grp) {
        for_groups_at_least(w0 >> 6, w0 < w1 ? (w1 + 63) >> 6 : w0 >> 6, T, [&](int gi) {
          const int i = 64 * gi + lane;
          const uint32_t key = i < w1 ? gkeys[i] : 0u;
          cgt += __popcll(__ballot(i < w1 && key > T));
          ceq += __popcll(__ballot(i < w1 && key == T));
        });
      } else {
        for (int base = w0; base < w1; base += 64 * NE) {
          uint32_t key[NE];
#pragma unroll
          for (int j = 0; j < NE; ++j) {
            const int i = base + 64 * j + lane;
            key[j] = i < w1 ? gkeys[i] : 0u;
          }
#pragma unroll
          for (int j = 0; j < NE; ++j) {
            const int i = base + 64 * j + lane;
            cgt += __popcll(__ballot(i < w1 && key[j] > T));
            ceq += __popcll(__ballot(i < w1 && key[j] == T));
          }
        }
      }
      __syncthreads();
      if (lane == 0) {
        hist[wave] = cgt;
        hist[NW + wave] = ceq;
      }
      __syncthreads();
      uint32_t gt_before = 0, eq_before = 0, gt_total = 0;
      for (int w = 0; w < NW; ++w) {
        gt_total += hist[w];
        if (w < wave) {
          gt_before += hist[w];
          eq_before += hist[NW + w];
        }
      }
      const uint32_t need_eq = (uint32_t)kk - gt_total;  // keys equal to T to take, lowest positions first (>= 1)
      const unsigned long long lt_mask = (1ull << lane) - 1ull;
      // the 64 positions from `base` on, their keys in `key`: kept ones go to their ranks
      auto emit64 = [&](int base, uint32_t key) {
        const int i = base + lane;
        const bool gt = i < w1 && key > T, eq = i < w1 && key == T;
        const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
        if ((bgt | beq) == 0) return;
        const uint32_t gtb = gt_before + __popcll(bgt & lt_mask);
        const uint32_t eqb = eq_before + __popcll(beq & lt_mask);
        if (gt) idx[gtb + min(eqb, need_eq)] = i;
        if (eq && eqb < need_eq) idx[gtb + eqb] = i;
        gt_before += __popcll(bgt);
        eq_before += __popcll(beq);
      };
      if (use_grp) {
        for_groups_at_least(w0 >> 6, w0 < w1 ? (w1 + 63) >> 6 : w0 >> 6, T, [&](int gi) {
          const int i = 64 * gi + lane;
          emit64(64 * gi, i < w1 ? gkeys[i] : 0u);
        });
      } else {
        for (int base = w0; base < w1; base += 64 * NE) {
          uint32_t key[NE];
#pragma unroll
          for (int j = 0; j < NE; ++j) {
            const int i = base + 64 * j + lane;
            key[j] = i < w1 ? gkeys[i] : 0u;
          }
#pragma unroll
          for (int j = 0; j < NE; ++j) emit64(base + 64 * j, key[j]);
        }
      }
    }
  }
  for (int t = tid; t < alpha; t += NT) idx[kk + t] = npre + t;
}

// fuse_gather: once the unit's kept positions are written, the same workgroup copies the unit's K and V rows
// (a7): for the few hundred rows of a small budget a launch of its own costs more than the copy.
__global__ __launch_bounds__(NT) void pool_select_batch_kernel(const SelectBatchArgs a, const GatherBatchArgs ga,
                                                               const int fuse_gather) {
  extern __shared__ uint32_t lkeys[];  // kLdsKeys entries
  __shared__ uint32_t hist[HIST];
  __shared__ uint32_t scan32[2 * NW];
  __shared__ uint32_t sel[2];

  const int tid = threadIdx.x;
  const int BH = a.B * a.Hkv;
  const int u = blockIdx.x;
  const int l = u / BH;
  const int bg = u - l * BH;
  const int b = bg / a.Hkv;
  const int g = bg - b * a.Hkv;
  const SelectLayer& ly = a.layer[l];
  int n = a.N;
  if (a.seq_lens) {
    n = a.seq_lens[b];
    n = n < 0 ? 0 : (n > a.N ? a.N : n);
  }
  const int count = ly.k_l < n ? ly.k_l : n;
  // a scoring kernel that gave up a wait leaves meaningless scores: the caller learns it from the count
  if (g == 0 && tid == 0) ly.count_out[b] = (a.err && *a.err != 0) ? -1 : count;
  int32_t* idx = ly.idx_out + (size_t)bg * ly.k_cap;
  auto gather_unit = [&]() {
    if (!fuse_gather) return;
    __syncthreads();  // the unit's kept positions are complete (all of them written by this workgroup)
    const GatherLayer& gl = ga.layer[l];
    const int sh = ga.d == 128 ? 4 : 3;  // 16 or 8 lanes per row
    const int total = gl.k_cap << sh;
    // four row segments per thread and round, each stage (positions, rows, stores) issued for all four before the
    // next one: three memory round trips per round instead of twelve
    constexpr int NB = 4;
    const size_t head_off = (size_t)b * ga.kv_sb + (size_t)g * ga.kv_sh;
    const size_t out_off = (size_t)b * gl.o_sb + (size_t)g * gl.o_sh;
    const int32_t* pos = gl.idx + ((size_t)b * ga.Hkv + g) * gl.k_cap;
    for (int t0 = tid; t0 < total; t0 += NB * NT) {
      int src[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int t = t0 + u * NT;
        src[u] = t < total ? pos[t >> sh] : -1;
      }
      uint4 kv[NB], vv[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int seg = (t0 + u * NT) & ((1 << sh) - 1);
        kv[u] = make_uint4(0, 0, 0, 0);
        vv[u] = kv[u];
        if ((uint32_t)src[u] < (uint32_t)ga.N) {  // -1: unused slot; nothing outside [0, N) is dereferenced
          const size_t off = head_off + (size_t)src[u] * ga.kv_st + seg * 8;
          kv[u] = *reinterpret_cast<const uint4*>(gl.K + off);
          vv[u] = *reinterpret_cast<const uint4*>(gl.V + off);
        }
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int t = t0 + u * NT;
        if (t < total) {
          const size_t o = out_off + (size_t)(t >> sh) * gl.o_st + (t & ((1 << sh) - 1)) * 8;
          *reinterpret_cast<uint4*>(gl.K_out + o) = kv[u];
          *reinterpret_cast<uint4*>(gl.V_out + o) = vv[u];
        }
      }
    }
  };
  if (ly.k_l >= n) {  // keep everything
    for (int j = tid; j < ly.k_cap; j += NT) idx[j] = j < n ? j : -1;
    gather_unit();
    return;
  }
  const int npre = n - a.alpha;
  const int kk = ly.k_l - a.alpha;  // prefix tokens to select; kk < npre
  const size_t rb_stride = (size_t)BH * a.N;
  const float* raw = a.raw + ((size_t)l * a.nrb * BH + bg) * a.N;
  float* pooled = ly.pooled + (size_t)bg * a.N;
  if (npre <= 8 * NT)
    select_unit<true, 8>(raw, a.nrb, rb_stride, a.inv_G, pooled, ly.write_pooled != 0, idx, npre, kk, a.alpha, a.pool,
                         a.pool_w, lkeys, hist, scan32, sel);
  else if (npre <= 16 * NT)
    select_unit<true, 16>(raw, a.nrb, rb_stride, a.inv_G, pooled, ly.write_pooled != 0, idx, npre, kk, a.alpha,
                          a.pool, a.pool_w, lkeys, hist, scan32, sel);
  else if (npre <= kLdsKeys)
    select_unit<true, kLdsKeys / NT>(raw, a.nrb, rb_stride, a.inv_G, pooled, ly.write_pooled != 0, idx, npre, kk,
                                     a.alpha, a.pool, a.pool_w, lkeys, hist, scan32, sel);
  else
    select_unit<false, kLdsKeys / NT>(raw, a.nrb, rb_stride, a.inv_G, pooled, true, idx, npre, kk, a.alpha, a.pool,
                                      a.pool_w, lkeys, hist, scan32, sel);
  gather_unit();
}

}  // namespace

hipError_t launch_pool_select_batch(const SelectBatchArgs& a, const GatherBatchArgs& ga, bool fuse_gather, int nlayers,
                                    hipStream_t s) {
  static bool attr_set[kMaxDevices];
  const size_t dyn = (size_t)kLdsKeys * sizeof(uint32_t);
  const int dev = current_device_slot();
  if (dev < 0) return hipErrorInvalidDevice;
  if (!attr_set[dev]) {  // allow 128 KB of dynamic LDS, once per device (idempotent; no allocation)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pool_select_batch_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);
    if (e != hipSuccess) return e;
    attr_set[dev] = true;
  }
  hipLaunchKernelGGL(pool_select_batch_kernel, dim3(nlayers * a.B * a.Hkv), dim3(NT), dyn, s, a, ga,
                     fuse_gather ? 1 : 0);
  return hipGetLastError();
}

// ---- attention recall rate (appendix, "Attention Recall Rate Experiment") ----
// The attention of a window query over all keys it sees sums to 1, so the share that falls on the kept keys is
// 1 - (mass on the dropped prefix keys); averaged over the G * alpha queries of a KV head that is
//   recall = 1 - (sum_{i < n-alpha} s_i - sum_{kept prefix i} s_i) / alpha
// with the un-pooled group-mean window scores s_i (the window keys are always kept).  One workgroup per
// (layer, sequence, KV head): one coalesced pass over the scores, one gather over the kept positions.
namespace {
__global__ __launch_bounds__(256) void recall_kernel(const RecallArgs a) {
  const RecallLayer& ly = a.layer[blockIdx.y];
  const int bg = blockIdx.x;
  const int b = bg / a.Hkv;
  const int BH = a.B * a.Hkv;
  int n = a.N;
  if (a.seq_lens) {
    n = a.seq_lens[b];
    n = n < 0 ? 0 : (n > a.N ? a.N : n);
  }
  __shared__ float red[2][256];
  float all = 0.f, kept = 0.f;
  if (ly.k_l < n) {
    const int npre = n - a.alpha, kk = ly.k_l - a.alpha;
    for (int p = 0; p < a.nrb; ++p) {
      const float* row = a.raw + (((size_t)blockIdx.y * a.nrb + p) * BH + bg) * a.N;
      for (int i = threadIdx.x; i < npre; i += 256) all += row[i];
      for (int j = threadIdx.x; j < kk; j += 256) {
        const int i = ly.idx[(size_t)bg * ly.k_cap + j];
        if ((uint32_t)i < (uint32_t)npre) kept += row[i];
      }
    }
  }
  red[0][threadIdx.x] = all;
  red[1][threadIdx.x] = kept;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      red[0][threadIdx.x] += red[0][threadIdx.x + s];
      red[1][threadIdx.x] += red[1][threadIdx.x + s];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0)
    ly.recall[bg] = (ly.k_l < n) ? 1.f - (red[0][0] - red[1][0]) * a.inv_G / (float)a.alpha : 1.f;
}
}  // namespace

hipError_t launch_recall(const RecallArgs& a, int nlayers, hipStream_t s) {
  hipLaunchKernelGGL(recall_kernel, dim3(a.B * a.Hkv, nlayers), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace pkv
