// Register-resident window scoring (Sec. 4.2.2, Eq. Al and Eq. att_score) for MI355X: K is read from
// HBM exactly once.
//
// The score of a key needs the softmax normaliser of every window query, which is known only after
// all keys of the head have been seen; so the product Q K^T has to be formed twice (statistics, then
// normalised scores).  Re-reading K for the second sweep costs as much as the first (the 4 MB L2 per
// XCD cannot hold a head, and the memory-side cache streams no faster than HBM), so K stays on chip
// between the sweeps: 512 persistent 256-thread workgroups, two per compute unit, each hold 512 keys
// as MFMA operand fragments in their vector registers (4 waves x 4 tiles x 32 keys).
//
// Work split.  A "unit" is (layer, sequence, KV head); it is cut into parts of 512 keys, one part per
// workgroup.  The grid is divided into groups of 64..512 workgroups (the smallest power of two that
// holds a unit); a group works through its own list of units at its own pace, so groups drift apart
// and while one streams keys from HBM others compute.  The two workgroups of a compute unit belong to
// different groups, and the second set of groups starts late, so that a compute unit rarely has both
// of its workgroups waiting at the same time.
//
// Per unit a workgroup
//   1. loads its keys straight into MFMA operand layout (each lane: 16 bytes of one key row per
//      load; 32 loads in flight per lane) and stages the 128-row block of Q in LDS;
//   2. sweep 1: for every 32-row tile of Q and every resident 32-key tile, logits -> per-row
//      (reference, sum exp2) per lane; merged over the wave halves, the 4 waves (LDS) and written as the
//      part's statistics;
//   3. arrives at the unit's counter.  The last part to arrive folds all parts into the per-row
//      normaliser c_r = max + log2(sum) and publishes it, tagged with the unit number; the others poll
//      the tagged words.  (Agent-scope relaxed atomics: written through, never served from a stale line.)
//   4. sweep 2: same products from the same registers, s_i = sum_r exp2(kappa q_r.k_i - c_r), written
//      once per key (already divided by the group size).
//
// Inner loops.  Products are v_mfma_f32_32x32x16_bf16 (the 16x16x32 shape does not overlap with vector
// work on this chip and runs at two thirds of the rate).  A sweep is bound by the vector pipe: per
// logit one multiply-add, one v_exp_f32 and one add.  The 8 MFMAs of the next 32x32 product are issued
// one by one between the exponentials of the current product (explicit scheduling groups), so the
// matrix pipe runs in the shadow of the vector pipe.  Sweep 1 uses a provisional per-lane reference
// exponent taken from the first tile instead of a running maximum (no branch, no second exponential);
// a row tile whose sums leave a safe range is recomputed with the exact running-maximum update, and so
// are tiles that touch the causal window or the end of the sequence (they need masks).
//
// Every wait is bounded: a workgroup that spins too long raises the error word and carries on, so the
// grid always drains.  The launch uses exactly 512 workgroups, two per compute unit (register- and
// LDS-limited), which the host checks against the device before choosing this path.
#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// 16 bytes as a native vector (HIP's uint4 class keeps such values out of registers when staged in arrays)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kTiles = 4;          // 32-key tiles held by one wave
constexpr int kRowBlock = 128;     // rows of Q staged in LDS at a time
constexpr int kSpinLimit = 1 << 20;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ bf16x8 as_frag(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }
#define PKV_MFMA32(A, B, C) __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B, C, 0, 0, 0)
// scheduling groups: the next N instructions of a class, in this order
#define PKV_SG_MFMA(n) __builtin_amdgcn_sched_group_barrier(0x008, n, 0)
#define PKV_SG_VALU(n) __builtin_amdgcn_sched_group_barrier(0x002, n, 0)
#define PKV_SG_TRANS(n) __builtin_amdgcn_sched_group_barrier(0x400, n, 0)
#define PKV_SG_DSR(n) __builtin_amdgcn_sched_group_barrier(0x100, n, 0)

// The Q block is kept in LDS with a row pitch of SEG + 1 sixteen-byte segments: consecutive rows then
// start 4 banks apart (mod 64), so the 16 rows that one ds_read_b128 phase touches hit all banks once,
// and the segment index stays a compile-time address offset.
template <int SEG>
__device__ __forceinline__ constexpr int lds_pitch() { return SEG + 1; }

__device__ __forceinline__ void merge_stats(float& m, float& z, float m2, float z2) {
  const float M = fmaxf(m, m2);
  const float Ms = (M == -INFINITY) ? 0.f : M;
  z = z * fast_exp2(m - Ms) + z2 * fast_exp2(m2 - Ms);
  m = M;
}

__device__ __forceinline__ void st64(u64* p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ u64 ld64(const u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Accumulator element v of a lane (half h) belongs to tile row mrow(v, h) (32x32 MFMA output layout).
__device__ __forceinline__ constexpr int mrow0(int v) { return 8 * (v >> 2) + (v & 3); }

template <int D>
__global__ __launch_bounds__(kThreads, 2) void score_resident_kernel(const ResidentArgs a) {
  constexpr int KS = D / 16;   // 32x32x16 MFMA k-steps per dot product
  constexpr int SEG = D / 8;   // 16-byte segments per row
  constexpr int TPM = 16 / KS; // logits per lane handled between two MFMAs
  constexpr int PITCH = lds_pitch<SEG>();
  constexpr int QLD = kRowBlock * SEG / kThreads;  // 16-byte loads per thread for one block of Q
  constexpr int RPP = kThreads / SEG;              // rows covered by one pass of the workgroup
  __shared__ u32x4 qs[kRowBlock * PITCH];        // current 128-row block of Q
  __shared__ float2 red[kWaves][kRowBlock];
  __shared__ __attribute__((aligned(16))) float cst[kResidentMaxRows];
  __shared__ int qoff[kRowBlock];
  __shared__ int s_last;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps addressing in scalar registers
  const int l32 = lane & 31;
  const int hf = lane >> 5;
  const int BH = a.B * a.Hkv;

  // ---- which group, which slot ----
  // blockIdx -> XCD is blockIdx % 8, and an XCD fills every compute unit once before any gets a second
  // workgroup; so set 0 / set 1 are the first / second workgroup of each compute unit.  (Only speed
  // depends on this placement, never the result.)
  const int xcd = blockIdx.x & 7, kk = blockIdx.x >> 3;
  const int set = kk >> 5, cu = kk & 31;
  int group, slot;
  if (a.ngroups >= 2) {
    const int xpc = 16 / a.ngroups;  // XCDs per group cluster
    group = (xcd / xpc) * 2 + set;
    slot = (xcd % xpc) * 32 + cu;
  } else {
    group = 0;
    slot = set * 256 + xcd * 32 + cu;
  }
  const int sub = slot / a.TPU;
  const int part_id = slot - sub * a.TPU;
  if (sub >= a.UPG) return;  // no work for this workgroup at this shape
  const int slot_id = group * a.UPG + sub;  // one of nslots concurrent units
  const int nslots = a.ngroups * a.UPG;
  float2* part_base = a.part + (size_t)slot_id * a.TPU * a.Rpad;
  u64* cbuf = a.cbuf + (size_t)slot_id * a.Rpad;

#ifdef PKV_RES_TIMING
  long long tstamp[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  tstamp[5] = -(long long)clock64();
  tstamp[6] = -(long long)wall_clock64();
  // absolute phase-boundary times of a few workgroups (the two of one compute unit, on two XCDs)
  const int trace_id = (blockIdx.x == 0) ? 0 : (blockIdx.x == 256) ? 1 : (blockIdx.x == 1) ? 2 : (blockIdx.x == 257) ? 3 : -1;
  int trace_n = 0;
#define PKV_TRACE() do { if (trace_id >= 0 && trace_n < 240 && tid == 0 && a.dbg) a.dbg[kResidentGrid * 8 + trace_id * 256 + trace_n] = wall_clock64(); ++trace_n; } while (0)
#define PKV_T(i) do { tstamp[i] += wall_clock64(); PKV_TRACE(); } while (0)
#define PKV_TN(i) do { tstamp[i] -= wall_clock64(); if (i == 0) PKV_TRACE(); } while (0)
#else
#define PKV_T(i)
#define PKV_TN(i)
#endif

#ifdef PKV_RES_TIMING
  if (set == 1 && a.stagger < 0) return;  // measurement: one workgroup per compute unit
#endif
  if (set == 1 && a.stagger > 0) {  // late start of the second set: a plain timed wait
    const long long t0 = wall_clock64();
    while (wall_clock64() - t0 < a.stagger) __builtin_amdgcn_s_sleep(16);
  }

  for (int u = slot_id; u < a.U; u += nslots) {
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
    const int wkey0 = key0 + wave * (kTiles * 32);
    const bool has_keys = wkey0 < n;                      // wave-uniform
    const bool whole = wkey0 + kTiles * 32 <= n;
    // tile t needs masks iff it reaches beyond the prefix (causal window, end of the sequence)
    int dirty_mask = 0;
#pragma unroll
    for (int t = 0; t < kTiles; ++t) dirty_mask |= (wkey0 + 32 * t + 32 > npre) ? (1 << t) : 0;
    const uint16_t* Qbase = a.layer[l].Q + (size_t)b * a.q_sb + (size_t)(g * a.G) * a.q_sh;
    const uint16_t* Kbase = a.layer[l].K + (size_t)b * a.kv_sb + (size_t)g * a.kv_sh;

    // Stage a 128-row block of Q in LDS.  qoff[row] = byte offset of the row (-1: padding row).
    // Thread -> (row tid / SEG + RPP * i, segment tid % SEG): 16 bytes per load, rows fully coalesced.
    const int q_row0 = tid / SEG, q_seg = tid - q_row0 * SEG;
    auto stage_q_issue = [&](int rb, u32x4 (&v)[QLD]) {
      if (tid < kRowBlock) {
        const int r = rb * kRowBlock + tid;
        int off = -1;
        if (r < a.R) {
          const int hh = r / a.alpha, t = r - hh * a.alpha;
          off = (int)(hh * a.q_sh + t * a.q_st) * 2;
        }
        qoff[tid] = off;
      }
      __syncthreads();
      const char* qb = reinterpret_cast<const char*>(Qbase) + q_seg * 16;
#pragma unroll
      for (int i = 0; i < QLD; ++i) {
        const int off = qoff[q_row0 + RPP * i];
        v[i] = u32x4{0u, 0u, 0u, 0u};
        if (off >= 0) v[i] = *reinterpret_cast<const u32x4*>(qb + (uint32_t)off);
      }
    };
    auto stage_q_commit = [&](const u32x4 (&v)[QLD]) {
      u32x4* dst = qs + q_row0 * PITCH + q_seg;
#pragma unroll
      for (int i = 0; i < QLD; ++i) dst[RPP * i * PITCH] = v[i];
    };

    // ---- 1. Q block 0 -> LDS, keys -> registers (fragment layout, no staging) ----
    PKV_TN(0);
    bf16x8 kf[kTiles][KS];
    {
      u32x4 qv[QLD];
      stage_q_issue(0, qv);  // issued first: loads return in order, and the Q block is needed first
      if (has_keys) {
        // 32-bit byte offsets from the head's first key (the host admits only shapes where they fit)
        const char* kb = reinterpret_cast<const char*>(Kbase) + 16 * hf;
        const uint32_t row_bytes = (uint32_t)a.kv_st * 2u;
#pragma unroll
        for (int t = 0; t < kTiles; ++t) {
          int key = wkey0 + 32 * t + l32;
          if (!whole) key = min(key, n - 1);  // rows at or beyond n are never read
          const char* rowp = kb + (uint32_t)key * row_bytes;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) kf[t][ks] = as_frag(*reinterpret_cast<const u32x4*>(rowp + 32 * ks));
        }
      }
      stage_q_commit(qv);
    }
    __syncthreads();
    PKV_T(0);
    PKV_TN(1);

    // LDS reads of one 32-row tile of Q as MFMA operand fragments
    const u32x4* q_lane = qs + l32 * PITCH + hf;
    auto q_frag = [&](int rt, int ks) { return as_frag(q_lane[32 * rt * PITCH + 2 * ks]); };

    // ---- 2. sweep 1: per-row statistics over this workgroup's keys ----
    // Products: rows = keys (element v of a lane: key mrow0(v) + 4*hf of the tile), columns = query rows
    // (lane & 31).  Per lane and row tile: reference exponent m (log2 domain) and z = sum exp2(x - m).
    float2* part = part_base + (size_t)part_id * a.Rpad;
    for (int rb = 0; rb < a.nrb; ++rb) {
      if (rb > 0) {
        u32x4 qv[QLD];
        __syncthreads();  // everyone is done with the previous block
        stage_q_issue(rb, qv);
        stage_q_commit(qv);
        __syncthreads();
      }
      const int rows_here = min(kRowBlock, a.R - rb * kRowBlock);
      const int nrt = (rows_here + 31) / 32;
      if (has_keys) {
        // exact update of (m, z) with the 16 logits of one product; masked elements excluded
        auto exact_update = [&](const f32x16& acc, int t, bool masked, int lim_rel, float& m, float& z) {
          float x[16];
          float tm = -INFINITY;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            x[v] = acc[v] * a.kappa;
            if (masked && 32 * t + mrow0(v) > lim_rel) x[v] = -INFINITY;
            tm = fmaxf(tm, x[v]);
          }
          const float mn = fmaxf(m, tm);
          const float ms = (mn == -INFINITY) ? 0.f : mn;
          float s = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) s += fast_exp2(x[v] - ms);
          z = z * fast_exp2(m - ms) + s;
          m = mn;
        };
        auto finish_rt = [&](int rt, float m, float z) {
          const float m2 = __shfl_xor(m, 32), z2 = __shfl_xor(z, 32);
          merge_stats(m, z, m2, z2);
          if (hf == 0) red[wave][32 * rt + l32] = make_float2(m, z);
        };
        // last key (relative to this wave's first key and half) that the lane's query of row tile rt sees
        auto lim_rel_of = [&](int rt) {
          const int r = rb * kRowBlock + 32 * rt + l32;
          const int lim = (r < a.R) ? npre + (r % a.alpha) : npre + a.alpha - 1;  // padding rows: statistics unused
          return lim - wkey0 - 4 * hf;
        };

        bf16x8 qf[KS];
        f32x16 cur, nxt;
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = q_frag(0, ks);
        cur = zero16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) cur = PKV_MFMA32(kf[0][ks], qf[ks], cur);
        int redo = 0;  // row tiles whose provisional reference failed (wave-uniform bit mask)
#pragma unroll 1
        for (int rt = 0; rt < nrt; ++rt) {
          const int rt_next = (rt + 1 < nrt) ? rt + 1 : 0;  // after the last tile one unused product is issued
          float m = -INFINITY, z = 0.f;  // m: reference exponent of this lane (not necessarily the maximum)
          const int lim_rel = lim_rel_of(rt);
#pragma unroll
          for (int t = 0; t < kTiles; ++t) {
            const int tn = (t + 1) % kTiles;
            if (dirty_mask & (1 << t)) {
              // slow variant of the step (masks, exact update); the next product is still issued first
              nxt = zero16;
#pragma unroll
              for (int ks = 0; ks < KS; ++ks) {
                nxt = PKV_MFMA32(kf[tn][ks], qf[ks], nxt);
                if (t == kTiles - 2) qf[ks] = q_frag(rt_next, ks);
              }
              exact_update(cur, t, true, lim_rel, m, z);
            } else {
              float nref;
              if (t == 0) {  // provisional reference: the largest of three of the lane's logits
                m = a.kappa * fmaxf(fmaxf(cur[0], cur[5]), cur[10]);
                z = 0.f;
              }
              nref = -m;
              float s0 = 0.f, s1 = 0.f;
              nxt = zero16;
#pragma unroll
              for (int ks = 0; ks < KS; ++ks) {
                nxt = PKV_MFMA32(kf[tn][ks], qf[ks], nxt);
                if (t == kTiles - 2) qf[ks] = q_frag(rt_next, ks);  // last use of this fragment was the MFMA above
                float x[TPM], e[TPM];
#pragma unroll
                for (int j = 0; j < TPM; ++j) x[j] = __builtin_fmaf(cur[TPM * ks + j], a.kappa, nref);
#pragma unroll
                for (int j = 0; j < TPM; ++j) e[j] = fast_exp2(x[j]);
#pragma unroll
                for (int j = 0; j < TPM; ++j) {
                  if (j & 1) s1 += e[j]; else s0 += e[j];
                }
                PKV_SG_MFMA(1);
                if (t == kTiles - 2) PKV_SG_DSR(1);
                PKV_SG_VALU(TPM);
                PKV_SG_TRANS(TPM);
                PKV_SG_VALU(TPM);
              }
              z += s0 + s1;
            }
            cur = nxt;
          }
          // a sum outside the safe range (or NaN) means the provisional reference was too far off
          if (__any(!(z <= 0x1p100f))) redo |= 1 << rt;
          finish_rt(rt, m, z);
        }
        // rare: recompute flagged row tiles with the exact running-maximum update (pipeline is drained here)
        for (int rt = 0; redo != 0 && rt < nrt; ++rt) {
          if (!(redo & (1 << rt))) continue;
          bf16x8 q2[KS];
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) q2[ks] = q_frag(rt, ks);
          float m = -INFINITY, z = 0.f;
          const int lim_rel = lim_rel_of(rt);
#pragma unroll
          for (int t = 0; t < kTiles; ++t) {
            f32x16 acc = zero16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = PKV_MFMA32(kf[t][ks], q2[ks], acc);
            exact_update(acc, t, (dirty_mask >> t) & 1, lim_rel, m, z);
          }
          finish_rt(rt, m, z);
        }
      } else {
        for (int r = lane; r < kRowBlock; r += 64) red[wave][r] = make_float2(-INFINITY, 0.f);
      }
      __syncthreads();
      if (tid < rows_here) {
        float m = red[0][tid].x, z = red[0][tid].y;
#pragma unroll
        for (int w = 1; w < kWaves; ++w) merge_stats(m, z, red[w][tid].x, red[w][tid].y);
        // device-scope store: written through, so that other XCDs see it without an L2 write-back
        st64(reinterpret_cast<u64*>(part + rb * kRowBlock + tid), ((u64)__float_as_uint(z) << 32) | __float_as_uint(m));
      }
    }
    __syncthreads();  // also waits for the stores above to be acknowledged
    PKV_T(1);
    PKV_TN(2);

    // ---- 3. arrive; the last part folds all parts into the per-row normaliser and publishes it ----
    const unsigned tag = (unsigned)u + 1u;
    if (tid == 0) {
      const int prev = __hip_atomic_fetch_add(&a.cnt[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = (prev == nparts - 1);
    }
    __syncthreads();
    if (s_last) {
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
                const u64 bits = ld64(reinterpret_cast<const u64*>(part_base + (size_t)p * a.Rpad + r));
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
          // kept as -c_r/kappa (see sweep 2); padding rows get -inf and contribute exp2(-inf) = 0
          const float c = (r < a.R) ? -(m + fast_log2(z)) * a.inv_kappa : -INFINITY;
          cst[r] = c;
          if (r < a.R) st64(&cbuf[r], ((u64)tag << 32) | __float_as_uint(c));
        }
        __syncthreads();
      }
    } else {
      for (int r = tid; r < a.Rpad; r += kThreads) {
        float c = -INFINITY;
        if (r < a.R) {
          int spins = 0;
          u64 w;
          for (;;) {
            w = ld64(&cbuf[r]);
            if ((unsigned)(w >> 32) == tag) break;
            __builtin_amdgcn_s_sleep(1);
            if (++spins > kSpinLimit || ((spins & 1023) == 0 && __hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
              __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              break;
            }
          }
          c = __uint_as_float((unsigned)w);
        }
        cst[r] = c;
      }
      __syncthreads();
    }
    PKV_T(2);
    PKV_TN(4);

    // ---- 4. sweep 2: normalised probabilities summed over the query rows ----
    // Here the product's rows are query rows (element v of a lane: row mrow0(v) + 4*hf of the tile) and its
    // columns keys (lane & 31).  cst[] holds -c_r/kappa and is the initial accumulator of each product, so the
    // product comes out as (q.k - c_r/kappa) and one multiply + exp2 + add per logit remain.
    float e[kTiles];
#pragma unroll
    for (int t = 0; t < kTiles; ++t) e[t] = 0.f;
    for (int rb = 0; rb < a.nrb; ++rb) {
      if (a.nrb > 1) {
        u32x4 qv[QLD];
        __syncthreads();
        stage_q_issue(rb, qv);
        stage_q_commit(qv);
        __syncthreads();
      }
      const int rows_here = min(kRowBlock, a.R - rb * kRowBlock);
      const int nrt = (rows_here + 31) / 32;
      if (has_keys) {
        bf16x8 qf[KS];
        f32x16 cinit, cur, nxt;
        auto load_cinit = [&](int rt, int j) {
          const f32x4 c = *reinterpret_cast<const f32x4*>(&cst[rb * kRowBlock + 32 * rt + 8 * j + 4 * hf]);
          cinit[4 * j + 0] = c[0]; cinit[4 * j + 1] = c[1]; cinit[4 * j + 2] = c[2]; cinit[4 * j + 3] = c[3];
        };
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = q_frag(0, ks);
#pragma unroll
        for (int j = 0; j < 4; ++j) load_cinit(0, j);
        cur = cinit;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) cur = PKV_MFMA32(qf[ks], kf[0][ks], cur);
#pragma unroll 1
        for (int rt = 0; rt < nrt; ++rt) {
          const int rt_next = (rt + 1 < nrt) ? rt + 1 : 0;
#pragma unroll
          for (int t = 0; t < kTiles; ++t) {
            const int tn = (t + 1) % kTiles;
            float s0 = 0.f, s1 = 0.f;
            nxt = cinit;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
              nxt = PKV_MFMA32(qf[ks], kf[tn][ks], nxt);
              if (t == kTiles - 2) {  // this row tile's fragments and normalisers are free: fetch the next tile's
                qf[ks] = q_frag(rt_next, ks);
                if (ks < 4) load_cinit(rt_next, ks);
              }
              float x[TPM], ee[TPM];
#pragma unroll
              for (int j = 0; j < TPM; ++j) x[j] = cur[TPM * ks + j] * a.kappa;
#pragma unroll
              for (int j = 0; j < TPM; ++j) ee[j] = fast_exp2(x[j]);
#pragma unroll
              for (int j = 0; j < TPM; ++j) {
                if (j & 1) s1 += ee[j]; else s0 += ee[j];
              }
              PKV_SG_MFMA(1);
              if (t == kTiles - 2) {
                if (ks < 4) PKV_SG_DSR(2); else PKV_SG_DSR(1);
              }
              PKV_SG_VALU(TPM);
              PKV_SG_TRANS(TPM);
              PKV_SG_VALU(TPM);
            }
            e[t] += s0 + s1;
            cur = nxt;
          }
        }
      }
    }
    if (has_keys) {
      float* raw = a.raw + (size_t)u * a.N;
#pragma unroll
      for (int t = 0; t < kTiles; ++t) {
        float tot = e[t];
        tot += __shfl_xor(tot, 32);
        const int key = wkey0 + 32 * t + l32;
        if (hf == 0 && key < npre) raw[key] = tot * a.inv_G;
      }
    }
    __syncthreads();  // cst / qs / red are reused by the next unit
    PKV_T(4);
  }
#ifdef PKV_RES_TIMING
  tstamp[5] += clock64();
  tstamp[6] += wall_clock64();
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
  // the counters, the error word and the tagged normaliser words must start at zero
  const int nz = a.sync_words;
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
