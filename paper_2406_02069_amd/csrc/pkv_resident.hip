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
//      When a unit has 4 parts or more, every part takes part in every unit of its group (one beyond the end
//      of a shorter sequence contributes neutral statistics) and there is no counter: the statistics
//      words carry a phase bit, and part p folds the rows p, p + nparts, ... as soon as their words show
//      it.
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
// Every wait is bounded by wall-clock time: a workgroup that has waited too long raises the error word and
// carries on, so the grid always drains.  The launch uses exactly 512 workgroups, two per compute unit (register- and
// LDS-limited), which the host checks against the device before choosing this path.
//
// One-sweep variant (second template argument): when the caller supplies the softmax denominators of the
// window queries (the log-sum-exp its attention kernel computed during prefill), steps 2 and 3 fall away
// and the kernel is step 4 alone over a stream of keys: no workgroup waits for another, the (unit, part)
// items are handed out from a counter, and the next item's keys, Q block and denominators travel while the
// current item is computed.  Bound by HBM instead of the vector pipe.
#include <type_traits>

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

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ bf16x8 as_frag(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }
#define PKV_MFMA32(A, B, C) __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B, C, 0, 0, 0)
// End of a hand-ordered chunk (one MFMA, the exponentials that run in its shadow, at most one LDS read):
// nothing is scheduled across this point, so the interleaving written in the source is what is emitted.
#define PKV_CHUNK_END() __builtin_amdgcn_sched_barrier(0)
// The same, and the two running sums are pinned here: without that the optimiser sinks the exponentials of
// all chunks to the place where the sums are finally used, behind the last MFMA.
#define PKV_CHUNK_END_SUMS(s0, s1)                 \
  do {                                             \
    asm volatile("" : "+v"(s0), "+v"(s1));         \
    __builtin_amdgcn_sched_barrier(0);             \
  } while (0)

// The Q block is kept in LDS with a row pitch of SEG + 1 sixteen-byte segments: consecutive rows then
// start 4 banks apart (mod 64), so the 16 rows that one ds_read_b128 phase touches hit all banks once,
// and the segment index stays a compile-time address offset.
template <int SEG>
__host__ __device__ __forceinline__ constexpr int lds_pitch() { return SEG + 1; }

__device__ __forceinline__ void merge_stats(float& m, float& z, float m2, float z2) {
  const float M = fmaxf(m, m2);
  const float Ms = (M == -INFINITY) ? 0.f : M;
  z = z * fast_exp2(m - Ms) + z2 * fast_exp2(m2 - Ms);
  m = M;
}

// -c/kappa as three bf16 summands (hi + mid + lo reproduces the fp32 value to 2^-24): the layout of the
// first three k-elements of an MFMA operand.  -inf stays -inf (padding rows).
__device__ __forceinline__ u64 split3(float c) {
  const __bf16 hi = (__bf16)c;
  float r = c - (float)hi;
  if (c == -INFINITY) r = 0.f;
  const __bf16 mid = (__bf16)r;
  r -= (float)mid;
  const __bf16 lo = (__bf16)r;
  const uint32_t w0 = (uint32_t)__builtin_bit_cast(uint16_t, hi) | ((uint32_t)__builtin_bit_cast(uint16_t, mid) << 16);
  const uint32_t w1 = (uint32_t)__builtin_bit_cast(uint16_t, lo);
  return ((u64)w1 << 32) | w0;
}

// A value the compiler must treat as new: lane constants derived from it are recomputed where they are
// used instead of being kept (and spilled) across the whole unit loop.
__device__ __forceinline__ int fresh(int v) {
  asm volatile("" : "+v"(v));
  return v;
}

// Workgroup barrier that orders LDS traffic only.  A full __syncthreads() carries fences over global memory as
// well, and the waits the compiler builds for them include, since memory operations retire in order, every key
// load requested before: exactly the loads that are meant to stay in flight across the barrier.  (Neither kind
// of barrier waits for the acknowledgement of outstanding global stores: where another workgroup is told that
// data is ready, the storing waves wait for vmcnt(0) themselves.)
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ void st64(u64* p, u64 v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ u64 ld64(const u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Accumulator element v of a lane (half h) belongs to tile row mrow(v, h) (32x32 MFMA output layout).
__device__ __forceinline__ constexpr int mrow0(int v) { return 8 * (v >> 2) + (v & 3); }

// LSE: the per-row softmax denominators come from the caller (natural-log sums, one per window query); sweep 1
// and the exchange between the workgroups are not needed then and every key is used once: a plain stream over K.
template <int D, bool LSE>
__global__ __launch_bounds__(kThreads, 2) void score_resident_kernel(const ResidentArgs a) {
  constexpr int KS = D / 16;   // 32x32x16 MFMA k-steps per dot product
  constexpr int SEG = D / 8;   // 16-byte segments per row
  constexpr int TPM = 16 / KS; // logits per lane handled between two MFMAs
  constexpr int PITCH = lds_pitch<SEG>();
  constexpr int QLD = kRowBlock * SEG / kThreads;  // 16-byte loads per thread for one block of Q
  constexpr int RPP = kThreads / SEG;              // rows covered by one pass of the workgroup
  constexpr int QBUF = kRowBlock * PITCH;          // 16-byte slots of one Q buffer
  extern __shared__ u32x4 qsmem[];                 // two buffers for 128-row blocks of Q
  // sweep-1 statistics per wave, wave half and row.  Between sweeps the same memory serves as scratch for
  // the fold, as the row-offset table of the Q staging and as the "last to arrive" flag (never at once).
  __shared__ float2 stat_mem[kWaves * 2 * kRowBlock];
  // per-row normalisers, ready for the matrix pipe: -c_r/kappa split into three bf16 (hi | mid << 16, lo)
  __shared__ u64 cfr[kResidentMaxRows];
  float2 (*stat)[2][kRowBlock] = reinterpret_cast<float2 (*)[2][kRowBlock]>(stat_mem);
  // With supplied denominators there are no statistics: the memory holds a second normaliser table instead (the
  // next unit's is filled while the current one is in use), and behind it the row-offset tables.
  static_assert(sizeof(stat_mem) >= kResidentMaxRows * sizeof(u64) + 2 * kRowBlock * sizeof(int), "LDS reuse");
  u64* cfr_alt = reinterpret_cast<u64*>(stat_mem);                                // [kResidentMaxRows], LSE only
  int* qoff = reinterpret_cast<int*>(stat_mem) + (LSE ? 2 * kResidentMaxRows : 0);  // [kRowBlock]
  int* qoff0 = qoff + kRowBlock;                                                  // [kRowBlock], LSE only: block 0, kept
  int* s_last_p = reinterpret_cast<int*>(stat_mem + kWaves * 2 * kRowBlock) - 1;  // last word
#define s_last (*s_last_p)

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps addressing in scalar registers
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
  if (!LSE && sub >= a.UPG) return;  // no work for this workgroup at this shape
  const int slot_id = group * a.UPG + sub;  // one of nslots concurrent units
  const int nslots = a.ngroups * a.UPG;
  float2* part_base = a.part + (size_t)slot_id * a.TPU * a.Rpad;
  u64* cbuf = a.cbuf + (size_t)slot_id * a.Rpad;
  const int key0 = part_id * kResidentKeys;
  const int wkey0 = key0 + wave * (kTiles * 32);


  if (a.stagger > 0 && a.ngroups >= 2) {
    // Staggered start (a plain timed wait): the groups begin evenly spread over one period, the two
    // groups that share compute units half a period apart.
    const int rank = (group >> 1) + (a.ngroups >> 1) * set;
    const long long t0 = wall_clock64(), wait = (long long)a.stagger * rank;
    while (wall_clock64() - t0 < wait) __builtin_amdgcn_s_sleep(16);
  }

  // One unit as this workgroup sees it (all fields wave-uniform).
  struct Unit {
    int u, n, npre, nparts;
    int j;  // position of the unit in the list of the group pair (two-sweep path)
    const uint16_t* Q;
    const uint16_t* K;
    const float* lse;  // the unit's G * alpha denominators (row r = head * alpha + t), LSE only
    int wkey0;         // first key of this wave in the unit, LSE only (there the part changes from unit to unit)
  };
  // Which units a group works on.  The units are dealt round-robin to the pairs of groups that share compute units
  // (first and second workgroup of every unit of an XCD cluster), and a pair's list is split between its two
  // groups in the ratio (32 - w) : w.  The second workgroup of a compute unit gets the issue slots the first one
  // leaves, so its group needs about a tenth longer per unit; with equal shares the first groups would sit idle
  // at the end.  (Only speed depends on the split; w = 16 alternates.)
  const bool paired = a.ngroups >= 2;
  const int npairs = paired ? nslots / 2 : nslots;
  const int pair_slot = paired ? (group >> 1) * a.UPG + sub : slot_id;
  auto mine = [&](int j) { return !paired || ((((j + 1) * a.set1_w) >> 5) != ((j * a.set1_w) >> 5)) == ((group & 1) != 0); };
  // First unit at or after position j of the pair's list that is this group's and in which this workgroup has
  // keys to score.
  auto find_unit = [&](int j, Unit& d) {
    for (;; ++j) {
      const int u = pair_slot + j * npairs;
      if (u >= a.U) break;
      if (!mine(j)) continue;
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
      // no keys here: with the arrival counter this part is not counted and moves on; with the tagged exchange
      // every part takes part in every unit of its group (neutral statistics, its share of the fold, the wait)
      if (!a.tagged && key0 >= n) continue;
      d.u = u;
      d.j = j;
      d.n = n;
      d.npre = n - a.alpha;
      d.nparts = a.tagged ? a.TPU : (n + kResidentKeys - 1) / kResidentKeys;
      d.Q = a.layer[l].Q + (size_t)b * a.q_sb + (size_t)(g * a.G) * a.q_sh;
      d.K = a.layer[l].K + (size_t)b * a.kv_sb + (size_t)g * a.kv_sh;
      if (LSE) d.lse = a.layer[l].lse + ((size_t)b * a.Hq + (size_t)g * a.G) * a.alpha;
      return;
    }
    d.u = a.U;
  };
  // LSE: nothing ties a workgroup to a group or a part, so the (unit, part) items are handed out on demand: item
  // j = unit j / TPU, part j % TPU.  Every workgroup starts with the items blockIdx and 512 + blockIdx and draws
  // further ones from a counter; a workgroup slowed down by its neighbours or its memory channels just takes
  // fewer.  An item without work (sequence kept whole, part beyond its end) is skipped.
  const int n_items = a.U * a.TPU;
  // four words: [0], [1] for the draws made ahead (used alternately), [2] for replacement draws, [3] spare
  int* s_item = reinterpret_cast<int*>(stat_mem + kWaves * 2 * kRowBlock) - 4;
  auto decode = [&](int item, Unit& d) -> bool {
    const int u = item / a.TPU, part = item - u * a.TPU;
    const int l = u / BH;
    const int bg = u - l * BH;
    const int b = bg / a.Hkv;
    const int g = bg - b * a.Hkv;
    int n = a.N;
    if (a.seq_lens) {
      n = a.seq_lens[b];
      n = n < 0 ? 0 : (n > a.N ? a.N : n);
    }
    if (a.layer[l].k_l >= n || part * kResidentKeys >= n) return false;
    d.u = u;
    d.n = n;
    d.npre = n - a.alpha;
    d.nparts = 0;
    d.Q = a.layer[l].Q + (size_t)b * a.q_sb + (size_t)(g * a.G) * a.q_sh;
    d.K = a.layer[l].K + (size_t)b * a.kv_sb + (size_t)g * a.kv_sh;
    d.lse = a.layer[l].lse + ((size_t)b * a.Hq + (size_t)g * a.G) * a.alpha;
    d.wkey0 = part * kResidentKeys + wave * (kTiles * 32);
    return true;
  };
  // The item `it`, or the next one with work, as unit d (d.u = U when the items have run out).  Called by all
  // threads together; drawing a replacement involves the whole workgroup (rare).
  auto take = [&](int it, Unit& d) {
    while (it < n_items && !decode(it, d)) {
      __syncthreads();  // everyone holds the same `it` and is done with the previous replacement
      if (tid == 0)
        s_item[2] = 2 * kResidentGrid + __hip_atomic_fetch_add(&a.cnt[0], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __syncthreads();
      it = s_item[2];
    }
    if (it >= n_items) d.u = a.U;
  };

  // Stage a 128-row block of Q in LDS.  qoff[row] = byte offset of the row (-1: padding row).
  // Thread -> (row tid / SEG + RPP * i, segment tid % SEG): 16 bytes per load, rows fully coalesced.
  // Callers put a workgroup barrier between this and the first read of the buffer.
  auto stage_q = [&](const Unit& d, int rb, u32x4* qb) {
    const int tid_ = fresh(tid);
    const int q_row0 = tid_ / SEG, q_seg = tid_ - q_row0 * SEG;
    if (tid < kRowBlock) {
      const int r = rb * kRowBlock + tid;
      int off = -1;
      if (r < a.R) {
        const int hh = r / a.alpha, t = r - hh * a.alpha;
        off = (int)(hh * a.q_sh + t * a.q_st) * 2;
      }
      qoff[tid] = off;
    }
    lds_barrier();
    const char* src = reinterpret_cast<const char*>(d.Q) + q_seg * 16;
    u32x4 v[QLD];
#pragma unroll
    for (int i = 0; i < QLD; ++i) {
      const int off = qoff[q_row0 + RPP * i];
      v[i] = u32x4{0u, 0u, 0u, 0u};
      if (off >= 0) v[i] = *reinterpret_cast<const u32x4*>(src + (uint32_t)off);
    }
    u32x4* dst = qb + q_row0 * PITCH + q_seg;
#pragma unroll
    for (int i = 0; i < QLD; ++i) dst[RPP * i * PITCH] = v[i];
  };

  // LSE: block 0 of a unit's Q goes to LDS in two halves (H = 0, 1: every second group of rows), each requested
  // into registers at one point and written to LDS at a later one, so that the loads travel in the shadow of a
  // pass while only a few registers wait for them.  Row offsets come from the kept table; no barrier here.
  constexpr int QH = QLD / 2;
  auto q_request = [&](const Unit& d, auto H, u32x4 (&v)[QH]) {
    const int tid_ = fresh(tid);
    const int q_row0 = tid_ / SEG, q_seg = tid_ - q_row0 * SEG;
    const char* src = reinterpret_cast<const char*>(d.Q) + q_seg * 16;
#pragma unroll
    for (int i = 0; i < QH; ++i) {
      const int off = qoff0[q_row0 + RPP * (2 * i + decltype(H)::value)];
      v[i] = u32x4{0u, 0u, 0u, 0u};
      if (off >= 0) v[i] = *reinterpret_cast<const u32x4*>(src + (uint32_t)off);
    }
  };
  auto q_commit = [&](const u32x4 (&v)[QH], auto H, u32x4* qb) {
    const int tid_ = fresh(tid);
    const int q_row0 = tid_ / SEG, q_seg = tid_ - q_row0 * SEG;
    u32x4* dst = qb + q_row0 * PITCH + q_seg;
#pragma unroll
    for (int i = 0; i < QH; ++i) dst[RPP * (2 * i + decltype(H)::value) * PITCH] = v[i];
  };
  // LSE: the unit's supplied denominators.  Table entry of row r: -c_r/kappa with c_r = lse_r * log2(e) (the logits
  // are kept in the log2 domain); padding rows -inf.
  constexpr int NL = kResidentMaxRows / kThreads;
  auto lse_request = [&](const Unit& d, float (&lv)[NL]) {
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int r = tid + kThreads * j;
      lv[j] = INFINITY;
      if (r < a.R) lv[j] = d.lse[r];
    }
  };
  auto lse_commit = [&](const float (&lv)[NL], u64* table) {
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int r = tid + kThreads * j;
      if (r < a.Rpad) table[r] = split3(-(lv[j] * 1.44269504088896340736f) * a.inv_kappa);
    }
  };

  // The wave's keys as MFMA operand fragments: kf[t][ks] = for key 32*t + (lane & 31), the 8 elements at
  // 16*ks + 8*(lane >> 5).  Loaded straight from global memory in this layout.
  bf16x8 kf[kTiles][KS];
  // Request fragments [KLO, KHI) of key tile T of unit d.  Branch-free: keys at or beyond n are clamped to the
  // last valid row (never read beyond it); a wave without keys in that unit just fetches that row.
  auto issue_k = [&](const Unit& d, auto T, auto KLO, auto KHI) {
    constexpr int t = decltype(T)::value;
    const int lane_ = fresh(lane);
    const int l32 = lane_ & 31, hf = lane_ >> 5;
    const int key = min((LSE ? d.wkey0 : wkey0) + 32 * t + l32, d.n - 1);
    // 32-bit byte offsets from the head's first key (the host admits only shapes where they fit)
    const char* rowp = reinterpret_cast<const char*>(d.K) + 16 * hf + (uint32_t)key * ((uint32_t)a.kv_st * 2u);
#pragma unroll
    for (int ks = decltype(KLO)::value; ks < decltype(KHI)::value; ++ks)
      kf[t][ks] = as_frag(*reinterpret_cast<const u32x4*>(rowp + 32 * ks));
  };
  using IKS = std::integral_constant<int, KS>;
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  using INONE = std::integral_constant<int, -1>;
  // While a pass works on one pair of key tiles, the other pair can be refilled: half a tile (RFT, or none if
  // negative) after the middle chunk of a step, at fixed places of the first two row-tile iterations, so that
  // the loads trickle out in the shadow of the arithmetic instead of stalling the wave at the memory
  // pipeline's entrance.  (Unconditional loads at fixed places: loads under a run-time condition keep the
  // old and the new fragments alive side by side, which the register budget cannot afford.)
  auto refill = [&](const Unit& ru, auto RFT, auto HALF) {
    if constexpr (decltype(RFT)::value >= 0) {
      using LO = std::integral_constant<int, decltype(HALF)::value * (KS / 2)>;
      using HI = std::integral_constant<int, decltype(HALF)::value * (KS / 2) + KS / 2>;
      issue_k(ru, RFT, LO{}, HI{});
      PKV_CHUNK_END();
    }
  };

  // Every wait for another workgroup is bounded by wall-clock time (the grid must drain even if its workgroups are
  // not resident together).  Called after a failed probe: true once the wait has lasted wait_ticks (10 ns each)
  // or another workgroup has already given up.  The clock is read every 16th probe (a probe is a memory round trip).
  auto waited_too_long = [&](int& spins, long long& t0) -> bool {
    if (a.wait_ticks == 0) return true;
    if (spins++ == 0) {
      t0 = wall_clock64();
      return false;
    }
    if ((spins & 15) != 0) return false;
    return wall_clock64() - t0 > (long long)a.wait_ticks ||
           __hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
  };

  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  if (tid == 0) qsmem[SEG] = u32x4{0u, 0u, 0u, 0u};  // pad slot of row 0: never written by the staging
  Unit cur_u, nxt_u;
  int drawn = 0;  // LSE: the counter's value at this unit's draw (the item is 1024 + that)
  int seqpos = 0; // units this workgroup has worked on (two-sweep path, tagged mode: all parts of a group agree)
  if constexpr (LSE) {
    take((int)blockIdx.x, cur_u);
    if (cur_u.u < a.U) take(kResidentGrid + (int)blockIdx.x, nxt_u);
  } else {
    find_unit(0, cur_u);
  }
  if (cur_u.u >= a.U) return;
  int buf = 0;
  if (LSE && tid < kRowBlock) {  // row offsets of block 0: the same for every unit
    int off = -1;
    if (tid < a.R) {
      const int hh = tid / a.alpha, t = tid - hh * a.alpha;
      off = (int)(hh * a.q_sh + t * a.q_st) * 2;
    }
    qoff0[tid] = off;
  }
  stage_q(cur_u, 0, qsmem);
  if (LSE) {
    float lv[NL];
    lse_request(cur_u, lv);
    lse_commit(lv, cfr);
  }
  issue_k(cur_u, I0{}, I0{}, IKS{});
  issue_k(cur_u, I1{}, I0{}, IKS{});
  // LSE: the unit loop is entered as it comes round: first half of the keys arrived, second half in flight.  (Else
  // the first pass, which sees both ways in, would wait for part of the second half in every unit.)
  if constexpr (LSE) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  issue_k(cur_u, I2{}, I0{}, IKS{});
  issue_k(cur_u, I3{}, I0{}, IKS{});
  __syncthreads();

  while (cur_u.u < a.U) {
    const int u = cur_u.u, n = cur_u.n, npre = cur_u.npre, nparts = cur_u.nparts;
    if constexpr (!LSE) find_unit(cur_u.j + 1, nxt_u);
    const bool has_next = nxt_u.u < a.U;
    const uint32_t phase = (uint32_t)(seqpos & 1) ^ 1u;  // tagged mode: the bit this unit's statistics carry
    ++seqpos;
    const int wkey = LSE ? cur_u.wkey0 : wkey0;
    const bool has_keys = wkey < n;                       // wave-uniform
    // tile t needs masks iff it reaches beyond the prefix (causal window, end of the sequence)
    int dirty_mask = 0;
#pragma unroll
    for (int t = 0; t < kTiles; ++t) dirty_mask |= (wkey0 + 32 * t + 32 > npre) ? (1 << t) : 0;
    u32x4* qb = qsmem + buf * QBUF;
    const int lane_u = fresh(lane);
    const int l32 = lane_u & 31, hf = lane_u >> 5;
    const u32x4* q_lane = qb + l32 * PITCH + hf;
    // normaliser table of this unit; LSE: the two tables alternate like the Q buffers
    const u64* cfr_cur = (LSE && buf) ? cfr_alt : cfr;
    u64* cfr_nxt = (LSE && !buf) ? cfr_alt : cfr;
    bool q_staged = false;
    // LDS reads of one 32-row tile of Q as MFMA operand fragments
    auto q_frag = [&](int rt, int ks) { return as_frag(q_lane[32 * rt * PITCH + 2 * ks]); };

    if constexpr (!LSE) {
    // ---- sweep 1: per-row statistics over this workgroup's keys ----
    // Products: rows = keys (element v of a lane: key mrow0(v) + 4*hf of the tile), columns = query rows
    // (lane & 31).  Per lane and row tile: reference exponent m (log2 domain) and z = sum exp2(x - m), kept in
    // LDS between the two passes over the row tiles (first the tiles 0,1 of the keys, then 2,3: the second
    // half of the keys may still be in flight during the first pass).
    float2* part = part_base + (size_t)part_id * a.Rpad;
    for (int rb = 0; rb < a.nrb; ++rb) {
      if (rb > 0) {
        __syncthreads();  // everyone is done with the previous block
        stage_q(cur_u, rb, qb);
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
        // last key (relative to this wave's first key and half) that the lane's query of row tile rt sees
        auto lim_rel_of = [&](int rt) {
          const int r = rb * kRowBlock + 32 * rt + l32;
          const int lim = (r < a.R) ? npre + (r % a.alpha) : npre + a.alpha - 1;  // padding rows: statistics unused
          return lim - wkey0 - 4 * hf;
        };

        bf16x8 qf[KS];
        f32x16 cur, nxt;
        int redo = 0;  // row tiles whose provisional reference failed (wave-uniform bit mask)
        // One step of the pipeline: issue the MFMAs of the product (TN, current qf) and meanwhile turn the
        // finished product `cur` of tile TC into exponentials.  RELOAD: the issued product is the last use
        // of qf, which is refilled for row tile rt_next as the MFMAs go out.
        auto step = [&](auto TC, auto TN, auto FIRST, auto RELOAD, auto ISSUE, auto RFT, auto HALF, const Unit& ru, int rt,
                        int rt_next, float& m, float& z) {
          constexpr int tc = decltype(TC)::value, tn = decltype(TN)::value;
          constexpr bool issue = decltype(ISSUE)::value;  // false: the pass ends here, no further product
          const bool dirty = (dirty_mask & (1 << tc)) != 0;
          if (dirty && decltype(FIRST)::value) {
            // A masked tile that also has to found the lane's reference exponent (no earlier tile of the wave in
            // this unit): exact running-maximum update; the next product is still issued first.
            nxt = zero16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
              if (issue) nxt = PKV_MFMA32(kf[tn][ks], qf[ks], nxt);
              if (decltype(RELOAD)::value) qf[ks] = q_frag(rt_next, ks);
            }
            refill(ru, RFT, HALF);
            exact_update(cur, tc, true, lim_rel_of(rt), m, z);
          } else {
            // The pipelined variant; MASKED: the tile reaches beyond the prefix (causal window, end of the
            // sequence), logits of keys the lane's query does not see become -inf before the exponential.  The
            // reference exponent then comes from an earlier, unmasked tile of the wave.
            auto fast = [&](auto MASKED) {
              constexpr bool masked = decltype(MASKED)::value;
              if (decltype(FIRST)::value) {  // provisional reference: the largest of three of the lane's logits
                m = a.kappa * fmaxf(fmaxf(cur[0], cur[5]), cur[10]);
                z = 0.f;
              }
              const float nref = -m;
              const int lim = masked ? lim_rel_of(rt) - 32 * tc : 0;  // last visible key, relative to this tile and half
              float s0 = 0.f, s1 = 0.f;
              nxt = zero16;
#pragma unroll
              for (int ks = 0; ks < KS; ++ks) {
                if (issue) nxt = PKV_MFMA32(kf[tn][ks], qf[ks], nxt);
                if (decltype(RELOAD)::value) qf[ks] = q_frag(rt_next, ks);  // last use of this fragment was the MFMA above
                float x[TPM], e[TPM];
#pragma unroll
                for (int j = 0; j < TPM; ++j) {
                  x[j] = __builtin_fmaf(cur[TPM * ks + j], a.kappa, nref);
                  if (masked && mrow0(TPM * ks + j) > lim) x[j] = -INFINITY;
                }
#pragma unroll
                for (int j = 0; j < TPM; ++j) e[j] = fast_exp2(x[j]);
#pragma unroll
                for (int j = 0; j < TPM; ++j) {
                  if (j & 1) s1 += e[j]; else s0 += e[j];
                }
                PKV_CHUNK_END_SUMS(s0, s1);
                if (ks == KS / 2 - 1) refill(ru, RFT, HALF);
              }
              z += s0 + s1;
            };
            if (dirty) fast(std::true_type{});
            else fast(std::false_type{});
          }
          cur = nxt;
        };
        using F = std::false_type;
        using T = std::true_type;
        // both products of one row tile with the key tiles (TA, TB); RFT: key tile refilled meanwhile
        auto iter = [&](auto TA, auto TB, auto FIRSTPASS, auto RFT, const Unit& ru, int rt) {
          const int rt_next = (rt + 1 < nrt) ? rt + 1 : 0;  // (the last reload of the pass is not used)
          float m = -INFINITY, z = 0.f;  // m: reference exponent of this lane (not necessarily the maximum)
          if (!decltype(FIRSTPASS)::value) {
            const float2 st = stat[wave][hf][32 * rt + l32];
            m = st.x;
            z = st.y;
          }
          step(TA, TB, FIRSTPASS, T{}, T{}, RFT, I0{}, ru, rt, rt_next, m, z);
          if (rt + 1 < nrt) step(TB, TA, F{}, F{}, T{}, RFT, I1{}, ru, rt, rt_next, m, z);
          else step(TB, TA, F{}, F{}, F{}, RFT, I1{}, ru, rt, rt_next, m, z);  // last product of the pass
          stat[wave][hf][32 * rt + l32] = make_float2(m, z);
          // a sum outside the safe range (or NaN) means the provisional reference was too far off
          if (!decltype(FIRSTPASS)::value && __any(!(z <= 0x1p100f))) redo |= 1 << rt;
        };
        // pass over the row tiles with the key tiles (TA, TB); REFILL: key tiles (F0, F1) are requested for ru
        auto pass = [&](auto TA, auto TB, auto FIRSTPASS, auto REFILL, auto F0, auto F1, const Unit& ru) {
          constexpr int ta = decltype(TA)::value;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) qf[ks] = q_frag(0, ks);
          cur = zero16;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) cur = PKV_MFMA32(kf[ta][ks], qf[ks], cur);
          int rt = 0;
          if constexpr (decltype(REFILL)::value) {
            iter(TA, TB, FIRSTPASS, F0, ru, 0);
            if (nrt > 1) iter(TA, TB, FIRSTPASS, F1, ru, 1);
            else issue_k(ru, F1, I0{}, IKS{});
            rt = 2;
          }
#pragma unroll 1
          for (; rt < nrt; ++rt) iter(TA, TB, FIRSTPASS, INONE{}, ru, rt);
        };
        pass(I0{}, I1{}, T{}, F{}, I2{}, I3{}, cur_u);
        pass(I2{}, I3{}, F{}, F{}, I0{}, I1{}, cur_u);
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
          stat[wave][hf][32 * rt + l32] = make_float2(m, z);
        }
      } else {
        for (int r = lane; r < 2 * kRowBlock; r += 64) stat[wave][r >> 7][r & 127] = make_float2(-INFINITY, 0.f);
      }
      // From here to the start of sweep 2 the wave has little to issue and most of it sits on the critical path of
      // the whole group (statistics, arrival, fold, release): it goes first at the issue port that it shares with
      // a wave of another group that is in the middle of a sweep.
      __builtin_amdgcn_s_setprio(3);
      lds_barrier();
      if (tid < rows_here) {
        float m = -INFINITY, z = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          merge_stats(m, z, stat[w][0][tid].x, stat[w][0][tid].y);
          merge_stats(m, z, stat[w][1][tid].x, stat[w][1][tid].y);
        }
        // device-scope store: written through, so that other XCDs see it without an L2 write-back.  Tagged mode:
        // the sign bit of the sum (never negative) carries the unit's phase bit, so the word announces itself.
        uint32_t zb = __float_as_uint(z);
        if (a.tagged) zb = (zb & 0x7FFFFFFFu) | (phase << 31);
        st64(reinterpret_cast<u64*>(part + rb * kRowBlock + tid), ((u64)zb << 32) | __float_as_uint(m));
      }
    }
    if (a.tagged) {
      lds_barrier();  // (nobody waits for these stores: their readers look at the tag)
    } else {
      // Release: the arrival below tells the last arriver that this part's statistics can be read, so every
      // wave first waits until its own statistics stores have been acknowledged (a workgroup barrier alone
      // does not wait for outstanding global stores), and only then does the workgroup meet.
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
      __syncthreads();
    }

    // ---- arrive; the last part folds all parts into the per-row normaliser and publishes it ----
    // Tagged mode (every part takes part in every unit of its group): no counter and no last arriver.  Part p folds
    // the rows p, p + nparts, ..., one wave per row and one lane per part: a lane probes its part's word of the row
    // until it shows this unit's phase bit.  Two hops of the exchange fall away (the acknowledgement of the
    // statistics stores and the round trip of the arrival counter).
    const unsigned tag = (unsigned)u + 1u;
    bool last = false;
    if (a.tagged) {
      for (int r = part_id + wave * nparts; r < a.R; r += kWaves * nparts) {
        float m = -INFINITY, z = 0.f;
        for (int p = lane; p < nparts; p += 64) {
          const u64* src = reinterpret_cast<const u64*>(part_base + (size_t)p * a.Rpad + r);
          int spins = 0;
          long long t0 = 0;
          u64 w;
          for (;;) {
            w = ld64(src);
            if ((uint32_t)(w >> 63) == phase) break;
            __builtin_amdgcn_s_sleep(2);
            if (waited_too_long(spins, t0)) {
              __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              break;
            }
          }
          merge_stats(m, z, __uint_as_float((uint32_t)w), __uint_as_float((uint32_t)(w >> 32) & 0x7FFFFFFFu));
        }
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) {
          const float m2 = __shfl_xor(m, s), z2 = __shfl_xor(z, s);
          merge_stats(m, z, m2, z2);
        }
        if (lane == 0) st64(&cbuf[r], ((u64)tag << 32) | __float_as_uint(-(m + fast_log2(z)) * a.inv_kappa));
      }
    } else {
      if (tid == 0) {
        const int prev = __hip_atomic_fetch_add(&a.cnt[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == nparts - 1);
      }
      __syncthreads();
      last = s_last != 0;
    }
    if (last) {
      // NQ threads per row, each folds every NQ-th part (32 independent loads in flight), then they meet in LDS
      constexpr int NQ = kThreads / kRowBlock;
      constexpr int NLD = 32;
      const int q = tid >> 7, rl = tid & 127;
      float2* red = &stat[0][0][0];  // [NQ][kRowBlock]
      for (int r0 = 0; r0 < a.Rpad; r0 += kRowBlock) {
        const int r = r0 + rl;
        float m = -INFINITY, z = 0.f;
        if (r < a.R) {
          for (int p0 = q; p0 < nparts; p0 += NLD * NQ) {
            u64 bits[NLD];
#pragma unroll
            for (int k = 0; k < NLD; ++k) {
              const int p = min(p0 + NQ * k, nparts - 1);  // clamped: duplicates are skipped below
              bits[k] = ld64(reinterpret_cast<const u64*>(part_base + (size_t)p * a.Rpad + r));
            }
            float M = m;
#pragma unroll
            for (int k = 0; k < NLD; ++k)
              if (p0 + NQ * k < nparts) M = fmaxf(M, __uint_as_float((uint32_t)bits[k]));
            const float Ms = (M == -INFINITY) ? 0.f : M;
            z *= fast_exp2(m - Ms);
#pragma unroll
            for (int k = 0; k < NLD; ++k)
              if (p0 + NQ * k < nparts)
                z += __uint_as_float((uint32_t)(bits[k] >> 32)) * fast_exp2(__uint_as_float((uint32_t)bits[k]) - Ms);
            m = M;
          }
        }
        red[q * kRowBlock + rl] = make_float2(m, z);
        lds_barrier();
        if (q == 0) {
#pragma unroll
          for (int k = 1; k < NQ; ++k) merge_stats(m, z, red[k * kRowBlock + rl].x, red[k * kRowBlock + rl].y);
          // kept as -c_r/kappa (see sweep 2); padding rows get -inf and contribute exp2(-inf) = 0
          const float c = (r < a.R) ? -(m + fast_log2(z)) * a.inv_kappa : -INFINITY;
          cfr[r] = split3(c);
          if (r < a.R) st64(&cbuf[r], ((u64)tag << 32) | __float_as_uint(c));
        }
        lds_barrier();
      }
      if (has_next) {  // before this unit's sweep 2 requests the next keys: loads return in order
        stage_q(nxt_u, 0, qsmem + (buf ^ 1) * QBUF);
        q_staged = true;
      }
    } else {
      // while the others arrive: the next unit's first block of Q goes into the other LDS buffer
      if (has_next) {
        stage_q(nxt_u, 0, qsmem + (buf ^ 1) * QBUF);
        q_staged = true;
      }
      for (int r = tid; r < a.Rpad; r += kThreads) {
        float c = -INFINITY;
        if (r < a.R) {
          int spins = 0;
          long long t0 = 0;
          u64 w;
          for (;;) {
            w = ld64(&cbuf[r]);
            if ((unsigned)(w >> 32) == tag) break;
            __builtin_amdgcn_s_sleep(1);
            if (waited_too_long(spins, t0)) {
              __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              break;
            }
          }
          c = __uint_as_float((unsigned)w);
        }
        cfr[r] = split3(c);
      }
      lds_barrier();
    }
    __builtin_amdgcn_s_setprio(0);
    }  // !LSE

    // ---- sweep 2: normalised probabilities summed over the query rows ----
    // Here the product's rows are query rows (element v of a lane: row mrow0(v) + 4*hf of the tile) and its
    // columns keys (lane & 31).  -c_r/kappa enters each product through one extra MFMA (see below), so the
    // product comes out as (q.k - c_r/kappa) and one multiply + exp2 + add per logit remain.
    // Again two passes (key tiles 0,1, then 2,3): after a pass its keys are no longer needed, their scores are
    // written, and the next unit's keys are requested into the same registers.
    // Every load issued so far has long returned (sweep 1 consumed the keys).  Saying so here keeps the
    // compiler from waiting, in the second pass, for the next unit's keys requested after the first pass.
    // (With supplied denominators there was no sweep 1: the second half of the keys may still be in flight, and
    // should be.)
    if constexpr (!LSE) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    float* raw = a.raw + (size_t)u * a.N;
    float e[kTiles];
#pragma unroll
    for (int t = 0; t < kTiles; ++t) e[t] = 0.f;
    // LAST: the final row block; only there are scores written and the next keys requested (kept out of the
    // row-block loop so that no load appears to be pending on the keys when the loop comes round).
    auto s2_block = [&](int rb, auto LAST) {
      constexpr bool last_rb = decltype(LAST)::value;
      if (a.nrb > 1) {
        __syncthreads();
        stage_q(cur_u, rb, qb);
        __syncthreads();
      }
      const int rows_here = min(kRowBlock, a.R - rb * kRowBlock);
      const int nrt = (rows_here + 31) / 32;
      bf16x8 qf[KS];
      f32x16 cur, nxt;
      // The normalisers enter through one extra MFMA per product: operand A = (hi, mid, lo, 0...) of the
      // lane's query row in the first wave half (zeros in the second), operand B = (1, 1, 1, 0...).
      const u32x4 ones_u = (hf == 0) ? u32x4{0x3F803F80u, 0x00003F80u, 0u, 0u} : u32x4{0u, 0u, 0u, 0u};
      const bf16x8 ones = as_frag(ones_u);
      const u64* cfr_lane = (hf == 0) ? cfr_cur + rb * kRowBlock + l32 : reinterpret_cast<const u64*>(qsmem + SEG);  // second half: a zero word
      const int cfr_step = (hf == 0) ? 32 : 0;
      bf16x8 bfr;
      auto load_bias = [&](int rt) {
        const u64 w = cfr_lane[cfr_step * rt];
        bfr = as_frag(u32x4{(uint32_t)w, (uint32_t)(w >> 32), 0u, 0u});
      };
      // `fin` holds the finished product of tile TC; the product of tile TN goes into `out` (the two accumulators
      // swap roles from step to step, so nothing is ever copied)
      auto step = [&](auto TC, auto TN, auto RELOAD, auto ISSUE, auto RFT, auto HALF, const Unit& ru, int rt_next,
                      const f32x16& fin, f32x16& out) {
        constexpr int tc = decltype(TC)::value, tn = decltype(TN)::value;
        constexpr bool issue = decltype(ISSUE)::value;  // false: the pass ends here, no further product
        float s0 = 0.f, s1 = 0.f;
        // a scale factor of its own for every instance of this step: identical multiplies in the two arms of a
        // branch would otherwise be merged in front of it, away from the MFMAs they are meant to run under
        float kap = a.kappa;
        asm volatile("" : "+s"(kap));
        if (issue) out = PKV_MFMA32(bfr, ones, zero16);
        if (decltype(RELOAD)::value) load_bias(rt_next);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          if (issue) out = PKV_MFMA32(qf[ks], kf[tn][ks], out);
          if (decltype(RELOAD)::value) qf[ks] = q_frag(rt_next, ks);  // this row tile's fragments are free: fetch the next tile's
          float x[TPM], ee[TPM];
#pragma unroll
          for (int j = 0; j < TPM; ++j) x[j] = fin[TPM * ks + j] * kap;
#pragma unroll
          for (int j = 0; j < TPM; ++j) ee[j] = fast_exp2(x[j]);
#pragma unroll
          for (int j = 0; j < TPM; ++j) {
            if (j & 1) s1 += ee[j]; else s0 += ee[j];
          }
          PKV_CHUNK_END_SUMS(s0, s1);
          if (ks == KS / 2 - 1) refill(ru, RFT, HALF);
        }
        e[tc] += s0 + s1;
      };
      auto iter = [&](auto TA, auto TB, auto RFT, const Unit& ru, int rt) {
        const int rt_next = (rt + 1 < nrt) ? rt + 1 : 0;
        step(TA, TB, std::true_type{}, std::true_type{}, RFT, I0{}, ru, rt_next, cur, nxt);
        if (rt + 1 < nrt) step(TB, TA, std::false_type{}, std::true_type{}, RFT, I1{}, ru, rt_next, nxt, cur);
        else step(TB, TA, std::false_type{}, std::false_type{}, RFT, I1{}, ru, rt_next, nxt, cur);  // last product of the pass
      };
      auto pass = [&](auto TA, auto TB, auto REFILL, auto F0, auto F1, const Unit& ru) {
        constexpr int ta = decltype(TA)::value, tb = decltype(TB)::value;
        if (has_keys) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) qf[ks] = q_frag(0, ks);
          load_bias(0);
          cur = PKV_MFMA32(bfr, ones, zero16);
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) cur = PKV_MFMA32(qf[ks], kf[ta][ks], cur);
          int rt = 0;
          if constexpr (decltype(REFILL)::value) {
            iter(TA, TB, F0, ru, 0);
            if (nrt > 1) iter(TA, TB, F1, ru, 1);
            else issue_k(ru, F1, I0{}, IKS{});
            rt = 2;
          }
#pragma unroll 1
          for (; rt < nrt; ++rt) iter(TA, TB, INONE{}, ru, rt);
          if (last_rb) {
#pragma unroll
            for (int t = ta; t <= tb; ++t) {
              float tot = e[t];
              tot += __shfl_xor(tot, 32);
              const int key = wkey + 32 * t + l32;
              if (hf == 0 && key < npre) raw[key] = tot * a.inv_G;
            }
          }
        } else if constexpr (decltype(REFILL)::value) {  // a wave without keys in this unit still fetches the next unit's
          issue_k(ru, F0, I0{}, IKS{});
          issue_k(ru, F1, I0{}, IKS{});
        }
      };
      // LSE: the next unit's denominators and Q block travel while this unit is computed: the denominators and one
      // half of the rows during the first pass, the other half during the second.  Each is written to the other
      // LDS buffers (read from the start of the next unit, behind the barrier that ends this one) at a place where
      // the wave waits for nothing younger than what it needs there anyway.
      u32x4 qv[QH];
      float lv[NL];
      const bool prefetch = LSE && last_rb && has_next;
      const bool prefetch_q = prefetch && a.nrb == 1;
      if (prefetch) lse_request(nxt_u, lv);
      if (prefetch_q) q_request(nxt_u, I0{}, qv);
      pass(I0{}, I1{}, std::false_type{}, I2{}, I3{}, cur_u);
      if (prefetch) lse_commit(lv, cfr_nxt);
      if (prefetch_q) q_commit(qv, I0{}, qsmem + (buf ^ 1) * QBUF);
      // The item after the next one is drawn here: every earlier request of the wave has just been waited for and
      // every later one is younger, so that no wait for keys can mistake it for one of them, and the answer is
      // back long before the unit ends.  Two lanes draw, the second one adding nothing to the spare word beside
      // the error word (err + 2 is the first counter word): what a single lane asks for is moved to a scalar
      // register at once, and the wave would wait for the answer on the spot.
      if (LSE && last_rb && tid < 2)
        drawn = __hip_atomic_fetch_add(a.err + 2 - fresh(tid), 1 - fresh(tid), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (prefetch_q) q_request(nxt_u, I1{}, qv);
      // key tiles 0,1 are done: the next unit's are requested into the same registers during the second pass
      // (after the last unit the current ones are fetched once more: harmless, and the code stays branch-free)
      pass(I2{}, I3{}, LAST, I0{}, I1{}, has_next ? nxt_u : cur_u);
      // ... and key tiles 2,3 right after it: they are needed last, half a sweep from now
      if (prefetch_q) q_commit(qv, I1{}, qsmem + (buf ^ 1) * QBUF);
      if constexpr (last_rb) {
        issue_k(has_next ? nxt_u : cur_u, I2{}, I0{}, IKS{});
        issue_k(has_next ? nxt_u : cur_u, I3{}, I0{}, IKS{});
      }
    };
    for (int rb = 0; rb + 1 < a.nrb; ++rb) s2_block(rb, std::false_type{});
    s2_block(a.nrb - 1, std::true_type{});
    if (!LSE && has_next && !q_staged) stage_q(nxt_u, 0, qsmem + (buf ^ 1) * QBUF);
    if (LSE && tid < 2) s_item[tid == 0 ? buf : 3] = 2 * kResidentGrid + drawn;  // (lane 1: the spare word)
    lds_barrier();  // cfr / stat and the Q buffers change hands
    cur_u = nxt_u;
    if constexpr (LSE) {
      // (the word is written again two units from now, behind the next barrier: everyone has read it by then)
      if (has_next) take(s_item[buf], nxt_u);
    }
    buf ^= 1;
  }
}

// Clears n words at p and n2 words at p2 (p2 16-byte aligned, n2 a multiple of 4: four words per thread there).
__global__ void zero_kernel(int32_t* p, int n, int32_t* p2, int n2) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
  else if (4 * (i - n) < n2) reinterpret_cast<int4*>(p2)[i - n] = make_int4(0, 0, 0, 0);
}

}  // namespace

template <int D, bool LSE>
static hipError_t launch_resident(const ResidentArgs& a, hipStream_t s) {
  constexpr int SEG = D / 8;
  const size_t dyn = (size_t)2 * kRowBlock * lds_pitch<SEG>() * sizeof(u32x4);  // two Q buffers
  static bool attr_set[kMaxDevices];
  const int dev = current_device_slot();
  if (dev < 0) return hipErrorInvalidDevice;
  if (!attr_set[dev]) {  // raise the dynamic LDS limit once per device (idempotent; no allocation)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(score_resident_kernel<D, LSE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);
    if (e != hipSuccess) return e;
    attr_set[dev] = true;
  }
  hipLaunchKernelGGL((score_resident_kernel<D, LSE>), dim3(kResidentGrid), dim3(kThreads), dyn, s, a);
  return hipGetLastError();
}

hipError_t launch_score_resident(const ResidentArgs& a, hipStream_t s) {
  // the counters, the error word and the tagged normaliser words must start at zero (with supplied denominators
  // only the error word is looked at, by the selection kernel)
  // (tagged mode: the per-part statistics as well, whose words carry a phase bit)
  const int nz = a.sync_words, nz2 = a.tagged ? a.part_words : 0;  // (part_words: a multiple of 256)
  hipLaunchKernelGGL(zero_kernel, dim3((nz + nz2 / 4 + 255) / 256), dim3(256), 0, s, a.zero_base, nz,
                     reinterpret_cast<int32_t*>(a.part), nz2);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.lse_mode) {
    if (a.d == 128) return launch_resident<128, true>(a, s);
    if (a.d == 64) return launch_resident<64, true>(a, s);
  } else {
    if (a.d == 128) return launch_resident<128, false>(a, s);
    if (a.d == 64) return launch_resident<64, false>(a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace pkv
