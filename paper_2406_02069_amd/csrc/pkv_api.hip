// Host side of libpkv: budget allocation (Sec. 4.2.1), argument validation, workspace carve-up and
// the launch sequence (Sec. 4.2.2 + gather).  Nothing here touches device memory.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <vector>

#include "pkv_internal.h"

namespace pkv {

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// How a call is split over the device.  Derived from the shape and the layer count only (never from
// k_l), so that one workspace size serves every budget.
Plan make_plan(const pkv_layer_desc& d, int L) {
  Plan p;
  memset(&p, 0, sizeof(p));
  p.G = d.Hq / d.Hkv;
  p.R = p.G * d.alpha;
  p.BH = d.B * d.Hkv;
  p.L = L;
  // --- register-resident path ---
  p.res_Rpad = (p.R + 127) / 128 * 128;
  p.res_nrb = p.res_Rpad / 128;
  p.TPU = (d.N + kResidentKeys - 1) / kResidentKeys;
  // the kernel addresses keys and query rows with 32-bit byte offsets from the head's first element
  const bool offsets_fit = (int64_t)d.N * d.kv_st * 2 < ((int64_t)1 << 31) &&
                           ((int64_t)p.G * d.q_sh + (int64_t)d.alpha * d.q_st) * 2 < ((int64_t)1 << 31);
  p.resident_ok = p.res_Rpad <= kResidentMaxRows && p.TPU <= kResidentGrid && offsets_fit;
  int gs = 64;  // group size: the smallest power of two >= 64 that holds all parts of a unit
  while (gs < p.TPU && gs < kResidentGrid) gs *= 2;
  p.ngroups = kResidentGrid / gs;
  p.UPG = p.resident_ok ? gs / p.TPU : 1;
  // --- per-layer streaming path ---
  p.RT = p.R <= 32 ? 1 : (p.R <= 64 ? 2 : 4);
  p.RB = 32 * p.RT;
  p.nrb = (p.R + p.RB - 1) / p.RB;
  p.Rpad = p.nrb * p.RB;
  const long long keys_total = (long long)p.BH * p.nrb * d.N;
  long long kc = (keys_total / 1024 + 127) / 128 * 128;  // ~4 workgroups per compute unit
  if (kc < 128) kc = 128;
  if (kc > 1024) kc = 1024;
  p.KC = (int)kc;
  p.nchunk = (d.N + p.KC - 1) / p.KC;
  // --- workspace: large enough for either path ---
  const size_t U = (size_t)L * p.BH;
  const size_t nslots = (size_t)p.ngroups * p.UPG;
  const size_t part_res = p.resident_ok ? nslots * p.TPU * p.res_Rpad * sizeof(float2) : 0;
  const size_t part_str = (size_t)p.BH * p.Rpad * p.nchunk * sizeof(float2);
  const size_t raw_res = U * d.N * sizeof(float);
  const size_t raw_str = U * p.nrb * d.N * sizeof(float);
  size_t off = 0;
  p.off_cnt = off;
  // [error word, 8 bytes][U counters][pad to 8 bytes][nslots * Rpad tagged normaliser words]
  p.sync_bytes = 8 + (U * sizeof(int32_t) + 7) / 8 * 8 + nslots * p.res_Rpad * sizeof(uint64_t);
  off += align256(p.sync_bytes);
  p.off_part = off;
  off += align256(part_res > part_str ? part_res : part_str);
  p.off_cfin = off;
  off += align256((size_t)p.BH * p.Rpad * sizeof(float));
  p.off_raw = off;
  off += align256(raw_res > raw_str ? raw_res : raw_str);
  p.off_pooled = off;
  off += align256(U * d.N * sizeof(float));
  p.total = off;
  return p;
}

static int check_desc(const pkv_layer_desc* d) {
  if (!d) return PKV_ERR_INVALID_ARG;
  if (d->B < 1 || d->Hq < 1 || d->Hkv < 1 || d->Hq % d->Hkv != 0 || d->N < 1 || d->d < 1) return PKV_ERR_INVALID_ARG;
  if (d->alpha < 1 || d->k_l < d->alpha) return PKV_ERR_INVALID_ARG;
  if (d->pool != PKV_POOL_NONE && d->pool != PKV_POOL_MAX && d->pool != PKV_POOL_AVG) return PKV_ERR_INVALID_ARG;
  if (d->pool_w < 1 || d->pool_w % 2 == 0 || (d->flags & ~(int32_t)PKV_FLAG_ALL) != 0) return PKV_ERR_INVALID_ARG;
  const int64_t strides[9] = {d->q_sb, d->q_sh, d->q_st, d->kv_sb, d->kv_sh, d->kv_st, d->o_sb, d->o_sh, d->o_st};
  for (int i = 0; i < 9; ++i)
    if (strides[i] < 0 || strides[i] % 8 != 0) return PKV_ERR_INVALID_ARG;  // 16-byte row alignment
  if (d->q_st < d->d || d->kv_st < d->d || d->o_st < d->d) return PKV_ERR_INVALID_ARG;
  if (d->d != 64 && d->d != 128) return PKV_ERR_UNSUPPORTED;
  if (d->alpha > kMaxAlpha || d->pool_w > kMaxPoolW) return PKV_ERR_UNSUPPORTED;
  if ((int64_t)d->B * d->Hkv > 65535 || d->N > (1 << 26) || d->Hq / d->Hkv > 1024) return PKV_ERR_UNSUPPORTED;
  return PKV_OK;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

struct LayerPtrs {
  const void* Q;
  const void* K;
  const void* V;
  void* K_out;
  void* V_out;
  int32_t* idx_out;
  int32_t* count_out;
  float* scores_out;
  const float* lse;  // supplied softmax denominators, or null
  const int32_t* table;  // paged output: the layer's block table (K_out, V_out are then the page pools), or null
};

static int check_ptrs(const LayerPtrs& p) {
  if (!p.Q || !p.K || !p.V || !p.K_out || !p.V_out || !p.idx_out || !p.count_out) return PKV_ERR_INVALID_ARG;
  if (!aligned16(p.Q) || !aligned16(p.K) || !aligned16(p.V) || !aligned16(p.K_out) || !aligned16(p.V_out))
    return PKV_ERR_INVALID_ARG;
  if (((uintptr_t)p.idx_out & 3) || ((uintptr_t)p.count_out & 3) || ((uintptr_t)p.scores_out & 3))
    return PKV_ERR_INVALID_ARG;
  if (((uintptr_t)p.lse & 3) || ((uintptr_t)p.table & 3)) return PKV_ERR_INVALID_ARG;
  return PKV_OK;
}

static int check_workspace(const Plan& plan, const void* ws, size_t bytes) {
  if (!ws || ((uintptr_t)ws & 255) || bytes < plan.total) return PKV_ERR_WORKSPACE;
  return PKV_OK;
}

// Optional event trail for pkv_compress_layers_profiled.
struct Recorder {
  void* const* events;
  int32_t n_events;
  int32_t* kernel_ids;
  int32_t used;
  void begin(hipStream_t s) {
    used = 0;
    (void)hipEventRecord(static_cast<hipEvent_t>(events[used++]), s);
  }
  void after(int id, hipStream_t s) {
    if (used >= n_events) return;
    kernel_ids[used - 1] = id;
    (void)hipEventRecord(static_cast<hipEvent_t>(events[used++]), s);
  }
};

// The register-resident kernel needs one co-resident workgroup on each of 256 compute units.
static bool device_fits_resident() {
  static int cached[64];  // 0 unknown, 1 yes, 2 no
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
  if (cached[dev] == 0) {
    int cus = 0;
    const hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    cached[dev] = (e == hipSuccess && cus >= kResidentCUs) ? 1 : 2;
  }
  return cached[dev] == 1;
}

// Start offset between consecutive workgroup groups of the two-sweep resident kernel, in 10 ns ticks.
constexpr int kResidentStagger = 250;

// Largest per-layer budget up to which the kept rows are copied by the selection kernel itself.
constexpr int kFuseGatherRows = 512;
// ... or number of units (layers x sequences x KV heads) of a launch from which on it does so whatever the budget.
constexpr int kFuseGatherUnits = 1024;

// Share (of 32) of a group pair's units that the group of second workgroups takes.  Measured on the 32k workload:
// with the arrival counter 15 beats equal shares (16) by 1.7 %; with the tagged exchange the second workgroups wait
// less and equal shares are ahead by 0.7 %.
static int resident_set1_weight(bool tagged) { return tagged ? 16 : 15; }

// Wall-clock bound of every wait between workgroups, in 10 ns ticks: 50 ms, several thousand times what a wait
// takes when the grid is resident.
constexpr int kResidentWaitTicks = 5000000;

// lse_mode: with supplied denominators the workgroups of the persistent kernel never wait for each other, so it
// runs on a device of any size.
static bool use_resident(const Plan& plan, bool lse_mode, int32_t flags) {
  if (flags & PKV_FLAG_STREAM_SCORING) return false;
  return plan.resident_ok && (lse_mode || device_fits_resident());
}

// Queue the kernels of L layers.  All arguments have been validated.
static int run_layers(int32_t L, const pkv_layer_desc* descs, const Plan& plan, const LayerPtrs* ptrs,
                      const int32_t* seq_lens, void* workspace, hipStream_t stream, Recorder* rec,
                      const pkv_paged_desc* paged) {
  const pkv_layer_desc& d = descs[0];
  char* ws = static_cast<char*>(workspace);
  float* raw = reinterpret_cast<float*>(ws + plan.off_raw);
  float* pooled_ws = reinterpret_cast<float*>(ws + plan.off_pooled);
  const float kappa = (float)(1.4426950408889634 / sqrt((double)d.d));
  const bool lse_mode = ptrs[0].lse != nullptr;  // all layers or none (checked by the caller)
  const bool resident = use_resident(plan, lse_mode, d.flags);
  bool any_scores = false;
  for (int32_t l = 0; l < L; ++l) any_scores = any_scores || descs[l].k_l < d.N;
  if (rec) rec->begin(stream);

  // ---- scoring: un-pooled group-mean scores of every prefix key -> raw ----
  if (any_scores && resident) {
    for (int32_t l0 = 0; l0 < L; l0 += kResidentMaxLayers) {
      const int32_t nl = L - l0 < kResidentMaxLayers ? L - l0 : kResidentMaxLayers;
      ResidentArgs ra;
      memset(&ra, 0, sizeof(ra));
      for (int32_t i = 0; i < nl; ++i) {
        ra.layer[i].Q = static_cast<const uint16_t*>(ptrs[l0 + i].Q);
        ra.layer[i].K = static_cast<const uint16_t*>(ptrs[l0 + i].K);
        ra.layer[i].lse = ptrs[l0 + i].lse;
        ra.layer[i].k_l = descs[l0 + i].k_l;
      }
      ra.lse_mode = lse_mode ? 1 : 0;
      ra.seq_lens = seq_lens;
      ra.U = nl * plan.BH;
      ra.raw = raw + (size_t)l0 * plan.BH * d.N;
      ra.part = reinterpret_cast<float2*>(ws + plan.off_part);
      // the error word is cleared by the first launch of the call only: a later launch must not hide an earlier give-up
      ra.err = reinterpret_cast<int32_t*>(ws + plan.off_cnt);
      ra.cnt = ra.err + 2;
      const size_t cbuf_off = 8 + ((size_t)ra.U * sizeof(int32_t) + 7) / 8 * 8;
      ra.cbuf = reinterpret_cast<unsigned long long*>(ws + plan.off_cnt + cbuf_off);
      const int32_t all_words = (int32_t)((cbuf_off + (size_t)plan.ngroups * plan.UPG * plan.res_Rpad * sizeof(uint64_t)) / 4);
      ra.zero_base = l0 == 0 ? ra.err : ra.cnt;
      ra.sync_words = l0 == 0 ? all_words : all_words - 2;
      ra.L = nl; ra.B = d.B; ra.Hq = d.Hq; ra.Hkv = d.Hkv; ra.G = plan.G; ra.alpha = d.alpha; ra.N = d.N;
      ra.R = plan.R; ra.Rpad = plan.res_Rpad; ra.nrb = plan.res_nrb; ra.TPU = plan.TPU;
      ra.ngroups = plan.ngroups; ra.UPG = plan.UPG;
      // staggered starts pay when a group has many units to drift apart over (32k workload, 32 units per group:
      // 2.5 % faster than a common start); on a short launch the delay itself weighs more than the drift gains
      // (8k workload, 8 units per group: 5 % slower; tiny workload: 25 %)
      ra.stagger = (lse_mode || ra.U < 16 * plan.ngroups * plan.UPG) ? 0 : kResidentStagger;
      ra.wait_ticks = (d.flags & PKV_FLAG_NO_WAIT) ? 0 : kResidentWaitTicks;
      // the tagged exchange (every part of a group takes part in every unit, also one that lies beyond the end of a
      // shorter sequence) is worth it when a unit has a few parts to spread the rows over (measured at 4, 8, 12, 15
      // and 16 parts per unit: 3 - 5 % faster than the arrival counter or equal; 2 and 3 parts: no difference)
      ra.tagged = (!lse_mode && plan.TPU >= 4 && !(d.flags & PKV_FLAG_COUNTER_EXCHANGE)) ? 1 : 0;
      ra.part_words = (int32_t)((size_t)plan.ngroups * plan.UPG * plan.TPU * plan.res_Rpad * 2);
      ra.set1_w = resident_set1_weight(ra.tagged != 0);
      ra.d = d.d;
      ra.q_sb = d.q_sb; ra.q_sh = d.q_sh; ra.q_st = d.q_st;
      ra.kv_sb = d.kv_sb; ra.kv_sh = d.kv_sh; ra.kv_st = d.kv_st;
      ra.kappa = kappa;
      ra.inv_kappa = 1.0f / kappa;
      ra.inv_G = 1.0f / (float)plan.G;
      if (launch_score_resident(ra, stream) != hipSuccess) return PKV_ERR_HIP;
      if (rec) rec->after(PKV_KERNEL_SCORE_RESIDENT, stream);
    }
  } else if (any_scores) {
    for (int32_t l = 0; l < L; ++l) {
      if (descs[l].k_l >= d.N) continue;
      ScoreArgs sa;
      sa.Q = static_cast<const uint16_t*>(ptrs[l].Q);
      sa.K = static_cast<const uint16_t*>(ptrs[l].K);
      sa.seq_lens = seq_lens;
      sa.part = reinterpret_cast<float2*>(ws + plan.off_part);
      sa.cfin = reinterpret_cast<float*>(ws + plan.off_cfin);
      sa.raw = raw + (size_t)l * plan.nrb * plan.BH * d.N;
      sa.B = d.B; sa.Hq = d.Hq; sa.Hkv = d.Hkv; sa.G = plan.G; sa.alpha = d.alpha; sa.N = d.N;
      sa.k_l = descs[l].k_l;
      sa.R = plan.R; sa.Rpad = plan.Rpad; sa.nrb = plan.nrb; sa.KC = plan.KC; sa.nchunk = plan.nchunk;
      sa.RT = plan.RT; sa.d = d.d;
      sa.q_sb = d.q_sb; sa.q_sh = d.q_sh; sa.q_st = d.q_st;
      sa.kv_sb = d.kv_sb; sa.kv_sh = d.kv_sh; sa.kv_st = d.kv_st;
      sa.kappa = kappa;
      sa.lse = ptrs[l].lse;
      if (!lse_mode) {
        if (launch_score_stats(sa, stream) != hipSuccess) return PKV_ERR_HIP;
        if (rec) rec->after(PKV_KERNEL_SCORE_STATS, stream);
      }
      // (with supplied denominators this only converts them into the per-row normaliser table)
      if (launch_score_finalize(sa, stream) != hipSuccess) return PKV_ERR_HIP;
      if (rec) rec->after(PKV_KERNEL_SCORE_FINALIZE, stream);
      if (launch_score_accum(sa, stream) != hipSuccess) return PKV_ERR_HIP;
      if (rec) rec->after(PKV_KERNEL_SCORE_ACCUM, stream);
    }
  }

  // ---- pooling + per-head top-k, then gather; all layers per launch ----
  for (int32_t l0 = 0; l0 < L; l0 += kBatchMaxLayers) {
    const int32_t nl = L - l0 < kBatchMaxLayers ? L - l0 : kBatchMaxLayers;
    SelectBatchArgs se;
    GatherBatchArgs ga;
    memset(&se, 0, sizeof(se));
    memset(&ga, 0, sizeof(ga));
    int32_t k_cap_max = 0;
    for (int32_t i = 0; i < nl; ++i) {
      const int32_t l = l0 + i;
      const int32_t k_cap = descs[l].k_l < d.N ? descs[l].k_l : d.N;
      k_cap_max = k_cap > k_cap_max ? k_cap : k_cap_max;
      se.layer[i].pooled = ptrs[l].scores_out ? ptrs[l].scores_out : pooled_ws + (size_t)l * plan.BH * d.N;
      se.layer[i].idx_out = ptrs[l].idx_out;
      se.layer[i].count_out = ptrs[l].count_out;
      se.layer[i].k_l = descs[l].k_l;
      se.layer[i].k_cap = k_cap;
      se.layer[i].write_pooled = ptrs[l].scores_out ? 1 : 0;
      ga.layer[i].K = static_cast<const uint16_t*>(ptrs[l].K);
      ga.layer[i].V = static_cast<const uint16_t*>(ptrs[l].V);
      ga.layer[i].K_out = static_cast<uint16_t*>(ptrs[l].K_out);
      ga.layer[i].V_out = static_cast<uint16_t*>(ptrs[l].V_out);
      ga.layer[i].idx = ptrs[l].idx_out;
      ga.layer[i].table = ptrs[l].table;
      ga.layer[i].count_out = ptrs[l].count_out;
      ga.layer[i].o_sb = descs[l].o_sb; ga.layer[i].o_sh = descs[l].o_sh; ga.layer[i].o_st = descs[l].o_st;
      ga.layer[i].k_cap = k_cap;
    }
    const int nrb = resident ? 1 : plan.nrb;
    se.raw = raw + (size_t)l0 * nrb * plan.BH * d.N;
    se.seq_lens = seq_lens;
    se.B = d.B; se.Hkv = d.Hkv; se.N = d.N; se.alpha = d.alpha;
    se.pool = (d.pool_w == 1) ? PKV_POOL_NONE : d.pool;
    se.pool_w = d.pool_w;
    se.nrb = nrb;
    se.inv_G = resident ? 1.0f : 1.0f / (float)plan.G;
    // the error word of this call's scoring launches
    se.err = (any_scores && resident) ? reinterpret_cast<const int32_t*>(ws + plan.off_cnt) : nullptr;
    ga.L = nl; ga.B = d.B; ga.Hkv = d.Hkv; ga.d = d.d; ga.k_cap_max = k_cap_max; ga.N = d.N;
    ga.kv_sb = d.kv_sb; ga.kv_sh = d.kv_sh; ga.kv_st = d.kv_st;
    if (paged) {
      ga.page_size = paged->page_size; ga.num_pages = paged->num_pages; ga.max_pages = paged->max_pages;
    }
    // Few kept rows per head: the selection workgroup of a unit copies them itself (a gather launch of its own costs
    // more than the copy; 8k workload: select + gather 34 -> 26.5 us).  So it does when there are several units per
    // compute unit anyway (ragged batch at average budget 2048: 0.976 -> 0.909 ms).  Many rows of few units (32k
    // workload at average budget 2048: the fused copy would take 0.165 instead of 0.045 + 0.089 ms), or page pools
    // (whose bad-page report must come after the counts are written): the gather kernel, spread over the chip.
    const bool fuse_gather = !paged && (k_cap_max <= kFuseGatherRows || (int64_t)nl * plan.BH >= kFuseGatherUnits);
    if (launch_pool_select_batch(se, ga, fuse_gather, nl, stream) != hipSuccess) return PKV_ERR_HIP;
    if (rec) rec->after(PKV_KERNEL_POOL_SELECT, stream);
    if (!fuse_gather) {
      if (launch_gather_batch(ga, stream) != hipSuccess) return PKV_ERR_HIP;
      if (rec) rec->after(PKV_KERNEL_GATHER, stream);
    }
  }
  return PKV_OK;
}

static int compress_layers_impl(int32_t L, const pkv_layer_desc* descs, const void* const* Q_win,
                                const void* const* K, const void* const* V, const int32_t* seq_lens,
                                void* const* K_out, void* const* V_out, int32_t* const* idx_out,
                                int32_t* const* count_out, float* const* scores_out, void* workspace,
                                size_t workspace_bytes, void* stream, Recorder* rec,
                                const float* const* lse = nullptr, bool want_lse = false,
                                const pkv_paged_desc* paged = nullptr, const int32_t* const* tables = nullptr) {
  if (L < 1 || L > kMaxLayers || !descs || !Q_win || !K || !V || !K_out || !V_out || !idx_out || !count_out)
    return PKV_ERR_INVALID_ARG;
  if (want_lse && !lse) return PKV_ERR_INVALID_ARG;
  if (paged) {
    if (!tables || paged->page_size < 1 || paged->num_pages < 1 || paged->max_pages < 1 || paged->reserved != 0)
      return PKV_ERR_INVALID_ARG;
  }
  if ((uintptr_t)seq_lens & 3) return PKV_ERR_INVALID_ARG;
  LayerPtrs ptrs[kMaxLayers];
  for (int32_t l = 0; l < L; ++l) {
    int rc = check_desc(&descs[l]);
    if (rc != PKV_OK) return rc;
    const pkv_layer_desc &a = descs[0], &b = descs[l];
    if (a.B != b.B || a.Hq != b.Hq || a.Hkv != b.Hkv || a.d != b.d || a.N != b.N || a.alpha != b.alpha ||
        a.pool != b.pool || a.pool_w != b.pool_w || a.flags != b.flags || a.q_sb != b.q_sb || a.q_sh != b.q_sh || a.q_st != b.q_st ||
        a.kv_sb != b.kv_sb || a.kv_sh != b.kv_sh || a.kv_st != b.kv_st)
      return PKV_ERR_INVALID_ARG;
    ptrs[l] = {Q_win[l], K[l], V[l], K_out[l], V_out[l], idx_out[l], count_out[l],
               scores_out ? scores_out[l] : nullptr, want_lse ? lse[l] : nullptr, paged ? tables[l] : nullptr};
    if (want_lse && !ptrs[l].lse) return PKV_ERR_INVALID_ARG;
    if (paged) {  // the block table must reach as far as this layer's budget
      if (!ptrs[l].table) return PKV_ERR_INVALID_ARG;
      const int64_t k_cap = descs[l].k_l < descs[l].N ? descs[l].k_l : descs[l].N;
      if ((k_cap + paged->page_size - 1) / paged->page_size > paged->max_pages) return PKV_ERR_INVALID_ARG;
    }
    rc = check_ptrs(ptrs[l]);
    if (rc != PKV_OK) return rc;
  }
  const Plan plan = make_plan(descs[0], L);
  const int rc = check_workspace(plan, workspace, workspace_bytes);
  if (rc != PKV_OK) return rc;
  if (rec) {
    if (!rec->events || !rec->kernel_ids || rec->n_events < 5 * L + 1) return PKV_ERR_INVALID_ARG;
    for (int32_t i = 0; i < 5 * L + 1; ++i)
      if (!rec->events[i]) return PKV_ERR_INVALID_ARG;
  }
  return run_layers(L, descs, plan, ptrs, seq_lens, workspace, static_cast<hipStream_t>(stream), rec, paged);
}

// Built-in scratch buffer of pkv_compress_layer_noalloc: part of the device image, so every device the library
// runs on holds its own copy at its own address until the process ends.  In host code the array's name is only a
// stand-in for the symbol; the device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[PKV_NOALLOC_SCRATCH_BYTES];

static int noalloc_scratch(void** out) {
  static std::atomic<void*> device_ptr[kMaxDevices];
  const int dev = current_device_slot();
  if (dev < 0) return PKV_ERR_HIP;
  void* p = device_ptr[dev].load(std::memory_order_acquire);
  if (!p) {  // first call on this device (which is current); two racing first calls find the same address
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PKV_ERR_HIP;
    device_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return PKV_OK;
}

}  // namespace pkv

using namespace pkv;

extern "C" {

int pkv_budgets(int32_t L, int32_t avg_budget, int32_t beta, int32_t alpha, int32_t* k_out) {
  if (L < 1 || beta < 1 || alpha < 0 || avg_budget < alpha || !k_out) return PKV_ERR_INVALID_ARG;
  const int64_t A = (int64_t)avg_budget - alpha;  // per-layer budget left after the window
  if (L == 1) {
    k_out[0] = avg_budget;
    return PKV_OK;
  }
  // r_l = A * [(2 beta - 1)(L - 1) - 2 (beta - 1) l] / (beta (L - 1)): from A/beta at the top layer to
  // 2A - A/beta at the bottom one.  Work on the integer numerators over the common denominator.
  const int64_t den = (int64_t)beta * (L - 1);
  int64_t floor_sum = 0;
  for (int32_t l = 0; l < L; ++l) {
    const int64_t num = A * ((2 * (int64_t)beta - 1) * (L - 1) - 2 * ((int64_t)beta - 1) * l);
    k_out[l] = (int32_t)(num / den);
    floor_sum += num / den;
  }
  // The fractional parts sum to an integer `extra` < L.  Give one unit each to the `extra` layers with
  // the largest fraction; among equal fractions the lower layer goes first.
  const int64_t extra = (int64_t)L * A - floor_sum;
  for (int64_t given = 0; given < extra; ++given) {
    int32_t pick = -1;
    int64_t pick_frac = -1;
    for (int32_t l = 0; l < L; ++l) {
      const int64_t num = A * ((2 * (int64_t)beta - 1) * (L - 1) - 2 * ((int64_t)beta - 1) * l);
      if (k_out[l] != (int32_t)(num / den)) continue;  // already bumped
      if (num % den > pick_frac) {
        pick_frac = num % den;
        pick = l;
      }
    }
    k_out[pick] += 1;
  }
  for (int32_t l = 0; l < L; ++l) k_out[l] += alpha;
  return PKV_OK;
}

size_t pkv_workspace_bytes(const pkv_layer_desc* desc, int32_t L) {
  if (L < 1 || L > kMaxLayers || check_desc(desc) != PKV_OK) return 0;
  return make_plan(*desc, L).total;
}

int pkv_compress_layer(const pkv_layer_desc* desc, const void* Q_win, const void* K, const void* V,
                       const int32_t* seq_lens, void* K_out, void* V_out, int32_t* idx_out, int32_t* count_out,
                       float* scores_out, void* workspace, size_t workspace_bytes, void* stream) {
  float* const* so = scores_out ? &scores_out : nullptr;
  return compress_layers_impl(1, desc, &Q_win, &K, &V, seq_lens, &K_out, &V_out, &idx_out, &count_out, so,
                              workspace, workspace_bytes, stream, nullptr);
}

int pkv_compress_layer_noalloc(const pkv_layer_desc* desc, const void* Q_win, const void* K, const void* V,
                               const int32_t* seq_lens, void* K_out, void* V_out, int32_t* idx_out,
                               int32_t* count_out, float* scores_out, void* stream) {
  const int drc = check_desc(desc);
  if (drc != PKV_OK) return drc;
  if (make_plan(*desc, 1).total > PKV_NOALLOC_SCRATCH_BYTES) return PKV_ERR_SCRATCH;
  void* ws = nullptr;
  const int src = noalloc_scratch(&ws);
  if (src != PKV_OK) return src;
  float* const* so = scores_out ? &scores_out : nullptr;
  return compress_layers_impl(1, desc, &Q_win, &K, &V, seq_lens, &K_out, &V_out, &idx_out, &count_out, so, ws,
                              PKV_NOALLOC_SCRATCH_BYTES, stream, nullptr);
}

int pkv_compress_layers(int32_t L, const pkv_layer_desc* descs, const void* const* Q_win, const void* const* K,
                        const void* const* V, const int32_t* seq_lens, void* const* K_out, void* const* V_out,
                        int32_t* const* idx_out, int32_t* const* count_out, float* const* scores_out,
                        void* workspace, size_t workspace_bytes, void* stream) {
  return compress_layers_impl(L, descs, Q_win, K, V, seq_lens, K_out, V_out, idx_out, count_out, scores_out,
                              workspace, workspace_bytes, stream, nullptr);
}

int pkv_compress_layers_lse(int32_t L, const pkv_layer_desc* descs, const void* const* Q_win, const void* const* K,
                            const void* const* V, const float* const* lse, const int32_t* seq_lens,
                            void* const* K_out, void* const* V_out, int32_t* const* idx_out,
                            int32_t* const* count_out, float* const* scores_out, void* workspace,
                            size_t workspace_bytes, void* stream) {
  return compress_layers_impl(L, descs, Q_win, K, V, seq_lens, K_out, V_out, idx_out, count_out, scores_out,
                              workspace, workspace_bytes, stream, nullptr, lse, true);
}

int pkv_compress_layers_paged(int32_t L, const pkv_layer_desc* descs, const void* const* Q_win, const void* const* K,
                              const void* const* V, const float* const* lse, const int32_t* seq_lens,
                              const pkv_paged_desc* paged, void* const* K_pages, void* const* V_pages,
                              const int32_t* const* block_tables, int32_t* const* idx_out,
                              int32_t* const* count_out, float* const* scores_out, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (!paged) return PKV_ERR_INVALID_ARG;
  return compress_layers_impl(L, descs, Q_win, K, V, seq_lens, K_pages, V_pages, idx_out, count_out, scores_out,
                              workspace, workspace_bytes, stream, nullptr, lse, lse != nullptr, paged, block_tables);
}

static int check_decode_desc(const pkv_decode_desc* desc) {
  if (!desc) return PKV_ERR_INVALID_ARG;
  const pkv_decode_desc& d = *desc;
  if (d.B < 1 || d.Hq < 1 || d.Hkv < 1 || d.Hq % d.Hkv != 0 || d.k_cap < 1 || d.reserved != 0) return PKV_ERR_INVALID_ARG;
  if (d.page_size < 0) return PKV_ERR_INVALID_ARG;
  if (d.page_size > 0) {
    if (d.num_pages < 1 || d.max_pages < ((int64_t)d.k_cap + d.page_size - 1) / d.page_size) return PKV_ERR_INVALID_ARG;
  } else {
    const int64_t st[3] = {d.c_sb, d.c_sh, d.c_st};
    for (int i = 0; i < 3; ++i)
      if (st[i] < 0 || st[i] % 8 != 0) return PKV_ERR_INVALID_ARG;
    if (d.c_st < d.d) return PKV_ERR_INVALID_ARG;
  }
  if (d.d != 64 && d.d != 128) return PKV_ERR_UNSUPPORTED;
  if (d.Hq / d.Hkv > 8 || d.k_cap > kDecodeMaxRows || d.B > 65535) return PKV_ERR_UNSUPPORTED;
  return PKV_OK;
}

size_t pkv_decode_workspace_bytes(const pkv_decode_desc* desc) {
  if (check_decode_desc(desc) != PKV_OK) return 0;
  const int S = decode_splits(desc->B, desc->Hkv, desc->k_cap);
  if (S == 1) return 0;
  return (size_t)desc->B * desc->Hkv * S * (8 * (size_t)desc->d + 16) * sizeof(float);
}

int pkv_decode_attention(const pkv_decode_desc* desc, const void* q, const void* K_cache, const void* V_cache,
                         const int32_t* block_table, const int32_t* count, float* out, float* lse_out,
                         void* workspace, size_t workspace_bytes, void* stream) {
  if (!desc || !q || !K_cache || !V_cache || !count || !out) return PKV_ERR_INVALID_ARG;
  const int drc = check_decode_desc(desc);
  if (drc != PKV_OK) return drc;
  const pkv_decode_desc& d = *desc;
  if (!aligned16(q) || !aligned16(K_cache) || !aligned16(V_cache) || ((uintptr_t)count & 3) || ((uintptr_t)out & 3) ||
      ((uintptr_t)lse_out & 3) || ((uintptr_t)block_table & 3))
    return PKV_ERR_INVALID_ARG;
  if (d.page_size > 0 && !block_table) return PKV_ERR_INVALID_ARG;
  const size_t need = pkv_decode_workspace_bytes(desc);
  if (need > 0 && (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need)) return PKV_ERR_WORKSPACE;
  DecodeArgs da;
  memset(&da, 0, sizeof(da));
  da.S = decode_splits(d.B, d.Hkv, d.k_cap);
  da.chunk = ((d.k_cap + da.S - 1) / da.S + 31) / 32 * 32;
  da.part_o = static_cast<float*>(workspace);
  da.part_mz = da.part_o ? da.part_o + (size_t)d.B * d.Hkv * da.S * 8 * d.d : nullptr;
  da.q = static_cast<const uint16_t*>(q);
  da.K = static_cast<const uint16_t*>(K_cache);
  da.V = static_cast<const uint16_t*>(V_cache);
  da.table = block_table;
  da.count = count;
  da.out = out;
  da.lse = lse_out;
  da.B = d.B; da.Hq = d.Hq; da.Hkv = d.Hkv; da.G = d.Hq / d.Hkv; da.d = d.d; da.k_cap = d.k_cap;
  da.page_size = d.page_size; da.num_pages = d.num_pages; da.max_pages = d.max_pages;
  da.c_sb = d.c_sb; da.c_sh = d.c_sh; da.c_st = d.c_st;
  da.scale_log2 = (float)(1.4426950408889634 / sqrt((double)d.d));
  return launch_decode_attention(da, static_cast<hipStream_t>(stream)) == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

// How the layers of a decoding step are cut into key ranges (from the descriptors alone).
namespace {
struct DecodeLayersPlan {
  int chunk_target;
  int64_t records;  // partial-result records of the layers with more than one range
  bool ok;
};
DecodeLayersPlan decode_layers_plan(int32_t L, const pkv_decode_desc* descs) {
  DecodeLayersPlan p = {0, 0, false};
  if (L < 1 || L > kMaxLayers || !descs) return p;
  int64_t rows = 0;
  for (int32_t l = 0; l < L; ++l) {
    if (check_decode_desc(&descs[l]) != PKV_OK) return p;
    const pkv_decode_desc &d = descs[l], &d0 = descs[0];
    if (d.B != d0.B || d.Hq != d0.Hq || d.Hkv != d0.Hkv || d.d != d0.d || d.page_size != d0.page_size) return p;
    rows += (int64_t)d.B * d.Hkv * d.k_cap;
  }
  p.chunk_target = decode_layers_chunk(rows);
  for (int32_t l = 0; l < L; ++l) {
    int chunk;
    const int S = decode_layers_splits(descs[l].k_cap, p.chunk_target, &chunk);
    if (S > 1) p.records += (int64_t)descs[l].B * descs[l].Hkv * S;
  }
  p.ok = true;
  return p;
}
}  // namespace

size_t pkv_decode_layers_workspace_bytes(int32_t L, const pkv_decode_desc* descs) {
  const DecodeLayersPlan p = decode_layers_plan(L, descs);
  if (!p.ok) return 0;
  return (size_t)p.records * (8 * (size_t)descs[0].d + 16) * sizeof(float);
}

int pkv_decode_attention_layers(int32_t L, const pkv_decode_desc* descs, const void* const* q,
                                const void* const* K_cache, const void* const* V_cache,
                                const int32_t* const* block_tables, const int32_t* const* count, float* const* out,
                                float* const* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (L < 1 || L > kMaxLayers || !descs || !q || !K_cache || !V_cache || !count || !out) return PKV_ERR_INVALID_ARG;
  for (int32_t l = 0; l < L; ++l) {
    const int drc = check_decode_desc(&descs[l]);
    if (drc != PKV_OK) return drc;
  }
  const DecodeLayersPlan plan = decode_layers_plan(L, descs);
  if (!plan.ok) return PKV_ERR_INVALID_ARG;  // the layers differ in B, heads, d or page size
  const pkv_decode_desc& d0 = descs[0];
  if (d0.page_size > 0 && !block_tables) return PKV_ERR_INVALID_ARG;
  for (int32_t l = 0; l < L; ++l) {
    if (!q[l] || !K_cache[l] || !V_cache[l] || !count[l] || !out[l]) return PKV_ERR_INVALID_ARG;
    if (!aligned16(q[l]) || !aligned16(K_cache[l]) || !aligned16(V_cache[l]) || ((uintptr_t)count[l] & 3) ||
        ((uintptr_t)out[l] & 3) || (lse_out && ((uintptr_t)lse_out[l] & 3)))
      return PKV_ERR_INVALID_ARG;
    if (d0.page_size > 0 && (!block_tables[l] || ((uintptr_t)block_tables[l] & 3))) return PKV_ERR_INVALID_ARG;
  }
  const size_t need = (size_t)plan.records * (8 * (size_t)d0.d + 16) * sizeof(float);
  if (need > 0 && (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need)) return PKV_ERR_WORKSPACE;
  float* part_o = static_cast<float*>(workspace);
  float* part_mz = part_o ? part_o + (size_t)plan.records * 8 * d0.d : nullptr;
  int64_t part0 = 0;
  for (int32_t l0 = 0; l0 < L; l0 += kDecodeMaxLayers) {
    const int32_t nl = L - l0 < kDecodeMaxLayers ? L - l0 : kDecodeMaxLayers;
    DecodeBatchArgs a;
    memset(&a, 0, sizeof(a));
    a.part_o = part_o;
    a.part_mz = part_mz;
    a.L = nl; a.B = d0.B; a.Hq = d0.Hq; a.Hkv = d0.Hkv; a.G = d0.Hq / d0.Hkv; a.d = d0.d; a.page_size = d0.page_size;
    a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)d0.d));
    int64_t wg = 0;
    int max_chunk = 0;
    bool any_split = false;
    for (int32_t i = 0; i < nl; ++i) {
      const pkv_decode_desc& d = descs[l0 + i];
      DecodeLayer& ly = a.layer[i];
      ly.q = static_cast<const uint16_t*>(q[l0 + i]);
      ly.K = static_cast<const uint16_t*>(K_cache[l0 + i]);
      ly.V = static_cast<const uint16_t*>(V_cache[l0 + i]);
      ly.table = d0.page_size > 0 ? block_tables[l0 + i] : nullptr;
      ly.count = count[l0 + i];
      ly.out = out[l0 + i];
      ly.lse = lse_out ? lse_out[l0 + i] : nullptr;
      ly.c_sb = d.c_sb; ly.c_sh = d.c_sh; ly.c_st = d.c_st;
      ly.k_cap = d.k_cap; ly.num_pages = d.num_pages; ly.max_pages = d.max_pages;
      ly.S = decode_layers_splits(d.k_cap, plan.chunk_target, &ly.chunk);
      ly.wg0 = (int32_t)wg;
      ly.part0 = (int32_t)part0;
      wg += (int64_t)d.B * d.Hkv * ly.S;
      if (ly.S > 1) {
        part0 += (int64_t)d.B * d.Hkv * ly.S;
        any_split = true;
      }
      if (ly.chunk > max_chunk) max_chunk = ly.chunk;
    }
    if (wg > 0x7FFFFFFF || part0 > 0x7FFFFFFF) return PKV_ERR_UNSUPPORTED;
    if (launch_decode_attention_layers(a, (int)wg, max_chunk, any_split, static_cast<hipStream_t>(stream)) != hipSuccess)
      return PKV_ERR_HIP;
  }
  return PKV_OK;
}

int pkv_budgets_schedule(int32_t L, int32_t avg_budget, int32_t beta, int32_t alpha, int32_t schedule,
                         int32_t* k_out) {
  if (schedule == PKV_SCHEDULE_LINEAR) return pkv_budgets(L, avg_budget, beta, alpha, k_out);
  if (L < 1 || L > kMaxLayers || beta < 1 || alpha < 0 || avg_budget < alpha || !k_out) return PKV_ERR_INVALID_ARG;
  if (schedule != PKV_SCHEDULE_GEOMETRIC && schedule != PKV_SCHEDULE_UNIFORM) return PKV_ERR_INVALID_ARG;
  std::fill(k_out, k_out + L, avg_budget);
  if (schedule == PKV_SCHEDULE_UNIFORM || L == 1 || beta == 1) return PKV_OK;
  // Geometric decay over the budget left after the window: r_l = r_0 q^l.  The ratio of top to bottom layer is the
  // linear pyramid's, q^(L-1) = 1/(2 beta - 1), and the layers share L * rest units, so by the closed form of the
  // geometric series r_0 = L * rest * (1 - q) / (1 - q^L).  The values follow from r_0 by repeated multiplication.
  const int64_t rest = (int64_t)avg_budget - alpha;
  const double ln_ratio = -log(2.0 * beta - 1.0);
  const double q = exp(ln_ratio / (L - 1));
  const double qL = exp(ln_ratio * L / (L - 1));
  struct Share { double frac; int32_t layer; };
  std::vector<Share> share(L);
  int64_t missing = (int64_t)L * rest;
  double r = (double)L * (double)rest * (1.0 - q) / (1.0 - qL);
  for (int32_t l = 0; l < L; ++l, r *= q) {
    const double whole = floor(r);
    k_out[l] = alpha + (int32_t)whole;
    missing -= (int64_t)whole;
    share[l] = {r - whole, l};
  }
  // Integer budgets as for the linear schedule: the units the floors leave over go, one each, to the layers with the
  // largest fractional parts (equal parts: the lower layer first).  Rounding of the series can leave the count one
  // off the number of layers at most; the clamp keeps the sum exact in any case.
  std::stable_sort(share.begin(), share.end(), [](const Share& x, const Share& y) { return x.frac > y.frac; });
  for (int64_t i = 0; i < missing; ++i) k_out[share[(size_t)(i % L)].layer] += 1;
  for (int64_t i = 0; i > missing; --i) k_out[share[(size_t)(L - 1 + i % L)].layer] -= 1;
  return PKV_OK;
}

int pkv_attention_recall(int32_t L, const pkv_layer_desc* descs, int32_t lse_supplied, const int32_t* seq_lens,
                         const int32_t* const* idx_out, float* const* recall_out, const void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (L < 1 || L > kMaxLayers || !descs || !idx_out || !recall_out) return PKV_ERR_INVALID_ARG;
  if ((uintptr_t)seq_lens & 3) return PKV_ERR_INVALID_ARG;
  for (int32_t l = 0; l < L; ++l) {
    const int rc = check_desc(&descs[l]);
    if (rc != PKV_OK) return rc;
    const pkv_layer_desc &a = descs[0], &b = descs[l];
    if (a.B != b.B || a.Hq != b.Hq || a.Hkv != b.Hkv || a.d != b.d || a.N != b.N || a.alpha != b.alpha ||
        a.flags != b.flags)
      return PKV_ERR_INVALID_ARG;
    if (!idx_out[l] || !recall_out[l] || ((uintptr_t)idx_out[l] & 3) || ((uintptr_t)recall_out[l] & 3))
      return PKV_ERR_INVALID_ARG;
  }
  const pkv_layer_desc& d = descs[0];
  const Plan plan = make_plan(d, L);
  const int wrc = check_workspace(plan, workspace, workspace_bytes);
  if (wrc != PKV_OK) return wrc;
  // where the compress call left the un-pooled scores: one array per layer (resident path, already divided by the
  // group size) or one partial per row block (streaming path)
  const bool resident = use_resident(plan, lse_supplied != 0, d.flags);
  const int nrb = resident ? 1 : plan.nrb;
  const float* raw = reinterpret_cast<const float*>(static_cast<const char*>(workspace) + plan.off_raw);
  for (int32_t l0 = 0; l0 < L; l0 += kBatchMaxLayers) {
    const int32_t nl = L - l0 < kBatchMaxLayers ? L - l0 : kBatchMaxLayers;
    RecallArgs ra;
    memset(&ra, 0, sizeof(ra));
    for (int32_t i = 0; i < nl; ++i) {
      ra.layer[i].idx = idx_out[l0 + i];
      ra.layer[i].recall = recall_out[l0 + i];
      ra.layer[i].k_l = descs[l0 + i].k_l;
      ra.layer[i].k_cap = descs[l0 + i].k_l < d.N ? descs[l0 + i].k_l : d.N;
    }
    ra.raw = raw + (size_t)l0 * nrb * plan.BH * d.N;
    ra.seq_lens = seq_lens;
    ra.B = d.B; ra.Hkv = d.Hkv; ra.N = d.N; ra.alpha = d.alpha; ra.nrb = nrb;
    ra.inv_G = resident ? 1.0f : 1.0f / (float)plan.G;
    if (launch_recall(ra, nl, static_cast<hipStream_t>(stream)) != hipSuccess) return PKV_ERR_HIP;
  }
  return PKV_OK;
}

int pkv_compress_layers_profiled(int32_t L, const pkv_layer_desc* descs, const void* const* Q_win,
                                 const void* const* K, const void* const* V, const float* const* lse,
                                 const int32_t* seq_lens, const pkv_paged_desc* paged,
                                 const int32_t* const* block_tables,
                                 void* const* K_out, void* const* V_out, int32_t* const* idx_out,
                                 int32_t* const* count_out, float* const* scores_out, void* workspace,
                                 size_t workspace_bytes, void* stream, void* const* events, int32_t n_events,
                                 int32_t* kernel_ids, int32_t* n_used) {
  if (!n_used) return PKV_ERR_INVALID_ARG;
  Recorder rec = {events, n_events, kernel_ids, 0};
  const int rc = compress_layers_impl(L, descs, Q_win, K, V, seq_lens, K_out, V_out, idx_out, count_out,
                                      scores_out, workspace, workspace_bytes, stream, &rec, lse, lse != nullptr,
                                      paged, block_tables);
  *n_used = rec.used;
  return rc;
}

int pkv_probe_read(const void* buf, size_t bytes, uint32_t* sink, void* stream) {
  if (!buf || !sink || bytes == 0 || bytes % 16 != 0 || ((uintptr_t)buf & 15) || ((uintptr_t)sink & 3)) return PKV_ERR_INVALID_ARG;
  return launch_probe_read(buf, bytes, sink, static_cast<hipStream_t>(stream)) == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

const char* pkv_status_string(int status) {
  switch (status) {
    case PKV_OK: return "ok";
    case PKV_ERR_INVALID_ARG: return "invalid argument";
    case PKV_ERR_UNSUPPORTED: return "unsupported shape";
    case PKV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case PKV_ERR_HIP: return "HIP launch failed";
    case PKV_ERR_SCRATCH: return "shape needs more scratch than the built-in buffer holds";
    default: return "unknown status";
  }
}

}  // extern "C"
