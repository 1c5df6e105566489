// Internal declarations shared by the translation units of libpkv (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pkv.h"
#include "pkv_measure.h"

namespace pkv {

// Upper bounds the kernels are written for; the host rejects anything beyond them.
constexpr int kMaxAlpha = 64;
constexpr int kMaxPoolW = 63;
constexpr int kKeysPerTile = 32;     // one MFMA tile of keys
constexpr int kWavesPerBlock = 4;    // score kernels
constexpr int kSelectThreads = 1024; // pool + select kernel

constexpr int kMaxLayers = 1024;     // layers per call

// How a call is split over the device; derived from the shape and the layer count only (never from
// k_l), so that one workspace size serves every budget.
struct Plan {
  int G;         // query heads per KV head
  int R;         // query rows sharing one KV head: G * alpha
  int BH;        // B * Hkv
  int L;
  // register-resident scoring
  bool resident_ok;
  int res_Rpad, res_nrb;  // rows padded to 128-row blocks
  int TPU;       // 512-key parts per unit
  int ngroups;   // independent workgroup groups (512 / group size)
  int UPG;       // units in flight per group
  // per-layer streaming scoring
  int RT;        // 32-row MFMA tiles per row block (1, 2 or 4)
  int RB;        // rows per row block: 32 * RT
  int nrb;       // row blocks: ceil(R / RB)
  int Rpad;      // nrb * RB
  int KC;        // keys per score workgroup (multiple of 128)
  int nchunk;    // ceil(N / KC)
  // workspace carve-up (byte offsets, each 256-aligned)
  size_t off_cnt, off_part, off_cfin, off_raw, off_pooled, total;
  size_t sync_bytes;  // error word + counters + tagged normalisers (zeroed before each resident launch)
};

Plan make_plan(const pkv_layer_desc& d, int L);

struct ScoreArgs {
  const uint16_t* Q;
  const uint16_t* K;
  const int32_t* seq_lens;
  float2* part;  // [BH][Rpad][nchunk] per-chunk softmax statistics (max, sum) in the log2 domain
  float* cfin;   // [BH][Rpad] per-row log2 normaliser: max + log2(sum)
  float* raw;    // [nrb][BH][N] un-pooled scores, one partial per row block
  int32_t B, Hq, Hkv, G, alpha, N, k_l, R, Rpad, nrb, KC, nchunk, RT, d;
  int64_t q_sb, q_sh, q_st, kv_sb, kv_sh, kv_st;
  float kappa;   // log2(e) / sqrt(d)
  const float* lse;  // [B][Hq][alpha] supplied natural-log softmax denominators, or null
};


// ---- register-resident scoring over many layers (pkv_resident.hip) ----
constexpr int kResidentCUs = 256;       // compute units the persistent grid is sized for
constexpr int kResidentGrid = 512;      // persistent workgroups: two per compute unit, one wave per SIMD each
constexpr int kResidentKeys = 512;      // keys held in registers by one workgroup (4 waves x 4 tiles x 32)
constexpr int kResidentMaxRows = 512;   // G * alpha (padded to 128) the LDS normaliser table can hold
constexpr int kResidentMaxLayers = 96;  // per launch (kernel-argument table)

struct ResidentLayer {
  const uint16_t* Q;
  const uint16_t* K;
  const float* lse;  // [B][Hq][alpha] supplied natural-log softmax denominators, or null (two-sweep scoring)
  int32_t k_l;
  int32_t pad;
};

struct ResidentArgs {
  ResidentLayer layer[kResidentMaxLayers];
  const int32_t* seq_lens;
  float* raw;     // [U][N] un-pooled scores
  float2* part;   // [nslots][TPU][Rpad] per-part softmax statistics (log2 domain), reused from unit to unit
  int32_t* cnt;   // [U] arrivals per unit
  int32_t* err;   // in front of cnt: set to 1 if a bounded wait gave up; cleared by the first launch of a call only
  int32_t* zero_base;  // start of the words to zero before the launch (err or cnt)
  unsigned long long* cbuf;  // [nslots][Rpad] (unit tag << 32 | normaliser bits), behind err, 8-byte aligned
  int32_t sync_words;  // 32-bit words to zero from zero_base: (error word,) counters, cbuf
  int32_t L, B, Hq, Hkv, G, alpha, N, R, Rpad, nrb, TPU, U, d;
  int32_t ngroups;  // independent groups of workgroups: 512 / group size
  int32_t UPG;      // units a group works on at the same time: group size / TPU
  int32_t tagged;   // 1: statistics words carry a phase bit, parts fold their own rows (no arrival counter)
  int32_t part_words;  // 32-bit words of the per-part statistics (zeroed before a tagged launch)
  int32_t set1_w;   // share (of 32) of a group pair's units that goes to the group of second workgroups
  int32_t stagger;  // start offset between consecutive groups, in 10 ns ticks
  int32_t lse_mode;    // 1: every layer carries lse; one sweep, no exchange between workgroups
  int32_t wait_ticks;  // wall-clock bound (10 ns ticks) of a wait for other workgroups; beyond it the workgroup
                       // raises the error word and carries on (0: give up at once)
  int64_t q_sb, q_sh, q_st, kv_sb, kv_sh, kv_st;
  float kappa, inv_kappa, inv_G;
};

// ---- pooling + selection and gather over many layers ----
constexpr int kBatchMaxLayers = 32;  // per launch (kernel-argument tables: selection + gather together < 4 KB)

struct SelectLayer {
  float* pooled;       // [BH][N]: scores_out of the layer, else workspace
  int32_t* idx_out;    // [BH][k_cap]
  int32_t* count_out;  // [B]
  int32_t k_l, k_cap;
  int32_t write_pooled;  // the caller asked for scores_out
  int32_t pad;
};

struct SelectBatchArgs {
  SelectLayer layer[kBatchMaxLayers];
  const float* raw;    // [L][nrb][BH][N], first layer of this launch
  const int32_t* seq_lens;
  int32_t B, Hkv, N, alpha, pool, pool_w;
  int32_t nrb;         // partial score arrays to add per layer
  float inv_G;         // factor applied to the sum of the partials
  const int32_t* err;  // error word of the scoring kernel (non-zero: a wait was given up), or null
};

struct GatherLayer {
  const uint16_t* K;
  const uint16_t* V;
  uint16_t* K_out;
  uint16_t* V_out;
  const int32_t* idx;
  const int32_t* table;  // paged output: [B][max_pages] page numbers of this layer, else null
  int32_t* count_out;    // paged output: [B], set to -2 where a page number is out of range
  int64_t o_sb, o_sh, o_st;
  int32_t k_cap, pad;
};

struct GatherBatchArgs {
  GatherLayer layer[kBatchMaxLayers];
  int32_t L, B, Hkv, d, k_cap_max;
  int32_t N;  // rows per head in K and V: positions outside [0, N) are never dereferenced
  int32_t page_size, num_pages, max_pages;  // page_size 0: compact output through the o_* strides
  int64_t kv_sb, kv_sh, kv_st;
};

// 16 bytes (segment seg) of kept row j of (sequence b, KV head g): from the cache into the compact cache or the
// layer's page pool.  An index outside [0, N) is never dereferenced: the compact slot is cleared, a pool slot is
// left alone.  d / 8 neighbouring lanes move one row.
__device__ __forceinline__ void gather_row_segment(const GatherBatchArgs& a, const GatherLayer& ly, int b, int g, int j,
                                                   int seg) {
  const int src = ly.idx[((size_t)b * a.Hkv + g) * ly.k_cap + j];
  if (a.page_size > 0) {
    if ((uint32_t)src >= (uint32_t)a.N) return;  // unused slot: the pool keeps its content
    const int q = j / a.page_size, slot = j - q * a.page_size;
    const int pg = q < a.max_pages ? ly.table[(size_t)b * a.max_pages + q] : -1;
    if ((uint32_t)pg >= (uint32_t)a.num_pages) {  // never written through a bad page number: reported instead
      ly.count_out[b] = -2;
      return;
    }
    const size_t off = (size_t)b * a.kv_sb + (size_t)g * a.kv_sh + (size_t)src * a.kv_st + seg * 8;
    const size_t o = (((size_t)pg * a.Hkv + g) * a.page_size + slot) * a.d + seg * 8;
    *reinterpret_cast<uint4*>(ly.K_out + o) = *reinterpret_cast<const uint4*>(ly.K + off);
    *reinterpret_cast<uint4*>(ly.V_out + o) = *reinterpret_cast<const uint4*>(ly.V + off);
    return;
  }
  uint4 kv = make_uint4(0, 0, 0, 0), vv = kv;
  if ((uint32_t)src < (uint32_t)a.N) {  // -1 marks an unused slot; anything else out of range is not dereferenced either
    const size_t off = (size_t)b * a.kv_sb + (size_t)g * a.kv_sh + (size_t)src * a.kv_st + seg * 8;
    kv = *reinterpret_cast<const uint4*>(ly.K + off);
    vv = *reinterpret_cast<const uint4*>(ly.V + off);
  }
  const size_t o = (size_t)b * ly.o_sb + (size_t)g * ly.o_sh + (size_t)j * ly.o_st + seg * 8;
  *reinterpret_cast<uint4*>(ly.K_out + o) = kv;
  *reinterpret_cast<uint4*>(ly.V_out + o) = vv;
}

// ---- attention recall of the kept set, from the un-pooled scores a compress call left in its workspace ----
struct RecallLayer {
  const int32_t* idx;  // [BH][k_cap] kept positions of the layer
  float* recall;       // [BH]
  int32_t k_l, k_cap;
};

struct RecallArgs {
  RecallLayer layer[kBatchMaxLayers];
  const float* raw;    // [L][nrb][BH][N], first layer of this launch
  const int32_t* seq_lens;
  int32_t B, Hkv, N, alpha, nrb;
  float inv_G;         // factor applied to the sum of the partials
};

// ---- decoding attention over a compacted (possibly paged) cache ----
constexpr int kDecodeMaxRows = 4096;  // kept rows per sequence the LDS probability table can hold
struct DecodeArgs {
  const uint16_t* q;     // [B][Hq][d]
  const uint16_t* K;     // compact [B][Hkv][k_cap][d] (strides c_*) or pool [num_pages][Hkv][page_size][d]
  const uint16_t* V;
  const int32_t* table;  // [B][max_pages], paged only
  const int32_t* count;  // [B]
  float* out;            // [B][Hq][d]
  float* lse;            // [B][Hq] or null
  float* part_o;         // [B][Hkv][S][8][d] un-normalised partial outputs (S > 1)
  float* part_mz;        // [B][Hkv][S][8][2] reference exponent and sum of the partial result
  int32_t B, Hq, Hkv, G, d, k_cap, page_size, num_pages, max_pages;
  int32_t S, chunk;      // key ranges per (sequence, head); keys per range (multiple of 32)
  int64_t c_sb, c_sh, c_st;
  float scale_log2;      // log2(e) / sqrt(d)
};
int decode_splits(int B, int Hkv, int k_cap);
hipError_t launch_decode_attention(const DecodeArgs& a, hipStream_t s);

// The same over the caches of several layers in one launch (per-layer pointers and cache sizes; shape shared).
struct DecodeLayer {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;
  const int32_t* table;
  const int32_t* count;
  float* out;
  float* lse;
  int64_t c_sb, c_sh, c_st;
  int32_t k_cap, num_pages, max_pages;
  int32_t S, chunk;  // key ranges of this layer; keys per range
  int32_t wg0;       // first workgroup of this layer in the launch: layers follow one another, [b][g][range] inside
  int32_t part0;     // first partial-result record of this layer in the workspace ([b][g][range] inside)
  int32_t pad;
};
constexpr int kDecodeMaxLayers = 32;  // per launch (kernel-argument table)
struct DecodeBatchArgs {
  DecodeLayer layer[kDecodeMaxLayers];
  float* part_o;   // [records][8][d]
  float* part_mz;  // [records][8][2]
  int32_t L, B, Hq, Hkv, G, d, page_size;
  float scale_log2;
};
int decode_layers_chunk(int64_t rows_total);
int decode_layers_splits(int k_cap, int chunk_target, int* chunk);
hipError_t launch_decode_attention_layers(const DecodeBatchArgs& a, int total_wgs, int max_chunk, bool any_split,
                                          hipStream_t s);

// Index of the current device for per-device launch state (dynamic LDS limits are set per device), or -1.
constexpr int kMaxDevices = 64;
inline int current_device_slot() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
  return dev;
}

hipError_t launch_score_resident(const ResidentArgs& a, hipStream_t s);
hipError_t launch_recall(const RecallArgs& a, int nlayers, hipStream_t s);
// fuse_gather: the selection workgroup of a unit also copies the unit's kept rows (compact output only)
hipError_t launch_pool_select_batch(const SelectBatchArgs& a, const GatherBatchArgs& ga, bool fuse_gather, int nlayers,
                                    hipStream_t s);
hipError_t launch_gather_batch(const GatherBatchArgs& a, hipStream_t s);
hipError_t launch_probe_read(const void* buf, size_t bytes, uint32_t* sink, hipStream_t s);

// Each returns hipSuccess or the launch error.
hipError_t launch_score_stats(const ScoreArgs& a, hipStream_t s);
hipError_t launch_score_finalize(const ScoreArgs& a, hipStream_t s);
hipError_t launch_score_accum(const ScoreArgs& a, hipStream_t s);

}  // namespace pkv
