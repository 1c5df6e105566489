// Internal declarations shared by the translation units of libpkv (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pkv.h"

namespace pkv {

// Upper bounds the kernels are written for; the host rejects anything beyond them.
constexpr int kMaxAlpha = 64;
constexpr int kMaxPoolW = 63;
constexpr int kKeysPerTile = 32;     // one MFMA tile of keys
constexpr int kWavesPerBlock = 4;    // score kernels
constexpr int kSelectThreads = 1024; // pool + select kernel

// How one layer call is split over the device; derived from the shape only (never from k_l), so
// that one workspace serves every layer of a model.
struct Plan {
  int G;         // query heads per KV head
  int R;         // query rows sharing one KV head: G * alpha
  int RT;        // 32-row MFMA tiles per row block (1, 2 or 4)
  int RB;        // rows per row block: 32 * RT
  int nrb;       // row blocks: ceil(R / RB)
  int Rpad;      // nrb * RB
  int KC;        // keys per score workgroup (multiple of 128)
  int nchunk;    // ceil(N / KC)
  int BH;        // B * Hkv
  // workspace carve-up (byte offsets, each 256-aligned)
  size_t off_part, off_cfin, off_raw, off_pooled, total;
};

Plan make_plan(const pkv_layer_desc& d);

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
};

struct SelectArgs {
  const float* raw;       // [nrb][BH][N]
  float* pooled;          // [BH][N]: scores_out if the caller wants it, else workspace
  const int32_t* seq_lens;
  int32_t* idx_out;       // [BH][k_cap]
  int32_t* count_out;     // [B]
  int32_t B, Hkv, N, alpha, k_l, k_cap, nrb, pool, pool_w;
  float inv_G;
};

struct GatherArgs {
  const uint16_t* K;
  const uint16_t* V;
  uint16_t* K_out;
  uint16_t* V_out;
  const int32_t* idx;     // [BH][k_cap]
  int32_t B, Hkv, k_cap, d;
  int64_t kv_sb, kv_sh, kv_st, o_sb, o_sh, o_st;
};

// Each returns hipSuccess or the launch error.
hipError_t launch_score_stats(const ScoreArgs& a, hipStream_t s);
hipError_t launch_score_finalize(const ScoreArgs& a, hipStream_t s);
hipError_t launch_score_accum(const ScoreArgs& a, hipStream_t s);
hipError_t launch_pool_select(const SelectArgs& a, hipStream_t s);
hipError_t launch_gather(const GatherArgs& a, hipStream_t s);

}  // namespace pkv
