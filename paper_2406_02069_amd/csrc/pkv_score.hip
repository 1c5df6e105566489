// Window-attention scoring kernels (Sec. 4.2.2, Eq. Al and Eq. att_score) for gfx950.
//
// For one KV head, the R = G*alpha query rows (G query heads of the group x alpha instruction
// tokens) all multiply the same keys, so they are stacked into one MFMA operand: a 32-key tile of K
// is multiplied with up to 128 query rows at once (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// The softmax normaliser of a query row is known only after every visible key has been seen, and it
// differs per row, so the score  s_i = sum_rows exp(l_ri - c_r)  cannot be formed in one sweep.
// Two sweeps over K are made; logits are never stored:
//   stats    : per row, running (max, sum exp) over a chunk of keys       -> part[row][chunk]
//   finalize : per row, c_r = max + log2(sum) over all chunks             -> cfin[row]
//   accum    : per key, sum over rows of exp2(kappa*q.k - c_r)            -> raw[key]
// Everything is kept in the log2 domain (kappa = log2(e)/sqrt(d)) so that v_exp_f32 applies directly.
//
// Work split: grid = (key chunk, row block, sequence x KV head); a workgroup has 4 waves, each wave
// owns whole 32-key tiles of the chunk and all rows of the row block.  K tiles are read from HBM with
// fully coalesced 16-byte loads (one 256-byte row per 16 lanes), staged through a wave-private,
// XOR-swizzled LDS tile and re-read as MFMA fragments; the next tile's global loads are issued before
// the current tile's matrix work.  Q fragments live in registers for the whole chunk.
#include "pkv_internal.h"

namespace pkv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// 16 bytes as a native vector (HIP's uint4 class keeps such values out of registers when staged in arrays)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ bf16x8 as_frag(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

// Position of 16-byte segment `seg` of tile row `row` inside an LDS tile with SEG segments per row.
// The XOR spreads the 16 rows that one ds_read_b128 phase touches over 16 different bank groups.
template <int SEG>
__device__ __forceinline__ int lds_slot(int row, int seg) {
  const int swz = (SEG == 16) ? (row & 15) : ((row >> 1) & 7);
  return row * SEG + (seg ^ swz);
}

// LDS traffic of one wave to its own tile needs ordering only inside the wave.
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

// PASS 1: statistics.  PASS 2: accumulation of normalised probabilities over the rows.
template <int D, int RT, int PASS>
__global__ __launch_bounds__(256) void score_kernel(const ScoreArgs a) {
  constexpr int KS = D / 16;   // MFMA k-steps per dot product
  constexpr int SEG = D / 8;   // 16-byte segments per row
  constexpr int RB = 32 * RT;  // query rows of this workgroup
  constexpr int NLD = SEG / 2; // global loads per lane per 32-key tile
  constexpr int TILE_U4 = 32 * SEG;
  constexpr int LDS_U4 = (RB * SEG > kWavesPerBlock * TILE_U4) ? RB * SEG : kWavesPerBlock * TILE_U4;
  __shared__ u32x4 lds[LDS_U4];
  __shared__ float2 red[kWavesPerBlock][RB];
  __shared__ float cst[RB];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps addressing in scalar registers
  const int idx32 = lane & 31;
  const int half = lane >> 5;

  const int chunk = blockIdx.x;
  const int rb = blockIdx.y;
  const int bg = blockIdx.z;
  const int b = bg / a.Hkv;
  const int g = bg - b * a.Hkv;

  int n = a.N;
  if (a.seq_lens) {
    n = a.seq_lens[b];
    n = n < 0 ? 0 : (n > a.N ? a.N : n);
  }
  if (a.k_l >= n) return;  // whole sequence kept: nothing to score
  const int npre = n - a.alpha;
  const int chunk_start = chunk * a.KC;
  const int range_end = (PASS == 1) ? n : npre;
  const int row0 = rb * RB;
  float2* part = a.part + ((size_t)bg * a.Rpad + row0) * a.nchunk + chunk;

  if (chunk_start >= range_end) {
    if (PASS == 1) {
      for (int r = tid; r < RB; r += 256) part[(size_t)r * a.nchunk] = make_float2(-INFINITY, 0.f);
    }
    return;
  }
  const int chunk_end = min(chunk_start + a.KC, range_end);
  const int ntiles = (chunk_end - chunk_start + kKeysPerTile - 1) / kKeysPerTile;

  // ---- Q block -> LDS (coalesced) -> per-wave register fragments ----
  for (int e = tid; e < RB * SEG; e += 256) {
    const int row = e / SEG, seg = e - row * SEG;
    const int r = row0 + row;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (r < a.R) {
      const int hh = r / a.alpha, t = r - hh * a.alpha;
      const uint16_t* src = a.Q + (size_t)b * a.q_sb + (size_t)(g * a.G + hh) * a.q_sh + (size_t)t * a.q_st + seg * 8;
      v = *reinterpret_cast<const u32x4*>(src);
    }
    lds[lds_slot<SEG>(row, seg)] = v;
  }
  if (PASS == 2) {
    for (int r = tid; r < RB; r += 256) cst[r] = a.cfin[(size_t)bg * a.Rpad + row0 + r];
  }
  __syncthreads();
  bf16x8 qf[RT][KS];
#pragma unroll
  for (int j = 0; j < RT; ++j)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[j][ks] = as_frag(lds[lds_slot<SEG>(32 * j + idx32, ks * 2 + half)]);

  // Accumulator element v of a lane belongs to tile row mrow(v) (32x32 MFMA output layout).
  auto mrow = [&](int v) { return 8 * (v >> 2) + 4 * half + (v & 3); };

  float cv[PASS == 2 ? RT : 1][16];
  if (PASS == 2) {
#pragma unroll
    for (int j = 0; j < RT; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) cv[j][v] = cst[32 * j + mrow(v)];
  }
  __syncthreads();  // Q block consumed; the same LDS now stages K tiles

  const uint16_t* Kbase = a.K + (size_t)b * a.kv_sb + (size_t)g * a.kv_sh;
  u32x4* tile = lds + wave * TILE_U4;
  const int kmax = n - 1;

  auto load_tile = [&](int tt, u32x4 (&st)[NLD]) {
    const int tile_base = chunk_start + tt * kKeysPerTile;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int e = i * 64 + lane;
      const int row = e / SEG, seg = e - row * SEG;
      const int key = min(tile_base + row, kmax);  // rows at or beyond n are never read
      st[i] = *reinterpret_cast<const u32x4*>(Kbase + (size_t)key * a.kv_st + seg * 8);
    }
  };

  // pass 1 state: per lane, per row tile j: statistics of query row 32j+idx32 over this lane's keys
  float sm[RT], sz[RT];
  int limit[RT];
#pragma unroll
  for (int j = 0; j < RT; ++j) {
    sm[j] = -INFINITY;
    sz[j] = 0.f;
    const int r = row0 + 32 * j + idx32;
    limit[j] = (r < a.R) ? npre + (r % a.alpha) : -1;  // last key visible to this query (causal)
  }

  u32x4 stage[NLD];
  if (wave < ntiles) load_tile(wave, stage);

  for (int tt = wave; tt < ntiles; tt += kWavesPerBlock) {
    const int tile_base = chunk_start + tt * kKeysPerTile;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int e = i * 64 + lane;
      const int row = e / SEG, seg = e - row * SEG;
      tile[lds_slot<SEG>(row, seg)] = stage[i];
    }
    wave_lds_fence();
    if (tt + kWavesPerBlock < ntiles) load_tile(tt + kWavesPerBlock, stage);
    bf16x8 kf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kf[ks] = as_frag(tile[lds_slot<SEG>(idx32, ks * 2 + half)]);
    wave_lds_fence();

    f32x16 acc[RT];
#pragma unroll
    for (int j = 0; j < RT; ++j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (PASS == 1)  // rows of the product = keys, columns = query rows
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[j][ks], acc[j], 0, 0, 0);
        else            // rows = query rows, columns = keys
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[j][ks], kf[ks], acc[j], 0, 0, 0);
      }
    }

    if (PASS == 1) {
      const bool full = tile_base + kKeysPerTile <= npre;  // every key visible to every query row
#pragma unroll
      for (int j = 0; j < RT; ++j) {
        if (!full) {
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (tile_base + mrow(v) > limit[j]) acc[j][v] = -INFINITY;
        }
        float tm = acc[j][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tm = fmaxf(tm, acc[j][v]);
        const float mn = fmaxf(sm[j], tm * a.kappa);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        float sum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += fast_exp2(__builtin_fmaf(acc[j][v], a.kappa, -ms));
        sz[j] = sz[j] * fast_exp2(sm[j] - ms) + sum;
        sm[j] = mn;
      }
    } else {
      float e = 0.f;
#pragma unroll
      for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) e += fast_exp2(__builtin_fmaf(acc[j][v], a.kappa, -cv[j][v]));
      e += __shfl_xor(e, 32);
      const int key = tile_base + idx32;
      if (half == 0 && key < npre) a.raw[((size_t)rb * a.B * a.Hkv + bg) * a.N + key] = e;
    }
  }

  if (PASS == 1) {
    // lanes l and l+32 hold the same query rows over different keys; then merge the 4 waves
#pragma unroll
    for (int j = 0; j < RT; ++j) {
      const float m2 = __shfl_xor(sm[j], 32), z2 = __shfl_xor(sz[j], 32);
      merge_stats(sm[j], sz[j], m2, z2);
      if (half == 0) red[wave][32 * j + idx32] = make_float2(sm[j], sz[j]);
    }
    __syncthreads();
    for (int r = tid; r < RB; r += 256) {
      float m = red[0][r].x, z = red[0][r].y;
#pragma unroll
      for (int w = 1; w < kWavesPerBlock; ++w) merge_stats(m, z, red[w][r].x, red[w][r].y);
      part[(size_t)r * a.nchunk] = make_float2(m, z);
    }
  }
}

// One thread per query row: fold the per-chunk statistics into the row's log2 normaliser.
__global__ __launch_bounds__(256) void finalize_kernel(const ScoreArgs a) {
  const int bg = blockIdx.x;
  const int b = bg / a.Hkv;
  int n = a.N;
  if (a.seq_lens) {
    n = a.seq_lens[b];
    n = n < 0 ? 0 : (n > a.N ? a.N : n);
  }
  if (a.k_l >= n) return;
  for (int r = threadIdx.x; r < a.Rpad; r += blockDim.x) {
    float c = INFINITY;  // padding rows contribute exp2(-inf) = 0
    if (r < a.R && a.lse) {
      // supplied natural-log denominator of row r = head * alpha + t of this group, into the log2 domain
      const int g = bg - b * a.Hkv;
      c = a.lse[((size_t)b * a.Hq + (size_t)g * a.G) * a.alpha + r] * 1.44269504088896340736f;
    } else if (r < a.R) {
      const float2* p = a.part + ((size_t)bg * a.Rpad + r) * a.nchunk;
      float m = -INFINITY, z = 0.f;
      for (int ch = 0; ch < a.nchunk; ++ch) merge_stats(m, z, p[ch].x, p[ch].y);
      c = m + fast_log2(z);
    }
    a.cfin[(size_t)bg * a.Rpad + r] = c;
  }
}

template <int PASS>
hipError_t launch_score(const ScoreArgs& a, hipStream_t s) {
  dim3 grid(a.nchunk, a.nrb, a.B * a.Hkv), block(256);
#define PKV_CASE(DD, RR)                                              \
  if (a.d == DD && a.RT == RR) {                                      \
    hipLaunchKernelGGL((score_kernel<DD, RR, PASS>), grid, block, 0, s, a); \
    return hipGetLastError();                                         \
  }
  PKV_CASE(128, 4) PKV_CASE(128, 2) PKV_CASE(128, 1) PKV_CASE(64, 4) PKV_CASE(64, 2) PKV_CASE(64, 1)
#undef PKV_CASE
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_score_stats(const ScoreArgs& a, hipStream_t s) { return launch_score<1>(a, s); }
hipError_t launch_score_accum(const ScoreArgs& a, hipStream_t s) { return launch_score<2>(a, s); }
hipError_t launch_score_finalize(const ScoreArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(finalize_kernel, dim3(a.B * a.Hkv), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace pkv
