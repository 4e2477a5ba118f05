// Internal definitions shared by the encoder and decoder translation units of
// libcvlc (gfx950).  Nothing here is part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cvlc.h"

namespace cvlc {

// ---- stream format (packet layout of Sec. IV-D, made concrete) ----------------
constexpr uint32_t kMagic = 0x434C5643u;  // "CVLC"
constexpr uint32_t kVersion = 1u;
constexpr uint32_t kGlobalHeaderWords = 8u;  // magic, version|quant, d, R, s, B, client, total_words
constexpr uint32_t kSegHeaderWords = 4u;     // y_r, P_r, min_r, max_r  (H = 128 bits of Eq. (3))
constexpr uint32_t kGlobalHeaderBits = 32u * kGlobalHeaderWords;
constexpr uint32_t kSegHeaderBits = 32u * kSegHeaderWords;

// ---- encoder geometry --------------------------------------------------------
constexpr uint32_t kBlock = 256;           // threads per workgroup (4 wavefronts)
constexpr uint32_t kWave = 64;
constexpr uint32_t kWavesPerBlock = kBlock / kWave;
constexpr uint32_t kSubTile = 1024;        // coordinates one wavefront holds in registers (16 per lane)
constexpr uint32_t kRegion = 8192;         // coordinates one wavefront filters as a unit (8 sub-tiles)
constexpr uint32_t kSpan = 512;            // candidates one wavefront classifies as a unit (8 rows of 64)
constexpr uint32_t kChunkSpans = 8;        // spans per emit chunk (4096 candidates, one workgroup)
constexpr uint32_t kSampleBins = 8192;     // sample histogram on key >> 18 (8 exponent + 5 mantissa bits)
constexpr uint32_t kSampleShift = 18;
constexpr uint32_t kL1Bins = 2048;         // level-1 digit: key >> 20 (8 exponent + 3 mantissa bits)
constexpr uint32_t kDigitBins = 1024;      // level-2 and level-3 digits: 10 bits each
constexpr uint32_t kSlotGroup = 15;        // boundaries refined per level-2/3 launch (60 KB of LDS) for plans of up to 15 groups
constexpr uint32_t kSlotGroupWide = 31;    // ... for plans of more groups: all boundaries at once (124 KB of LDS)
constexpr uint32_t kSamplePieceQuads = 16;    // a piece of the sample: 16 float4 = 64 coordinates = 256 bytes (random 64-byte
                                              // reads run at a fifth of what HBM gives 256-byte ones: 21 against 14 us for the pass)
constexpr uint32_t kSamplePiece = 4u * kSamplePieceQuads;  // coordinates per piece
constexpr uint32_t kSampleChunksMax = 4096;   // pieces in the sample (256 Ki coordinates)
constexpr uint32_t kTieCap = 2048;         // boundary-class members kept per histogram slot for tie resolution
constexpr uint32_t kSampleBlocks = 16;     // workgroups per client in the sample pass
constexpr uint32_t kStatsStride = CVLC_STATS_STRIDE;
constexpr uint32_t kNormLimbs = 20;        // 32-bit limbs of an exact sum of up to 2^31 squares of fp32 values

// Per-client inputs of one encode call, written to the workspace by small
// upload kernels (kernel arguments are the only host->device path that needs
// neither pinned memory nor a synchronisation).
struct ClientParams {
  const float* update;
  uint32_t* stream;
  uint32_t client_id;
  uint32_t R;            // coded groups
  uint32_t k;            // Z_R = P_1 + ... + P_R
  uint32_t total_words;  // stream size
  uint32_t sample_rank;  // rank in the sample that places the candidate threshold (0: keep all)
  float B;
  uint32_t Z[CVLC_MAX_CODED];  // cumulative group boundaries Z_r
  uint8_t y[32];               // code lengths
};
static_assert(sizeof(ClientParams) % 8 == 0, "ClientParams must stay 8-byte granular");

// Per-client scratch state, zero-filled at the start of every encode call.
struct ClientCtl {
  uint32_t tau_lo;           // candidate threshold key from the sample (0: keep every coordinate)
  uint32_t n_cand;           // candidates kept by the filter pass that counts
  uint32_t keep_all;         // 1: the sampled threshold kept fewer than k: every coordinate is a candidate, read from the vector
  uint32_t n_nz;             // regions that kept at least one coordinate
  uint32_t dead;             // 1: more candidates than the workspace has room for; nothing further is done for the client
  uint32_t claim;            // regions of the filter's claimed part taken so far
  uint32_t emit_claim;       // chunks of the packing pass taken beyond every workgroup's first
  double seg_sumsq[32];      // energy of every coded group; entry R: candidates below the last boundary (atomic)
  uint32_t tie_cnt[32];      // kept-aside class members per histogram slot
  uint32_t sel_prefix[2][32];  // key prefix of boundary r after level 1 (11 bits) and level 2 (21 bits); 0xFFFFFFFF: Z_r = 0
  uint32_t sel_rem[2][32];     // rank of the boundary element inside that prefix class, 1-based from the top
  uint32_t tau[32];          // Z_r-th largest key (0xFFFFFFFF: Z_r = 0)
  uint32_t iota[32];         // last of the key == tau_r candidates inside the top Z_r, by its number in the position-ordered list
  uint32_t seg_max_enc[32];  // max over the group of ordered(x); 0 = empty
  uint32_t seg_negmin_enc[32];  // max over the group of ~ordered(x); 0 = empty
  uint32_t hist_sample[kSampleBins];  // sample histogram, accumulated with device-wide atomics
  uint32_t hist_l1[kL1Bins];    // level-1 digit counts of the candidates (device-wide atomics from the filter)
};

// ---- decoder -------------------------------------------------------------------
constexpr uint32_t kDecTile = 4096;  // output coordinates per decode workgroup

struct ListDesc {       // one (client, coded group) record list
  const uint32_t* payload;
  double weight;        // w_i
  uint32_t P, W, s, y;
  float m, step;
};

// ---- device helpers ----------------------------------------------------------------
__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ uint32_t wave_id() { return threadIdx.x / kWave; }

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {  // popcount of mask over lower lanes
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
  const uint32_t lane = lane_id();
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t t = __shfl_up(v, o, 64);
    if (lane >= (uint32_t)o) v += t;
  }
  return v;
}

// Exclusive prefix sum of one value per thread over a workgroup of NW
// wavefronts, in thread order; *total receives the sum.  `scratch` holds NW words.
template <uint32_t NW>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* scratch, uint32_t* total) {
  const uint32_t incl = wave_incl_scan_u32(v);
  const uint32_t wave = threadIdx.x / kWave;
  __syncthreads();
  if (lane_id() == kWave - 1) scratch[wave] = incl;
  __syncthreads();
  uint32_t before = 0, sum = 0;
#pragma unroll
  for (uint32_t w = 0; w < NW; ++w) {
    const uint32_t t = scratch[w];
    if (w < wave) before += t;
    sum += t;
  }
  *total = sum;
  return before + incl - v;
}

// hist[bin] += 1 for every lane with `active`, using one LDS atomic per distinct
// bin in the wavefront (lanes that share a bin elect the lowest one).  Must be
// reached by all lanes of the wavefront.  `bin` must fit in NBITS bits.
template <int NBITS>
__device__ __forceinline__ void wave_hist_add(uint32_t* hist, uint32_t bin, bool active) {
  uint64_t same = __ballot(active);
#pragma unroll
  for (int bit = 0; bit < NBITS; ++bit) {
    const uint64_t set = __ballot((bin >> bit) & 1u);
    same &= ((bin >> bit) & 1u) ? set : ~set;
  }
  if (active && lane_id() == (uint32_t)__builtin_ctzll(same)) atomicAdd(&hist[bin], (uint32_t)__popcll(same));
}

// Loads/stores that other workgroups of the same kernel must observe.
__device__ __forceinline__ uint32_t load_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t load_agent(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent(uint64_t* p, uint64_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Monotone map float -> uint32 (larger float, larger code); never 0 or ~0 for finite input.
__device__ __forceinline__ uint32_t ordered_bits(float x) {
  uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}

__host__ __device__ __forceinline__ uint32_t position_bits(uint32_t d) {
  uint32_t s = 0;
  while (s < 32 && ((uint64_t)1 << s) < (uint64_t)d) ++s;
  return s < 1 ? 1 : s;
}

__host__ __device__ __forceinline__ bool code_len_supported(uint32_t y) {
  return (y >= 1 && y <= 16) || y == 32;
}

__host__ __device__ __forceinline__ uint64_t payload_words(uint32_t P, uint32_t W) {
  return ((uint64_t)P * W + 31u) / 32u;
}

// Spacing of the 2^y uniform centroids on [m, M] and its inverse: one correctly
// rounded fp32 division each; a single-valued (or empty) group has one centroid.
__host__ __device__ __forceinline__ void centroid_spacing(float m, float M, uint32_t y, float* step, float* inv) {
  float range = M - m;
  float top = (float)(((uint64_t)1 << y) - 1u);
  if (range > 0.0f) {
    *step = range / top;
    *inv = top / range;
  } else {
    *step = 0.0f;
    *inv = 0.0f;
  }
}

int hip_check(hipError_t e);  // hipSuccess -> CVLC_OK, else CVLC_ERR_DEVICE

// Brackets a stage of a call with HIP events while profiling is switched on
// (cvlc_profile_start); does nothing otherwise.
void profile_mark(int stage, bool begin, hipStream_t stream);
struct StageScope {
  int stage;
  hipStream_t stream;
  StageScope(int stage_, hipStream_t stream_) : stage(stage_), stream(stream_) { profile_mark(stage, true, stream); }
  ~StageScope() { profile_mark(stage, false, stream); }
};

}  // namespace cvlc
