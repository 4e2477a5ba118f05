// Encoder of libcvlc for gfx950: one client's update vector -> one
// variable-length stream (Sec. IV-B sparsification + quantisation, the final
// loop of Algorithm 1, packet format of Sec. IV-D).
//
// The paper ranks all d updates; here the ranking is never materialised.  The
// kernels find, for every group boundary Z_r, the exact Z_r-th largest
// magnitude (radix-histogram selection) and classify coordinates against those
// thresholds, which yields the same groups as a full sort with ties broken by
// position.  Launch chain per batch of clients (no kernel waits on another
// workgroup and none needs a memory fence; every dependency is a kernel
// boundary):
//   upload        per-client parameters as kernel arguments; clears the
//                 call's control blocks
//   sample_hist   strided sample of |U| -> histogram of the top 13 key bits
//   sample_walk   conservative candidate threshold tau_lo from that histogram
//   filter        the one full pass over U.  Every wavefront owns regions of
//                 8192 consecutive coordinates and writes the coordinates with
//                 key >= tau_lo to the front of the region's slot, in position
//                 order; it also counts the level-1 digit (top 11 key bits) of
//                 what it keeps and sums the squares of what it drops
//   scan_l1       prefix over the region counts, list of the non-empty runs;
//                 level-1 bins of the boundaries (for a client whose sample
//                 misjudged, every coordinate becomes a candidate here)
//   gather_l2     copies the runs into one dense, position-ordered candidate
//                 list, spans of 512 candidates per wavefront, and histograms
//                 level 2 (the next 10 key bits) of the boundaries
//   select_pass3  level 3: LDS histograms of the last 10 key bits of the
//                 candidates that match a boundary's 21-bit prefix
//   select_walk   adds up the histograms, fixes the next digit of every
//                 boundary; after level 3 the exact boundary keys and, where a
//                 boundary cuts a class of equal magnitudes, the position of
//                 its last member inside the boundary
//   count         per span: group of every candidate and its number among the
//                 span's members of that group (left for emit, 16 bits per
//                 candidate), per-group count, min/max/sum of squares; for the
//                 QSGD quantiser also every group's exact sum of squares in
//                 integer limbs
//   layout        prefix of the per-span counts, headers (QSGD: the group norms
//                 from the exact sums), statistics
//   emit          per chunk of 8 spans: record number from prefix and span
//                 number, stochastic rounding (Philox4x32-10) and bit packing;
//                 on request the error energy of every group
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <type_traits>

#include "cvlc_common.h"

namespace cvlc {
namespace {

// ------------------------------------------------------------------ workspace layout
// Per-client, per-group constants of the last stages, written by the layout kernel.
struct GroupInfo {
  uint32_t payload[32];  // first stream word of the group's records
  uint32_t P[32], W[32], y[32];
  float m[32], inv[32];  // smallest value and reciprocal centroid spacing
  float step[32];        // centroid spacing, as the decoder derives it from the header
};

struct EncodeLayout {
  size_t status, ctl, params, region_cnt, region_sumsq, cand_idx, cand_val, dense_idx, dense_val, nz_off, nz_run, span_first, span_cnt, group_info,
      tie_list, sel_part, l3_hist, norm_limbs, total;
  size_t zero_bytes;        // [status, params) is cleared at the start of a call
  uint32_t n_regions, max_spans;
  uint32_t dense_cap;       // candidates the dense list of a client has room for
  uint32_t sel_blocks;      // workgroups per client in a level-2/3 selection pass
};

size_t align256(size_t v) { return (v + 255u) & ~(size_t)255u; }

// Workgroups per client in the filter pass: all of them resident at once
// (`resident` workgroups fit the device), every wavefront the same number of regions.
constexpr uint32_t kFilterBlocksCap = 2048;  // 8 workgroups on each of 256 CUs
uint32_t filter_blocks_per_client(uint32_t n_regions, uint32_t n, uint32_t resident) {
  const uint32_t max_blocks = resident / n > 0 ? resident / n : 1u;
  const uint32_t max_waves = max_blocks * kWavesPerBlock;
  const uint32_t rounds = (n_regions + max_waves - 1) / max_waves;
  const uint32_t waves = (n_regions + rounds - 1) / rounds;
  return (waves + kWavesPerBlock - 1) / kWavesPerBlock;
}

// `cap`: candidates (coordinates at or above the sampled threshold) a client may have; the filter's own
// output is laid out by region and stays d long, everything behind it is as long as the candidates.
EncodeLayout encode_layout(uint32_t d, uint32_t n, uint32_t cap) {
  EncodeLayout L;
  L.n_regions = (uint32_t)(((uint64_t)d + kRegion - 1) / kRegion);
  L.dense_cap = cap < d ? cap : d;
  L.max_spans = (uint32_t)(((uint64_t)L.dense_cap + kSpan - 1) / kSpan);
  {
    uint32_t b = (512u + n - 1) / n;
    L.sel_blocks = b < 2 ? 2u : (b > 32 ? 32u : b);
  }
  size_t off = 0;
  L.status = off; off = align256(off + 256);
  L.ctl = off; off = align256(off + (size_t)n * sizeof(ClientCtl));
  L.l3_hist = off; off = align256(off + (size_t)n * kSlotGroupWide * kDigitBins * sizeof(uint32_t));
  L.norm_limbs = off; off = align256(off + (size_t)n * 32 * kNormLimbs * sizeof(uint64_t));
  L.zero_bytes = off;
  L.params = off; off = align256(off + (size_t)n * sizeof(ClientParams));
  L.region_cnt = off; off = align256(off + (size_t)n * L.n_regions * sizeof(uint32_t));
  L.region_sumsq = off; off = align256(off + (size_t)n * L.n_regions * sizeof(double));
  L.cand_idx = off; off = align256(off + (size_t)n * d * sizeof(uint16_t));
  L.cand_val = off; off = align256(off + (size_t)n * d * sizeof(uint32_t));
  L.dense_idx = off; off = align256(off + (size_t)n * L.dense_cap * sizeof(uint32_t));
  L.dense_val = off; off = align256(off + (size_t)n * L.dense_cap * sizeof(uint32_t));
  L.nz_off = off; off = align256(off + (size_t)n * (L.n_regions + 1) * sizeof(uint32_t));
  L.nz_run = off; off = align256(off + (size_t)n * (L.n_regions + 1) * sizeof(uint32_t));
  L.span_first = off; off = align256(off + (size_t)n * (L.max_spans + 1) * sizeof(uint32_t));
  L.span_cnt = off; off = align256(off + (size_t)n * (L.max_spans + 1) * 32 * sizeof(uint32_t));
  L.group_info = off; off = align256(off + (size_t)n * sizeof(GroupInfo));
  L.tie_list = off; off = align256(off + (size_t)n * kSlotGroupWide * kTieCap * sizeof(uint2));
  L.sel_part = off; off = align256(off + (size_t)n * L.sel_blocks * kSlotGroupWide * kDigitBins * sizeof(uint32_t));
  L.total = off;
  return L;
}

struct Workspace {  // device pointers into the caller's workspace
  uint32_t* status;
  ClientParams* params;
  ClientCtl* ctl;
  uint32_t* region_cnt;
  double* region_sumsq;
  uint16_t* cand_idx;  // positions of the kept coordinates inside their region: a run at the front of every region's slot
  uint32_t* cand_val;  // their value bits, same layout
  uint32_t* dense_idx; // the same candidates, contiguous per client, in position order: positions (read by emit only)
  uint32_t* dense_val;
  uint32_t* nz_off;      // the non-empty runs in position order: number of the run's first candidate ...
  uint32_t* nz_run;      // ... and its region; entry n_nz of nz_off holds the number of candidates
  uint32_t* span_first;  // index (into the non-empty runs) of the run that holds candidate 512 s, per span s
  uint32_t* span_cnt;  // per span of 512 candidates: members of every group, then their exclusive prefix
  GroupInfo* group_info;
  uint2* tie_list;
  uint32_t* sel_part;
  uint32_t* l3_hist;   // level-3 digit counts per (client, slot), zero between uses
  unsigned long long* norm_limbs;  // QSGD: per (client, group) the exact sum of squares in 32-bit limbs
  uint32_t d, n_regions, max_spans, dense_cap, filter_blocks, sel_blocks;
};

// ------------------------------------------------------------------ parameter upload
// The per-client parameter blocks travel as kernel arguments (no pinned memory,
// no synchronisation).  Clients of a batch mostly share a plan, so a chunk holds
// every distinct block once, with pointers and client id left out ("template"),
// and six words per client: update pointer, stream pointer, client id, template.
constexpr uint32_t kUploadWords = 960;
constexpr uint32_t kParamWords = sizeof(ClientParams) / 4u;
constexpr uint32_t kRefWords = 6;
static_assert(sizeof(ClientParams) % 4 == 0 && offsetof(ClientParams, update) == 0 &&
                  offsetof(ClientParams, stream) == 8 && offsetof(ClientParams, client_id) == 16,
              "the upload kernel patches words 0..4 of a parameter block");
struct UploadChunk {
  uint32_t n_clients, first_client, n_templates, pad;
  uint32_t data[kUploadWords];  // n_templates parameter blocks, then n_clients references
};

// Workgroup 0 expands the chunk into the clients' parameter blocks; all
// workgroups clear zero_n16 16-byte pieces from `zero` on (the call's state that
// starts at zero, in the call's first launch; a plain kernel, so that a caller
// may capture the call in a graph).
__global__ __launch_bounds__(256) void upload_kernel(uint32_t* dst, UploadChunk c, uint4* zero, uint32_t zero_n16) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < zero_n16; i += gridDim.x * blockDim.x)
    zero[i] = make_uint4(0u, 0u, 0u, 0u);
  if (blockIdx.x == 0) {
    const uint32_t* refs = c.data + c.n_templates * kParamWords;
    for (uint32_t i = threadIdx.x; i < c.n_clients * kParamWords; i += blockDim.x) {
      const uint32_t client = i / kParamWords, w = i % kParamWords;
      const uint32_t* ref = refs + client * kRefWords;
      const uint32_t v = w < 5 ? ref[w] : c.data[ref[5] * kParamWords + w];
      dst[(size_t)(c.first_client + client) * kParamWords + w] = v;
    }
  }
}

// ------------------------------------------------------------------ small device helpers
// Number of set bits of the four masks in lanes below the caller's.
__device__ __forceinline__ uint32_t lanes_below4(uint64_t m0, uint64_t m1, uint64_t m2, uint64_t m3) {
  uint32_t acc = __builtin_amdgcn_mbcnt_lo((uint32_t)m0, 0u);
  acc = __builtin_amdgcn_mbcnt_hi((uint32_t)(m0 >> 32), acc);
  acc = __builtin_amdgcn_mbcnt_lo((uint32_t)m1, acc);
  acc = __builtin_amdgcn_mbcnt_hi((uint32_t)(m1 >> 32), acc);
  acc = __builtin_amdgcn_mbcnt_lo((uint32_t)m2, acc);
  acc = __builtin_amdgcn_mbcnt_hi((uint32_t)(m2 >> 32), acc);
  acc = __builtin_amdgcn_mbcnt_lo((uint32_t)m3, acc);
  acc = __builtin_amdgcn_mbcnt_hi((uint32_t)(m3 >> 32), acc);
  return acc;
}

// Pointers read from the parameter block are generic; the update vectors live in
// global memory, and saying so lets the loads be issued as global loads.
typedef const float __attribute__((address_space(1))) * GlobalFloatPtr;
typedef float __attribute__((ext_vector_type(4))) Float4V;
typedef const Float4V __attribute__((address_space(1))) * GlobalFloat4Ptr;

constexpr uint32_t kWideBlock = 1024;
constexpr uint32_t kWideWaves = kWideBlock / kWave;

// ------------------------------------------------------------------ 1. sample histogram
// Reads n_s 256-byte pieces spread evenly over the vector and histograms the
// magnitude keys on their top 13 bits.  kSampleBlocks workgroups per client each
// take a slice of the pieces, issue their loads eight deep, and add their
// non-empty bins to the client's histogram.
__global__ __launch_bounds__(kBlock) void sample_hist_kernel(const ClientParams* __restrict__ params,
                                                             ClientCtl* __restrict__ ctls, uint32_t n_s,
                                                             uint64_t piece_step) {
  __shared__ uint32_t hist[kSampleBins];
  const uint32_t client = blockIdx.y;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  if (p.sample_rank == 0) return;  // keep-all plan: the threshold stays 0
  for (uint32_t i = threadIdx.x; i < kSampleBins; i += kBlock) hist[i] = 0;
  __syncthreads();
  GlobalFloat4Ptr src = (GlobalFloat4Ptr)p.update;
  const uint32_t total_q = n_s * kSamplePieceQuads;
  const uint32_t per_block = (total_q + gridDim.x - 1) / gridDim.x;
  const uint32_t q_begin = blockIdx.x * per_block;
  const uint32_t q_end = min(total_q, q_begin + per_block);
  for (uint32_t base = q_begin; base < q_end; base += kBlock * 8u) {
    Float4V v[8];
    bool live[8];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) {
      const uint32_t q = base + u * kBlock + threadIdx.x;
      live[u] = q < q_end;
      v[u] = Float4V{0.0f, 0.0f, 0.0f, 0.0f};
      if (live[u]) {
        const uint32_t j = q / kSamplePieceQuads, part = q % kSamplePieceQuads;
        const uint64_t piece = ((uint64_t)j * piece_step) >> 32;  // piece_step = 2^32 * pieces / n_s, rounded down
        v[u] = src[piece * kSamplePieceQuads + part];
      }
    }
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) {
      if (live[u]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) atomicAdd(&hist[(__float_as_uint(v[u][c]) & 0x7FFFFFFFu) >> kSampleShift], 1u);
      }
    }
  }
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < kSampleBins; i += kBlock) {
    const uint32_t h = hist[i];
    if (h) atomicAdd(&ctl->hist_sample[i], h);
  }
}

// One workgroup per client walks the sample histogram from the large keys down
// to the sample rank the host derived from k/d plus a 6-sigma margin.  The
// lower edge of that bin becomes the candidate threshold.
__global__ __launch_bounds__(kWideBlock) void sample_walk_kernel(const ClientParams* __restrict__ params,
                                                                 ClientCtl* __restrict__ ctls) {
  __shared__ uint32_t scan_tmp[kWideWaves];
  const uint32_t client = blockIdx.x;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  if (p.sample_rank == 0) return;
  // thread t owns `per` bins ending at top = kSampleBins - 1 - per * t, largest keys first
  constexpr uint32_t per = kSampleBins / kWideBlock;
  const uint32_t top = kSampleBins - 1 - per * threadIdx.x;
  uint32_t h[per], mine = 0;
#pragma unroll
  for (uint32_t i = 0; i < per; ++i) {
    h[i] = ctl->hist_sample[top - i];
    mine += h[i];
  }
  uint32_t total;
  const uint32_t above = block_excl_scan<kWideWaves>(mine, scan_tmp, &total);
  const uint32_t target = p.sample_rank;
  if (above < target && target <= above + mine) {
    uint32_t acc = above, bin = top;
#pragma unroll
    for (uint32_t i = 0; i < per; ++i) {
      acc += h[i];
      if (acc >= target) { bin = top - i; break; }
    }
    ctl->tau_lo = bin << kSampleShift;
  }
  // target beyond the sample: tau_lo keeps its cleared value 0 (everything is a candidate)
}

// ------------------------------------------------------------------ 2. filter (the full pass)
// A wavefront streams a region in sub-tiles of 1024 coordinates, read as four
// float4 per lane (the j-th at j*256 + lane*4), so position order inside a
// sub-tile is (j, lane, component).  The next sub-tile's loads are issued
// before the current one is processed.
struct SubTile {
  float v[4][4];
};

__device__ __forceinline__ void load_subtile(SubTile& t, GlobalFloatPtr U, uint32_t sbase, uint32_t lane, uint32_t d) {
  if (sbase + kSubTile <= d) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // read once, never again: keep the stream out of the way of what the caches hold
      const Float4V q = __builtin_nontemporal_load(reinterpret_cast<GlobalFloat4Ptr>(U + sbase + j * 256u + lane * 4u));
      t.v[j][0] = q.x; t.v[j][1] = q.y; t.v[j][2] = q.z; t.v[j][3] = q.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t e0 = sbase + j * 256u + lane * 4u;
#pragma unroll
      for (int c = 0; c < 4; ++c) t.v[j][c] = (e0 + c < d) ? U[e0 + c] : 0.0f;
    }
  }
}

// Kept coordinates are staged per wavefront in LDS and leave in rows of 64 (one
// coalesced 512-byte store each); a row also feeds the level-1 histogram.  Loads
// and stores share one outstanding-operation counter on this hardware, so a
// wavefront that has just stored must wait for the store's acknowledgement
// before it can consume its next loads: rows are therefore held back until the
// stage could not take another four float4 per lane, or the region ends.
constexpr uint32_t kStageCap = 448;
constexpr uint32_t kStageFlushAt = kStageCap - 256;  // more staged than this: flush

static_assert(kRegion <= 65536 && (kRegion & (kRegion - 1)) == 0, "positions inside a region are kept in 16 bits");

struct FilterWave {
  uint2* stage;            // this wavefront's staging rows in LDS
  uint16_t* __restrict__ out_idx;  // the region's slot in global memory: positions inside the region (13 bits)
  uint32_t* __restrict__ out_val;  // ... and value bits
  uint32_t* hist;          // the workgroup's level-1 histogram in LDS
  uint32_t fill;           // staged entries (uniform)
  uint32_t run;            // entries already written to `out` (uniform)
  uint32_t nonfinite;      // a kept key was Inf or NaN (per lane)
};

// LDS accesses of one wavefront complete in order; this keeps the compiler from
// moving them across the point where lanes read what other lanes wrote.
__device__ __forceinline__ void wave_lds_fence() { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); }

__device__ __forceinline__ void flush_rows(FilterWave& w, uint32_t lane, bool all) {
  wave_lds_fence();
  uint32_t g = 0;
  for (; g + kWave <= w.fill; g += kWave) {
    const uint2 e = w.stage[g + lane];
    w.out_idx[w.run + g + lane] = (uint16_t)(e.x & (kRegion - 1u));
    w.out_val[w.run + g + lane] = e.y;
    atomicAdd(&w.hist[(e.y & 0x7FFFFFFFu) >> 20], 1u);
    w.nonfinite |= (e.y & 0x7FFFFFFFu) >= 0x7F800000u ? 1u : 0u;
  }
  const uint32_t left = w.fill - g;  // < 64
  if (left) {
    uint2 e = make_uint2(0u, 0u);
    if (lane < left) e = w.stage[g + lane];
    if (all) {
      if (lane < left) {
        w.out_idx[w.run + g + lane] = (uint16_t)(e.x & (kRegion - 1u));
        w.out_val[w.run + g + lane] = e.y;
        atomicAdd(&w.hist[(e.y & 0x7FFFFFFFu) >> 20], 1u);
        w.nonfinite |= (e.y & 0x7FFFFFFFu) >= 0x7F800000u ? 1u : 0u;
      }
      g += left;
    } else if (g) {  // move the partial row to the front
      wave_lds_fence();
      if (lane < left) w.stage[lane] = e;
    }
  }
  w.run += g;
  w.fill -= g;
  wave_lds_fence();
}

// Stages the coordinates of one sub-tile whose key reaches tau_lo, in position
// order.  The squares of the others go to *sq.  Inf and NaN have the largest
// keys, so they are always among the kept ones, where flush_rows sees them.
template <bool TAIL>
__device__ __forceinline__ void filter_subtile(const SubTile& t, uint32_t sbase, uint32_t lane, uint32_t d,
                                               uint32_t tau_lo, FilterWave& w, double* sq) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t e0 = sbase + j * 256u + lane * 4u;
    uint32_t bits[4];
    bool keep[4];
    uint64_t m[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      bits[c] = __float_as_uint(t.v[j][c]);
      const uint32_t key = bits[c] & 0x7FFFFFFFu;
      keep[c] = key >= tau_lo && (!TAIL || e0 + c < d);
      m[c] = __ballot(keep[c]);
      const double dropped = (double)(keep[c] ? 0.0f : t.v[j][c]);  // coordinates past d were loaded as 0
      *sq = fma(dropped, dropped, *sq);
    }
    if (m[0] | m[1] | m[2] | m[3]) {
      uint32_t pos = w.fill + lanes_below4(m[0], m[1], m[2], m[3]);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (keep[c]) {
          w.stage[pos] = make_uint2(e0 + c, bits[c]);
          ++pos;
        }
      }
      w.fill += (uint32_t)(__popcll(m[0]) + __popcll(m[1]) + __popcll(m[2]) + __popcll(m[3]));
      if (w.fill > kStageFlushAt) flush_rows(w, lane, false);
    }
  }
}

__global__ __launch_bounds__(kBlock) void filter_kernel(const ClientParams* __restrict__ params,
                                                        ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ uint32_t s_hist[kL1Bins];
  __shared__ uint2 s_stage[kWavesPerBlock][kStageCap];
  // workgroups start in the order of their number, and the older ones get ahead: every client gets its share of both
  const uint32_t lin = blockIdx.y * gridDim.x + blockIdx.x;
  const uint32_t client = lin % gridDim.y, block_x = lin / gridDim.y;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  const uint32_t tau_lo = ctl->tau_lo;
  const uint32_t d = ws.d, n_regions = ws.n_regions;
  GlobalFloatPtr U = (GlobalFloatPtr)p.update;
  const uint32_t lane = lane_id();
  for (uint32_t i = threadIdx.x; i < kL1Bins; i += kBlock) s_hist[i] = 0;
  __syncthreads();

  double sq = 0.0;
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  FilterWave w;
  w.stage = s_stage[wave_id()];
  w.hist = s_hist;
  w.nonfinite = 0;
  // Software pipeline over all sub-tiles of all of this wavefront's regions: the
  // loads of the next sub-tile (of the next region, at a region's end) are issued
  // before the current one is processed, so the rare row stores sit behind loads
  // that are already in flight.
  const uint32_t wave_global = block_x * kWavesPerBlock + wave_id();
  // Which regions a wavefront takes.  The first half of the rounds is dealt out (region = wavefront + round x
  // wavefronts: all wavefronts read one moving window); the rest is claimed from a counter of the client's, one
  // region at a time and one region ahead, so that the wavefronts that get ahead (the memory system serves
  // the oldest first) take over from those that fall behind and all end together: 285 -> 273 us.  (Claiming
  // every region: 278 us; a quarter of them: 276 us.)
  const uint32_t rounds = n_regions / n_waves;
  const uint32_t n_static = rounds >= 4u ? (rounds - rounds / 2u) * n_waves : n_regions;
  auto claim = [&]() {  // the next region nobody has taken yet (a per-lane value, lane 0's counts; not waited for here)
    uint32_t got = 0;
    if (lane == 0) got = atomicAdd(&ctl->claim, 1u);
    return got;
  };
  uint32_t region = wave_global;
  if (region >= n_static) region = n_static < n_regions ? n_static + (uint32_t)__builtin_amdgcn_readfirstlane(claim()) : n_regions;
  if (region < n_regions) {
    SubTile cur, nxt;
    bool upcoming_static = false;
    uint32_t claimed = 0;
    uint32_t sbase = region * kRegion;
    load_subtile(cur, U, sbase, lane, d);
    while (true) {
      const uint32_t rbase = region * kRegion;
      const uint32_t rend = (d - rbase < kRegion) ? d : rbase + kRegion;
      if (sbase == rbase) {
        w.out_idx = ws.cand_idx + (size_t)client * d + rbase;
        w.out_val = ws.cand_val + (size_t)client * d + rbase;
        w.fill = 0;
        w.run = 0;
        // the region after this one: the next of the wavefront's own, or one that is claimed now and known by the time this one ends
        upcoming_static = region < n_static && region + n_waves < n_static;
        if (!upcoming_static && n_static < n_regions) claimed = claim();
      }
      // where the pipeline goes next
      const bool last_of_region = sbase + kSubTile >= rend;
      uint32_t next_region = region;
      if (last_of_region)
        next_region = upcoming_static ? region + n_waves
                                      : (n_static < n_regions ? n_static + (uint32_t)__builtin_amdgcn_readfirstlane(claimed) : n_regions);
      const uint32_t next_sbase = last_of_region ? next_region * kRegion : sbase + kSubTile;
      const bool more = next_region < n_regions;
      if (more) load_subtile(nxt, U, next_sbase, lane, d);
      if (sbase + kSubTile <= d) {
        filter_subtile<false>(cur, sbase, lane, d, tau_lo, w, &sq);
      } else {
        filter_subtile<true>(cur, sbase, lane, d, tau_lo, w, &sq);
      }
      if (last_of_region) {
        flush_rows(w, lane, true);
        const double total = wave_sum_f64(sq);
        sq = 0.0;
        if (lane == 0) {
          ws.region_cnt[(size_t)client * n_regions + region] = w.run;
          ws.region_sumsq[(size_t)client * n_regions + region] = total;
        }
      }
      if (!more) break;
      cur = nxt;
      region = next_region;
      sbase = next_sbase;
    }
  }
  // a threshold in the Inf/NaN range can only come from a sample that held such values
  if (w.nonfinite || tau_lo > 0x7F800000u) atomicOr(ws.status, CVLC_DEV_NONFINITE);
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < kL1Bins; i += kBlock) {
    const uint32_t h = s_hist[i];
    if (h) atomicAdd(&ctl->hist_l1[i], h);
  }
}

// ------------------------------------------------------------------ 3. region prefix + selection level 1
// One workgroup per client.  Turns the region counts into exclusive offsets
// and lists the non-empty runs with the number of their first candidate (the
// candidates' position-ordered numbering; the gather works in spans of 512
// candidates, and the run holding every span's first candidate is noted), then reads the level-1
// histogram the filter's workgroups accumulated and locates, for every boundary
// Z_r, the bin holding the Z_r-th largest key and the rank left inside it.
// Should the sampled threshold have kept fewer than k coordinates (the sample
// misjudged: six standard deviations, or a vector built against the sampling
// pattern), every coordinate becomes a candidate: the runs are then the regions
// themselves, read from the vector, and this workgroup counts the level-1
// digits of the whole vector on its own: slow, and next to never needed.
__global__ __launch_bounds__(kWideBlock) void scan_l1_kernel(const ClientParams* __restrict__ params,
                                                             ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ uint32_t hist[kL1Bins];
  __shared__ uint32_t incl[kL1Bins];  // keys in bins >= b
  __shared__ uint32_t scan_tmp[kWideWaves];
  const uint32_t client = blockIdx.x, tid = threadIdx.x;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  const uint32_t n_regions = ws.n_regions;
  const uint32_t* cnt = ws.region_cnt + (size_t)client * n_regions;
  uint32_t* nz_off = ws.nz_off + (size_t)client * (n_regions + 1);
  uint32_t* nz_run = ws.nz_run + (size_t)client * (n_regions + 1);
  uint32_t* span_first = ws.span_first + (size_t)client * (ws.max_spans + 1);
  // one workgroup per client, all latency: the first two rounds' counts and the level-1 histogram are
  // requested before anything is waited for
  const uint32_t ahead0 = tid < n_regions ? cnt[tid] : 0u;
  const uint32_t ahead1 = tid + kWideBlock < n_regions ? cnt[tid + kWideBlock] : 0u;
  const uint32_t l1_even = ctl->hist_l1[2u * tid], l1_odd = ctl->hist_l1[2u * tid + 1];
  uint32_t run = 0, n_nz = 0;
  for (uint32_t base = 0; base < n_regions; base += kWideBlock) {
    const uint32_t j = base + tid;
    const uint32_t v = base == 0 ? ahead0 : (base == kWideBlock ? ahead1 : (j < n_regions ? cnt[j] : 0u));
    uint32_t tot, tot_nz;
    const uint32_t excl = block_excl_scan<kWideWaves>(v, scan_tmp, &tot);
    const uint32_t q = n_nz + block_excl_scan<kWideWaves>(v ? 1u : 0u, scan_tmp, &tot_nz);
    if (j < n_regions) {
      if (v) {
        const uint32_t begin = run + excl, end = begin + v;
        nz_off[q] = begin;
        nz_run[q] = j;
        // spans whose first candidate lies in this run (those the workspace has room for; more: see below)
        for (uint32_t sp = (begin + kSpan - 1) / kSpan; (uint64_t)sp * kSpan < end && sp <= ws.max_spans; ++sp)
          span_first[sp] = q;
      }
    }
    run += tot;
    n_nz += tot_nz;
  }
  const bool keep_all = run < p.k;  // uniform
  if (run > ws.dense_cap || (keep_all && ws.d > ws.dense_cap)) {  // the caller's workspace is too short for this vector: no stream, and say so
    if (tid == 0) {
      nz_off[0] = 0;
      ctl->n_cand = 0;
      ctl->n_nz = 0;
      ctl->dead = 1u;
      p.stream[0] = 0u;  // not a stream header
      atomicOr(ws.status, CVLC_DEV_WORKSPACE);
    }
    return;
  }
  if (!keep_all) {
    if (tid == 0) {
      nz_off[n_nz] = run;
      ctl->n_cand = run;
      ctl->n_nz = n_nz;
    }
    hist[2u * tid] = l1_even;
    hist[2u * tid + 1] = l1_odd;
  } else {
    const uint32_t d = ws.d;
    __syncthreads();  // the runs written above are overwritten
    double* rsq = ws.region_sumsq + (size_t)client * n_regions;
    for (uint32_t j = tid; j < n_regions; j += kWideBlock) {
      nz_off[j] = j * kRegion;
      nz_run[j] = j;
      rsq[j] = 0.0;  // nothing is dropped before the selection
    }
    for (uint32_t sp = tid; (uint64_t)sp * kSpan < d; sp += kWideBlock) span_first[sp] = sp / (kRegion / kSpan);
    if (tid == 0) {
      nz_off[n_regions] = d;
      ctl->n_cand = d;
      ctl->n_nz = n_regions;
      ctl->keep_all = 1u;
    }
    hist[2u * tid] = 0;
    hist[2u * tid + 1] = 0;
    __syncthreads();
    const uint32_t* __restrict__ bits = reinterpret_cast<const uint32_t*>(p.update);
    bool nonfinite = false;
    for (uint32_t base = 0; base < d; base += kWideBlock * 8u) {
      uint32_t v[8];
#pragma unroll
      for (uint32_t u = 0; u < 8; ++u) v[u] = bits[min(base + u * kWideBlock + tid, d - 1u)];
#pragma unroll
      for (uint32_t u = 0; u < 8; ++u) {
        if (base + u * kWideBlock + tid < d) {
          const uint32_t key = v[u] & 0x7FFFFFFFu;
          nonfinite |= key >= 0x7F800000u;
          atomicAdd(&hist[key >> 20], 1u);
        }
      }
    }
    if (nonfinite) atomicOr(ws.status, CVLC_DEV_NONFINITE);
  }
  __syncthreads();
  const uint32_t top = kL1Bins - 1 - 2u * tid;
  const uint32_t h0 = hist[top], h1 = hist[top - 1];
  uint32_t total;
  const uint32_t above = block_excl_scan<kWideWaves>(h0 + h1, scan_tmp, &total);
  incl[top] = above + h0;
  incl[top - 1] = above + h0 + h1;
  __syncthreads();
  if (tid < 32) {
    uint32_t pre = 0xFFFFFFFFu, rem = 0;
    if (tid < p.R) {
      const uint32_t Z = p.Z[tid];
      if (Z > total) atomicOr(ws.status, CVLC_DEV_INTERNAL);  // cannot happen once the filter kept >= k
      if (Z != 0 && Z <= total) {
        uint32_t lo = 0, hi = kL1Bins - 1;  // largest bin b with incl[b] >= Z
        while (lo < hi) {
          const uint32_t mid = (lo + hi + 1) >> 1;
          if (incl[mid] >= Z) lo = mid; else hi = mid - 1;
        }
        pre = lo;
        rem = Z - (incl[lo] - hist[lo]);
      }
    }
    ctl->sel_prefix[0][tid] = pre;
    ctl->sel_rem[0][tid] = rem;
    ctl->tau[tid] = 0xFFFFFFFFu;  // boundaries with Z_r = 0 keep "nothing inside"
    ctl->iota[tid] = 0u;
  }
}

// ------------------------------------------------------------------ 4. selection, levels 2 and 3
// LEVEL 2 refines bits 19..10, LEVEL 3 bits 9..0 of the boundary keys.  The
// kernels come in two sizes SG: room for 15 boundaries (plans of up to 15
// groups: 60 KB of counters, two workgroups to a CU) or for all 31 (124 KB, one
// workgroup to a CU).  Boundaries that share a prefix share a histogram
// ("slot").  The pass (level 2: the gather) histograms, in LDS, the next digit
// of every candidate whose key starts with a slot's prefix; level 2 stores one
// partial histogram per workgroup, level 3 adds its few counts to one table per
// client; the walk kernel (one workgroup per slot and client) adds them up and
// reads off every boundary's digit.
// During level 3 the few candidates matching a boundary's 21-bit prefix are
// also kept aside, so that a boundary cutting through a class of equal keys
// can find the position of the last member inside it (ties rank by position).
constexpr uint32_t kNoSlot = 0xFFFFFFFFu;

template <uint32_t SG>
struct SlotTable {
  uint32_t prefix[SG];  // slot -> key prefix (11 bits at level 2, 21 bits at level 3)
  uint32_t leader[SG];  // boundary inside the group -> its slot, kNoSlot for Z_r = 0
  uint32_t n;
};

// Lane of the first of the lanes 0..SG-1 that are `valid` and hold the
// caller's value (the caller's own lane if none is earlier).  Whole wavefront;
// the result means something for valid lanes below SG only.
template <uint32_t SG>
__device__ __forceinline__ uint32_t first_equal_lane(uint32_t value, bool valid) {
  const uint64_t vmask = __ballot(valid);
  const uint32_t lane = lane_id();
  uint32_t first = lane;
#pragma unroll
  for (int j = (int)SG - 1; j >= 0; --j) {
    const uint32_t vj = __builtin_amdgcn_readlane(value, j);
    if (((vmask >> j) & 1u) && (uint32_t)j < lane && vj == value) first = (uint32_t)j;
  }
  return first;
}

// Slots in order of first appearance among the group's boundaries.  Run by one
// whole wavefront whose lane b < nb holds boundary b's prefix.  Returns the
// caller's slot (kNoSlot: Z_r = 0 or no boundary) and whether it opens it.
template <uint32_t SG>
__device__ __forceinline__ uint32_t build_slots(SlotTable<SG>& st, uint32_t pre, uint32_t nb, bool* opens) {
  const uint32_t lane = lane_id();
  const bool valid = lane < nb && pre != 0xFFFFFFFFu;
  const uint32_t first = first_equal_lane<SG>(pre, valid);
  const bool leader = valid && first == lane;
  const uint64_t leaders = __ballot(leader);
  const uint32_t slot = valid ? (uint32_t)__popcll(leaders & ((1ull << first) - 1ull)) : kNoSlot;
  if (leader) st.prefix[slot] = pre;
  if (lane < SG) st.leader[lane] = slot;
  if (lane == 0) st.n = (uint32_t)__popcll(leaders);
  *opens = leader;
  return slot;
}

constexpr uint32_t kNoDigit = 0xFFFFFFFFu;
constexpr uint32_t kTieStage = 64;  // kept-aside candidates a workgroup stages per slot
static_assert(kTieStage <= kWave, "one wavefront moves a slot's staged candidates in one step");

// LEVEL 2 counts every candidate of a boundary's level-1 bin: a full histogram per slot.  LEVEL 3 counts the
// handful of candidates that share a boundary's 21-bit prefix (more only when many keys are equal, and
// equal keys share the digit): per slot one digit with its count, met first by the workgroup; candidates
// with another digit are added straight to the client's table.
template <uint32_t SG, int LEVEL>
struct SelectShared {
  uint32_t hist[LEVEL == 2 ? SG * kDigitBins : 1];
  uint32_t l3_digit[SG], l3_count[SG];
  // level 3: the candidates kept aside wait here and join the client's lists when the workgroup is done (one
  // device-wide atomic per slot and workgroup instead of one per wavefront row that holds such a candidate:
  // a client's counters share a cache line, and atomics to one line queue up); what does not fit goes directly
  uint2 tie_stage[LEVEL == 3 ? SG : 1][kTieStage];
  uint32_t tie_n[SG];
  SlotTable<SG> slots;
  // top 11 key bits -> 1 + (level 2: slot, level 3: bin id); 4 bits each for up to 15 slots, 8 bits beyond
  static constexpr uint32_t kTagBits = SG <= 15 ? 4u : 8u, kTagsPerWord = 32u / kTagBits;
  uint32_t bin_slot[kL1Bins / kTagsPerWord];
  uint32_t digit_map[SG][kDigitBins / 32];  // level 3: second digits present per bin id
  uint32_t tie_full[SG];                 // this workgroup has seen the slot's kept-aside list overflow

  __device__ __forceinline__ uint32_t bin_tag(uint32_t top11) const {
    return (bin_slot[top11 / kTagsPerWord] >> ((top11 % kTagsPerWord) * kTagBits)) & ((1u << kTagBits) - 1u);
  }
  __device__ __forceinline__ void set_bin_tag(uint32_t top11, uint32_t tag) {  // once per top11, tag <= SG
    atomicOr(&bin_slot[top11 / kTagsPerWord], tag << ((top11 % kTagsPerWord) * kTagBits));
  }
};
// Level 2 for up to 15 boundaries: two workgroups to a CU.  All 31 at once: one workgroup.
static_assert(sizeof(SelectShared<kSlotGroup, 2>) <= 65536 && sizeof(SelectShared<kSlotGroupWide, 2>) <= 160 * 1024 - 2048,
              "SelectShared must fit the CU's LDS");

// Counts one candidate per lane (`live` lanes only); dense_i is its number in the
// position-ordered candidate list (which ranks equal keys just as positions do).
// Must be reached by all lanes of the wavefront.
template <int LEVEL, uint32_t SG>
__device__ __forceinline__ void select_count(SelectShared<SG, LEVEL>& S, uint32_t key, uint32_t dense_i, bool live,
                                             uint32_t* tie_cnt, uint2* __restrict__ ties, uint32_t* table) {
  uint32_t q = kNoSlot;
  if (live) {
    const uint32_t tag = S.bin_tag(key >> 20);
    if (tag) {
      if (LEVEL == 2) {
        atomicAdd(&S.hist[(tag - 1) * kDigitBins + ((key >> 10) & (kDigitBins - 1))], 1u);
      } else {
        const uint32_t second = (key >> 10) & (kDigitBins - 1);
        if ((S.digit_map[tag - 1][second >> 5] >> (second & 31u)) & 1u) {
          const uint32_t pre = key >> 10, ns = S.slots.n;
          for (uint32_t qq = 0; qq < ns; ++qq)
            if (S.slots.prefix[qq] == pre) q = qq;
        }
      }
    }
  }
  if (LEVEL == 3) {
    const uint32_t digit = key & (kDigitBins - 1);
    uint64_t todo = __ballot(q != kNoSlot);
    while (todo) {  // one round per distinct (slot, last digit) present in the wavefront
      const uint32_t leader = (uint32_t)__builtin_ctzll(todo);
      const uint32_t qs = __builtin_amdgcn_readlane(q, leader), ds = __builtin_amdgcn_readlane(digit, leader);
      const bool mine = q == qs && digit == ds;
      const uint64_t peers = __ballot(mine);
      const uint32_t n_peers = (uint32_t)__popcll(peers);
      uint32_t staged = 0;
      if (lane_id() == leader) {
        const uint32_t seen = atomicCAS(&S.l3_digit[qs], kNoDigit, ds);
        if (seen == kNoDigit || seen == ds) atomicAdd(&S.l3_count[qs], n_peers);
        else atomicAdd(&table[qs * kDigitBins + ds], n_peers);
        staged = atomicAdd(&S.tie_n[qs], n_peers);  // grows past kTieStage once the stage is full
      }
      staged = __builtin_amdgcn_readlane(staged, leader);
      const uint32_t place = staged + lanes_below(peers);
      if (mine && place < kTieStage) S.tie_stage[qs][place] = make_uint2(dense_i, digit);
      const uint64_t over = __ballot(mine && place >= kTieStage);
      if (over) {  // uniform
        const uint32_t first_over = (uint32_t)__builtin_ctzll(over);
        uint32_t base = kTieCap;
        if (lane_id() == first_over && !S.tie_full[qs]) {
          base = atomicAdd(&tie_cnt[qs], (uint32_t)__popcll(over));
          if (base >= kTieCap) S.tie_full[qs] = 1u;  // the count is past the cap for good: stop adding to it
        }
        base = __builtin_amdgcn_readlane(base, first_over);
        if (mine && place >= kTieStage) {
          const uint32_t pos = base + lanes_below(over);
          if (pos < kTieCap) ties[qs * kTieCap + pos] = make_uint2(dense_i, digit);
        }
      }
      todo &= ~peers;
    }
  }
}

// ---- walking the filter's output in position order
constexpr uint32_t kNoGroup = 0xFFFFFFFFu;
constexpr uint32_t kEmitBlock = kSpan * kChunkSpans / 8u;  // threads of a count/emit workgroup: 8 candidates each
constexpr uint32_t kEmitWaves = kEmitBlock / kWave;
constexpr uint32_t kPerLane = kSpan / kWave;              // candidates per lane per span
static_assert(kEmitWaves == kChunkSpans && kPerLane == 8, "one wavefront per span, eight rows of 64");

// The candidates of one client in position order, as the filter left them:
// candidate i is entry i - nz_off[q] of the run of region nz_run[q], q the last
// non-empty run with nz_off[q] <= i.
struct CandView {
  const uint32_t* __restrict__ val;         // region slots: value bits
  const uint16_t* __restrict__ idx;         // region slots: positions inside the region
  const uint32_t* __restrict__ nz_off;      // n_nz + 1 entries, the last = n
  const uint32_t* __restrict__ nz_run;
  const uint32_t* __restrict__ span_first;  // q of candidate 512 s
  uint32_t n_nz, n;
};

__device__ __forceinline__ CandView cand_view(const Workspace& ws, const ClientCtl* ctl, uint32_t client) {
  CandView view;
  view.val = ws.cand_val + (size_t)client * ws.d;
  view.idx = ws.cand_idx + (size_t)client * ws.d;
  view.nz_off = ws.nz_off + (size_t)client * (ws.n_regions + 1);
  view.nz_run = ws.nz_run + (size_t)client * (ws.n_regions + 1);
  view.span_first = ws.span_first + (size_t)client * (ws.max_spans + 1);
  view.n_nz = ctl->n_nz;
  view.n = ctl->n_cand;
  return view;
}

// Places of the candidates of span `span` in the region slots: row j of the
// span is candidate span*512 + j*64 + lane.  The runs that follow the span's
// first one are fetched 64 at a time, one per lane; every run that starts
// inside the span moves the rows at or after its first candidate on to it.
struct SpanWindow {  // the first 64 runs at or after a span's first candidate, one per lane
  uint32_t base, wo, wr;
};

__device__ __forceinline__ SpanWindow span_window(const CandView& cv, uint32_t span) {
  SpanWindow w;
  w.base = cv.span_first[span];
  w.wo = cv.nz_off[min(w.base + lane_id(), cv.n_nz)];
  w.wr = cv.nz_run[min(w.base + lane_id(), cv.n_nz)];  // entry n_nz is never selected: its offset is n >= end
  return w;
}

// A span that lies in a stretch of nearly empty regions crosses hundreds of runs (it has 512 candidates, so up
// to 512 of them): walking those one by one, a memory round trip per 63, made single wavefronts the last to
// finish by far.  So: few runs inside the window (the rule) are walked one by one; many are searched by every
// row at once (the window's 64 offsets ascend: six shuffle steps); the window after is asked for before
// the current one is worked on.
constexpr uint32_t kSerialRuns = 8;

__device__ __forceinline__ void span_slots(const CandView& cv, uint32_t span, const SpanWindow& win,
                                           uint32_t (&slot)[kPerLane]) {
  const uint32_t lane = lane_id();
  const uint32_t begin = span * kSpan;
  const uint32_t end = min(begin + kSpan, cv.n);
  uint32_t base = win.base, wo = win.wo, wr = win.wr;
  // slot of candidate i in run (region r, first candidate o): r * kRegion + (i - o); kept as i + shift
  const uint32_t shift0 = __builtin_amdgcn_readlane(wr, 0) * kRegion - __builtin_amdgcn_readlane(wo, 0);
#pragma unroll
  for (uint32_t j = 0; j < kPerLane; ++j) slot[j] = shift0;
  while (true) {
    // entries 1..m of the window start inside the span (offsets ascend strictly; the entry after the last run holds n >= end)
    const uint32_t m = (uint32_t)__popcll(__ballot(wo < end) & ~1ull);
    const bool more = m == kWave - 1u;  // the window's last entry still starts inside: look at the next window too
    uint32_t nwo = 0, nwr = 0;
    if (more) {  // uniform
      nwo = cv.nz_off[min(base + (kWave - 1u) + lane, cv.n_nz)];
      nwr = cv.nz_run[min(base + (kWave - 1u) + lane, cv.n_nz)];
    }
    if (m <= kSerialRuns) {
      for (uint32_t t = 1; t <= m; ++t) {
        const uint32_t ot = __builtin_amdgcn_readlane(wo, t);
        const uint32_t shift = __builtin_amdgcn_readlane(wr, t) * kRegion - ot;
#pragma unroll
        for (uint32_t j = 0; j < kPerLane; ++j) {
          const uint32_t i = begin + j * kWave + lane;
          if (i >= ot) slot[j] = shift;
        }
      }
    } else {
      const uint32_t first_here = __builtin_amdgcn_readlane(wo, 1);  // rows before it keep what they have
#pragma unroll
      for (uint32_t j = 0; j < kPerLane; ++j) {
        const uint32_t i = begin + j * kWave + lane;
        uint32_t pos = 0;  // last entry in 0..m whose offset is <= i
#pragma unroll
        for (uint32_t step = kWave / 2u; step; step >>= 1) {
          const uint32_t probe = (uint32_t)__shfl((int)wo, (int)min(pos + step, kWave - 1u), kWave);
          if (pos + step <= m && probe <= i) pos += step;
        }
        const uint32_t ro = (uint32_t)__shfl((int)wo, (int)pos, kWave), rr = (uint32_t)__shfl((int)wr, (int)pos, kWave);
        if (i >= first_here) slot[j] = rr * kRegion - ro;
      }
    }
    if (!more) break;
    base += kWave - 1;  // entry 63 of this window is entry 0 of the next
    wo = nwo;
    wr = nwr;
  }
#pragma unroll
  for (uint32_t j = 0; j < kPerLane; ++j) slot[j] += begin + j * kWave + lane;  // meaningless for i >= n, never used there
}

// A workgroup's partial level-2 histogram is stored in 16-bit counters when no workgroup can
// see more than 65535 candidates (the gather: whole spans dealt round the wavefronts; the
// later passes: an equal share each): half the bytes written and read back.
__device__ __forceinline__ bool narrow_partials(uint32_t n_cand, uint32_t blocks) { return n_cand <= 32768u * blocks; }

__device__ __forceinline__ void store_partials(const uint32_t* hist, uint32_t used, uint32_t* part, bool narrow) {
  if (narrow) {
    for (uint32_t i = threadIdx.x; i < used / 2u; i += kWideBlock) part[i] = hist[2u * i] | (hist[2u * i + 1u] << 16);
  } else {
    for (uint32_t i = threadIdx.x; i < used; i += kWideBlock) part[i] = hist[i];
  }
}

// Fills the workgroup's slot tables for the plan's boundaries.
template <int LEVEL, uint32_t SG>
__device__ __forceinline__ void select_setup(SelectShared<SG, LEVEL>& S, const ClientCtl* ctl, uint32_t nb) {
  const uint32_t tid = threadIdx.x;
  if (LEVEL == 2)
    for (uint32_t i = tid; i < SG * kDigitBins; i += kWideBlock) S.hist[i] = 0;
  if (tid < SG) {
    S.l3_digit[tid] = kNoDigit;
    S.l3_count[tid] = 0;
    S.tie_n[tid] = 0;
  }
  for (uint32_t i = tid; i < kL1Bins / SelectShared<SG, LEVEL>::kTagsPerWord; i += kWideBlock) S.bin_slot[i] = 0;
  for (uint32_t i = tid; i < SG * (kDigitBins / 32); i += kWideBlock) (&S.digit_map[0][0])[i] = 0;
  if (tid < SG) S.tie_full[tid] = 0;
  uint32_t pre = 0xFFFFFFFFu;
  if (tid < nb) pre = ctl->sel_prefix[LEVEL - 2][tid];
  __syncthreads();
  if (tid < kWave) {  // the first wavefront, lane b = boundary b
    bool opens;
    const uint32_t slot = build_slots<SG>(S.slots, pre, nb, &opens);
    if (LEVEL == 2) {
      if (opens) S.set_bin_tag(pre, slot + 1);
    } else {
      // the slots' top 11 bits are numbered in order of first appearance as well
      const uint32_t top11 = pre >> 10, second = pre & (kDigitBins - 1);
      const uint32_t first = first_equal_lane<SG>(top11, opens);
      const uint64_t bin_openers = __ballot(opens && first == tid);
      if (opens) {
        const uint32_t bin = (uint32_t)__popcll(bin_openers & ((1ull << first) - 1ull));
        if (first == tid) S.set_bin_tag(top11, bin + 1);
        atomicOr(&S.digit_map[bin][second >> 5], 1u << (second & 31u));
      }
    }
  }
  __syncthreads();
}

// Level 2, fused with the gather: every
// wavefront takes spans of 512 candidates (gw, gw + wavefronts, ...), collects
// them from the region runs they lie in, stores them at their place in the
// dense position-ordered candidate list and counts the level-2 digits on the
// way.  Every span is the same amount of work wherever its candidates lie.
// The wavefronts do not wait for each other until the histogram is stored.
template <uint32_t SG>
__global__ __launch_bounds__(kWideBlock) void gather_l2_kernel(const ClientParams* __restrict__ params,
                                                               ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ SelectShared<SG, 2> S;
  const uint32_t client = blockIdx.y, tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  if (ctl->dead) return;  // the workspace was too short for this client (whole workgroup)
  const uint32_t nb = min(p.R, SG);
  select_setup<2, SG>(S, ctl, nb);
  const CandView cv = cand_view(ws, ctl, client);
  uint32_t* __restrict__ dst_idx = ws.dense_idx + (size_t)client * ws.dense_cap;
  uint32_t* __restrict__ dst_val = ws.dense_val + (size_t)client * ws.dense_cap;
  const uint32_t n_spans = (cv.n + kSpan - 1) / kSpan;
  // keep_all: a slot is a region of the vector itself and a candidate's place in it its position
  auto copy_spans = [&](auto keep_all) {
    const uint32_t* __restrict__ src_val = keep_all.value ? reinterpret_cast<const uint32_t*>(p.update) : cv.val;
    for (uint32_t span = blockIdx.x * kWideWaves + wave; span < n_spans; span += gridDim.x * kWideWaves) {
      uint32_t slot[kPerLane], v[kPerLane], x[kPerLane];
      span_slots(cv, span, span_window(cv, span), slot);
#pragma unroll
      for (uint32_t j = 0; j < kPerLane; ++j) {
        // rows past the last candidate read some valid place instead of branching, so that the
        // sixteen loads of a span go out together
        const uint32_t sl = min(slot[j], ws.d - 1u);
        v[j] = src_val[sl];
        x[j] = keep_all.value ? sl : (sl & ~(kRegion - 1u)) + cv.idx[sl];  // a slot starts where its region starts
      }
#pragma unroll
      for (uint32_t j = 0; j < kPerLane; ++j) {
        const uint32_t i = span * kSpan + j * kWave + lane;
        if (i - lane >= cv.n) break;  // uniform
        if (i < cv.n) {
          dst_val[i] = v[j];
          dst_idx[i] = x[j];
        }
        if (nb) select_count<2, SG>(S, v[j] & 0x7FFFFFFFu, 0u, i < cv.n, nullptr, nullptr, nullptr);
      }
    }
  };
  if (ctl->keep_all) copy_spans(std::true_type{}); else copy_spans(std::false_type{});
  __syncthreads();
  if (nb == 0) return;
  uint32_t* part = ws.sel_part + ((size_t)client * gridDim.x + blockIdx.x) * SG * kDigitBins;
  store_partials(S.hist, S.slots.n * kDigitBins, part, narrow_partials(cv.n, gridDim.x));
}

// Level 3 reads the dense list.  (With 31 slots the compiler would keep 90 scalar registers, and past 80 or so a
// CU takes one workgroup of 1024 threads instead of two: capped.)
template <uint32_t SG>
__global__ __launch_bounds__(kWideBlock) __attribute__((amdgpu_num_sgpr(64))) void select_pass3_kernel(const ClientParams* __restrict__ params,
                                                                  ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ SelectShared<SG, 3> S;
  const uint32_t client = blockIdx.y, tid = threadIdx.x, wave = tid / kWave;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  if (ctl->dead) return;  // the workspace was too short for this client (whole workgroup)
  if (p.R == 0) return;  // nothing is coded
  const uint32_t nb = min(p.R, SG);
  const uint32_t* __restrict__ val = ws.dense_val + (size_t)client * ws.dense_cap;
  uint2* ties = ws.tie_list + (size_t)client * SG * kTieCap;
  uint32_t* tie_cnt = ctl->tie_cnt;
  uint32_t* table = ws.l3_hist + (size_t)client * SG * kDigitBins;
  select_setup<3, SG>(S, ctl, nb);

  const uint32_t n = ctl->n_cand;
  const uint32_t span = (uint32_t)(((uint64_t)n + gridDim.x - 1) / gridDim.x);
  const uint64_t begin64 = (uint64_t)blockIdx.x * span;
  const uint32_t begin = (uint32_t)(begin64 < n ? begin64 : n);
  const uint32_t end = (uint32_t)(begin64 + span < n ? begin64 + span : n);
  for (uint32_t base = begin; base < end; base += kWideBlock * 8u) {
    uint32_t v[8];
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) {
      const uint32_t i = base + u * kWideBlock + tid;
      v[u] = 0;
      if (i < end) v[u] = val[i];
    }
#pragma unroll
    for (uint32_t u = 0; u < 8; ++u) {
      const uint32_t i = base + u * kWideBlock + tid;
      if (base + u * kWideBlock + wave * kWave >= end) break;  // uniform per wavefront
      select_count<3, SG>(S, v[u] & 0x7FFFFFFFu, i, i < end, tie_cnt, ties, table);
    }
  }
  __syncthreads();
  // the slots' own digits go to the client's table now, the staged candidates to the kept-aside lists
  if (tid < S.slots.n && S.l3_count[tid]) atomicAdd(&table[tid * kDigitBins + S.l3_digit[tid]], S.l3_count[tid]);
  const uint32_t lane = lane_id();
  for (uint32_t q = wave; q < S.slots.n; q += kWideWaves) {  // a wavefront per slot
    const uint32_t n_staged = min(S.tie_n[q], kTieStage);
    if (n_staged == 0) continue;
    uint32_t base = kTieCap;
    if (lane == 0) base = atomicAdd(&tie_cnt[q], n_staged);  // a count past the cap only says "too many"
    base = __builtin_amdgcn_readlane(base, 0);
    if (lane < n_staged && base + lane < kTieCap) ties[q * kTieCap + base + lane] = S.tie_stage[q][lane];
  }
}

// One workgroup per (histogram slot, client): thread t owns digit t.  The
// partial histograms are added up, a suffix sum from the largest digit gives
// "keys with digit >= t", and every boundary that shares the slot reads off its
// digit and the rank left inside it.
template <int LEVEL, uint32_t SG>
__global__ __launch_bounds__(kWideBlock) void select_walk_kernel(const ClientParams* __restrict__ params,
                                                                 ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ SlotTable<SG> slots;
  __shared__ uint32_t s_digit[SG], s_quota[SG], s_need[SG], s_rem[SG];
  __shared__ uint32_t s_found;
  __shared__ uint32_t scan_tmp[kWideWaves];
  __shared__ uint2 s_list[LEVEL == 3 ? kTieCap : 1];
  const uint32_t slot = blockIdx.x, client = blockIdx.y, tid = threadIdx.x;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  if (ctl->dead) return;  // the workspace was too short for this client (whole workgroup)
  const uint32_t n_cand = ctl->n_cand;  // asked for together with R
  if (p.R == 0) return;
  const uint32_t nb = min(p.R, SG);
  const uint32_t n_parts = ws.sel_blocks;
  const uint32_t* parts = ws.sel_part + (size_t)client * n_parts * SG * kDigitBins;
  // Everything the walk reads from global memory is requested here, before the
  // first wait.  Thread t takes digit 1023 - t, so that the scan runs from the top
  // digit down; a slot past the last one in use adds up stale partials for nothing.
  uint32_t pre = 0xFFFFFFFFu, rem_in = 0;
  if (tid < nb) {
    pre = ctl->sel_prefix[LEVEL - 2][tid];
    rem_in = ctl->sel_rem[LEVEL - 2][tid];
    // the level's results go to arrays of their own: other workgroups of this launch may still have to read its inputs
    if (LEVEL == 2 && slot == 0 && pre == 0xFFFFFFFFu) ctl->sel_prefix[1][tid] = pre;
  }
  const uint32_t kept = LEVEL == 3 ? ctl->tie_cnt[slot] : 0u;
  const uint32_t digit = kDigitBins - 1 - tid;
  uint32_t h = 0;
  if (LEVEL == 3) {  // one table per client; left cleared for the next call
    uint32_t* mine = ws.l3_hist + ((size_t)client * SG + slot) * kDigitBins + digit;
    h = *mine;
    *mine = 0;
  } else {
    if (narrow_partials(n_cand, n_parts)) {
      const uint16_t* narrow = reinterpret_cast<const uint16_t*>(parts);
#pragma unroll 8
      for (uint32_t b = 0; b < n_parts; ++b)
        h += narrow[((size_t)b * SG * kDigitBins) * 2u + (size_t)slot * kDigitBins + digit];
    } else {
#pragma unroll 8
      for (uint32_t b = 0; b < n_parts; ++b) h += parts[((size_t)b * SG + slot) * kDigitBins + digit];
    }
  }
  if (tid < SG) {
    s_need[tid] = 0;
    s_rem[tid] = rem_in;
  }
  if (tid < kWave) {
    bool opens;
    build_slots<SG>(slots, pre, nb, &opens);
  }
  __syncthreads();
  if (slot >= slots.n) return;
  uint32_t total;
  const uint32_t above = block_excl_scan<kWideWaves>(h, scan_tmp, &total);  // keys with a larger digit
  const uint32_t prefix = slots.prefix[slot];
  for (uint32_t b = 0; b < nb; ++b) {
    if (slots.leader[b] != slot) continue;
    const uint32_t r = b;
    const uint32_t rem = s_rem[b];
    if (rem > total && tid == 0) atomicOr(ws.status, CVLC_DEV_INTERNAL);  // histogram short of the rank
    if (above < rem && rem <= above + h) {  // exactly one thread
      const uint32_t quota = rem - above;   // rank inside the digit class, 1-based
      const uint32_t full = (prefix << 10) | digit;
      if (LEVEL == 2) {
        ctl->sel_prefix[1][r] = full;
        ctl->sel_rem[1][r] = quota;
      } else {
        ctl->tau[r] = full;
        ctl->iota[r] = 0xFFFFFFFFu;  // every member of the class is inside unless it straddles Z_r
        s_digit[b] = digit;
        s_quota[b] = quota;
        s_need[b] = quota < h ? 1u : 0u;
      }
    }
  }
  if (LEVEL == 3) {
    __syncthreads();
    // a class of equal keys straddles the boundary: find its quota-th member in position order
    const uint2* list = ws.tie_list + ((size_t)client * SG + slot) * kTieCap;
    const uint32_t* __restrict__ val = ws.dense_val + (size_t)client * ws.dense_cap;
    const uint32_t n = ctl->n_cand;
    for (uint32_t b = 0; b < nb; ++b) {
      if (!s_need[b]) continue;  // uniform
      const uint32_t r = b, w_digit = s_digit[b], w_quota = s_quota[b];
      if (kept <= kTieCap) {
        // position-order rank of every kept-aside member of the class, all threads, list in LDS
        __syncthreads();
        for (uint32_t e = tid; e < kept; e += kWideBlock) s_list[e] = list[e];
        __syncthreads();
        for (uint32_t e = tid; e < kept; e += kWideBlock) {
          const uint2 me = s_list[e];
          if (me.y != w_digit) continue;
          uint32_t before = 0;
          for (uint32_t o = 0; o < kept; ++o) {
            const uint2 other = s_list[o];
            before += (other.y == w_digit && other.x < me.x) ? 1u : 0u;
          }
          if (before + 1 == w_quota) ctl->iota[r] = me.x;
        }
      } else {
        // too many to keep aside: walk the whole candidate list.  Every wavefront counts the members
        // of the class in a contiguous sixteenth of the list; the one whose share holds the
        // quota-th member then walks it again, row by row.  No workgroup barrier inside the walks.
        const uint32_t tau = (prefix << 10) | w_digit;
        const uint32_t lane = lane_id(), wave = tid / kWave;
        const uint32_t share = ((n + kWideBlock - 1) / kWideBlock) * kWave;  // a multiple of 64
        const uint32_t w_begin = min(wave * share, n), w_end = min(w_begin + share, n);
        __syncthreads();
        if (tid == 0) s_found = 0;
        uint32_t mine = 0;
        for (uint32_t base = w_begin; base < w_end; base += kWave * 8u) {
          uint32_t v[8];
#pragma unroll
          for (uint32_t u = 0; u < 8; ++u) v[u] = val[min(base + u * kWave + lane, n - 1u)];
#pragma unroll
          for (uint32_t u = 0; u < 8; ++u)
            mine += (uint32_t)__popcll(__ballot(base + u * kWave + lane < w_end && (v[u] & 0x7FFFFFFFu) == tau));
        }
        if (lane == 0) scan_tmp[wave] = mine;
        __syncthreads();
        uint32_t before = 0;
        for (uint32_t w = 0; w < wave; ++w) before += scan_tmp[w];
        if (before < w_quota && w_quota <= before + mine) {  // uniform per wavefront: exactly one takes this
          uint32_t left = w_quota - before;
          for (uint32_t base = w_begin; base < w_end; base += kWave) {
            const uint32_t i = base + lane;
            const bool hit = i < w_end && (val[min(i, n - 1u)] & 0x7FFFFFFFu) == tau;
            const uint64_t m = __ballot(hit);
            const uint32_t c = (uint32_t)__popcll(m);
            if (left <= c) {
              if (hit && lanes_below(m) + 1u == left) {
                ctl->iota[r] = i;
                s_found = 1;
              }
              break;
            }
            left -= c;
          }
        }
        __syncthreads();
        if (tid == 0 && !s_found) atomicOr(ws.status, CVLC_DEV_INTERNAL);
      }
    }
  }
}

// ------------------------------------------------------------------ 5. classification of the candidates
struct Thresholds {  // group boundaries in LDS
  uint32_t tau[32];
  uint32_t iota[32];
  uint32_t cut[32];  // key < cut[r]  <=>  key <= tau[r] for r < R; 0 (never) for r >= R
  uint32_t above[33];  // the boundary key just above group g: tau[g - 1]; no key (all ones) above group 0
};

__device__ __forceinline__ void load_thresholds(Thresholds& t, const ClientCtl* ctl, uint32_t R) {
  if (threadIdx.x < 32) {
    const bool live = threadIdx.x < R;
    const uint32_t tau = live ? ctl->tau[threadIdx.x] : 0xFFFFFFFFu;
    t.tau[threadIdx.x] = tau;
    t.iota[threadIdx.x] = live ? ctl->iota[threadIdx.x] : 0u;
    t.cut[threadIdx.x] = live ? (tau == 0xFFFFFFFFu ? tau : tau + 1u) : 0u;  // keys stay below 2^31
    t.above[threadIdx.x + 1] = tau;
    if (threadIdx.x == 0) t.above[0] = 0xFFFFFFFFu;
  }
}

// Group of a candidate, 0-based: the first boundary r whose top-Z_r set holds
// it (key above tau_r, or equal and not after candidate iota_r); R if none (dropped).
// tau is non-increasing in r, so "key <= tau_r" holds for the first g boundaries
// and for no later one, g being the number of boundaries with tau_r >= key: a
// binary search over the boundaries (entries past R never hold) finds it in
// log2 R probes per candidate.  The position is only needed (and only read)
// when the key equals a boundary key.
template <uint32_t N>
__device__ __forceinline__ void classify_keys(const Thresholds& t, uint32_t R, const uint32_t (&key)[N],
                                              uint32_t (&grp)[N]) {
#pragma unroll
  for (uint32_t j = 0; j < N; ++j) grp[j] = 0;
  // largest power of two <= R: the probes reach entry 2 * top - 2 <= 30 at most, the result 2 * top - 1 >= R
  for (uint32_t step = R ? 1u << (31 - __builtin_clz(R)) : 0u; step; step >>= 1) {
    uint32_t probe[N];  // all N reads of a step before the first comparison: one LDS round trip per step
#pragma unroll
    for (uint32_t j = 0; j < N; ++j) probe[j] = t.cut[grp[j] + step - 1u];
#pragma unroll
    for (uint32_t j = 0; j < N; ++j) grp[j] += key[j] < probe[j] ? step : 0u;
  }
}

// Second step for a key that equals the boundary key just above its group:
// boundaries with that key decide by position, i.e. by the candidate's number
// in the position-ordered list against that of the last member inside.
__device__ __forceinline__ uint32_t classify_tie(const Thresholds& t, uint32_t key, uint32_t g, uint32_t dense_i) {
  while (g > 0 && t.tau[g - 1] == key && dense_i <= t.iota[g - 1]) --g;
  return g;
}

// Lanes that hold a candidate of the caller's group (group ids below 2^ID_BITS); lanes
// with g == kNoGroup match nobody.  Must be reached by the whole wavefront.
// Per bit of the id: the lanes that have it set, against an all-ones / all-zeros word of the
// caller's own bit; what differs in any bit is not the caller's group.
template <uint32_t ID_BITS>
__device__ __forceinline__ uint64_t same_group_lanes(uint32_t g) {
  const uint64_t coded = __ballot(g != kNoGroup);
  uint32_t differ_lo = 0, differ_hi = 0;
#pragma unroll
  for (uint32_t bit = 0; bit < ID_BITS; ++bit) {
    const uint32_t mine = (uint32_t)__builtin_amdgcn_sbfe((int32_t)g, bit, 1u);  // the bit, sign-extended
    const uint64_t set = __ballot(mine != 0u);
    differ_lo |= (uint32_t)set ^ mine;
    differ_hi |= (uint32_t)(set >> 32) ^ mine;
  }
  return coded & ~(((uint64_t)differ_hi << 32) | differ_lo);
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, (uint32_t)__shfl_xor(v, o, 64));
  return v;
}

// Loads span `span` of the dense list (kPerLane candidates per lane, row j at
// span*512 + j*64 + lane, i.e. in position order).  No branch around the loads (a lane past
// the end reads the last candidate again): all eight are in flight before the first is waited for.
__device__ __forceinline__ void load_span(const uint32_t* __restrict__ list, uint32_t n, uint32_t span,
                                          uint32_t (&out)[kPerLane]) {
  const uint32_t mine = span * kSpan + lane_id();
#pragma unroll
  for (uint32_t j = 0; j < kPerLane; ++j) out[j] = list[min(mine + j * kWave, n - 1u)];
}

// Classifies the loaded value bits of span `span`; grp[j] = kNoGroup past the end of the list.
__device__ __forceinline__ void classify_loaded(const Thresholds& thr, uint32_t R, uint32_t n, uint32_t span,
                                                const uint32_t (&v)[kPerLane], uint32_t (&grp)[kPerLane]) {
  const uint32_t mine = span * kSpan + lane_id();
  uint32_t key[kPerLane];
#pragma unroll
  for (uint32_t j = 0; j < kPerLane; ++j) key[j] = v[j] & 0x7FFFFFFFu;
  classify_keys<kPerLane>(thr, R, key, grp);
  // the boundary key just above every candidate's group, all eight read before the first is looked at:
  // only a key that equals it (next to none) goes on to the tie rule
  uint32_t above[kPerLane];
#pragma unroll
  for (uint32_t j = 0; j < kPerLane; ++j) above[j] = thr.above[grp[j]];
#pragma unroll
  for (uint32_t j = 0; j < kPerLane; ++j) {
    const uint32_t i = mine + j * kWave;
    uint32_t g = grp[j];
    if (above[j] == key[j]) g = classify_tie(thr, key[j], g, i);
    grp[j] = i < n ? g : kNoGroup;
  }
}

// ------------------------------------------------------------------ 6. group counts and statistics
// QSGD's header carries the group's l2-norm, and the stream must not depend on
// the order squares are added in: the sum of squares is kept exactly, as a
// fixed-point number in units of 2^-298 (the square of the smallest denormal)
// spread over 32-bit limbs, each limb summed in a 64-bit counter of its own.
// x = m * 2^(q - 149) with m < 2^24, so x^2 = m^2 << 2q: three limbs from 2q / 32.
struct SquareLimbs {
  uint32_t word;     // first limb
  uint32_t part[3];  // the pieces of m^2 << (2q mod 32), each below 2^32
};
__device__ __forceinline__ SquareLimbs square_limbs(uint32_t value_bits) {
  const uint32_t b = value_bits & 0x7FFFFFFFu, e = b >> 23, frac = b & 0x7FFFFFu;
  const uint64_t m = e ? (frac | 0x800000u) : frac;
  const uint32_t off = 2u * (e ? e - 1u : 0u), sh = off & 31u;
  const uint64_t sq = m * m, low = sq << sh;  // the top bits that leave `low` are part[2]
  SquareLimbs r;
  r.word = off >> 5;
  r.part[0] = (uint32_t)low;
  r.part[1] = (uint32_t)(low >> 32);
  r.part[2] = sh ? (uint32_t)(sq >> (64u - sh)) : 0u;
  return r;
}

// What the counting pass leaves for the packing pass, 16 bits per candidate of the dense list: its group
// (5 bits) and above it its number among the members of that group in its span of 512 (9 bits); kNoPlace
// for a dropped candidate.  The array takes the place of the filter's region-slot positions, which nothing
// reads once the gather has run (d entries per client, the dense list has at most as many).
constexpr uint32_t kPlaceShift = 5;
constexpr uint16_t kNoPlace = 0xFFFFu;
__device__ __forceinline__ uint16_t* span_places(const Workspace& ws, uint32_t client) {
  return ws.cand_idx + (size_t)client * ws.d;
}

constexpr uint32_t kLimbBanks = 2;  // copies of a workgroup's limb counters, to thin out colliding LDS atomics

// Every wavefront takes spans of 512 candidates (gw, gw + wavefronts, ...) and
// writes, per span, the number of members of every group and, per candidate,
// its group and its number among the span's members of that group (together
// with the layout's prefix over the spans: its record's place in the stream;
// the packing pass neither classifies nor counts again).  Min, max and sum of
// squares of the groups go to LDS
// columns private to a lane id, so that the LDS atomics of one instruction never
// collide; they are reduced once at the end.  Wavefronts do not wait for each
// other before that.
// QSGD: also the exact sum of squares of every group (see above).
template <bool QSGD>
__global__ __launch_bounds__(kEmitBlock) void count_kernel(const ClientParams* __restrict__ params,
                                                           ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ Thresholds thr;
  __shared__ unsigned long long s_limb[QSGD ? kLimbBanks : 1][QSGD ? 32 : 1][kNormLimbs];  // bank = lane mod kLimbBanks
  __shared__ uint32_t s_max[33][kWave], s_negmin[33][kWave];
  __shared__ double s_sq[33][kWave];
  __shared__ uint32_t s_cnt[kEmitWaves][32];
  const uint32_t client = blockIdx.y, tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  if (ctl->dead) return;  // the workspace was too short for this client (whole workgroup)
  const uint32_t R = p.R, n = ctl->n_cand;
  const uint32_t n_spans = (n + kSpan - 1) / kSpan;
  const uint32_t* __restrict__ val = ws.dense_val + (size_t)client * ws.dense_cap;
  uint32_t* __restrict__ span_cnt = ws.span_cnt + (size_t)client * (ws.max_spans + 1) * 32;
  load_thresholds(thr, ctl, R);
  if (tid < kEmitWaves * 32) (&s_cnt[0][0])[tid] = 0;
  for (uint32_t i = tid; i < 33 * kWave; i += kEmitBlock) {
    (&s_max[0][0])[i] = 0;
    (&s_negmin[0][0])[i] = 0;
    (&s_sq[0][0])[i] = 0.0;
  }
  if (QSGD)
    for (uint32_t i = tid; i < kLimbBanks * 32 * kNormLimbs; i += kEmitBlock) (&s_limb[0][0][0])[i] = 0;
  __syncthreads();
  uint16_t* __restrict__ place = span_places(ws, client);
  uint32_t* running = s_cnt[wave];  // members of every group (the dropped ones last) in the rows so far
  const uint32_t span_step = gridDim.x * kEmitWaves;
  uint32_t ahead[kPerLane];  // the next span's value bits, asked for before the current span is worked on
  if (blockIdx.x * kEmitWaves + wave < n_spans) load_span(val, n, blockIdx.x * kEmitWaves + wave, ahead);
  for (uint32_t span = blockIdx.x * kEmitWaves + wave; span < n_spans; span += span_step) {
    uint32_t v[kPerLane], grp[kPerLane];
#pragma unroll
    for (uint32_t j = 0; j < kPerLane; ++j) v[j] = ahead[j];
    if (span + span_step < n_spans) load_span(val, n, span + span_step, ahead);
    classify_loaded(thr, R, n, span, v, grp);
    // Every candidate's number among the span's members of its group (row after row, lanes in order): a
    // row's members of a group read the group's running number and the lowest of them adds the row's
    // members to it.  This wavefront alone touches the counters and its LDS accesses complete in the order
    // they are issued, so no row waits for the one before.  What the counters hold after the last row are
    // the span's group sizes.
    uint32_t start[kPerLane], below[kPerLane];
    auto number_rows = [&](auto id_bits) {
#pragma unroll
      for (uint32_t j = 0; j < kPerLane; ++j) {
        const uint64_t same = same_group_lanes<decltype(id_bits)::value>(grp[j]);
        below[j] = lanes_below(same);
        start[j] = 0;
        if (grp[j] != kNoGroup) {
          start[j] = running[grp[j]];
          if (below[j] == 0) atomicAdd(&running[grp[j]], (uint32_t)__popcll(same));
        }
        asm volatile("" ::: "memory");  // the rows' LDS accesses stay in this order; nothing to wait for
      }
    };
    if (R < 8u) number_rows(std::integral_constant<uint32_t, 3>());  // ids 0 .. R, R for the dropped
    else if (R < 16u) number_rows(std::integral_constant<uint32_t, 4>());
    else number_rows(std::integral_constant<uint32_t, 5>());
#pragma unroll
    for (uint32_t j = 0; j < kPerLane; ++j) {
      const uint32_t i = span * kSpan + j * kWave + lane;
      if (i < n) place[i] = grp[j] < R ? (uint16_t)(grp[j] | ((start[j] + below[j]) << kPlaceShift)) : kNoPlace;
    }
    wave_lds_fence();
    if (lane < 32) {
      span_cnt[(size_t)span * 32 + lane] = running[lane];
      running[lane] = 0;
    }
    wave_lds_fence();
#pragma unroll
    for (uint32_t j = 0; j < kPerLane; ++j) {
      const uint32_t g = grp[j];
      if (g != kNoGroup) {
        const float x = __uint_as_float(v[j]);
        const uint32_t o = ordered_bits(x);
        atomicMax(&s_max[g][lane], o);
        atomicMax(&s_negmin[g][lane], ~o);
        atomicAdd(&s_sq[g][lane], (double)x * (double)x);
        if (QSGD && g < R) {
          const SquareLimbs sl = square_limbs(v[j]);  // word + 2 <= 17
          unsigned long long* mine = s_limb[lane % kLimbBanks][g] + sl.word;
          atomicAdd(mine, (unsigned long long)sl.part[0]);
          if (sl.part[1]) atomicAdd(mine + 1, (unsigned long long)sl.part[1]);
          if (sl.part[2]) atomicAdd(mine + 2, (unsigned long long)sl.part[2]);
        }
      }
    }
  }
  __syncthreads();
  if (QSGD) {  // a workgroup sees fewer than 2^31 candidates, so no counter has wrapped
    unsigned long long* dst = ws.norm_limbs + (size_t)client * 32 * kNormLimbs;
    for (uint32_t i = tid; i < R * kNormLimbs; i += kEmitBlock) {
      unsigned long long t = 0;
      for (uint32_t b = 0; b < kLimbBanks; ++b) t += (&s_limb[b][0][0])[i];
      if (t) atomicAdd(&dst[i], t);
    }
  }
  // group g's columns are reduced by wavefront g mod 8; finite values never code to 0, so 0 = no member here
  for (uint32_t g = wave; g <= R; g += kEmitWaves) {
    const uint32_t mx = wave_max_u32(s_max[g][lane]);
    const uint32_t ng = wave_max_u32(s_negmin[g][lane]);
    const double sq = wave_sum_f64(s_sq[g][lane]);
    if (lane == 0 && mx != 0) {
      atomicMax(&ctl->seg_max_enc[g], mx);
      atomicMax(&ctl->seg_negmin_enc[g], ng);
      atomicAdd(&ctl->seg_sumsq[g], sq);
    }
  }
}

// ------------------------------------------------------------------ 7. layout: prefix, headers, statistics
typedef uint32_t __attribute__((address_space(1))) * GlobalWordPtr;

// One workgroup of 1024 threads per client.  Turns the per-span counts of the
// groups into exclusive prefixes (in place; the row after the last span
// receives the totals), checks the totals against the plan, and
// clears the first and the last stream word of every (chunk, group) record run,
// a chunk being 8 spans: those two words can be shared with the neighbouring
// chunks, which OR their bits in; all other payload words have one owner and are
// stored whole.  Then the headers and the statistics block.
__global__ __launch_bounds__(kWideBlock) void layout_kernel(const ClientParams* __restrict__ params,
                                                            ClientCtl* __restrict__ ctls, Workspace ws,
                                                            cvlc_seg_stats_t* __restrict__ stats_out, uint32_t quant) {
  __shared__ double s_tail[kWideWaves];
  __shared__ uint32_t s_sum[32][kNormLimbs];  // QSGD: a group's sum of squares, limbs below 2^32
  __shared__ uint32_t s_payload[32];
  __shared__ uint32_t s_tot[kWideWaves][32];
  const uint32_t client = blockIdx.x, tid = threadIdx.x;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  if (ctl->dead) return;  // the workspace was too short for this client (whole workgroup)
  const uint32_t R = p.R, sbits = position_bits(ws.d);
  const uint32_t n_spans = (ctl->n_cand + kSpan - 1) / kSpan;
  const uint32_t lane = lane_id(), wave = tid / kWave;
  GlobalWordPtr stream = (GlobalWordPtr)p.stream;
  uint32_t* cnt = ws.span_cnt + (size_t)client * (ws.max_spans + 1) * 32;
  // What the headers and the statistics at the end need from memory is asked for here: this kernel is one
  // workgroup per client and all latency.
  uint32_t enc_max = 0, enc_negmin = 0;
  if (tid < R) {
    enc_max = ctl->seg_max_enc[tid];
    enc_negmin = ctl->seg_negmin_enc[tid];
  }
  const double* rsq = ws.region_sumsq + (size_t)client * ws.n_regions;  // energy the filter dropped, region by region
  const double tail0 = tid < ws.n_regions ? rsq[tid] : 0.0;
  const double tail1 = tid + kWideBlock < ws.n_regions ? rsq[tid + kWideBlock] : 0.0;
  if (tid < 32) {  // first stream word of every group's records: exclusive prefix of the payload sizes
    uint32_t words = 0;
    if (tid < R) words = (uint32_t)payload_words(p.Z[tid] - (tid ? p.Z[tid - 1] : 0u), sbits + p.y[tid]);
    const uint32_t incl = wave_incl_scan_u32(words);
    s_payload[tid] = kGlobalHeaderWords + kSegHeaderWords * R + incl - words;
  }
  __syncthreads();
  // Exclusive prefix of the per-span counts over the spans, per group, in place.
  // Wavefront w takes a contiguous range of spans (a whole number of chunks); a
  // lane takes group (lane & 31) of every second span, so that one load covers
  // two whole rows of the table.
  const uint32_t g = lane & 31u, half = lane >> 5;
  const uint32_t W = g < R ? sbits + p.y[g] : 0u;
  const uint32_t P = g < R ? p.Z[g] - (g ? p.Z[g - 1] : 0u) : 0u;
  const uint32_t per_wave = (((n_spans + kWideWaves - 1) / kWideWaves + kChunkSpans - 1) / kChunkSpans) * kChunkSpans;
  const uint32_t s0 = min(wave * per_wave, n_spans), s1 = min(s0 + per_wave, n_spans);
  constexpr uint32_t kBatch = 8;  // loads in flight per lane and batch
  // A lane's counts of one batch of 2 * kBatch spans from span c on (0 past the wavefront's range); the
  // loads are not branched around (a lane past the end reads the range's last row), so that they all go out
  // together.
  auto load_batch = [&](uint32_t c, uint32_t (&vs)[kBatch]) {
#pragma unroll
    for (uint32_t u = 0; u < kBatch; ++u) {
      const uint32_t cc = c + 2 * u + half;
      const uint32_t x = cnt[(size_t)min(cc, s1 - 1u) * 32 + g];
      vs[u] = cc < s1 ? x : 0u;
    }
  };
  // The counts are read twice, for the wavefronts' totals and for the prefix; the first kKeep batches of a
  // wavefront (all of them up to 768 spans per client) stay in registers in between: this kernel is one
  // workgroup per client and all latency.
  constexpr uint32_t kKeep = 3;
  uint32_t keep[kKeep][kBatch];
  {
    uint32_t acc = 0;
#pragma unroll
    for (uint32_t b = 0; b < kKeep; ++b) {
      if (s0 + b * 2 * kBatch < s1) {  // uniform
        load_batch(s0 + b * 2 * kBatch, keep[b]);
      } else {
#pragma unroll
        for (uint32_t u = 0; u < kBatch; ++u) keep[b][u] = 0;
      }
    }
#pragma unroll
    for (uint32_t b = 0; b < kKeep; ++b)
#pragma unroll
      for (uint32_t u = 0; u < kBatch; ++u) acc += keep[b][u];
    for (uint32_t c = s0 + kKeep * 2 * kBatch; c < s1; c += 2 * kBatch) {
      uint32_t vs[kBatch];
      load_batch(c, vs);
#pragma unroll
      for (uint32_t u = 0; u < kBatch; ++u) acc += vs[u];
    }
    acc += __shfl_xor(acc, 32, 64);
    if (half == 0) s_tot[wave][g] = acc;
  }
  __syncthreads();
  uint32_t run = 0, total = 0;
  for (uint32_t w = 0; w < kWideWaves; ++w) {
    const uint32_t t = s_tot[w][g];
    if (w < wave) run += t;
    total += t;
  }
  // The first and the last word of a (chunk, group) record run [b, e); a consistent selection
  // never passes the planned size, and the test keeps the two stores inside the group's
  // payload even if an internal check has failed.
  auto clear_edges = [&](uint32_t b, uint32_t e) {
    if (half == 0 && e > b && e <= P) {
      const uint64_t bit0 = (uint64_t)b * W, bit1 = (uint64_t)e * W;
      stream[s_payload[g] + (uint32_t)(bit0 >> 5)] = 0;
      stream[s_payload[g] + (uint32_t)((bit1 - 1) >> 5)] = 0;
    }
  };
  uint32_t chunk_begin = run;
  auto prefix_batch = [&](uint32_t c, const uint32_t (&vs)[kBatch]) {
#pragma unroll
    for (uint32_t u = 0; u < kBatch; ++u) {
      const uint32_t cp = c + 2 * u;  // the pair's first span
      if (cp >= s1) break;            // uniform
      if (cp % kChunkSpans == 0 && cp > s0) {
        clear_edges(chunk_begin, run);
        chunk_begin = run;
      }
      const uint32_t v = vs[u], other = __shfl_xor(v, 32, 64);
      if (cp + half < s1) cnt[(size_t)(cp + half) * 32 + g] = half ? run + other : run;
      run += v + other;
    }
  };
#pragma unroll
  for (uint32_t b = 0; b < kKeep; ++b)
    if (s0 + b * 2 * kBatch < s1) prefix_batch(s0 + b * 2 * kBatch, keep[b]);  // uniform
  for (uint32_t c = s0 + kKeep * 2 * kBatch; c < s1; c += 2 * kBatch) {
    uint32_t vs[kBatch];
    load_batch(c, vs);
    prefix_batch(c, vs);
  }
  if (s1 > s0) clear_edges(chunk_begin, run);
  if (wave == 0 && half == 0) {
    cnt[(size_t)n_spans * 32 + g] = total;
    if (g < R && total != P) atomicOr(ws.status, CVLC_DEV_INTERNAL);
  }
  // energy of the coordinates the filter dropped
  double acc = tail0 + tail1;
  for (uint32_t t = tid + 2u * kWideBlock; t < ws.n_regions; t += kWideBlock) acc += rsq[t];
  acc = wave_sum_f64(acc);
  if (lane == 0) s_tail[wave] = acc;
  __syncthreads();

  if (tid < R) {
    const uint32_t r = tid;
    const uint32_t P = p.Z[r] - (r ? p.Z[r - 1] : 0u);
    float m = 0.0f, M = 0.0f;
    if (P > 0 && enc_max != 0) {
      M = from_ordered_bits(enc_max);
      m = from_ordered_bits(~enc_negmin);
    } else if (P > 0) {
      atomicOr(ws.status, CVLC_DEV_INTERNAL);
    }
    if (!(fabsf(M - m) <= 3.4028234664e38f)) atomicOr(ws.status, CVLC_DEV_NONFINITE);
    float norm = 0.0f;
    if (quant == CVLC_QUANT_QSGD) {
      // carry the 64-bit counters into 32-bit limbs, then look for the smallest fp32 value whose
      // square reaches the sum: squares grow with the bit pattern, so a binary search over it
      const unsigned long long* src = ws.norm_limbs + ((size_t)client * 32 + r) * kNormLimbs;
      unsigned long long carry = 0;
      int top = -1;  // highest limb that is not zero
      for (uint32_t i = 0; i < kNormLimbs; ++i) {
        const unsigned long long t = src[i] + carry;
        s_sum[r][i] = (uint32_t)t;
        if ((uint32_t)t) top = (int)i;
        carry = t >> 32;
      }
      auto reaches = [&](uint32_t key) {  // key^2 >= sum, compared limb by limb from the top
        const SquareLimbs sl = square_limbs(key);
        const int from = max(top, (int)sl.word + 2);
        for (int i = from; i >= 0; --i) {
          const uint32_t j = (uint32_t)i - sl.word;  // wraps to a large value below sl.word
          const uint32_t mine = j < 3u ? sl.part[j] : 0u;
          const uint32_t theirs = s_sum[r][i];
          if (mine != theirs) return mine > theirs;
        }
        return true;
      };
      uint32_t lo = 0, hi = 0x7F7FFFFFu;
      if (!reaches(hi)) {
        atomicOr(ws.status, CVLC_DEV_NONFINITE);  // the norm overflows fp32
        lo = hi;
      } else if (top >= 0) {
        // a floating-point estimate from the three top limbs brackets the answer within a few
        // patterns; the exact comparison decides, and the full range stays as the fallback
        double head = (double)s_sum[r][top];
        if (top >= 1) head = head * 4294967296.0 + (double)s_sum[r][top - 1];
        if (top >= 2) head = head * 4294967296.0 + (double)s_sum[r][top - 2];
        const float guess = (float)sqrt(ldexp(head, 32 * (top - (top >= 2 ? 2 : top)) - 298));
        const uint32_t g = min(__float_as_uint(guess), 0x7F7FFFFFu);
        const uint32_t glo = g > 2u ? g - 2u : 0u, ghi = g < 0x7F7FFFFDu ? g + 2u : 0x7F7FFFFFu;
        if (reaches(ghi) && (glo == 0u || !reaches(glo - 1u))) {
          lo = glo;
          hi = ghi;
        }
      } else {
        hi = 0;  // an all-zero group
      }
      while (lo < hi) {
        const uint32_t mid = lo + (hi - lo) / 2u;
        if (reaches(mid)) hi = mid; else lo = mid + 1u;
      }
      norm = __uint_as_float(lo);
    }
    GlobalWordPtr hdr = stream + kGlobalHeaderWords + kSegHeaderWords * r;
    hdr[0] = p.y[r];
    hdr[1] = P;
    hdr[2] = quant == CVLC_QUANT_QSGD ? __float_as_uint(norm) : __float_as_uint(m);
    hdr[3] = quant == CVLC_QUANT_QSGD ? 0u : __float_as_uint(M);
    if (stats_out) {
      cvlc_seg_stats_t* st = stats_out + (size_t)client * kStatsStride + r;
      st->min = m; st->max = M; st->sumsq = ctl->seg_sumsq[r]; st->count = P; st->reserved = 0;
      st->errsq = 0.0;  // the pack kernel adds the group's error energy when asked to
    }
    GroupInfo* gi = ws.group_info + client;
    float step, inv;
    if (quant == CVLC_QUANT_QSGD) {  // levels 0 .. s on [0, norm]: the same spacing rule with s = 2^(y-1) - 1 steps
      centroid_spacing(0.0f, norm, p.y[r] == 32 ? 1u : p.y[r] - 1u, &step, &inv);
      m = 0.0f;
    } else {
      centroid_spacing(m, M, p.y[r] == 32 ? 1u : p.y[r], &step, &inv);
    }
    gi->payload[r] = s_payload[r];
    gi->P[r] = P;
    gi->W[r] = sbits + p.y[r];
    gi->y[r] = p.y[r];
    gi->m[r] = m;
    gi->inv[r] = inv;
    gi->step[r] = step;
  }
  if (tid == 32) {
    stream[0] = kMagic;
    stream[1] = kVersion | (quant << 16);
    stream[2] = ws.d;
    stream[3] = R;
    stream[4] = sbits;
    stream[5] = __float_as_uint(p.B);
    stream[6] = p.client_id;
    stream[7] = p.total_words;
    if (stats_out) {
      double tail = 0.0;
      for (uint32_t w = 0; w < kWideWaves; ++w) tail += s_tail[w];
      cvlc_seg_stats_t* st = stats_out + (size_t)client * kStatsStride + R;
      st->min = 0.0f; st->max = 0.0f; st->sumsq = tail + ctl->seg_sumsq[R]; st->count = ws.d - p.k; st->reserved = 0;
      st->errsq = st->sumsq;  // dropped whole
    }
  }
}

// ------------------------------------------------------------------ 8. emit: quantise + pack
// a ^ b ^ c in one instruction (three-operand bitwise op with the truth table of the parity).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32-10 (Salmon et al., SC'11), first output word.
__device__ __forceinline__ uint32_t philox_word0(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1) {
  uint32_t c2 = 0, c3 = 0;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    c0 = xor3(hi1, c1, k0);
    c1 = lo1;
    c2 = xor3(hi0, c3, k1);
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}

// Unbiased rounding to one of 2^y uniform centroids on [m, M] (PQ): position
// t = (x - m) * inv in fp32, lower centroid floor(t), one up with probability
// frac(t) resolved against a 24-bit uniform.
__device__ __forceinline__ uint32_t quantise(float x, float m, float inv, uint32_t y, uint32_t u24) {
  const float top = (float)((1u << y) - 1u);
  float t = __fmul_rn(__fsub_rn(x, m), inv);
  if (!(t > 0.0f)) t = 0.0f;
  if (t > top) t = top;
  const float fl = floorf(t);
  const uint32_t j = (uint32_t)fl;
  const float frac = __fsub_rn(t, fl);
  const uint32_t thr = (uint32_t)__fmul_rn(frac, 16777216.0f);
  const uint32_t cid = j + (u24 < thr ? 1u : 0u);
  const uint32_t last = (1u << y) - 1u;
  return cid > last ? last : cid;
}




constexpr uint32_t kChunkCands = kSpan * kChunkSpans;         // 4096
constexpr uint32_t kEdgeChunks = 8;                           // chunks whose shared stream words a workgroup holds back
constexpr uint32_t kStageWords = kChunkCands * 2 + 2 * 32;    // every record is < 64 bits; two edge words per group

struct alignas(16) EmitGroup {  // per (chunk, group)
  uint32_t first, lim;   // the chunk's record run [first, lim) of the group
  uint32_t W, y;
  float m, inv;
  uint32_t stage_bit;    // bit of record `first` in the workgroup's staged image of the stream
  float step;            // centroid spacing (only read when the error energy is measured)
};

// One workgroup per chunk of 4096 candidates, one wavefront per span.  Every
// coded candidate gets its record number inside its group (members in earlier
// spans from the layout's prefix, plus its number inside the span, which the
// counting pass left with its group in 16 bits), is quantised and OR-ed into an
// LDS image of the stream words its group's run covers.  The image is then
// written out: a group's first and last word can be shared with a neighbouring
// chunk and are OR-ed into the (cleared) stream, all others are stored whole.
// ERR: every record also adds (xtilde / B - x)^2 to its group's error energy in
// the statistics block (Lemma 1's left side for this draw), xtilde being the
// centroid value the decoder will compute from the header.
// QSGD: the code is the level of |x| on [0, norm] with the sign bit above it.
template <bool ERR, bool QSGD>
__global__ __launch_bounds__(kEmitBlock, 6) void emit_kernel(const ClientParams* __restrict__ params,
                                                          ClientCtl* __restrict__ ctls, Workspace ws, uint64_t seed,
                                                          cvlc_seg_stats_t* __restrict__ stats_out) {
  __shared__ double s_err[ERR ? kEmitWaves : 1][32];  // per wavefront, per group
  __shared__ uint32_t s_stage[kStageWords];
  // A chunk's tables, two sets: the next chunk's are filled while the current one is written out.
  __shared__ uint32_t s_wrun[2][kEmitWaves][32];   // per wavefront, per group: record number of its span's first member
  __shared__ EmitGroup s_grp[2][32];               // what a record of the group needs, read as two 16-byte pieces
  __shared__ uint32_t s_word0[2][32];              // first stream word (group-relative) the chunk touches
  __shared__ uint32_t s_nwords[2][32];             // words the chunk touches in each group
  __shared__ uint32_t s_stage_off[2][33];
  __shared__ uint32_t s_payload[32];
  __shared__ uint32_t s_next;                      // the chunk the workgroup takes after the current one
  // The first and the last word of a (chunk, group) run are OR-ed into the stream by device-wide atomics.
  // Whatever the wavefront loads next waits for their acknowledgement (the counter of outstanding memory
  // operations does not tell loads from atomics), so they are held back, kEdgeChunks chunks' worth, and
  // issued together.
  __shared__ uint32_t s_edge_word[kEdgeChunks][32][2];  // the bits; 0: nothing to OR
  __shared__ uint32_t s_edge_at[kEdgeChunks][32][2];    // the stream word they belong to
  // Workgroups are dispatched in the order of their linear index and a CU serves its oldest first: the
  // clients' workgroups are interleaved in that order, so that every client has workgroups of every age.
  const uint32_t linear = blockIdx.y * gridDim.x + blockIdx.x;
  const uint32_t client = linear % gridDim.y, block_x = linear / gridDim.y;
  const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  if (ctl->dead) return;  // the workspace was too short for this client (whole workgroup)
  const uint32_t n = ctl->n_cand;
  const uint32_t n_spans = (n + kSpan - 1) / kSpan;
  const uint32_t R = p.R, sbits = position_bits(ws.d);
  const uint32_t* __restrict__ val = ws.dense_val + (size_t)client * ws.dense_cap;
  const uint32_t* __restrict__ idx = ws.dense_idx + (size_t)client * ws.dense_cap;
  const uint16_t* __restrict__ place = span_places(ws, client);
  const uint32_t* __restrict__ prefix = ws.span_cnt + (size_t)client * (ws.max_spans + 1) * 32;
  GlobalWordPtr stream = (GlobalWordPtr)p.stream;
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32), client_id = p.client_id;

  uint32_t my_P = 0, my_W = 0, my_y = 0;
  float my_m = 0.0f, my_inv = 0.0f, my_step = 0.0f;
  if (tid < 32 && tid < R) {
    const GroupInfo* gi = ws.group_info + client;
    my_P = gi->P[tid];
    my_W = gi->W[tid];
    my_y = gi->y[tid];
    my_m = gi->m[tid];
    my_inv = gi->inv[tid];
    my_step = gi->step[tid];
    s_payload[tid] = gi->payload[tid];
  }
  const double inv_B = ERR ? 1.0 / (double)p.B : 0.0;  // the scaling operation of Sec. IV-B
  if (ERR && lane < 32) s_err[wave][lane] = 0.0;       // touched by this wavefront only until the end
  auto chunk_exists = [&](uint32_t c) { return (uint64_t)c * kChunkSpans < n_spans; };
  // What a chunk needs of the layout's prefix: the record numbers the wavefront's span starts at (lanes
  // 0..31: one group each) and, for the first 32 threads, the chunk's record run of a group.
  uint32_t ahead_row = 0, ahead_first = 0, ahead_last = 0;
  auto ask_prefix = [&](uint32_t c) {
    if (!chunk_exists(c)) return;  // uniform
    const uint32_t span = c * kChunkSpans + wave;
    if (lane < 32) ahead_row = span < n_spans ? prefix[(size_t)span * 32 + lane] : 0u;
    if (tid < R && tid < 32) {
      const uint32_t last_span = min((c + 1) * kChunkSpans, n_spans);
      ahead_first = prefix[(size_t)c * kChunkSpans * 32 + tid];
      ahead_last = prefix[(size_t)last_span * 32 + tid];
    }
  };
  // Value bits, position and place of the candidates of the wavefront's span.  Unconditional loads (a
  // lane past the end reads the last candidate again), so that all of them are in flight together.
  uint32_t v[kPerLane], pid[kPerLane], plc[kPerLane];
  auto ask_candidates = [&](uint32_t c) {
    if (!chunk_exists(c)) return;  // uniform
#pragma unroll
    for (uint32_t j = 0; j < kPerLane; ++j) {
      const uint32_t i = (c * kChunkSpans + wave) * kSpan + j * kWave + lane;
      const uint32_t at = min(i, n - 1u);
      v[j] = val[at];
      pid[j] = idx[at];
      plc[j] = i < n ? (uint32_t)place[at] : (uint32_t)kNoPlace;
    }
  };
  // Fills set `to` of the chunk tables from what ask_prefix brought.
  auto set_up = [&](uint32_t to) {
    if (lane < 32) s_wrun[to][wave][lane] = ahead_row;
    if (tid < 32) {
      const uint32_t r = tid;
      uint32_t nwords = 0, W = 0, first = 0, last = 0, bit_in_word = 0;
      if (r < R) {
        const uint32_t P = my_P;
        W = my_W;
        // the chunk's record run of group r: [first, last), clamped so that every write stays inside
        // the group's payload even if an internal check has failed
        first = ahead_first;
        last = ahead_last;
        if (last > P) last = P;
        if (first > last) first = last;
        if (last > first) {
          const uint64_t bit0 = (uint64_t)first * W, bit1 = (uint64_t)last * W;
          s_word0[to][r] = (uint32_t)(bit0 >> 5);
          bit_in_word = (uint32_t)(bit0 & 31u);
          nwords = (uint32_t)(((bit1 - 1) >> 5) - (bit0 >> 5) + 1);
        }
      }
      s_nwords[to][r] = nwords;
      // exclusive prefix of the staged word counts over the groups
      const uint32_t incl = wave_incl_scan_u32(nwords);
      s_stage_off[to][r] = incl - nwords;
      if (r == 31) s_stage_off[to][32] = incl;
      EmitGroup eg;
      eg.first = first;
      eg.lim = last;
      eg.W = W;
      eg.y = my_y;
      eg.m = my_m;
      eg.inv = my_inv;
      eg.stage_bit = (incl - nwords) * 32u + bit_in_word;  // bit of record `first` in the staged image
      eg.step = my_step;
      s_grp[to][r] = eg;
    }
  };
  // Which chunks a workgroup takes: its own first, then whichever chunk of the client nobody has
  // taken yet (a counter of the client's), so that the workgroups of a CU, of which the oldest is served
  // first, all stay until the work runs out instead of leaving one after the other.  The next chunk is
  // claimed when the current one begins and known (through s_next) when its records are done.
  // A chunk goes through two phases with a barrier before each: the records (all wavefronts OR into the
  // staged image); write the image out, leaving zeros behind.  The next chunk's candidates and prefix
  // are requested before the current chunk is written out, its tables filled after.
  for (uint32_t i = tid; i < kEdgeChunks * 64u; i += kEmitBlock) (&s_edge_word[0][0][0])[i] = 0;  // groups past R stay 0
  uint32_t held = 0;  // chunks whose edge words are held back
  auto release_edges = [&]() {  // by the whole workgroup, after a barrier
    for (uint32_t i = tid; i < held * 64u; i += kEmitBlock) {
      const uint32_t word = (&s_edge_word[0][0][0])[i];
      if (word) atomicOr((uint32_t*)(stream + (&s_edge_at[0][0][0])[i]), word);
    }
  };
  ask_prefix(block_x);
  ask_candidates(block_x);
  for (uint32_t i = tid; i < kStageWords; i += kEmitBlock) s_stage[i] = 0;
  set_up(0);
  uint32_t cur = 0;
  for (uint32_t c = block_x; chunk_exists(c); cur ^= 1u) {
    uint32_t claimed = 0;
    if (tid == 0) claimed = atomicAdd(&ctl->emit_claim, 1u);
    __syncthreads();  // the chunk before is written out (and its image cleared); this chunk's tables are in place
    const uint32_t* wrun = s_wrun[cur][wave];
#pragma unroll
    for (uint32_t j = 0; j < kPerLane; ++j) {
      if (plc[j] != kNoPlace) {
        const uint32_t g = plc[j] & ((1u << kPlaceShift) - 1u);
        const uint32_t e = wrun[g] + (plc[j] >> kPlaceShift);
        const EmitGroup eg = s_grp[cur][g];
        if (e < eg.lim) {
          const uint32_t y = eg.y, W = eg.W;
          uint32_t cid;
          if (y == 32) {
            cid = v[j];
          } else {
            const uint32_t u24 = philox_word0(pid[j], client_id, k0, k1) >> 8;
            if (QSGD)
              cid = quantise(fabsf(__uint_as_float(v[j])), 0.0f, eg.inv, y - 1u, u24) | ((v[j] >> 31) << (y - 1u));
            else
              cid = quantise(__uint_as_float(v[j]), eg.m, eg.inv, y, u24);
          }
          if (ERR) {
            const float x = __uint_as_float(v[j]);
            float xt = x;
            if (y != 32) {
              if (QSGD) {
                const float mag = __fmaf_rn((float)(cid & ((1u << (y - 1u)) - 1u)), eg.step, 0.0f);
                xt = (cid >> (y - 1u)) ? -mag : mag;
              } else {
                xt = __fmaf_rn((float)cid, eg.step, eg.m);
              }
            }
            const double err = (double)xt * inv_B - (double)x;
            atomicAdd(&s_err[wave][g], err * err);
          }
          const uint64_t record = (uint64_t)pid[j] | ((uint64_t)cid << sbits);
          // a chunk's run of a group is at most 4096 records of at most 63 bits: 32 bits hold the offset
          const uint32_t bit = eg.stage_bit + __umul24(e - eg.first, W);
          const uint32_t w0 = bit >> 5, sh = bit & 31u;
          const uint64_t lo = record << sh;
          atomicOr(&s_stage[w0], (uint32_t)lo);
          if (sh + W > 32u) atomicOr(&s_stage[w0 + 1], (uint32_t)(lo >> 32));
          if (sh + W > 64u) atomicOr(&s_stage[w0 + 2], (uint32_t)(record >> (64u - sh)));
        }
      }
    }
    if (tid == 0) s_next = gridDim.x + claimed;
    __syncthreads();
    const uint32_t c_next = s_next;
    ask_prefix(c_next);
    ask_candidates(c_next);
    // A wavefront writes whole groups' runs, lane l the l-th, l+64-th, ... word (with all 512 threads on one
    // group after the other most lanes had nothing to write in every group).  A group's size changes steadily
    // with its number, so the groups are dealt out going up and coming down in turn (wavefront w: w, 15 - w,
    // 16 + w, 31 - w).
    for (uint32_t k = 0; k * kEmitWaves < R; ++k) {
      const uint32_t g = k * kEmitWaves + ((k & 1u) ? kEmitWaves - 1u - wave : wave);
      if (g >= R) continue;  // uniform per wavefront
      const uint32_t nwords = s_nwords[cur][g];
      uint32_t* staged_words = s_stage + s_stage_off[cur][g];
      const uint32_t first_word = s_payload[g] + s_word0[cur][g];
      GlobalWordPtr dst = stream + first_word;
      if (lane < 2) s_edge_word[held][g][lane] = 0;  // (this wavefront's LDS accesses complete in order)
      for (uint32_t rel = lane; rel < nwords; rel += kWave) {
        const uint32_t word = staged_words[rel];
        staged_words[rel] = 0;  // the image is all zeros again when the next chunk begins
        if (rel == 0 || rel == nwords - 1) {
          const uint32_t which = rel == 0 ? 0u : 1u;
          s_edge_word[held][g][which] = word;
          s_edge_at[held][g][which] = first_word + rel;
        } else {
          dst[rel] = word;
        }
      }
    }
    set_up(cur ^ 1u);  // the next chunk's tables (after the last chunk: tables nobody reads)
    c = c_next;
    if (++held == kEdgeChunks) {  // uniform
      __syncthreads();
      release_edges();
      held = 0;
    }
  }  // chunks
  __syncthreads();
  release_edges();
  if (ERR) {
    __syncthreads();
    if (tid < R) {
      double sum = 0.0;
      for (uint32_t w = 0; w < kEmitWaves; ++w) sum += s_err[w][tid];
      if (sum != 0.0) atomicAdd(&stats_out[(size_t)client * kStatsStride + tid].errsq, sum);
    }
  }
}

// ------------------------------------------------------------------ host side
// Candidates per client a workspace of ws_bytes has room for: the largest cap <= d whose layout fits (the
// layout grows with cap), 0 if not even one does.
uint32_t candidate_room(uint32_t d, uint32_t n, size_t ws_bytes) {
  if (encode_layout(d, n, 1u).total > ws_bytes) return 0u;
  uint32_t lo = 1u, hi = d;  // lo fits
  while (lo < hi) {
    const uint32_t mid = lo + (hi - lo + 1u) / 2u;
    if (encode_layout(d, n, mid).total <= ws_bytes) lo = mid; else hi = mid - 1u;
  }
  return lo;
}

int validate_batch(uint32_t n, const cvlc_plan_t* plans, const float* const* d_updates,
                   const uint32_t* client_ids, void* const* d_streams, const size_t* capacities,
                   void* d_workspace, size_t ws_bytes) {
  if (n == 0 || !plans || !d_updates || !client_ids || !d_streams || !capacities || !d_workspace) return CVLC_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(d_workspace) % 256u) return CVLC_ERR_ARG;
  if (n > 65535u) return CVLC_ERR_ARG;  // clients index the grid's y dimension
  const uint32_t d = plans[0].d;
  for (uint32_t i = 0; i < n; ++i) {
    const int rc = cvlc_plan_validate(&plans[i]);
    if (rc) return rc;
    if (plans[i].d != d) return CVLC_ERR_ARG;
    if (!d_updates[i] || reinterpret_cast<uintptr_t>(d_updates[i]) % 16u) return CVLC_ERR_ARG;
    if (!d_streams[i] || reinterpret_cast<uintptr_t>(d_streams[i]) % 4u) return CVLC_ERR_ARG;
    if (capacities[i] < cvlc_stream_capacity(&plans[i])) return CVLC_ERR_CAPACITY;
    if (plans[i].total_bits / 32u > 0xFFFFFFFFull) return CVLC_ERR_PLAN;
  }
  uint32_t k_max = 0;
  for (uint32_t i = 0; i < n; ++i) {
    uint64_t k = 0;
    for (uint32_t r = 0; r < plans[i].n_coded; ++r) k += plans[i].count[r];
    if (k > k_max) k_max = (uint32_t)k;  // a valid plan keeps at most d
  }
  if (candidate_room(d, n, ws_bytes) < (k_max < 1 ? 1u : k_max)) return CVLC_ERR_CAPACITY;
  return CVLC_OK;
}

// Rank inside the sample at which the candidate threshold is read: the expected
// number of sampled coordinates inside the top k, plus six standard deviations
// of that count and a small constant.  0 = do not sample, keep every coordinate.
uint32_t sample_rank(uint32_t d, uint32_t k, uint32_t n_sampled) {
  if (n_sampled == 0) return 0u;
  const double expect = (double)k * (double)n_sampled / (double)d;
  const double want = std::ceil(expect + 6.0 * std::sqrt(expect) + 16.0);
  if (want >= (double)n_sampled) return 0u;
  return (uint32_t)want;
}

// Filter workgroups the current device holds at once, at most kFilterBlocksCap.
uint32_t filter_resident_blocks() {
  static uint32_t cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return kFilterBlocksCap / 2;
  if (cached[dev] == 0) {
    int cus = 0, per_cu = 0;
    uint32_t r = kFilterBlocksCap / 2;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, filter_kernel, kBlock, 0) == hipSuccess && cus > 0 &&
        per_cu > 0)
      r = (uint32_t)cus * (uint32_t)per_cu;
    cached[dev] = r > kFilterBlocksCap ? kFilterBlocksCap : r;
  }
  return cached[dev];
}

}  // namespace
}  // namespace cvlc

extern "C" {

size_t cvlc_encode_workspace_bytes(uint32_t d, uint32_t n_clients) {
  if (d < 1 || n_clients < 1) return 0;
  return cvlc::encode_layout(d, n_clients, d).total;
}

size_t cvlc_encode_workspace_bytes_for(uint32_t d, uint32_t n_clients, uint32_t max_candidates) {
  if (d < 1 || n_clients < 1) return 0;
  return cvlc::encode_layout(d, n_clients, max_candidates < 1 ? 1u : max_candidates).total;
}

uint32_t cvlc_plan_candidates_hint(const cvlc_plan_t* plan) {
  using namespace cvlc;
  if (!plan || cvlc_plan_validate(plan) != CVLC_OK) return 0;
  const uint32_t d = plan->d;
  uint64_t k = 0;
  for (uint32_t r = 0; r < plan->n_coded; ++r) k += plan->count[r];
  const uint32_t n_src = d / kSamplePiece;
  const uint32_t n_sampled = (n_src < kSampleChunksMax ? n_src : kSampleChunksMax) * kSamplePiece;
  const uint32_t rank = sample_rank(d, (uint32_t)k, n_sampled);
  if (rank == 0) return d;  // no threshold is sampled for this plan: every coordinate is a candidate
  // The share of the vector at or above the sample's rank-th largest key is rank / n_sampled give or take
  // sqrt(rank) / n_sampled; the threshold is that key rounded down to 13 bits, worth a few percent more.
  const double share = ((double)rank + 6.0 * std::sqrt((double)rank) + 16.0) / (double)n_sampled;
  const double want = std::ceil(1.25 * share * (double)d) + 4096.0;
  return want >= (double)d ? d : (uint32_t)want;
}

int cvlc_encode_batch(uint32_t n, const cvlc_plan_t* plans, const float* const* d_updates, uint64_t seed,
                      const uint32_t* client_ids, void* const* d_streams_out, const size_t* capacities,
                      void* d_workspace, size_t ws_bytes, cvlc_seg_stats_t* d_stats_out, uint32_t flags,
                      void* hip_stream) {
  using namespace cvlc;
  int rc = validate_batch(n, plans, d_updates, client_ids, d_streams_out, capacities, d_workspace, ws_bytes);
  if (rc) return rc;
  if (flags & ~CVLC_ENCODE_ERROR_STATS) return CVLC_ERR_ARG;
  const uint32_t quant = plans[0].quant;
  for (uint32_t i = 1; i < n; ++i)
    if (plans[i].quant != quant) return CVLC_ERR_ARG;
  if ((flags & CVLC_ENCODE_ERROR_STATS) && !d_stats_out) return CVLC_ERR_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const uint32_t d = plans[0].d;
  const EncodeLayout L = encode_layout(d, n, candidate_room(d, n, ws_bytes));
  char* base = static_cast<char*>(d_workspace);
  Workspace ws;
  ws.status = reinterpret_cast<uint32_t*>(base + L.status);
  ws.params = reinterpret_cast<ClientParams*>(base + L.params);
  ws.ctl = reinterpret_cast<ClientCtl*>(base + L.ctl);
  ws.region_cnt = reinterpret_cast<uint32_t*>(base + L.region_cnt);
  ws.region_sumsq = reinterpret_cast<double*>(base + L.region_sumsq);
  ws.cand_idx = reinterpret_cast<uint16_t*>(base + L.cand_idx);
  ws.cand_val = reinterpret_cast<uint32_t*>(base + L.cand_val);
  ws.dense_idx = reinterpret_cast<uint32_t*>(base + L.dense_idx);
  ws.dense_val = reinterpret_cast<uint32_t*>(base + L.dense_val);
  ws.nz_off = reinterpret_cast<uint32_t*>(base + L.nz_off);
  ws.nz_run = reinterpret_cast<uint32_t*>(base + L.nz_run);
  ws.span_first = reinterpret_cast<uint32_t*>(base + L.span_first);
  ws.span_cnt = reinterpret_cast<uint32_t*>(base + L.span_cnt);
  ws.group_info = reinterpret_cast<GroupInfo*>(base + L.group_info);
  ws.tie_list = reinterpret_cast<uint2*>(base + L.tie_list);
  ws.sel_part = reinterpret_cast<uint32_t*>(base + L.sel_part);
  ws.l3_hist = reinterpret_cast<uint32_t*>(base + L.l3_hist);
  ws.norm_limbs = reinterpret_cast<unsigned long long*>(base + L.norm_limbs);
  ws.d = d;
  ws.n_regions = L.n_regions;
  ws.max_spans = L.max_spans;
  ws.dense_cap = L.dense_cap;
  ws.filter_blocks = filter_blocks_per_client(L.n_regions, n, filter_resident_blocks());
  ws.sel_blocks = L.sel_blocks;

  // sample geometry: 256-byte pieces spread evenly; all of them when the vector is short
  const uint32_t n_src = d / kSamplePiece;
  const uint32_t n_s = n_src < kSampleChunksMax ? n_src : kSampleChunksMax;

  profile_mark(CVLC_STAGE_ENC_SETUP, true, stream);
  // the status word, the control blocks and the level-3 table start every call at zero
  uint32_t zero_n16 = (uint32_t)(L.zero_bytes / 16u);  // n <= 65535 clients: below 2^32 pieces

  // per-client parameters, shipped as kernel arguments
  uint32_t max_R = 0;
  bool any_sampled = false;
  {
    UploadChunk chunk;
    chunk.n_clients = 0;
    chunk.first_client = 0;
    chunk.n_templates = 0;
    chunk.pad = 0;
    uint32_t refs[kUploadWords];  // the chunk's references, appended behind its templates when it is sent
    auto send = [&]() {
      std::memcpy(&chunk.data[chunk.n_templates * kParamWords], refs, (size_t)chunk.n_clients * kRefWords * 4u);
      const uint32_t blocks = zero_n16 ? (zero_n16 + 1023u) / 1024u : 1u;
      hipLaunchKernelGGL(upload_kernel, dim3(blocks < 512u ? blocks : 512u), dim3(256), 0, stream,
                         reinterpret_cast<uint32_t*>(ws.params), chunk, reinterpret_cast<uint4*>(base + L.status),
                         zero_n16);
      zero_n16 = 0;  // cleared by the first launch
      chunk.first_client += chunk.n_clients;
      chunk.n_clients = 0;
      chunk.n_templates = 0;
    };
    for (uint32_t i = 0; i < n; ++i) {
      const cvlc_plan_t& pl = plans[i];
      ClientParams cp;
      std::memset(&cp, 0, sizeof(cp));  // pointers and client id stay out of the template
      cp.R = pl.n_coded;
      cp.total_words = (uint32_t)(pl.total_bits / 32u);
      cp.B = pl.B;
      uint32_t z = 0;
      for (uint32_t r = 0; r < pl.n_coded; ++r) {
        z += pl.count[r];
        cp.Z[r] = z;
        cp.y[r] = (uint8_t)pl.code_len[r];
      }
      cp.k = z;
      cp.sample_rank = sample_rank(d, z, n_s * kSamplePiece);
      any_sampled |= cp.sample_rank != 0;
      if (pl.n_coded > max_R) max_R = pl.n_coded;
      for (int attempt = 0; attempt < 2; ++attempt) {
        uint32_t t = 0;
        while (t < chunk.n_templates && std::memcmp(&chunk.data[t * kParamWords], &cp, sizeof(cp)) != 0) ++t;
        const uint32_t templates = t == chunk.n_templates ? t + 1 : chunk.n_templates;
        if (templates * kParamWords + (chunk.n_clients + 1) * kRefWords > kUploadWords) {
          send();  // no room: this client opens the next chunk (which always has room for one)
          continue;
        }
        if (t == chunk.n_templates) {
          std::memcpy(&chunk.data[t * kParamWords], &cp, sizeof(cp));
          chunk.n_templates = templates;
        }
        uint32_t* ref = refs + chunk.n_clients * kRefWords;
        const uint64_t up = reinterpret_cast<uint64_t>(d_updates[i]), sp = reinterpret_cast<uint64_t>(d_streams_out[i]);
        ref[0] = (uint32_t)up;
        ref[1] = (uint32_t)(up >> 32);
        ref[2] = (uint32_t)sp;
        ref[3] = (uint32_t)(sp >> 32);
        ref[4] = client_ids[i];
        ref[5] = t;
        ++chunk.n_clients;
        break;
      }
    }
    if (chunk.n_clients) send();
  }
  profile_mark(CVLC_STAGE_ENC_SETUP, false, stream);

  if (any_sampled) {
    StageScope scope(CVLC_STAGE_ENC_SAMPLE, stream);
    // n_src < 2^26 and n_s <= 2^12: the step is below 2^58 / n_s and j * step below 2^58
    hipLaunchKernelGGL(sample_hist_kernel, dim3(kSampleBlocks, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, n_s,
                       n_s ? ((uint64_t)n_src << 32) / n_s : 0u);
    hipLaunchKernelGGL(sample_walk_kernel, dim3(n), dim3(kWideBlock), 0, stream, ws.params, ws.ctl);
  }
  {
    StageScope scope(CVLC_STAGE_ENC_FILTER, stream);
    hipLaunchKernelGGL(filter_kernel, dim3(ws.filter_blocks, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, ws);
  }
  {
    StageScope scope(CVLC_STAGE_ENC_REFILTER, stream);
    hipLaunchKernelGGL(scan_l1_kernel, dim3(n), dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws);
  }
  {
    StageScope scope(CVLC_STAGE_ENC_SELECT, stream);
    const dim3 grid(L.sel_blocks, n);
    // The gather also builds the dense candidate list (also when nothing is coded).  Up to 15 boundaries:
    // 60 KB of LDS counters, two workgroups to a CU.  More: all of them in one round of launches with
    // 124 KB of counters, one workgroup to a CU, instead of three rounds over the candidates.
    if (max_R <= kSlotGroup) {
      constexpr uint32_t SG = kSlotGroup;
      hipLaunchKernelGGL(gather_l2_kernel<SG>, grid, dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws);
      hipLaunchKernelGGL((select_walk_kernel<2, SG>), dim3(SG, n), dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws);
      hipLaunchKernelGGL(select_pass3_kernel<SG>, grid, dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws);
      hipLaunchKernelGGL((select_walk_kernel<3, SG>), dim3(SG, n), dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws);
    } else {
      constexpr uint32_t SG = kSlotGroupWide;
      hipLaunchKernelGGL(gather_l2_kernel<SG>, grid, dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws);
      hipLaunchKernelGGL((select_walk_kernel<2, SG>), dim3(SG, n), dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws);
      hipLaunchKernelGGL(select_pass3_kernel<SG>, grid, dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws);
      hipLaunchKernelGGL((select_walk_kernel<3, SG>), dim3(SG, n), dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws);
    }
  }
  // count: wavefronts walk the spans; about what the device holds at once (four workgroups per CU)
  uint32_t g_count = (1024u + n - 1) / n;
  if (g_count > (L.max_spans + kEmitWaves - 1) / kEmitWaves) g_count = (L.max_spans + kEmitWaves - 1) / kEmitWaves;
  {
    StageScope scope(CVLC_STAGE_ENC_CLASSIFY, stream);
    if (quant == CVLC_QUANT_QSGD)
      hipLaunchKernelGGL(count_kernel<true>, dim3(g_count, n), dim3(kEmitBlock), 0, stream, ws.params, ws.ctl, ws);
    else
      hipLaunchKernelGGL(count_kernel<false>, dim3(g_count, n), dim3(kEmitBlock), 0, stream, ws.params, ws.ctl, ws);
  }
  {
    StageScope scope(CVLC_STAGE_ENC_LAYOUT, stream);
    hipLaunchKernelGGL(layout_kernel, dim3(n), dim3(kWideBlock), 0, stream, ws.params, ws.ctl, ws, d_stats_out, quant);
  }
  {
    // emit: workgroups walk the chunks; about what the device holds at once (three per CU)
    StageScope scope(CVLC_STAGE_ENC_EMIT, stream);
    uint32_t g_emit = (768u + n - 1) / n;
    const uint32_t max_chunks = (L.max_spans + kChunkSpans - 1) / kChunkSpans;
    if (g_emit > max_chunks) g_emit = max_chunks;
    const bool err = flags & CVLC_ENCODE_ERROR_STATS, qsgd = quant == CVLC_QUANT_QSGD;
    auto kernel = err ? (qsgd ? emit_kernel<true, true> : emit_kernel<true, false>)
                      : (qsgd ? emit_kernel<false, true> : emit_kernel<false, false>);
    hipLaunchKernelGGL(kernel, dim3(g_emit, n), dim3(kEmitBlock), 0, stream, ws.params, ws.ctl, ws, seed, d_stats_out);
  }
  return hip_check(hipGetLastError());
}

int cvlc_encode(const cvlc_plan_t* plan, const float* d_update, uint64_t seed, uint32_t client_id,
                void* d_stream_out, size_t capacity, void* d_workspace, size_t ws_bytes,
                cvlc_seg_stats_t* d_stats_out, uint32_t flags, void* hip_stream) {
  if (!plan) return CVLC_ERR_ARG;
  const float* updates[1] = {d_update};
  void* streams[1] = {d_stream_out};
  return cvlc_encode_batch(1, plan, updates, seed, &client_id, streams, &capacity, d_workspace, ws_bytes,
                           d_stats_out, flags, hip_stream);
}

int cvlc_device_status(const void* d_workspace, void* hip_stream, uint32_t* status_out) {
  if (!d_workspace || !status_out) return CVLC_ERR_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int rc = cvlc::hip_check(hipStreamSynchronize(stream));
  if (rc) return rc;
  return cvlc::hip_check(hipMemcpy(status_out, d_workspace, sizeof(uint32_t), hipMemcpyDeviceToHost));
}

}  // extern "C"
