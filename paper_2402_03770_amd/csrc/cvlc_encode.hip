// Encoder of libcvlc for gfx950: one client's update vector -> one
// variable-length stream (Sec. IV-B sparsification + quantisation, the final
// loop of Algorithm 1, packet format of Sec. IV-D).
//
// The paper ranks all d updates; here the ranking is never materialised.  The
// kernels find, for every group boundary Z_r, the exact Z_r-th largest
// magnitude (radix-histogram selection) and classify coordinates against those
// thresholds, which yields the same groups as a full sort with ties broken by
// position.  Launch chain per batch of clients:
//   sample_hist   strided sample of |U| -> conservative candidate threshold
//   filter        the one full pass over U: keep coordinates above the
//                 threshold, in position order (decoupled look-back scan)
//   select_l1/l23 three histogram levels (11+10+10 key bits) over the
//                 candidates -> exact boundary keys and tie quotas
//   tie_resolve   where a boundary cuts a class of equal magnitudes, the
//                 position of the last member inside the boundary
//   classify      per chunk: group of every candidate, per-group count,
//                 min/max/sum of squares
//   layout        prefix of the per-chunk counts, headers, statistics
//   emit          stochastic rounding (Philox4x32-10) and bit packing
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>

#include "cvlc_common.h"

namespace cvlc {
namespace {

// ------------------------------------------------------------------ workspace layout
struct EncodeLayout {
  size_t status, params, ctl, tile_state, tile_sumsq, cand_idx, cand_val, chunk_cnt, chunk_sumsq, total;
  size_t zero_begin, zero_end;  // [ctl, tile_state] is cleared at the start of a call
  uint32_t n_tiles, max_chunks;
};

size_t align256(size_t v) { return (v + 255u) & ~(size_t)255u; }

EncodeLayout encode_layout(uint32_t d, uint32_t n) {
  EncodeLayout L;
  L.n_tiles = (uint32_t)(((uint64_t)d + kTile - 1) / kTile);
  L.max_chunks = (uint32_t)(((uint64_t)d + kChunk - 1) / kChunk);
  size_t off = 0;
  L.status = off; off = align256(off + 256);
  L.params = off; off = align256(off + (size_t)n * sizeof(ClientParams));
  L.ctl = off; L.zero_begin = off; off = align256(off + (size_t)n * sizeof(ClientCtl));
  L.tile_state = off; off = align256(off + (size_t)n * 2 * L.n_tiles * sizeof(uint64_t));
  L.zero_end = off;
  L.tile_sumsq = off; off = align256(off + (size_t)n * L.n_tiles * sizeof(double));
  L.cand_idx = off; off = align256(off + (size_t)n * d * sizeof(uint32_t));
  L.cand_val = off; off = align256(off + (size_t)n * d * sizeof(float));
  L.chunk_cnt = off; off = align256(off + (size_t)n * L.max_chunks * 32 * sizeof(uint32_t));
  L.chunk_sumsq = off; off = align256(off + (size_t)n * L.max_chunks * 32 * sizeof(double));
  L.total = off;
  return L;
}

struct Workspace {  // device pointers into the caller's workspace
  uint32_t* status;
  ClientParams* params;
  ClientCtl* ctl;
  uint64_t* tile_state;
  double* tile_sumsq;
  uint32_t* cand_idx;
  float* cand_val;
  uint32_t* chunk_cnt;
  double* chunk_sumsq;
  uint32_t d, n_tiles, max_chunks;
};

// ------------------------------------------------------------------ parameter upload
constexpr uint32_t kUploadWords = 960;
struct UploadChunk {
  uint32_t n_words, dst_word;
  uint32_t data[kUploadWords];
};

__global__ void upload_kernel(uint32_t* dst, UploadChunk c) {
  for (uint32_t i = threadIdx.x; i < c.n_words; i += blockDim.x) dst[c.dst_word + i] = c.data[i];
}

// ------------------------------------------------------------------ small device helpers
__device__ __forceinline__ uint32_t final_ncand(const ClientCtl* ctl, const ClientParams& p) {
  const uint32_t n0 = ctl->n_cand[0];
  return n0 >= p.k ? n0 : ctl->n_cand[1];
}
__device__ __forceinline__ uint32_t final_pass(const ClientCtl* ctl, const ClientParams& p) {
  return ctl->n_cand[0] >= p.k ? 0u : 1u;
}

// Exclusive prefix sum of one value per thread over the workgroup (kBlock threads),
// in thread order; *total receives the sum.  `scratch` holds kWavesPerBlock words.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* scratch, uint32_t* total) {
  const uint32_t incl = wave_incl_scan_u32(v);
  __syncthreads();
  if (lane_id() == kWave - 1) scratch[wave_id()] = incl;
  __syncthreads();
  uint32_t before = 0, sum = 0;
#pragma unroll
  for (uint32_t w = 0; w < kWavesPerBlock; ++w) {
    const uint32_t t = scratch[w];
    if (w < wave_id()) before += t;
    sum += t;
  }
  *total = sum;
  return before + incl - v;
}

// The last workgroup of a (client, phase) to arrive gets true: everything the
// other workgroups wrote before arriving is then visible through agent-scope loads.
__device__ __forceinline__ bool arrive_last(uint32_t* counter, uint32_t expected) {
  __shared__ uint32_t s_last;
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) s_last = (atomicAdd(counter, 1u) == expected - 1u) ? 1u : 0u;
  __syncthreads();
  const bool last = s_last != 0;
  if (last) __threadfence();
  return last;
}

// ------------------------------------------------------------------ 1. sample histogram
// Reads n_s 64-byte pieces spread evenly over the vector and histograms the
// magnitude keys on their top 12 bits.  The last workgroup walks the histogram
// from the top to the sample rank the host derived from k/d plus a 6-sigma
// margin; the lower edge of that bin becomes the candidate threshold.
__global__ __launch_bounds__(kBlock) void sample_hist_kernel(const ClientParams* __restrict__ params,
                                                             ClientCtl* __restrict__ ctls, uint32_t n_s,
                                                             uint32_t n_src) {
  __shared__ uint32_t hist[kSampleBins];
  __shared__ uint32_t scan_tmp[kWavesPerBlock];
  const ClientParams& p = params[blockIdx.y];
  ClientCtl* ctl = ctls + blockIdx.y;
  if (p.sample_rank == 0) {  // keep-all plan: threshold stays 0
    return;
  }
  for (uint32_t i = threadIdx.x; i < kSampleBins; i += kBlock) hist[i] = 0;
  __syncthreads();
  const float4* src = reinterpret_cast<const float4*>(p.update);
  const uint32_t total_q = n_s * 4u;
  for (uint32_t q = blockIdx.x * kBlock + threadIdx.x; q < total_q; q += gridDim.x * kBlock) {
    const uint32_t j = q >> 2, part = q & 3u;
    const uint64_t piece = (uint64_t)j * n_src / n_s;
    const float4 v = src[piece * 4u + part];
    atomicAdd(&hist[(__float_as_uint(v.x) & 0x7FFFFFFFu) >> kSampleShift], 1u);
    atomicAdd(&hist[(__float_as_uint(v.y) & 0x7FFFFFFFu) >> kSampleShift], 1u);
    atomicAdd(&hist[(__float_as_uint(v.z) & 0x7FFFFFFFu) >> kSampleShift], 1u);
    atomicAdd(&hist[(__float_as_uint(v.w) & 0x7FFFFFFFu) >> kSampleShift], 1u);
  }
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < kSampleBins; i += kBlock)
    if (hist[i]) atomicAdd(&ctl->hist_sample[i], hist[i]);
  if (!arrive_last(&ctl->done_sample, gridDim.x)) return;

  // thread t owns the 16 bins [top-15, top], top = 4095 - 16 t: walk from large keys down
  constexpr uint32_t per = kSampleBins / kBlock;
  const uint32_t top = kSampleBins - 1 - per * threadIdx.x;
  uint32_t mine = 0;
  for (uint32_t i = 0; i < per; ++i) mine += load_agent(&ctl->hist_sample[top - i]);
  uint32_t total;
  const uint32_t above = block_excl_scan(mine, scan_tmp, &total);
  const uint32_t target = p.sample_rank;
  if (above < target && target <= above + mine) {
    uint32_t acc = above, bin = top;
    for (uint32_t i = 0; i < per; ++i) {
      acc += load_agent(&ctl->hist_sample[top - i]);
      if (acc >= target) { bin = top - i; break; }
    }
    ctl->tau_lo = bin << kSampleShift;
  }
  // target beyond the sample: tau_lo keeps its cleared value 0 (everything is a candidate)
}

// ------------------------------------------------------------------ 2. filter (the full pass)
constexpr uint64_t kFlagAgg = 1ull << 62;     // tile's own candidate count is published
constexpr uint64_t kFlagPrefix = 2ull << 62;  // inclusive prefix up to this tile is published
constexpr uint64_t kFlagMask = 3ull << 62;
constexpr uint32_t kSpinLimit = 1u << 24;

// Exclusive prefix of `agg` over the tiles before `tile` of the same client
// (decoupled look-back).  Called by all 64 lanes of one wavefront.  Tiles are
// claimed through an atomic counter, so every earlier tile already belongs to
// a running workgroup and publishes its count without waiting on anyone.  The
// spin is bounded: on expiry the internal-error bit is set and 0 is assumed.
__device__ uint32_t lookback_exclusive(uint64_t* state, uint32_t tile, uint32_t agg, uint32_t* status) {
  const uint32_t lane = lane_id();
  if (tile == 0) {
    if (lane == 0) store_agent(&state[0], kFlagPrefix | agg);
    return 0;
  }
  if (lane == 0) store_agent(&state[tile], kFlagAgg | agg);
  uint32_t excl = 0;
  int64_t base = (int64_t)tile - 1;
  while (true) {
    const int64_t idx = base - (int64_t)lane;
    uint64_t v = kFlagPrefix;  // positions before tile 0 act as an empty prefix
    if (idx >= 0) {
      uint32_t spins = 0;
      v = load_agent(&state[idx]);
      while ((v & kFlagMask) == 0 && ++spins < kSpinLimit) {
        __builtin_amdgcn_s_sleep(2);
        v = load_agent(&state[idx]);
      }
      if ((v & kFlagMask) == 0) {
        atomicOr(status, CVLC_DEV_INTERNAL);
        v = kFlagPrefix;
      }
    }
    const uint64_t has_prefix = __ballot((v & kFlagMask) == kFlagPrefix);
    const uint32_t first = has_prefix ? (uint32_t)__builtin_ctzll(has_prefix) : 64u;
    const uint32_t val = (lane <= first) ? (uint32_t)(v & 0xFFFFFFFFull) : 0u;
    excl += wave_sum_u32(val);
    if (has_prefix) break;
    base -= 64;
  }
  if (lane == 0) store_agent(&state[tile], kFlagPrefix | (uint64_t)(excl + agg));
  return excl;
}

// One tile = 4096 coordinates; wavefront w owns the contiguous 1024 starting at
// w*1024 and reads them as four float4 per lane (j-th load at j*256 + lane*4),
// so position order inside a wavefront is (j, lane, component).
template <int PASS>
__global__ __launch_bounds__(kBlock) void filter_kernel(const ClientParams* __restrict__ params,
                                                        ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ uint32_t s_tile, s_prefix;
  __shared__ uint32_t s_wtot[kWavesPerBlock];
  __shared__ double s_wsq[kWavesPerBlock];
  const uint32_t client = blockIdx.y;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  uint32_t tau_lo;
  if (PASS == 0) {
    tau_lo = ctl->tau_lo;
  } else {
    if (ctl->n_cand[0] >= p.k) return;  // the sampled threshold kept enough
    tau_lo = 0;
  }
  const uint32_t d = ws.d, n_tiles = ws.n_tiles;
  const float* __restrict__ U = p.update;
  uint64_t* state = ws.tile_state + ((size_t)client * 2 + PASS) * n_tiles;
  uint32_t* out_idx = ws.cand_idx + (size_t)client * d;
  float* out_val = ws.cand_val + (size_t)client * d;
  const uint32_t lane = lane_id(), wave = wave_id();

  while (true) {
    __syncthreads();
    if (threadIdx.x == 0) s_tile = atomicAdd(&ctl->tile_counter[PASS], 1u);
    __syncthreads();
    const uint32_t tile = s_tile;
    if (tile >= n_tiles) break;
    const uint32_t wbase = tile * kTile + wave * (kTile / kWavesPerBlock);

    float v[4][4];
    uint32_t flags[4];
    double sq = 0.0;
    bool bad = false;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t e0 = wbase + j * 256u + lane * 4u;
      if (e0 + 3u < d) {
        const float4 q = *reinterpret_cast<const float4*>(U + e0);
        v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[j][c] = (e0 + c < d) ? U[e0 + c] : 0.0f;
      }
      uint32_t f = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t key = __float_as_uint(v[j][c]) & 0x7FFFFFFFu;
        const bool in_range = e0 + c < d;
        bad |= key >= 0x7F800000u;
        if (in_range && key >= tau_lo) {
          f |= 1u << c;
        } else {
          sq += (double)v[j][c] * (double)v[j][c];  // padding contributes 0
        }
      }
      flags[j] = f;
    }
    if (bad) atomicOr(ws.status, CVLC_DEV_NONFINITE);

    // position-ordered offsets inside the wavefront
    uint32_t pre[4], wtot = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t cnt = __popc(flags[j]);
      const uint64_t b0 = __ballot(cnt & 1u), b1 = __ballot(cnt & 2u), b2 = __ballot(cnt & 4u);
      pre[j] = wtot + lanes_below(b0) + 2u * lanes_below(b1) + 4u * lanes_below(b2);
      wtot += (uint32_t)__popcll(b0) + 2u * (uint32_t)__popcll(b1) + 4u * (uint32_t)__popcll(b2);
    }
    sq = wave_sum_f64(sq);
    if (lane == 0) { s_wtot[wave] = wtot; s_wsq[wave] = sq; }
    __syncthreads();
    uint32_t woff = 0, agg = 0;
#pragma unroll
    for (uint32_t w = 0; w < kWavesPerBlock; ++w) {
      if (w < wave) woff += s_wtot[w];
      agg += s_wtot[w];
    }
    if (wave == 0) {
      const uint32_t excl = lookback_exclusive(state, tile, agg, ws.status);
      if (lane == 0) {
        s_prefix = excl;
        ws.tile_sumsq[(size_t)client * n_tiles + tile] = (s_wsq[0] + s_wsq[1]) + (s_wsq[2] + s_wsq[3]);
        if (tile == n_tiles - 1) ctl->n_cand[PASS] = excl + agg;
      }
    }
    __syncthreads();
    const uint32_t tile_off = s_prefix + woff;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t f = flags[j];
      if (f) {
        uint32_t pos = tile_off + pre[j];
        const uint32_t e0 = wbase + j * 256u + lane * 4u;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if (f & (1u << c)) {
            if (pos < d) {  // always true for a consistent prefix; guards the bounded-spin fallback
              out_idx[pos] = e0 + c;
              out_val[pos] = v[j][c];
            }
            ++pos;
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------ 3. selection, level 1
// Histogram of the candidates' top 11 key bits; the last workgroup locates, for
// every boundary Z_r, the bin holding the Z_r-th largest key and the rank left
// inside that bin.
__global__ __launch_bounds__(kBlock) void select_l1_kernel(const ClientParams* __restrict__ params,
                                                           ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ uint32_t hist[kL1Bins];
  __shared__ uint32_t incl[kL1Bins];  // count of keys in bins >= b
  __shared__ uint32_t scan_tmp[kWavesPerBlock];
  const uint32_t client = blockIdx.y;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  const uint32_t n = final_ncand(ctl, p);
  const float* val = ws.cand_val + (size_t)client * ws.d;
  for (uint32_t i = threadIdx.x; i < kL1Bins; i += kBlock) hist[i] = 0;
  __syncthreads();
  for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < n; i += gridDim.x * kBlock)
    atomicAdd(&hist[(__float_as_uint(val[i]) & 0x7FFFFFFFu) >> 20], 1u);
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < kL1Bins; i += kBlock)
    if (hist[i]) atomicAdd(&ctl->hist1[i], hist[i]);
  if (!arrive_last(&ctl->done_l1, gridDim.x)) return;

  constexpr uint32_t per = kL1Bins / kBlock;  // 8 bins per thread, from the top down
  const uint32_t top = kL1Bins - 1 - per * threadIdx.x;
  uint32_t h[per], mine = 0;
  for (uint32_t i = 0; i < per; ++i) { h[i] = load_agent(&ctl->hist1[top - i]); mine += h[i]; }
  uint32_t total;
  uint32_t run = block_excl_scan(mine, scan_tmp, &total);
  for (uint32_t i = 0; i < per; ++i) {
    run += h[i];
    hist[top - i] = h[i];
    incl[top - i] = run;
  }
  __syncthreads();
  if (threadIdx.x < p.R) {
    const uint32_t r = threadIdx.x, Z = p.Z[r];
    if (Z == 0 || Z > total) {  // Z > total cannot happen once the filter kept >= k
      ctl->sel_prefix[r] = 0xFFFFFFFFu;
      ctl->sel_rem[r] = 0;
      if (Z > total) atomicOr(ws.status, CVLC_DEV_INTERNAL);
    } else {
      uint32_t lo = 0, hi = kL1Bins - 1;  // largest bin b with incl[b] >= Z
      while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (incl[mid] >= Z) lo = mid; else hi = mid - 1;
      }
      ctl->sel_prefix[r] = lo;
      ctl->sel_rem[r] = Z - (incl[lo] - hist[lo]);
    }
  }
}

// ------------------------------------------------------------------ 4. selection, levels 2 and 3
// LEVEL 2 refines bits 19..10, LEVEL 3 bits 9..0 of the boundary keys of one
// group of up to kSlotGroup boundaries.  Boundaries that share a prefix share a
// histogram ("slot", the first such boundary of the group).
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void select_l23_kernel(const ClientParams* __restrict__ params,
                                                            ClientCtl* __restrict__ ctls, Workspace ws,
                                                            uint32_t group) {
  __shared__ uint32_t hist[kSlotGroup][kDigitBins];
  __shared__ uint32_t s_prefix[kSlotGroup];  // prefix per slot leader
  __shared__ uint32_t s_leader[kSlotGroup];  // local slot of every boundary in the group
  __shared__ uint32_t s_bitmap[kL1Bins / 32];
  __shared__ uint32_t s_nslots;
  constexpr uint32_t match_shift = LEVEL == 2 ? 20u : 10u;
  constexpr uint32_t digit_shift = LEVEL == 2 ? 10u : 0u;
  const uint32_t client = blockIdx.y;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  const uint32_t r0 = group * kSlotGroup;
  if (p.R <= r0) return;  // this client has no boundary in the group
  const uint32_t nb = min(p.R - r0, kSlotGroup);
  const uint32_t n = final_ncand(ctl, p);
  const float* val = ws.cand_val + (size_t)client * ws.d;

  for (uint32_t i = threadIdx.x; i < kSlotGroup * kDigitBins; i += kBlock) (&hist[0][0])[i] = 0;
  for (uint32_t i = threadIdx.x; i < kL1Bins / 32; i += kBlock) s_bitmap[i] = 0;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t ns = 0;
    for (uint32_t b = 0; b < nb; ++b) {
      const uint32_t pre = ctl->sel_prefix[r0 + b];
      uint32_t slot = 0xFFFFFFFFu;
      if (pre != 0xFFFFFFFFu) {
        for (uint32_t q = 0; q < ns; ++q)
          if (s_prefix[q] == pre) slot = q;
        if (slot == 0xFFFFFFFFu) {
          slot = ns++;
          s_prefix[slot] = pre;
          const uint32_t top11 = LEVEL == 2 ? pre : pre >> 10;
          s_bitmap[top11 >> 5] |= 1u << (top11 & 31u);
        }
      }
      s_leader[b] = slot;
    }
    s_nslots = ns;
  }
  __syncthreads();
  const uint32_t ns = s_nslots;
  if (ns > 0) {
    for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < n; i += gridDim.x * kBlock) {
      const uint32_t key = __float_as_uint(val[i]) & 0x7FFFFFFFu;
      const uint32_t top11 = key >> 20;
      if ((s_bitmap[top11 >> 5] >> (top11 & 31u)) & 1u) {
        const uint32_t pre = key >> match_shift;
        for (uint32_t q = 0; q < ns; ++q)
          if (s_prefix[q] == pre) {
            atomicAdd(&hist[q][(key >> digit_shift) & (kDigitBins - 1)], 1u);
            break;
          }
      }
    }
  }
  __syncthreads();
  uint32_t(*ghist)[kDigitBins] = LEVEL == 2 ? ctl->hist2 : ctl->hist3;
  for (uint32_t i = threadIdx.x; i < ns * kDigitBins; i += kBlock) {
    const uint32_t q = i / kDigitBins, b = i % kDigitBins;
    if (hist[q][b]) atomicAdd(&ghist[r0 + q][b], hist[q][b]);
  }
  if (!arrive_last(&ctl->done_l23[LEVEL - 2][group], gridDim.x)) return;

  // One wavefront per boundary: lane l owns the 16 digits [top-15, top], top = 1023 - 16 l.
  for (uint32_t b = wave_id(); b < nb; b += kWavesPerBlock) {
    const uint32_t r = r0 + b, slot = s_leader[b];
    if (slot == 0xFFFFFFFFu) {  // Z_r = 0: nothing is inside this boundary
      if (LEVEL == 3 && lane_id() == 0) { ctl->tau[r] = 0xFFFFFFFFu; ctl->iota[r] = 0; ctl->tie_need[r] = 0; }
      continue;
    }
    const uint32_t* gh = ghist[r0 + slot];
    const uint32_t top = kDigitBins - 1 - 16u * lane_id();
    uint32_t h[16], mine = 0;
    for (uint32_t i = 0; i < 16; ++i) { h[i] = load_agent(&gh[top - i]); mine += h[i]; }
    const uint32_t above = wave_incl_scan_u32(mine) - mine;
    const uint32_t rem = ctl->sel_rem[r];
    if (above < rem && rem <= above + mine) {
      uint32_t acc = above;
      for (uint32_t i = 0; i < 16; ++i) {
        if (acc + h[i] >= rem) {
          const uint32_t full = (s_prefix[slot] << 10) | (top - i);
          const uint32_t left = rem - acc;  // rank inside the digit class, 1-based
          if (LEVEL == 2) {
            ctl->sel_prefix[r] = full;
            ctl->sel_rem[r] = left;
          } else {
            ctl->tau[r] = full;
            ctl->sel_rem[r] = left;         // tie quota q_r
            const bool need = left < h[i];  // the class of equal keys straddles the boundary
            ctl->tie_need[r] = need ? 1u : 0u;
            ctl->iota[r] = 0xFFFFFFFFu;
            if (need) atomicOr(&ctl->need_tie, 1u);
          }
          break;
        }
        acc += h[i];
      }
    }
  }
}

// ------------------------------------------------------------------ 5. ties at a boundary
// For boundaries whose key class straddles Z_r: the position of the q_r-th
// member of the class in position order.  Each workgroup counts the class
// members in its slice of the candidate list; the last one finds the slice
// that holds the q_r-th member and walks it.
__global__ __launch_bounds__(kBlock) void tie_resolve_kernel(const ClientParams* __restrict__ params,
                                                             ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ uint32_t s_cnt[32];
  __shared__ uint32_t s_tau[32];
  __shared__ uint32_t s_need[32];
  __shared__ uint32_t scan_tmp[kWavesPerBlock];
  __shared__ uint32_t s_found;
  const uint32_t client = blockIdx.y;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  if (!ctl->need_tie) return;
  const uint32_t n = final_ncand(ctl, p);
  const float* val = ws.cand_val + (size_t)client * ws.d;
  const uint32_t* idx = ws.cand_idx + (size_t)client * ws.d;
  if (threadIdx.x < 32) {
    const bool live = threadIdx.x < p.R;
    s_cnt[threadIdx.x] = 0;
    s_tau[threadIdx.x] = live ? ctl->tau[threadIdx.x] : 0xFFFFFFFFu;
    s_need[threadIdx.x] = live ? ctl->tie_need[threadIdx.x] : 0u;
  }
  __syncthreads();
  const uint32_t span = (uint32_t)((((uint64_t)n + gridDim.x - 1) / gridDim.x + kBlock - 1) / kBlock * kBlock);
  const uint64_t begin64 = (uint64_t)blockIdx.x * span;
  const uint32_t begin = (uint32_t)(begin64 < n ? begin64 : n);
  const uint32_t end = (uint32_t)(begin64 + span < n ? begin64 + span : n);
  for (uint32_t i = begin + threadIdx.x; i < end; i += kBlock) {
    const uint32_t key = __float_as_uint(val[i]) & 0x7FFFFFFFu;
    for (uint32_t r = 0; r < p.R; ++r)
      if (s_need[r] && key == s_tau[r]) atomicAdd(&s_cnt[r], 1u);
  }
  __syncthreads();
  if (threadIdx.x < 32) store_agent(&ctl->tie_partial[blockIdx.x][threadIdx.x], s_cnt[threadIdx.x]);
  if (!arrive_last(&ctl->done_tie, gridDim.x)) return;

  for (uint32_t r = 0; r < p.R; ++r) {
    if (!s_need[r]) continue;
    const uint32_t quota = ctl->sel_rem[r];
    // slice holding the quota-th member
    uint32_t before = 0, slice = 0;
    for (slice = 0; slice < gridDim.x; ++slice) {
      const uint32_t c = load_agent(&ctl->tie_partial[slice][r]);
      if (before + c >= quota) break;
      before += c;
    }
    if (slice == gridDim.x) {  // fewer members than the quota: histogram and list disagree
      if (threadIdx.x == 0) atomicOr(ws.status, CVLC_DEV_INTERNAL);
      continue;
    }
    const uint64_t sb = (uint64_t)slice * span;
    const uint32_t s_begin = (uint32_t)(sb < n ? sb : n), s_end = (uint32_t)(sb + span < n ? sb + span : n);
    uint32_t left = quota - before;  // 1-based rank inside the slice
    __syncthreads();
    if (threadIdx.x == 0) s_found = 0;
    __syncthreads();
    for (uint32_t base = s_begin; base < s_end; base += kBlock) {
      const uint32_t i = base + threadIdx.x;
      const uint32_t hit = (i < s_end && (__float_as_uint(val[i]) & 0x7FFFFFFFu) == s_tau[r]) ? 1u : 0u;
      uint32_t tot;
      const uint32_t rank = block_excl_scan(hit, scan_tmp, &tot);
      if (hit && rank + 1 == left) {
        ctl->iota[r] = idx[i];
        s_found = 1;
      }
      __syncthreads();
      if (s_found || tot >= left) break;
      left -= tot;
    }
  }
}

// ------------------------------------------------------------------ classification
struct Thresholds {  // group boundaries in LDS
  uint32_t tau[32];
  uint32_t iota[32];
};

__device__ __forceinline__ void load_thresholds(Thresholds& t, const ClientCtl* ctl, uint32_t R) {
  if (threadIdx.x < 32) {
    const bool live = threadIdx.x < R;
    t.tau[threadIdx.x] = live ? ctl->tau[threadIdx.x] : 0xFFFFFFFFu;
    t.iota[threadIdx.x] = live ? ctl->iota[threadIdx.x] : 0u;
  }
}

// Group of a candidate, 0-based: the first boundary r whose top-Z_r set holds
// it (key above tau_r, or equal with position <= iota_r); R if none (dropped).
// Membership is monotone in r, so a binary search suffices.
__device__ __forceinline__ uint32_t classify(const Thresholds& t, uint32_t R, uint32_t key, uint32_t idx) {
  uint32_t lo = 0, hi = R;  // answer in [lo, hi]
  while (lo < hi) {
    const uint32_t mid = (lo + hi) >> 1;
    const uint32_t tau = t.tau[mid];
    const bool inside = key > tau || (key == tau && idx <= t.iota[mid]);
    if (inside) hi = mid; else lo = mid + 1;
  }
  return lo;
}

// ------------------------------------------------------------------ 6. classify + statistics
// Per chunk of kChunk candidates: count, min, max, sum of squares of every
// group (index R collects the candidates that end up dropped).  Also clears the
// stream buffer, which the emit pass ORs records into.
__global__ __launch_bounds__(kBlock) void classify_kernel(const ClientParams* __restrict__ params,
                                                          ClientCtl* __restrict__ ctls, Workspace ws) {
  __shared__ Thresholds thr;
  __shared__ uint32_t s_cnt[32], s_max[32], s_negmin[32];
  __shared__ double s_sq[32];
  const uint32_t client = blockIdx.y;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  const uint32_t n = final_ncand(ctl, p), R = p.R;
  const float* val = ws.cand_val + (size_t)client * ws.d;
  const uint32_t* idx = ws.cand_idx + (size_t)client * ws.d;

  for (uint32_t w = blockIdx.x * kBlock + threadIdx.x; w < p.total_words; w += gridDim.x * kBlock) p.stream[w] = 0;

  load_thresholds(thr, ctl, R);
  const uint32_t n_chunks = (n + kChunk - 1) / kChunk;
  for (uint32_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    __syncthreads();
    if (threadIdx.x < 32) { s_cnt[threadIdx.x] = 0; s_max[threadIdx.x] = 0; s_negmin[threadIdx.x] = 0; s_sq[threadIdx.x] = 0.0; }
    __syncthreads();
    for (uint32_t j = 0; j < kChunk / kBlock; ++j) {
      const uint32_t i = c * kChunk + wave_id() * (kChunk / kWavesPerBlock) + j * kWave + lane_id();
      if (i < n) {
        const float x = val[i];
        const uint32_t g = classify(thr, R, __float_as_uint(x) & 0x7FFFFFFFu, idx[i]);
        atomicAdd(&s_cnt[g], 1u);
        atomicAdd(&s_sq[g], (double)x * (double)x);
        const uint32_t o = ordered_bits(x);
        atomicMax(&s_max[g], o);
        atomicMax(&s_negmin[g], ~o);
      }
    }
    __syncthreads();
    if (threadIdx.x <= R) {
      const uint32_t g = threadIdx.x;
      const size_t slot = ((size_t)client * ws.max_chunks + c) * 32 + g;
      ws.chunk_cnt[slot] = s_cnt[g];
      ws.chunk_sumsq[slot] = s_sq[g];
      if (s_cnt[g] && g < R) {
        atomicMax(&ctl->seg_max_enc[g], s_max[g]);
        atomicMax(&ctl->seg_negmin_enc[g], s_negmin[g]);
      }
    }
  }
}

// ------------------------------------------------------------------ 7. layout: prefix, headers, statistics
// One workgroup of 1024 threads per client.  Wavefront w scans the per-chunk
// counts of groups w, w+16, ... into exclusive prefixes (in place) and adds up
// the per-chunk sums of squares in chunk order; then the headers and the
// statistics block are written.
__global__ __launch_bounds__(1024) void layout_kernel(const ClientParams* __restrict__ params,
                                                      ClientCtl* __restrict__ ctls, Workspace ws,
                                                      cvlc_seg_stats_t* __restrict__ stats_out) {
  __shared__ uint32_t s_total[32];
  __shared__ double s_sq[32];
  __shared__ double s_tail[16];
  const uint32_t client = blockIdx.x;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  const uint32_t n = final_ncand(ctl, p), R = p.R;
  const uint32_t n_chunks = (n + kChunk - 1) / kChunk;
  const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
  uint32_t* cnt = ws.chunk_cnt + (size_t)client * ws.max_chunks * 32;
  const double* csq = ws.chunk_sumsq + (size_t)client * ws.max_chunks * 32;

  for (uint32_t g = wave; g <= R; g += 16) {
    uint32_t run = 0;
    double sq = 0.0;
    for (uint32_t c0 = 0; c0 < n_chunks; c0 += kWave) {
      const uint32_t c = c0 + lane;
      const uint32_t v = c < n_chunks ? cnt[(size_t)c * 32 + g] : 0u;
      const double q = c < n_chunks ? csq[(size_t)c * 32 + g] : 0.0;
      const uint32_t incl = wave_incl_scan_u32(v);
      if (c < n_chunks) cnt[(size_t)c * 32 + g] = run + incl - v;
      run += __shfl(incl, 63, 64);
      sq += wave_sum_f64(q);
    }
    if (lane == 0) { s_total[g] = run; s_sq[g] = sq; }
  }
  // energy of the coordinates the filter dropped, in tile order
  {
    const double* tsq = ws.tile_sumsq + (size_t)client * ws.n_tiles;
    double acc = 0.0;
    for (uint32_t t = threadIdx.x; t < ws.n_tiles; t += 1024) acc += tsq[t];
    acc = wave_sum_f64(acc);
    if (lane == 0) s_tail[wave] = acc;
  }
  __syncthreads();

  uint32_t* stream = p.stream;
  if (threadIdx.x < R) {
    const uint32_t r = threadIdx.x;
    const uint32_t P = p.Z[r] - (r ? p.Z[r - 1] : 0u);
    if (s_total[r] != P) atomicOr(ws.status, CVLC_DEV_INTERNAL);
    float m = 0.0f, M = 0.0f;
    if (P > 0 && ctl->seg_max_enc[r] != 0) {
      M = from_ordered_bits(ctl->seg_max_enc[r]);
      m = from_ordered_bits(~ctl->seg_negmin_enc[r]);
    }
    if (!(fabsf(M - m) <= 3.4028234664e38f)) atomicOr(ws.status, CVLC_DEV_NONFINITE);
    uint32_t* hdr = stream + kGlobalHeaderWords + kSegHeaderWords * r;
    hdr[0] = p.y[r];
    hdr[1] = P;
    hdr[2] = __float_as_uint(m);
    hdr[3] = __float_as_uint(M);
    if (stats_out) {
      cvlc_seg_stats_t* st = stats_out + (size_t)client * kStatsStride + r;
      st->min = m; st->max = M; st->sumsq = s_sq[r]; st->count = P; st->reserved = 0;
    }
  }
  if (threadIdx.x == 0) {
    stream[0] = kMagic;
    stream[1] = kVersion;  // quantiser id 0 (PQ) in the upper half
    stream[2] = ws.d;
    stream[3] = R;
    stream[4] = position_bits(ws.d);
    stream[5] = __float_as_uint(p.B);
    stream[6] = p.client_id;
    stream[7] = p.total_words;
    if (stats_out) {
      double tail = 0.0;
      for (int w = 0; w < 16; ++w) tail += s_tail[w];
      cvlc_seg_stats_t* st = stats_out + (size_t)client * kStatsStride + R;
      st->min = 0.0f; st->max = 0.0f; st->sumsq = tail + s_sq[R]; st->count = ws.d - p.k; st->reserved = 0;
    }
  }
}

// ------------------------------------------------------------------ 8. emit: quantise + pack
// Philox4x32-10 (Salmon et al., SC'11), first output word.
__device__ __forceinline__ uint32_t philox_word0(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1) {
  uint32_t c2 = 0, c3 = 0;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
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

constexpr uint32_t kStageWords = kChunk * 2 + 2 * 32;  // every record is < 64 bits; two edge words per group

__global__ __launch_bounds__(kBlock) void emit_kernel(const ClientParams* __restrict__ params,
                                                      ClientCtl* __restrict__ ctls, Workspace ws, uint64_t seed) {
  __shared__ Thresholds thr;
  __shared__ uint32_t s_stage[kStageWords];
  __shared__ uint32_t s_wcnt[kWavesPerBlock][32];  // per wavefront, per group: members in this chunk
  __shared__ uint32_t s_base[32];                  // first record index of this chunk in each group
  __shared__ uint32_t s_lim[32];                   // one past this chunk's last record index in each group
  __shared__ uint32_t s_P[32];                     // planned group sizes
  __shared__ uint32_t s_word0[32];                 // first stream word (group-relative) this chunk touches
  __shared__ uint32_t s_nwords[32];                // words this chunk touches in each group
  __shared__ uint32_t s_stage_off[33];
  __shared__ uint32_t s_payload[32];               // first stream word of each group's payload
  __shared__ float s_m[32], s_inv[32];
  __shared__ uint32_t s_W[32];
  const uint32_t client = blockIdx.y;
  const ClientParams& p = params[client];
  ClientCtl* ctl = ctls + client;
  const uint32_t n = final_ncand(ctl, p), R = p.R;
  const uint32_t sbits = position_bits(ws.d);
  const float* val = ws.cand_val + (size_t)client * ws.d;
  const uint32_t* idx = ws.cand_idx + (size_t)client * ws.d;
  uint32_t* stream = p.stream;
  const uint32_t lane = lane_id(), wave = wave_id();
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);

  load_thresholds(thr, ctl, R);
  if (threadIdx.x < 32) {
    const uint32_t r = threadIdx.x;
    if (r < R) {
      const uint32_t* hdr = stream + kGlobalHeaderWords + kSegHeaderWords * r;  // written by the layout kernel
      const float m = __uint_as_float(hdr[2]), M = __uint_as_float(hdr[3]);
      float step, inv;
      centroid_spacing(m, M, p.y[r] == 32 ? 1u : p.y[r], &step, &inv);
      s_m[r] = m;
      s_inv[r] = inv;
      s_W[r] = sbits + p.y[r];
      s_P[r] = p.Z[r] - (r ? p.Z[r - 1] : 0u);
    }
  }
  if (threadIdx.x == 0) {
    uint32_t w = kGlobalHeaderWords + kSegHeaderWords * R;
    for (uint32_t r = 0; r < R; ++r) {
      s_payload[r] = w;
      const uint32_t P = p.Z[r] - (r ? p.Z[r - 1] : 0u);
      w += (uint32_t)payload_words(P, sbits + p.y[r]);
    }
  }
  const uint32_t n_chunks = (n + kChunk - 1) / kChunk;
  for (uint32_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < kWavesPerBlock * 32; i += kBlock) (&s_wcnt[0][0])[i] = 0;
    __syncthreads();
    // sweep 1: group of each of this thread's 8 candidates, per-wavefront group sizes
    float x[8];
    uint32_t pid[8], grp[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t i = c * kChunk + wave * (kChunk / kWavesPerBlock) + j * kWave + lane;
      grp[j] = 0xFFFFFFFFu;
      if (i < n) {
        x[j] = val[i];
        pid[j] = idx[i];
        grp[j] = classify(thr, R, __float_as_uint(x[j]) & 0x7FFFFFFFu, pid[j]);
        if (grp[j] < R) atomicAdd(&s_wcnt[wave][grp[j]], 1u);
      }
    }
    __syncthreads();
    if (threadIdx.x < 32) {
      const uint32_t r = threadIdx.x;
      uint32_t cnt = 0;
      if (r < R) {
        for (uint32_t w = 0; w < kWavesPerBlock; ++w) cnt += s_wcnt[w][r];
        uint32_t e0 = ws.chunk_cnt[((size_t)client * ws.max_chunks + c) * 32 + r];
        // a consistent selection never exceeds the planned size; the clamp keeps every
        // write inside the group's payload even if an internal check has failed
        if (e0 > s_P[r]) e0 = s_P[r];
        if (cnt > s_P[r] - e0) cnt = s_P[r] - e0;
        s_base[r] = e0;
        s_lim[r] = e0 + cnt;
        const uint64_t bit0 = (uint64_t)e0 * s_W[r], bit1 = (uint64_t)(e0 + cnt) * s_W[r];
        s_word0[r] = (uint32_t)(bit0 >> 5);
        s_nwords[r] = cnt ? (uint32_t)(((bit1 - 1) >> 5) - (bit0 >> 5) + 1) : 0u;
      } else {
        s_nwords[r] = 0;
      }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      uint32_t off = 0;
      for (uint32_t r = 0; r < 32; ++r) { s_stage_off[r] = off; off += s_nwords[r]; }
      s_stage_off[32] = off;
    }
    __syncthreads();
    const uint32_t staged = s_stage_off[32];
    for (uint32_t i = threadIdx.x; i < staged; i += kBlock) s_stage[i] = 0;
    __syncthreads();
    // sweep 2: rank inside (group, chunk) in position order, quantise, pack into LDS.
    // Lane g of a wavefront keeps the running rank of group g for that wavefront.
    uint32_t running = 0;
    if (lane < R)
      for (uint32_t w = 0; w < wave; ++w) running += s_wcnt[w][lane];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool coded = grp[j] < R;
      uint32_t my_rank = 0;
      uint64_t todo = __ballot(coded);
      while (todo) {
        const uint32_t leader = (uint32_t)__builtin_ctzll(todo);
        const uint32_t g = __shfl(grp[j], leader, 64);
        const uint64_t same = __ballot(coded && grp[j] == g);
        const uint32_t start = __shfl(running, g, 64);
        if (coded && grp[j] == g) my_rank = start + lanes_below(same);
        if (lane == g) running += (uint32_t)__popcll(same);
        todo &= ~same;
      }
      if (coded && s_base[grp[j]] + my_rank < s_lim[grp[j]]) {
        const uint32_t g = grp[j], y = p.y[g], W = s_W[g];
        uint32_t cid;
        if (y == 32) {
          cid = __float_as_uint(x[j]);
        } else {
          const uint32_t u24 = philox_word0(pid[j], p.client_id, k0, k1) >> 8;
          cid = quantise(x[j], s_m[g], s_inv[g], y, u24);
        }
        const uint64_t record = (uint64_t)pid[j] | ((uint64_t)cid << sbits);
        const uint64_t bit = (uint64_t)(s_base[g] + my_rank) * W - (uint64_t)s_word0[g] * 32u;
        const uint32_t w0 = s_stage_off[g] + (uint32_t)(bit >> 5), sh = (uint32_t)(bit & 31u);
        const uint64_t lo = record << sh;
        const uint32_t hi = sh ? (uint32_t)(record >> (64u - sh)) : 0u;
        atomicOr(&s_stage[w0], (uint32_t)lo);
        if (sh + W > 32u) atomicOr(&s_stage[w0 + 1], (uint32_t)(lo >> 32));
        if (sh + W > 64u) atomicOr(&s_stage[w0 + 2], hi);
      }
    }
    __syncthreads();
    // flush: interior words belong to this chunk alone; the two edge words of a
    // group may be shared with neighbouring chunks and are OR-ed in.
    for (uint32_t i = threadIdx.x; i < staged; i += kBlock) {
      uint32_t g = 0;
      while (i >= s_stage_off[g + 1]) ++g;
      const uint32_t rel = i - s_stage_off[g];
      uint32_t* dst = stream + s_payload[g] + s_word0[g] + rel;
      const uint32_t v = s_stage[i];
      if (rel == 0 || rel == s_nwords[g] - 1) {
        if (v) atomicOr(dst, v);
      } else {
        *dst = v;
      }
    }
  }
}

// ------------------------------------------------------------------ host side
int validate_batch(uint32_t n, const cvlc_plan_t* plans, const float* const* d_updates,
                   const uint32_t* client_ids, void* const* d_streams, const size_t* capacities,
                   void* d_workspace, size_t ws_bytes) {
  if (n == 0 || !plans || !d_updates || !client_ids || !d_streams || !capacities || !d_workspace) return CVLC_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(d_workspace) % 256u) return CVLC_ERR_ARG;
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
  if (ws_bytes < cvlc_encode_workspace_bytes(d, n)) return CVLC_ERR_CAPACITY;
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

}  // namespace
}  // namespace cvlc

extern "C" {

size_t cvlc_encode_workspace_bytes(uint32_t d, uint32_t n_clients) {
  if (d < 1 || n_clients < 1) return 0;
  return cvlc::encode_layout(d, n_clients).total;
}

int cvlc_encode_batch(uint32_t n, const cvlc_plan_t* plans, const float* const* d_updates, uint64_t seed,
                      const uint32_t* client_ids, void* const* d_streams_out, const size_t* capacities,
                      void* d_workspace, size_t ws_bytes, cvlc_seg_stats_t* d_stats_out, void* hip_stream) {
  using namespace cvlc;
  int rc = validate_batch(n, plans, d_updates, client_ids, d_streams_out, capacities, d_workspace, ws_bytes);
  if (rc) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const uint32_t d = plans[0].d;
  const EncodeLayout L = encode_layout(d, n);
  char* base = static_cast<char*>(d_workspace);
  Workspace ws;
  ws.status = reinterpret_cast<uint32_t*>(base + L.status);
  ws.params = reinterpret_cast<ClientParams*>(base + L.params);
  ws.ctl = reinterpret_cast<ClientCtl*>(base + L.ctl);
  ws.tile_state = reinterpret_cast<uint64_t*>(base + L.tile_state);
  ws.tile_sumsq = reinterpret_cast<double*>(base + L.tile_sumsq);
  ws.cand_idx = reinterpret_cast<uint32_t*>(base + L.cand_idx);
  ws.cand_val = reinterpret_cast<float*>(base + L.cand_val);
  ws.chunk_cnt = reinterpret_cast<uint32_t*>(base + L.chunk_cnt);
  ws.chunk_sumsq = reinterpret_cast<double*>(base + L.chunk_sumsq);
  ws.d = d;
  ws.n_tiles = L.n_tiles;
  ws.max_chunks = L.max_chunks;

  // sample geometry: 64-byte pieces spread evenly; all of them when the vector is short
  const uint32_t n_src = d / 16u;
  const uint32_t n_s = n_src < kSampleChunksMax ? n_src : kSampleChunksMax;

  profile_mark(CVLC_STAGE_ENC_SETUP, true, stream);
  if ((rc = hip_check(hipMemsetAsync(base + L.status, 0, 256, stream)))) return rc;
  if ((rc = hip_check(hipMemsetAsync(base + L.zero_begin, 0, L.zero_end - L.zero_begin, stream)))) return rc;

  // per-client parameters, shipped as kernel arguments
  uint32_t max_R = 0;
  bool any_sampled = false;
  {
    constexpr uint32_t words_per = sizeof(ClientParams) / 4u;
    const uint32_t per_chunk = kUploadWords / words_per;
    UploadChunk chunk;
    for (uint32_t first = 0; first < n; first += per_chunk) {
      const uint32_t cnt = (n - first < per_chunk) ? n - first : per_chunk;
      chunk.n_words = cnt * words_per;
      chunk.dst_word = first * words_per;
      for (uint32_t i = 0; i < cnt; ++i) {
        const cvlc_plan_t& pl = plans[first + i];
        ClientParams cp;
        std::memset(&cp, 0, sizeof(cp));
        cp.update = d_updates[first + i];
        cp.stream = static_cast<uint32_t*>(d_streams_out[first + i]);
        cp.client_id = client_ids[first + i];
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
        cp.sample_rank = sample_rank(d, z, n_s * 16u);
        any_sampled |= cp.sample_rank != 0;
        if (pl.n_coded > max_R) max_R = pl.n_coded;
        std::memcpy(&chunk.data[i * words_per], &cp, sizeof(cp));
      }
      hipLaunchKernelGGL(upload_kernel, dim3(1), dim3(256), 0, stream, reinterpret_cast<uint32_t*>(ws.params), chunk);
    }
  }

  profile_mark(CVLC_STAGE_ENC_SETUP, false, stream);

  auto spread = [n](uint32_t want_total, uint32_t cap) {  // workgroups per client
    uint32_t g = (want_total + n - 1) / n;
    if (g > cap) g = cap;
    return g < 1 ? 1u : g;
  };
  if (any_sampled) {
    StageScope scope(CVLC_STAGE_ENC_SAMPLE, stream);
    const uint32_t g = spread(512, (n_s * 4u + kBlock - 1) / kBlock);
    hipLaunchKernelGGL(sample_hist_kernel, dim3(g, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, n_s, n_src);
  }
  {
    const uint32_t g = spread(2048, L.n_tiles);
    {
      StageScope scope(CVLC_STAGE_ENC_FILTER, stream);
      hipLaunchKernelGGL(filter_kernel<0>, dim3(g, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, ws);
    }
    StageScope scope(CVLC_STAGE_ENC_REFILTER, stream);
    hipLaunchKernelGGL(filter_kernel<1>, dim3(g, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, ws);
  }
  const uint32_t g_sel = spread(1024, (d + kBlock * 8 - 1) / (kBlock * 8));
  {
    StageScope scope(CVLC_STAGE_ENC_SELECT, stream);
    hipLaunchKernelGGL(select_l1_kernel, dim3(g_sel, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, ws);
    const uint32_t groups = (max_R + kSlotGroup - 1) / kSlotGroup;
    // one launch per group of boundaries; clients with fewer boundaries leave it at once
    for (uint32_t gr = 0; gr < groups; ++gr)
      hipLaunchKernelGGL(select_l23_kernel<2>, dim3(g_sel, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, ws, gr);
    for (uint32_t gr = 0; gr < groups; ++gr)
      hipLaunchKernelGGL(select_l23_kernel<3>, dim3(g_sel, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, ws, gr);
    hipLaunchKernelGGL(tie_resolve_kernel, dim3(kTieBlocks, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, ws);
  }
  const uint32_t g_chunk = spread(2048, L.max_chunks);
  {
    StageScope scope(CVLC_STAGE_ENC_CLASSIFY, stream);
    hipLaunchKernelGGL(classify_kernel, dim3(g_chunk, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, ws);
  }
  {
    StageScope scope(CVLC_STAGE_ENC_LAYOUT, stream);
    hipLaunchKernelGGL(layout_kernel, dim3(n), dim3(1024), 0, stream, ws.params, ws.ctl, ws, d_stats_out);
  }
  {
    StageScope scope(CVLC_STAGE_ENC_EMIT, stream);
    hipLaunchKernelGGL(emit_kernel, dim3(g_chunk, n), dim3(kBlock), 0, stream, ws.params, ws.ctl, ws, seed);
  }
  return hip_check(hipGetLastError());
}

int cvlc_encode(const cvlc_plan_t* plan, const float* d_update, uint64_t seed, uint32_t client_id,
                void* d_stream_out, size_t capacity, void* d_workspace, size_t ws_bytes,
                cvlc_seg_stats_t* d_stats_out, void* hip_stream) {
  if (!plan) return CVLC_ERR_ARG;
  const float* updates[1] = {d_update};
  void* streams[1] = {d_stream_out};
  return cvlc_encode_batch(1, plan, updates, seed, &client_id, streams, &capacity, d_workspace, ws_bytes,
                           d_stats_out, hip_stream);
}

int cvlc_device_status(const void* d_workspace, void* hip_stream, uint32_t* status_out) {
  if (!d_workspace || !status_out) return CVLC_ERR_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int rc = cvlc::hip_check(hipStreamSynchronize(stream));
  if (rc) return rc;
  return cvlc::hip_check(hipMemcpy(status_out, d_workspace, sizeof(uint32_t), hipMemcpyDeviceToHost));
}

}  // extern "C"
