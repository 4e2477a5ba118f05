// cvlc_rank.hip -- the first step of Algorithm 1: the decay exponent alpha_i of
// Definition 1, fitted on the GPU from each client's update vector.
//
// Definition 1 bounds the l-th largest magnitude by phi * l^alpha.  The fit is
// the least-squares slope of ln|U{l}| on ln l at the ranks l = 1, 2, 4, ... and
// l = d (zero magnitudes left out), so what the GPU must deliver is the exact
// magnitude at about log2(d) ranks that reach all the way to the smallest
// entry: order statistics of the whole vector, not only of its top k.
//
// Three radix levels over the 31-bit magnitude key (fp32 bits without the
// sign): 13 bits, then 9, then 9.  Every level is one streaming pass over the
// vectors (HBM bound) that counts digits in LDS, followed by a one-workgroup
// walk per client that turns counts into the next key prefix of every rank.
//
//   init        pointers of the vectors -> workspace; clears the counters
//   hist1       all keys: counts of key >> 18 (8192 bins, 32 KB of LDS)
//   walk<1>     per rank: its level-1 bin and its rank inside that bin; ranks
//               that share a prefix form a class (at most 32 classes)
//   pass<2>     keys whose level-1 bin belongs to a class: counts of the next
//               9 bits per class (32 x 512 bins, 64 KB of LDS)
//   walk<2>     22-bit prefixes, ranks inside, classes again
//   pass<3>     keys that match a 22-bit prefix: counts of the last 9 bits
//   walk<3>     the keys themselves; the fit (fp64, one thread per client)
//
// Only a few percent of a vector's keys lie in a level-1 bin that holds one of
// the ranks.  Given a workspace with room for them (cvlc_fit_workspace_bytes_for)
// the second pass writes those keys out, every wavefront to a stretch of its
// own, and the third pass never happens:
//   collect     (after hist1) the level-1 walk, by every workgroup for itself;
//               all keys: those whose level-1 bin belongs to a class go to the
//               wavefront's list (rows of 64 through LDS) and are counted on
//               their next 9 bits (level 2)
//   walk<2>, pass<3>, walk<3>   as above, the pass reading the lists
#include <hip/hip_runtime.h>

#include <cmath>

#include "cvlc_common.h"

namespace cvlc {
namespace {

constexpr uint32_t kRanksMax = CVLC_FIT_RANKS_MAX;
constexpr uint32_t kTopBins = 8192;   // level 1: key >> 18
constexpr uint32_t kTopShift = 18;
constexpr uint32_t kSubBits = 9;      // levels 2 and 3
constexpr uint32_t kSubBins = 1u << kSubBits;
constexpr uint32_t kRankBlock = 1024;
constexpr uint32_t kRankWaves = kRankBlock / kWave;
constexpr uint32_t kDeep = 4;         // float4 loads a thread keeps in flight
constexpr uint32_t kNoClass = 0xFFu;
static_assert(kRanksMax == 32, "one lane of half a wavefront per rank");

typedef const float __attribute__((address_space(1))) * GlobalFloatPtr;
typedef float __attribute__((ext_vector_type(4))) Float4V;
typedef const Float4V __attribute__((address_space(1))) * GlobalFloat4Ptr;

struct RankSet {  // the ranks of one call, ascending, as kernel arguments
  uint32_t n;
  uint32_t rank[kRanksMax];
};

// Per-client state; cleared by the init kernel.
struct RankCtl {
  uint32_t top[kTopBins];               // level-1 counts of all d keys
  uint32_t sub[kRanksMax * kSubBins];   // per class: counts of the level's digit (cleared again by walk<2>)
  uint32_t prefix[kRanksMax];           // key prefix of rank j known so far (13, 22, 31 bits)
  uint32_t rem[kRanksMax];              // rank j counted inside its prefix class, 1-based from the largest key
  uint32_t cls[kRanksMax];              // class of rank j: classes number the distinct prefixes, largest first
  uint32_t cls_prefix[kRanksMax];
  uint32_t n_cls;
  uint32_t pad[3];
};

struct RankLayout {
  size_t status, ptrs, ctl, list_cnt, lists, total;
  size_t zero_bytes;  // [status, ptrs) and the ctl array are cleared at the start of a call
  uint32_t blocks;    // workgroups per client in the collecting pass
  uint32_t wave_cap;  // keys a wavefront's list has room for (0: no lists, three passes)
};

size_t align256(size_t v) { return (v + 255u) & ~(size_t)255u; }

uint32_t pass_blocks_per_client(uint32_t d, uint32_t n, uint32_t per_cu);

// d = 0: the layout without lists.  With lists, every wavefront of the collecting pass owns room for all
// the keys it reads (whole tiles, plus the last d % 4 coordinates), so nothing has to be counted first.
RankLayout rank_layout(uint32_t n, uint32_t d) {
  RankLayout L;
  size_t off = 0;
  L.status = off; off = align256(off + 256);
  L.ctl = off; off = align256(off + (size_t)n * sizeof(RankCtl));
  L.zero_bytes = off;
  L.ptrs = off; off = align256(off + (size_t)n * sizeof(const float*));
  L.list_cnt = L.lists = off;
  L.blocks = 0;
  L.wave_cap = 0;
  if (d) {
    L.blocks = pass_blocks_per_client(d, n, 2u);
    const uint32_t tiles = (d / 4u + kRankBlock * kDeep - 1) / (kRankBlock * kDeep);
    const uint32_t tiles_per_block = (tiles + L.blocks - 1) / L.blocks;
    L.wave_cap = tiles_per_block * (kDeep * kWave * 4u) + kWave;
    const size_t n_lists = (size_t)n * L.blocks * kRankWaves;
    L.list_cnt = off; off = align256(off + n_lists * sizeof(uint32_t));
    L.lists = off; off = align256(off + n_lists * L.wave_cap * sizeof(uint32_t));
  }
  L.total = off;
  return L;
}

// ------------------------------------------------------------------ init
constexpr uint32_t kPtrChunk = 448;
struct PtrChunk {
  uint32_t first, count;
  const float* ptr[kPtrChunk];
};
static_assert(sizeof(PtrChunk) <= 3800, "kernel arguments are limited to 4 KB");

__global__ __launch_bounds__(256) void rank_init_kernel(const float** dst, PtrChunk c, uint4* zero, size_t zero_n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < zero_n16; i += (size_t)gridDim.x * blockDim.x)
    zero[i] = make_uint4(0u, 0u, 0u, 0u);
  if (blockIdx.x == 0)
    for (uint32_t i = threadIdx.x; i < c.count; i += blockDim.x) dst[c.first + i] = c.ptr[i];
}

// ------------------------------------------------------------------ the streaming passes
// A workgroup takes every gridDim.x-th tile of kRankBlock * kDeep float4; thread t
// reads the t-th, t+1024-th, ... float4 of the tile (clamped, so that no load sits
// under a branch) and hands every in-range key to `visit`.  The last d % 4
// coordinates go to the first threads of workgroup 0.
template <class Visit>
__device__ __forceinline__ void stream_keys(const float* update, uint32_t d, Visit visit) {
  const uint32_t n_quads = d / 4u;
  GlobalFloat4Ptr src = (GlobalFloat4Ptr)update;
  constexpr uint32_t kTileQuads = kRankBlock * kDeep;
  for (uint32_t q0 = blockIdx.x * kTileQuads; q0 < n_quads; q0 += gridDim.x * kTileQuads) {
    Float4V v[kDeep];
#pragma unroll
    for (uint32_t u = 0; u < kDeep; ++u) {
      const uint32_t q = q0 + u * kRankBlock + threadIdx.x;
      v[u] = __builtin_nontemporal_load(src + min(q, n_quads - 1u));
    }
#pragma unroll
    for (uint32_t u = 0; u < kDeep; ++u) {
      const uint32_t q = q0 + u * kRankBlock + threadIdx.x;
      if (q < n_quads) {
#pragma unroll
        for (int c = 0; c < 4; ++c) visit(__float_as_uint(v[u][c]) & 0x7FFFFFFFu);
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < d - n_quads * 4u)
    visit(__float_as_uint(update[n_quads * 4u + threadIdx.x]) & 0x7FFFFFFFu);
}

__global__ __launch_bounds__(kRankBlock) void rank_hist1_kernel(const float* const* __restrict__ updates,
                                                                RankCtl* __restrict__ ctls, uint32_t d,
                                                                uint32_t* status) {
  __shared__ uint32_t hist[kTopBins];
  RankCtl* ctl = ctls + blockIdx.y;
  for (uint32_t i = threadIdx.x; i < kTopBins; i += kRankBlock) hist[i] = 0;
  __syncthreads();
  bool nonfinite = false;
  stream_keys(updates[blockIdx.y], d, [&](uint32_t key) {
    nonfinite |= key >= 0x7F800000u;
    atomicAdd(&hist[key >> kTopShift], 1u);
  });
  const int any_nonfinite = __syncthreads_or((int)nonfinite);
  if (any_nonfinite && threadIdx.x == 0) atomicOr(status, CVLC_DEV_NONFINITE);
  for (uint32_t i = threadIdx.x; i < kTopBins; i += kRankBlock) {
    const uint32_t h = hist[i];
    if (h) atomicAdd(&ctl->top[i], h);
  }
}

// LEVEL 2: prefix = level-1 bin, digit = bits 17..9.  LEVEL 3: prefix = top 22
// bits, digit = bits 8..0.  first_cls maps a level-1 bin to the first class whose
// prefix starts with it; classes are sorted, so the others follow it.
//
// LISTS: the keys come from the lists the collecting pass wrote (`lists`, `list_cnt`, `wave_cap`; a
// wavefront takes every (16 x workgroups)-th list of the client) instead of from the vectors.
struct KeyLists {
  const uint32_t* lists;
  const uint32_t* list_cnt;
  uint32_t per_client, wave_cap;
};

template <class Visit>
__device__ __forceinline__ void list_keys(const KeyLists& kl, Visit visit) {
  const uint32_t lane = lane_id();
  const uint32_t* __restrict__ cnts = kl.list_cnt + (size_t)blockIdx.y * kl.per_client;
  for (uint32_t l = blockIdx.x * kRankWaves + wave_id(); l < kl.per_client; l += gridDim.x * kRankWaves) {
    const uint32_t cnt = cnts[l];
    const uint32_t* __restrict__ keys = kl.lists + ((size_t)blockIdx.y * kl.per_client + l) * kl.wave_cap;
    for (uint32_t i0 = 0; i0 < cnt; i0 += kWave * 8u) {
      uint32_t k[8];
#pragma unroll
      for (uint32_t u = 0; u < 8; ++u) k[u] = keys[min(i0 + u * kWave + lane, cnt - 1u)];  // clamped: all in flight
#pragma unroll
      for (uint32_t u = 0; u < 8; ++u)
        if (i0 + u * kWave + lane < cnt) visit(k[u]);
    }
  }
}

template <int LEVEL, bool LISTS>
__global__ __launch_bounds__(kRankBlock) void rank_pass_kernel(const float* const* __restrict__ updates,
                                                               RankCtl* __restrict__ ctls, uint32_t d, KeyLists kl) {
  __shared__ uint32_t hist[kRanksMax * kSubBins];
  __shared__ alignas(16) uint8_t first_cls[kTopBins];
  __shared__ uint32_t cls_prefix[kRanksMax + 1];
  RankCtl* ctl = ctls + blockIdx.y;
  const uint32_t n_cls = ctl->n_cls;
  for (uint32_t i = threadIdx.x; i < n_cls * kSubBins; i += kRankBlock) hist[i] = 0;
  for (uint32_t i = threadIdx.x; i < kTopBins / 4u; i += kRankBlock)
    reinterpret_cast<uint32_t*>(first_cls)[i] = 0xFFFFFFFFu;
  if (threadIdx.x <= kRanksMax) cls_prefix[threadIdx.x] = threadIdx.x < n_cls ? ctl->cls_prefix[threadIdx.x] : 0xFFFFFFFFu;
  __syncthreads();
  if (threadIdx.x < n_cls) {
    const uint32_t c = threadIdx.x;
    const uint32_t bin = LEVEL == 2 ? cls_prefix[c] : cls_prefix[c] >> kSubBits;
    const uint32_t before = c == 0 ? 0xFFFFFFFFu : (LEVEL == 2 ? cls_prefix[c - 1] : cls_prefix[c - 1] >> kSubBits);
    if (bin != before) first_cls[bin] = (uint8_t)c;
  }
  __syncthreads();
  auto visit = [&](uint32_t key) {
    const uint32_t bin = key >> kTopShift;
    uint32_t c = first_cls[bin];
    if (c == kNoClass) return;
    if (LEVEL == 2) {
      atomicAdd(&hist[c * kSubBins + ((key >> kSubBits) & (kSubBins - 1u))], 1u);
    } else {
      const uint32_t mine = key >> kSubBits;
      // the entry after the last class never starts with a level-1 bin, so the walk ends
      for (uint32_t p = cls_prefix[c]; (p >> kSubBits) == bin; p = cls_prefix[++c])
        if (p == mine) {
          atomicAdd(&hist[c * kSubBins + (key & (kSubBins - 1u))], 1u);
          break;
        }
    }
  };
  if (LISTS) list_keys(kl, visit); else stream_keys(updates[blockIdx.y], d, visit);
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < n_cls * kSubBins; i += kRankBlock) {
    const uint32_t h = hist[i];
    if (h) atomicAdd(&ctl->sub[i], h);
  }
}

// ------------------------------------------------------------------ the walks
// Ranks ascend, so their prefixes never increase: classes are runs of equal
// prefixes.  Called by the first 32 threads of a workgroup with the new prefix
// and inside-rank of rank `lane` (in LDS); writes the client's state.
// `ctl` may be null (nothing is written then).  Returns the number of classes; *cls_out / *opens_out: the
// caller's rank's class and whether that rank is the first of it.
__device__ __forceinline__ uint32_t write_classes(RankCtl* ctl, const uint32_t* s_prefix, const uint32_t* s_rem,
                                                  uint32_t n_ranks, uint32_t* cls_out = nullptr,
                                                  bool* opens_out = nullptr) {
  const uint32_t j = threadIdx.x;  // < 64, the first wavefront
  const bool live = j < n_ranks;
  const uint32_t mine = live ? s_prefix[j] : 0u;
  const bool opens = live && (j == 0 || s_prefix[j - 1] != mine);
  const uint64_t open_mask = __ballot(opens);
  const uint32_t c = lanes_below(open_mask) + (opens ? 1u : 0u) - 1u;  // classes opened up to and including j
  if (live && ctl) {
    ctl->prefix[j] = mine;
    ctl->rem[j] = s_rem[j];
    ctl->cls[j] = c;
    if (opens) ctl->cls_prefix[c] = mine;
  }
  const uint32_t n_cls = (uint32_t)__popcll(open_mask);
  if (j == 0 && ctl) ctl->n_cls = n_cls;
  if (cls_out) *cls_out = c;
  if (opens_out) *opens_out = opens;
  return n_cls;
}

// Level 1, whole workgroup: from the client's counts of key >> 18, the bin of every rank and the rank inside it
// (into LDS, valid after the next barrier).
__device__ __forceinline__ void level1_walk(const RankCtl* ctl, const RankSet& ranks, uint32_t* scan_tmp,
                                            uint32_t* s_prefix, uint32_t* s_rem) {
  // thread t owns `per` bins ending at top = kTopBins - 1 - per * t, largest keys first
  constexpr uint32_t per = kTopBins / kRankBlock;
  const uint32_t top = kTopBins - 1 - per * threadIdx.x;
  uint32_t h[per], mine = 0;
#pragma unroll
  for (uint32_t i = 0; i < per; ++i) {
    h[i] = ctl->top[top - i];
    mine += h[i];
  }
  uint32_t total;
  const uint32_t above = block_excl_scan<kRankWaves>(mine, scan_tmp, &total);
  for (uint32_t j = 0; j < ranks.n; ++j) {
    const uint32_t target = ranks.rank[j];
    if (above < target && target <= above + mine) {
      uint32_t acc = above;
#pragma unroll
      for (uint32_t i = 0; i < per; ++i) {
        if (acc < target && target <= acc + h[i]) {
          s_prefix[j] = top - i;
          s_rem[j] = target - acc;
        }
        acc += h[i];
      }
    }
  }
}

// (The three-pass path; with room for the key lists the collecting pass does this walk itself.)
__global__ __launch_bounds__(kRankBlock) void rank_walk1_kernel(RankCtl* __restrict__ ctls, RankSet ranks) {
  __shared__ uint32_t scan_tmp[kRankWaves];
  __shared__ uint32_t s_prefix[kRanksMax], s_rem[kRanksMax];
  RankCtl* ctl = ctls + blockIdx.x;
  level1_walk(ctl, ranks, scan_tmp, s_prefix, s_rem);
  __syncthreads();
  if (threadIdx.x < kWave) write_classes(ctl, s_prefix, s_rem, ranks.n);
}

// Ordinary least squares of ln(magnitude) on ln(rank) over the keys (in LDS) of the ranks: the logarithms
// side by side, the sums by one thread with the ranks in ascending order.  Whole workgroup.
__device__ __forceinline__ void fit_exponent(const uint32_t* s_keys, const RankSet& ranks, double* alpha_out) {
  __shared__ double s_x[kRanksMax], s_y[kRanksMax];
  if (threadIdx.x < ranks.n) {
    const double mag = (double)__uint_as_float(s_keys[threadIdx.x]);
    s_x[threadIdx.x] = log((double)ranks.rank[threadIdx.x]);
    s_y[threadIdx.x] = mag > 0.0 ? log(mag) : 0.0;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double sx = 0.0, sy = 0.0, sxx = 0.0, sxy = 0.0;
    uint32_t m = 0;
    for (uint32_t j = 0; j < ranks.n; ++j) {
      if (s_keys[j] == 0u) continue;  // a zero magnitude has no logarithm
      const double x = s_x[j], y = s_y[j];
      sx += x; sy += y; sxx += x * x; sxy += x * y; ++m;
    }
    *alpha_out = m < 2 ? -1.0 : ((double)m * sxy - sx * sy) / ((double)m * sxx - sx * sx);
  }
}

// One wavefront per class: lane l holds the 8 digits ending at 511 - 8 l.
template <int LEVEL>
__global__ __launch_bounds__(kRankBlock) void rank_walk_kernel(RankCtl* __restrict__ ctls, RankSet ranks,
                                                               uint32_t* __restrict__ keys_out,
                                                               double* __restrict__ alpha_out) {
  __shared__ uint32_t s_old_prefix[kRanksMax], s_old_rem[kRanksMax], s_cls[kRanksMax];
  __shared__ uint32_t s_prefix[kRanksMax], s_rem[kRanksMax];
  RankCtl* ctl = ctls + blockIdx.x;
  const uint32_t n_cls = ctl->n_cls;
  if (threadIdx.x < ranks.n) {
    s_old_prefix[threadIdx.x] = ctl->prefix[threadIdx.x];
    s_old_rem[threadIdx.x] = ctl->rem[threadIdx.x];
    s_cls[threadIdx.x] = ctl->cls[threadIdx.x];
  }
  __syncthreads();
  constexpr uint32_t per = kSubBins / kWave;
  const uint32_t lane = lane_id();
  for (uint32_t c = wave_id(); c < n_cls; c += kRankWaves) {
    uint32_t* bins = ctl->sub + c * kSubBins;
    const uint32_t top = kSubBins - 1 - per * lane;
    uint32_t h[per], mine = 0;
#pragma unroll
    for (uint32_t i = 0; i < per; ++i) {
      h[i] = bins[top - i];
      mine += h[i];
    }
    if (LEVEL == 2) {  // the next level counts into the same bins
#pragma unroll
      for (uint32_t i = 0; i < per; ++i) bins[top - i] = 0;
    }
    const uint32_t above = wave_incl_scan_u32(mine) - mine;
    for (uint32_t j = 0; j < ranks.n; ++j) {
      if (s_cls[j] != c) continue;
      const uint32_t target = s_old_rem[j];
      if (above < target && target <= above + mine) {
        uint32_t acc = above;
#pragma unroll
        for (uint32_t i = 0; i < per; ++i) {
          if (acc < target && target <= acc + h[i]) {
            s_prefix[j] = (s_old_prefix[j] << kSubBits) | (top - i);
            s_rem[j] = target - acc;
          }
          acc += h[i];
        }
      }
    }
  }
  __syncthreads();
  if (LEVEL == 2) {
    if (threadIdx.x < kWave) write_classes(ctl, s_prefix, s_rem, ranks.n);
    return;
  }
  // level 3: s_prefix holds the keys
  if (keys_out && threadIdx.x < kRanksMax)
    keys_out[(size_t)blockIdx.x * kRanksMax + threadIdx.x] = threadIdx.x < ranks.n ? s_prefix[threadIdx.x] : 0u;
  fit_exponent(s_prefix, ranks, alpha_out + blockIdx.x);
}

// ------------------------------------------------------------------ two passes: collect, select
// The keys of the class bins, as the collecting pass leaves them: list (client, workgroup, wavefront) holds
// list_cnt[...] keys in no particular order.
constexpr uint32_t kCollectStage = 512;  // keys a wavefront stages in LDS; rows of 64 leave once 256 are there

//
// Every workgroup first does the level-1 walk for itself (the counts are in L2; a launch of its own for it costs
// more), workgroup 0 of a client also leaves the result where the later kernels look for it.  The keys it
// collects are counted on their next 9 bits as they pass (level 2, per class, 64 KB of LDS).  With its 104 KB
// of LDS one workgroup has a CU to itself, which suits a streaming pass (241 against 252 us with two).
__global__ __launch_bounds__(kRankBlock) void rank_collect_kernel(const float* const* __restrict__ updates,
                                                                  RankCtl* __restrict__ ctls, RankSet ranks,
                                                                  uint32_t d, uint32_t* __restrict__ lists,
                                                                  uint32_t* __restrict__ list_cnt, uint32_t wave_cap) {
  __shared__ alignas(16) uint8_t first_cls[kTopBins];
  __shared__ uint32_t stage[kRankWaves][kCollectStage];
  __shared__ uint32_t s_fill[kRankWaves];  // keys a wavefront has staged
  __shared__ uint32_t level2[kRanksMax * kSubBins];
  __shared__ uint32_t scan_tmp[kRankWaves];
  __shared__ uint32_t s_prefix[kRanksMax], s_rem[kRanksMax];
  __shared__ uint32_t s_n_cls;
  RankCtl* ctl = ctls + blockIdx.y;
  for (uint32_t i = threadIdx.x; i < kTopBins / 4u; i += kRankBlock)
    reinterpret_cast<uint32_t*>(first_cls)[i] = 0xFFFFFFFFu;
  level1_walk(ctl, ranks, scan_tmp, s_prefix, s_rem);
  __syncthreads();
  if (threadIdx.x < kWave) {
    uint32_t c;
    bool opens;
    const uint32_t n = write_classes(blockIdx.x == 0 ? ctl : nullptr, s_prefix, s_rem, ranks.n, &c, &opens);
    if (opens) first_cls[s_prefix[threadIdx.x]] = (uint8_t)c;  // level-1 classes: one per bin
    if (threadIdx.x == 0) s_n_cls = n;
  }
  __syncthreads();
  const uint32_t n_cls = s_n_cls;
  for (uint32_t i = threadIdx.x; i < n_cls * kSubBins; i += kRankBlock) level2[i] = 0;
  __syncthreads();
  const uint32_t lane = lane_id(), wave = wave_id();
  const size_t list = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * kRankWaves + wave;
  uint32_t* __restrict__ out = lists + list * wave_cap;
  uint32_t* mine = stage[wave];
  uint32_t fill = 0, run = 0;  // staged keys as of the last look, keys already written (uniform over the wavefront)
  // LDS accesses of a wavefront complete in order; the fences keep the compiler from moving them.
  auto lds_fence = [] { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); };
  if (lane == 0) s_fill[wave] = 0;
  lds_fence();
  // Class keys are few (a lane meets one in every sixteenth float4 or so): the lanes that hold some take
  // their places in the wavefront's stage with an LDS atomic; the order of the keys in a list is free.
  auto take = [&](const uint32_t* k, uint32_t n_keys, bool valid) {
    uint32_t hit = 0, cls[4];
    for (uint32_t c = 0; c < n_keys; ++c) {
      cls[c] = first_cls[k[c] >> kTopShift];
      hit |= (cls[c] != kNoClass ? 1u : 0u) << c;
    }
    if (valid && hit) {
      uint32_t pos = atomicAdd(&s_fill[wave], (uint32_t)__popc(hit));
      for (uint32_t c = 0; c < n_keys; ++c)
        if ((hit >> c) & 1u) {
          mine[pos++] = k[c];
          atomicAdd(&level2[cls[c] * kSubBins + ((k[c] >> kSubBits) & (kSubBins - 1u))], 1u);
        }
    }
  };
  auto look = [&] {
    lds_fence();
    fill = __builtin_amdgcn_readfirstlane(s_fill[wave]);
  };
  auto flush = [&](bool all) {
    lds_fence();
    uint32_t g = 0;
    for (; g + kWave <= fill; g += kWave) out[run + g + lane] = mine[g + lane];
    const uint32_t left = fill - g;
    if (left) {
      const uint32_t k = lane < left ? mine[g + lane] : 0u;
      if (all) {
        if (lane < left) out[run + g + lane] = k;
        g += left;
      } else if (g) {  // the partial row moves to the front
        lds_fence();
        if (lane < left) mine[lane] = k;
      }
    }
    run += g;
    fill -= g;
    if (lane == 0) s_fill[wave] = fill;
    lds_fence();
  };
  const float* update = updates[blockIdx.y];
  const uint32_t n_quads = d / 4u;
  GlobalFloat4Ptr src = (GlobalFloat4Ptr)update;
  constexpr uint32_t kTileQuads = kRankBlock * kDeep;
  for (uint32_t q0 = blockIdx.x * kTileQuads; q0 < n_quads; q0 += gridDim.x * kTileQuads) {
    Float4V v[kDeep];
#pragma unroll
    for (uint32_t u = 0; u < kDeep; ++u) {
      const uint32_t q = q0 + u * kRankBlock + threadIdx.x;
      v[u] = __builtin_nontemporal_load(src + min(q, n_quads - 1u));
    }
#pragma unroll
    for (uint32_t u = 0; u < kDeep; ++u) {
      const uint32_t q = q0 + u * kRankBlock + threadIdx.x;
      uint32_t k[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) k[c] = __float_as_uint(v[u][c]) & 0x7FFFFFFFu;
      take(k, 4u, q < n_quads);
      look();
      if (fill >= kCollectStage - 4u * kWave) flush(false);  // room for the next four keys of every lane
    }
  }
  if (blockIdx.x == 0 && wave == 0) {  // the last d % 4 coordinates
    const bool valid = lane < d - n_quads * 4u;
    const uint32_t k = valid ? __float_as_uint(update[n_quads * 4u + lane]) & 0x7FFFFFFFu : 0u;
    take(&k, 1u, valid);
  }
  look();
  flush(true);
  if (lane == 0) list_cnt[list] = run;
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < n_cls * kSubBins; i += kRankBlock) {
    const uint32_t h = level2[i];
    if (h) atomicAdd(&ctl->sub[i], h);
  }
}

// Workgroups per client in a streaming pass: per_cu 1024-thread workgroups on every CU, never more than
// there are tiles.
uint32_t pass_blocks_per_client(uint32_t d, uint32_t n, uint32_t per_cu) {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, found = 0;
    cus = 256;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&found, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && found > 0)
      cus = found;
  }
  const uint32_t tiles = (d / 4u + kRankBlock * kDeep - 1) / (kRankBlock * kDeep);
  uint32_t b = ((uint32_t)cus * per_cu + n - 1) / n;
  if (b > tiles) b = tiles;
  return b < 1 ? 1u : b;
}

}  // namespace
}  // namespace cvlc

extern "C" {

uint32_t cvlc_fit_ranks(uint32_t d, uint32_t* ranks_out) {
  if (d == 0) return 0;
  uint32_t n = 0;
  for (uint64_t l = 1; l < d; l *= 2) {
    if (ranks_out) ranks_out[n] = (uint32_t)l;
    ++n;
  }
  if (ranks_out) ranks_out[n] = d;
  return n + 1;
}

size_t cvlc_fit_workspace_bytes(uint32_t n_clients) { return cvlc::rank_layout(n_clients, 0).total; }

size_t cvlc_fit_workspace_bytes_for(uint32_t n_clients, uint32_t d) {
  if (n_clients == 0 || d == 0 || d > 0x7FFFFFFFu) return 0;
  return cvlc::rank_layout(n_clients, d).total;
}

int cvlc_fit_alpha(uint32_t n, const float* const* d_updates, uint32_t d, double* d_alpha_out, uint32_t* d_keys_out,
                   void* d_workspace, size_t ws_bytes, void* hip_stream) {
  using namespace cvlc;
  if (n == 0 || !d_updates || !d_alpha_out || !d_workspace) return CVLC_ERR_ARG;
  if (d == 0 || d > 0x7FFFFFFFu || n > 65535u) return CVLC_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(d_workspace) % 256u) return CVLC_ERR_ARG;
  for (uint32_t i = 0; i < n; ++i)
    if (!d_updates[i] || reinterpret_cast<uintptr_t>(d_updates[i]) % 16u) return CVLC_ERR_ARG;
  RankLayout L = rank_layout(n, d);  // with room for the collected keys: two passes
  if (ws_bytes < L.total) L = rank_layout(n, 0);
  if (ws_bytes < L.total) return CVLC_ERR_CAPACITY;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* base = static_cast<char*>(d_workspace);
  uint32_t* status = reinterpret_cast<uint32_t*>(base + L.status);
  RankCtl* ctls = reinterpret_cast<RankCtl*>(base + L.ctl);
  const float** ptrs = reinterpret_cast<const float**>(base + L.ptrs);
  RankSet ranks;
  for (uint32_t j = 0; j < kRanksMax; ++j) ranks.rank[j] = 0;
  ranks.n = cvlc_fit_ranks(d, ranks.rank);

  StageScope scope(CVLC_STAGE_FIT_ALPHA, stream);
  {
    PtrChunk chunk;
    for (uint32_t first = 0; first < n; first += kPtrChunk) {
      chunk.first = first;
      chunk.count = n - first < kPtrChunk ? n - first : kPtrChunk;
      for (uint32_t i = 0; i < kPtrChunk; ++i) chunk.ptr[i] = i < chunk.count ? d_updates[first + i] : nullptr;
      const size_t zero_n16 = first == 0 ? L.zero_bytes / 16u : 0u;
      size_t blocks = (zero_n16 + 2047u) / 2048u;  // eight pieces per thread, within 1..1024 workgroups
      blocks = blocks < 1 ? 1 : (blocks > 1024 ? 1024 : blocks);
      hipLaunchKernelGGL(rank_init_kernel, dim3((uint32_t)blocks), dim3(256), 0, stream, ptrs, chunk,
                         reinterpret_cast<uint4*>(base), zero_n16);
    }
  }
  const dim3 pass_grid(pass_blocks_per_client(d, n, 2u), n);
  hipLaunchKernelGGL(rank_hist1_kernel, pass_grid, dim3(kRankBlock), 0, stream, ptrs, ctls, d, status);
  KeyLists kl = {nullptr, nullptr, 0u, 0u};
  if (L.wave_cap) {  // two passes: the keys of the class bins are set aside, levels 2 and 3 count among those
    uint32_t* lists = reinterpret_cast<uint32_t*>(base + L.lists);
    uint32_t* list_cnt = reinterpret_cast<uint32_t*>(base + L.list_cnt);
    kl.lists = lists;
    kl.list_cnt = list_cnt;
    kl.per_client = L.blocks * kRankWaves;
    kl.wave_cap = L.wave_cap;
    hipLaunchKernelGGL(rank_collect_kernel, dim3(L.blocks, n), dim3(kRankBlock), 0, stream, ptrs, ctls, ranks, d, lists,
                       list_cnt, L.wave_cap);
    // a few workgroups per client: their cost is clearing and adding up the counters, not reading the keys
    const dim3 list_grid(L.blocks < 16u ? L.blocks : 16u, n);
    hipLaunchKernelGGL(rank_walk_kernel<2>, dim3(n), dim3(kRankBlock), 0, stream, ctls, ranks, (uint32_t*)nullptr,
                       (double*)nullptr);
    hipLaunchKernelGGL((rank_pass_kernel<3, true>), list_grid, dim3(kRankBlock), 0, stream, ptrs, ctls, d, kl);
    hipLaunchKernelGGL(rank_walk_kernel<3>, dim3(n), dim3(kRankBlock), 0, stream, ctls, ranks, d_keys_out, d_alpha_out);
    return hip_check(hipGetLastError());
  }
  hipLaunchKernelGGL(rank_walk1_kernel, dim3(n), dim3(kRankBlock), 0, stream, ctls, ranks);
  hipLaunchKernelGGL((rank_pass_kernel<2, false>), pass_grid, dim3(kRankBlock), 0, stream, ptrs, ctls, d, kl);
  hipLaunchKernelGGL(rank_walk_kernel<2>, dim3(n), dim3(kRankBlock), 0, stream, ctls, ranks, (uint32_t*)nullptr,
                     (double*)nullptr);
  hipLaunchKernelGGL((rank_pass_kernel<3, false>), pass_grid, dim3(kRankBlock), 0, stream, ptrs, ctls, d, kl);
  hipLaunchKernelGGL(rank_walk_kernel<3>, dim3(n), dim3(kRankBlock), 0, stream, ctls, ranks, d_keys_out, d_alpha_out);
  return hip_check(hipGetLastError());
}

}  // extern "C"
