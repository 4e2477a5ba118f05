// Parameter-server side of libcvlc for gfx950: decode n clients' streams and
// aggregate them into one dense fp32 vector (Sec. III step 3 with the 1/B
// scaling of Sec. IV-B):  out[j] = sum_i w_i * xhat_{i,j}.
//
// Records are stored per (client, group) in ascending position, so every such
// list is sorted.  Each workgroup owns a tile of output coordinates, pulls the
// slice of every list that falls into its tile, accumulates in LDS in fp64 and
// writes the tile once; nothing is scattered into global memory.
//   parse_headers  validate headers (which must name the quantiser the caller
//                  expects), build one descriptor per list
//   compact_lists  the non-empty lists, numbered consecutively, with the
//                  tile_table work items they need
//   tile_table     one streaming pass over all records: for every list, the
//                  first record of every output tile (and the order/range checks)
//   decode_tiles   fused decode + accumulate + single write of each tile (a second
//                  instance splits QSGD's sign bit from the level)
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>

#include "cvlc_common.h"

namespace cvlc {
namespace {

constexpr uint32_t kListsPerClient = 32;   // descriptor slots per client (CVLC_MAX_CODED used)
constexpr uint32_t kTabChunk = 512;        // records per tile_table work item (one wavefront, eight a lane)
constexpr uint32_t kListBatch = 512;       // lists a decode workgroup handles per sweep

struct CompactDesc {  // one non-empty (client, group) record list, 32 bytes
  const uint32_t* payload;
  double weight;  // w_i
  uint32_t P;
  uint32_t wsy;   // W | s << 8 | y << 16
  float m, step;
};
static_assert(sizeof(CompactDesc) == 32, "CompactDesc is copied to LDS as two 16-byte pieces");

struct DecodeCtl {  // written by compact_lists
  uint32_t n_active;  // non-empty lists
  uint32_t n_items;   // tile_table work items in all
};

struct DecodeLayout {
  size_t status, ctl, stream_bad, desc, cdesc, item_start, table, total;
  uint32_t n_tiles, n_lists;
};

size_t align256(size_t v) { return (v + 255u) & ~(size_t)255u; }

struct StreamArg {  // per-stream inputs, passed as kernel arguments
  const uint32_t* words;
  uint64_t n_words;
  double weight;
  uint32_t has_weight;  // 0: derive 1/(n*B) from the header
  uint32_t pad;
};

DecodeLayout decode_layout(uint32_t d, uint32_t n) {
  DecodeLayout L;
  L.n_tiles = (uint32_t)(((uint64_t)d + kDecTile - 1) / kDecTile);
  L.n_lists = n * kListsPerClient;
  size_t off = 0;
  L.status = off; off = align256(off + 256);
  L.ctl = off; off = align256(off + sizeof(DecodeCtl));
  L.stream_bad = off; off = align256(off + (size_t)n * sizeof(uint32_t));
  L.desc = off; off = align256(off + (size_t)L.n_lists * sizeof(ListDesc));
  L.cdesc = off; off = align256(off + (size_t)L.n_lists * sizeof(CompactDesc));
  L.item_start = off; off = align256(off + ((size_t)L.n_lists + 1) * sizeof(uint32_t));
  L.table = off; off = align256(off + (size_t)(L.n_tiles + 1) * L.n_lists * sizeof(uint32_t));
  L.total = off;
  return L;
}

// The streams' pointers, sizes and weights travel as kernel arguments of the
// header pass (no pinned memory, no synchronisation), up to kParseStreams a launch.
constexpr uint32_t kParseStreams = 112;
struct ParseChunk {
  uint32_t first, count, pad[2];
  StreamArg args[kParseStreams];
};
static_assert(sizeof(ParseChunk) <= 3800, "kernel arguments are limited to 4 KB");

// Bits [bit, bit + W) of a little-endian word array, W <= 63.  Reads the three
// words the field can touch; `n_words` bounds the reads.
template <typename WordPtr>
__device__ __forceinline__ uint64_t read_bits(WordPtr words, uint64_t n_words, uint64_t bit, uint32_t W) {
  const uint64_t w = bit >> 5;
  const uint32_t sh = (uint32_t)(bit & 31u);
  const uint64_t a = words[w];
  const uint64_t b = (w + 1 < n_words) ? words[w + 1] : 0u;
  const uint64_t c = (w + 2 < n_words) ? words[w + 2] : 0u;
  uint64_t v = ((a | (b << 32)) >> sh);
  if (sh) v |= c << (64u - sh);
  return v & ((1ull << W) - 1ull);
}

// ------------------------------------------------------------------ 1. headers
// One wavefront per stream; lane r reads and checks the header of group r, so
// that the group headers are fetched together.  A stream that fails any check
// contributes nothing: all its lists are marked empty and the status bit is set.
typedef const uint32_t __attribute__((address_space(1))) * GlobalConstWordPtr;

__device__ __forceinline__ uint64_t wave_incl_scan_u64(uint64_t v) {
  const uint32_t lane = lane_id();
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t lo = __shfl_up((uint32_t)v, o, 64), hi = __shfl_up((uint32_t)(v >> 32), o, 64);
    if (lane >= (uint32_t)o) v += ((uint64_t)hi << 32) | lo;
  }
  return v;
}

// Whole wavefront: the headers of one stream.
__device__ __forceinline__ void parse_stream(const StreamArg& sa, uint32_t client, ListDesc* descs, uint32_t d, uint32_t n,
                                             uint32_t* __restrict__ stream_bad, uint32_t quant) {
  const uint32_t t = lane_id();
  GlobalConstWordPtr w = (GlobalConstWordPtr)sa.words;
  ListDesc* out = descs + (size_t)client * kListsPerClient;
  bool ok = sa.n_words >= kGlobalHeaderWords;  // everything about `ok` is uniform over the wavefront
  uint32_t g[kGlobalHeaderWords] = {0, 0, 0, 0, 0, 0, 0, 0};
  // The group headers are asked for together with the global header, before the number of groups is known
  // (lane r: where group r's header would be, clamped to the stream), so that one memory round trip serves both.
  uint32_t hw[kSegHeaderWords] = {0, 0, 0, 0};
  if (ok) {
#pragma unroll
    for (uint32_t i = 0; i < kGlobalHeaderWords; ++i) g[i] = w[i];
#pragma unroll
    for (uint32_t i = 0; i < kSegHeaderWords; ++i)
      hw[i] = w[min((uint64_t)(kGlobalHeaderWords + kSegHeaderWords * min(t, CVLC_MAX_CODED - 1u) + i), sa.n_words - 1u)];
  }
  const uint32_t R = g[3], s = g[4];
  const float B = __uint_as_float(g[5]);
  ok = ok && g[0] == kMagic && g[1] == (kVersion | (quant << 16)) && g[2] == d && R <= CVLC_MAX_CODED && s == position_bits(d) &&
       B > 0.0f && fabsf(B) <= 3.4028234664e38f;
  const uint64_t first_payload = kGlobalHeaderWords + (uint64_t)kSegHeaderWords * R;
  ok = ok && sa.n_words >= first_payload;
  const bool mine = ok && t < R;
  uint32_t y = 0, P = 0;
  float m = 0.0f, M = 0.0f;
  if (mine) {  // t < R <= 31 and the stream holds all R headers: the words read above are group t's
    y = hw[0];
    P = hw[1];
    m = __uint_as_float(hw[2]);
    M = __uint_as_float(hw[3]);
  }
  bool header_ok = !mine || (code_len_supported(y) && fabsf(m) <= 3.4028234664e38f &&
                             fabsf(M) <= 3.4028234664e38f && fabsf(M - m) <= 3.4028234664e38f);
  if (quant == CVLC_QUANT_QSGD && mine)  // {norm, 0}; a sign bit and at least one level bit
    header_ok = header_ok && y >= 2 && m >= 0.0f && __float_as_uint(M) == 0u;
  ok = ok && __ballot(header_ok) == ~0ull;
  // where every group's records start, and what the stream must add up to (sizes of groups with a bad header
  // do not matter: the stream is rejected)
  const uint64_t words = mine && header_ok ? payload_words(P, s + y) : 0u;
  const uint64_t incl = wave_incl_scan_u64(words);
  const uint64_t k_incl = wave_incl_scan_u64(mine ? P : 0u);
  const uint64_t total = first_payload + (((uint64_t)__shfl((uint32_t)(incl >> 32), 63, 64) << 32) | __shfl((uint32_t)incl, 63, 64));
  const uint64_t k = ((uint64_t)__shfl((uint32_t)(k_incl >> 32), 63, 64) << 32) | __shfl((uint32_t)k_incl, 63, 64);
  ok = ok && k <= d && total == g[7] && sa.n_words >= total;
  if (t == 0) stream_bad[client] = ok ? 0u : 1u;  // gathered into the status word by the next kernel
  if (t < kListsPerClient) {
    ListDesc ld;
    ld.payload = nullptr; ld.weight = 0.0; ld.P = 0; ld.W = 0; ld.s = 0; ld.y = 0; ld.m = 0.0f; ld.step = 0.0f;
    if (ok && t < R) {
      float step = 0.0f, inv = 0.0f;
      if (y != 32) {
        if (quant == CVLC_QUANT_QSGD) {  // levels 0 .. 2^(y-1) - 1 on [0, norm]
          centroid_spacing(0.0f, m, y - 1u, &step, &inv);
          m = 0.0f;
        } else {
          centroid_spacing(m, M, y, &step, &inv);
        }
      }
      ld.payload = sa.words + (first_payload + incl - words);
      ld.weight = sa.has_weight ? sa.weight : 1.0 / ((double)n * (double)B);
      ld.P = P;
      ld.s = s;
      ld.y = y;
      ld.W = s + y;
      ld.m = m;
      ld.step = step;
    }
    out[t] = ld;
  }
}

__global__ __launch_bounds__(64) void parse_headers_kernel(ParseChunk chunk, ListDesc* descs, uint32_t d, uint32_t n,
                                                           uint32_t* __restrict__ stream_bad, uint32_t quant) {
  parse_stream(chunk.args[blockIdx.x], chunk.first + blockIdx.x, descs, d, n, stream_bad, quant);
}

// ------------------------------------------------------------------ 1b. the non-empty lists
// One workgroup of 1024 threads.  Lists with records are numbered in (client,
// group) order; item_start is the exclusive prefix of their tile_table work items.
__device__ __forceinline__ void compact_lists(const ListDesc* descs, uint32_t n_lists, CompactDesc* __restrict__ cdesc,
                                              uint32_t* __restrict__ item_start, DecodeCtl* ctl,
                                              const uint32_t* stream_bad, uint32_t n, uint32_t* status, uint32_t* scan_tmp) {
  const uint32_t tid = threadIdx.x;
  // the call's status word starts here: set if any stream failed its header checks
  uint32_t any_bad = 0;
  for (uint32_t i = tid; i < n; i += 1024) any_bad |= stream_bad[i];
  any_bad = __syncthreads_or((int)any_bad) ? 1u : 0u;
  if (tid == 0) *status = any_bad ? CVLC_DEV_STREAM : 0u;
  uint32_t lists_before = 0, items_before = 0;
  for (uint32_t base = 0; base < n_lists; base += 1024) {
    const uint32_t l = base + tid;
    ListDesc ld;
    ld.P = 0;
    if (l < n_lists) ld = descs[l];
    const uint32_t live = ld.P > 0 ? 1u : 0u;
    const uint32_t items = (ld.P + kTabChunk - 1) / kTabChunk;
    uint32_t tot_l, tot_i;
    const uint32_t pos = lists_before + block_excl_scan<16>(live, scan_tmp, &tot_l);
    const uint32_t first = items_before + block_excl_scan<16>(items, scan_tmp, &tot_i);
    if (live) {
      CompactDesc c;
      c.payload = ld.payload; c.weight = ld.weight; c.P = ld.P; c.wsy = ld.W | (ld.s << 8) | (ld.y << 16);
      c.m = ld.m; c.step = ld.step;
      cdesc[pos] = c;
      item_start[pos] = first;
    }
    lists_before += tot_l;
    items_before += tot_i;
  }
  if (tid == 0) {
    item_start[lists_before] = items_before;
    ctl->n_active = lists_before;
    ctl->n_items = items_before;
  }
}

__global__ __launch_bounds__(1024) void compact_lists_kernel(const ListDesc* __restrict__ descs, uint32_t n_lists,
                                                             CompactDesc* __restrict__ cdesc,
                                                             uint32_t* __restrict__ item_start, DecodeCtl* ctl,
                                                             const uint32_t* __restrict__ stream_bad, uint32_t n,
                                                             uint32_t* status) {
  __shared__ uint32_t scan_tmp[16];
  compact_lists(descs, n_lists, cdesc, item_start, ctl, stream_bad, n, status, scan_tmp);
}

// Both steps in one launch, for calls whose streams fit one set of kernel arguments: the sixteen wavefronts
// share out the streams, then the workgroup numbers the lists it has just described.
__global__ __launch_bounds__(1024) void setup_kernel(ParseChunk chunk, ListDesc* descs, uint32_t d, uint32_t quant,
                                                     CompactDesc* __restrict__ cdesc, uint32_t* __restrict__ item_start,
                                                     DecodeCtl* ctl, uint32_t* stream_bad, uint32_t* status) {
  __shared__ uint32_t scan_tmp[16];
  const uint32_t n = chunk.count;
  for (uint32_t i = threadIdx.x / kWave; i < n; i += 1024u / kWave)  // uniform per wavefront
    parse_stream(chunk.args[i], i, descs, d, n, stream_bad, quant);
  __threadfence_block();
  __syncthreads();  // the descriptors and flags written above are read below by other wavefronts of this workgroup
  compact_lists(descs, n * kListsPerClient, cdesc, item_start, ctl, stream_bad, n, status, scan_tmp);
}

// ------------------------------------------------------------------ 2. tile table
// table[list][t] = index of the first record of `list` whose position lies in
// output tile t or later; entry n_tiles holds the list length.  (List-major: a
// list's entries are written in ascending t by neighbouring threads.)  A work
// item is a run of kTabChunk records of one list and belongs to one wavefront:
// lane l reads the position fields of records l, l + 64, ... of the run straight
// from the stream (neighbouring lanes, neighbouring words), all of them in flight
// together, and compares each with the one before it.  Wavefronts never wait for
// each other.  The pass also checks that positions ascend and stay below d.
constexpr uint32_t kTabTurns = kTabChunk / kWave;  // records of an item a lane looks at

__global__ __launch_bounds__(kBlock, 8) void tile_table_kernel(const CompactDesc* __restrict__ cdesc,
                                                         const uint32_t* __restrict__ item_start,
                                                         const DecodeCtl* __restrict__ ctl, uint32_t* table,
                                                         uint32_t d, uint32_t n_tiles, uint32_t* status) {
  constexpr uint32_t kStartCache = 2048;
  __shared__ uint32_t s_start[kStartCache];
  const uint32_t tid = threadIdx.x, lane = lane_id();
  const uint32_t n_active = ctl->n_active, n_items = ctl->n_items;
  const bool cached = n_active <= kStartCache;
  if (cached)
    for (uint32_t i = tid; i < n_active; i += kBlock) s_start[i] = item_start[i];
  __syncthreads();
  const uint32_t n_waves = gridDim.x * kWavesPerBlock;
  bool bad = false;
  for (uint32_t q = blockIdx.x * kWavesPerBlock + tid / kWave; q < n_items; q += n_waves) {  // uniform per wavefront
    uint32_t a = 0, b = n_active;  // the list that owns item q: last list with item_start <= q
    while (b - a > 1) {
      const uint32_t mid = (a + b) >> 1;
      const uint32_t v = cached ? s_start[mid] : item_start[mid];
      if (v <= q) a = mid; else b = mid;
    }
    a = __builtin_amdgcn_readfirstlane(a);
    const uint32_t first_item = __builtin_amdgcn_readfirstlane(cached ? s_start[a] : item_start[a]);
    // the list's descriptor is the same for all lanes: keeping it in scalar registers keeps the address
    // arithmetic of the loads below off the vector unit
    const uint4* dsrc = reinterpret_cast<const uint4*>(cdesc + a);
    const uint4 d0 = dsrc[0], d1 = dsrc[1];
    GlobalConstWordPtr pay = (GlobalConstWordPtr)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane(d0.y) << 32) |
                                                  (uint32_t)__builtin_amdgcn_readfirstlane(d0.x));
    const uint32_t P = __builtin_amdgcn_readfirstlane(d1.x), wsy = __builtin_amdgcn_readfirstlane(d1.y);
    const uint32_t W = wsy & 0xFFu, s = (wsy >> 8) & 0xFFu;
    const uint32_t pid_mask = s >= 32 ? 0xFFFFFFFFu : (1u << s) - 1u;
    const uint32_t e0 = (q - first_item) * kTabChunk, cnt = min(P - e0, kTabChunk);
    uint32_t* row = table + (size_t)a * (n_tiles + 1);
    // The window of the item starts at the record before the run (the run's first record for the first
    // item of a list); records are addressed by their number in the window, bits by their offset from the
    // window's first word: both stay far below 2^24.
    const uint32_t lead = e0 ? 1u : 0u;
    const uint64_t bit0 = (uint64_t)(e0 - lead) * W;
    GlobalConstWordPtr src = pay + (bit0 >> 5);
    const uint32_t sh0 = (uint32_t)bit0 & 31u;
    const uint64_t words_left = ((((uint64_t)P * W + 31u) >> 5) - 1u) - (bit0 >> 5);  // the list's last word, from src
    const uint32_t rel_last = words_left < (1u << 24) ? (uint32_t)words_left : 1u << 24;
    // position field of record r of the window: its s <= 31 low bits lie in at most two words
    auto request = [&](uint32_t r, uint32_t& w0, uint32_t& w1) {
      const uint32_t bit = sh0 + __umul24(r, W), w = bit >> 5;
      w0 = src[w];
      w1 = src[min(w + 1u, rel_last)];
      return bit & 31u;
    };
    uint32_t lo[kTabTurns], hi[kTabTurns], sh[kTabTurns], c_lo, c_hi, c_sh;
    c_sh = request(0u, c_lo, c_hi);  // the record before the run (uniform)
#pragma unroll
    for (uint32_t i = 0; i < kTabTurns; ++i)  // no branch: a lane past the end reads the last record again
      sh[i] = request(lead + min(i * kWave + lane, cnt - 1u), lo[i], hi[i]);
    uint32_t carry = __builtin_amdgcn_alignbit(c_hi, c_lo, c_sh) & pid_mask;
#pragma unroll
    for (uint32_t i = 0; i < kTabTurns; ++i) {
      if (i * kWave >= cnt) break;  // uniform
      const uint32_t j = i * kWave + lane;
      const bool live = j < cnt;
      const uint32_t e = e0 + j;
      const uint32_t pid = __builtin_amdgcn_alignbit(hi[i], lo[i], sh[i]) & pid_mask;
      // the record before mine sits in the lane below; lane 0 takes the last one of the turn before
      const uint32_t prev = (uint32_t)__builtin_amdgcn_update_dpp((int)carry, (int)pid, 0x138 /* wave_shr:1 */, 0xF, 0xF, false);
      carry = __builtin_amdgcn_readlane(pid, kWave - 1);
      // a position past the end (an error, reported below) counts as lying behind the last tile
      const uint32_t t_cur = min(pid / kDecTile, n_tiles), t_prev = min(prev / kDecTile, n_tiles);
      const bool first = e == 0, last = e == P - 1;
      bad |= live && ((!first && prev >= pid) || pid >= d);  // positions must ascend strictly and stay below d
      // entries (tile of record e-1, tile of record e] point at e; past the last record they hold P
      const bool starts = live && (first || last || t_cur != t_prev);
      if (!__ballot(starts)) continue;
      const uint32_t t_first = first ? 0u : t_prev + 1u;
      const bool single = starts && !last && t_first == t_cur;  // nearly always: the next tile, one entry
      if (single) row[t_cur] = e;
      if (!__ballot(starts && !single)) continue;
      const bool run = starts && !single && t_cur >= t_first;
      uint32_t tail_first = 1, tail_last = 0;
      if (starts && last) {
        tail_first = t_cur + 1;
        tail_last = n_tiles;
      }
      // short runs of entries are written by the lane that found them, long ones (the stretch before a
      // list's first record, after its last, or across a region it skips) by the whole wavefront
      constexpr uint32_t kLong = 16;
      const bool long_run = run && t_cur - t_first >= kLong;
      const bool long_tail = tail_last >= tail_first;
      if (run && !long_run)
        for (uint32_t t = t_first; t <= t_cur; ++t) row[t] = e;
      uint64_t todo = __ballot(long_run);
      while (todo) {
        const uint32_t from = (uint32_t)__builtin_ctzll(todo);
        const uint32_t a0 = __builtin_amdgcn_readlane(t_first, from), a1 = __builtin_amdgcn_readlane(t_cur, from);
        const uint32_t val = __builtin_amdgcn_readlane(e, from);
        for (uint32_t t = a0 + lane; t <= a1; t += kWave) row[t] = val;
        todo &= todo - 1;
      }
      todo = __ballot(long_tail);
      while (todo) {
        const uint32_t from = (uint32_t)__builtin_ctzll(todo);
        const uint32_t a0 = __builtin_amdgcn_readlane(tail_first, from), a1 = __builtin_amdgcn_readlane(tail_last, from);
        for (uint32_t t = a0 + lane; t <= a1; t += kWave) row[t] = P;
        todo &= todo - 1;
      }
    }
  }
  if (bad) atomicOr(status, CVLC_DEV_STREAM);
}

// ------------------------------------------------------------------ 3. fused decode + accumulate
// Persistent workgroups walk the output tiles, neighbouring tiles at the same
// time on the same XCD (see tile_of below).  The records of a tile, over all lists, are numbered
// 0..total-1 list by list (an exclusive scan of the slice lengths); every
// wavefront takes a contiguous share of them, 64 at a time ("turn"), so the work
// is even however the records are spread over the lists and neighbouring lanes
// read neighbouring records.  Which list a lane's record belongs to: the
// non-empty slices that start inside the turn set a bit at their first record's
// place in a 64-bit mask, and a lane counts the bits at or below its own place;
// only the wavefront's first record needs a search.  List descriptors sit in LDS.
constexpr uint32_t kDecBlock = 512;  // threads of a decode workgroup
constexpr uint32_t kDecWaves = kDecBlock / kWave;
constexpr uint32_t kDecTurns = 6;    // turns of 64 records a wavefront works on together
constexpr uint32_t kChunkTiles = 16; // consecutive tiles decoded side by side on one XCD (more: less refetching, less even load)
constexpr uint32_t kFirstBits = 22;  // a tile's records over one batch of lists are numbered below 2^22 ...
constexpr uint32_t kFirstMask = (1u << kFirstBits) - 1u;
static_assert((uint64_t)kListBatch * kDecTile < (1ull << kFirstBits) && kListBatch <= (1u << (32 - kFirstBits)),
              "... and the list of a slice fits above that number in one word");
static_assert(kListBatch == kDecBlock, "one list per thread and batch");

struct DecodeShared {
  double acc[kDecTile];
  uint4 desc[kListBatch][2];       // CompactDesc, as loaded
  // per non-empty slice of the batch, in list order
  uint32_t begin[kListBatch];      // first record of the slice inside its list
  uint32_t first[kListBatch + 1];  // number of the slice's first record in the tile | list << kFirstBits; then the total
  unsigned long long turn_mask[kDecWaves][kDecTurns];  // per wavefront: starts of slices inside each of its current turns
  uint32_t scan_a[kDecWaves], scan_b[kDecWaves];
};

// Exclusive prefix sums of two values per thread over the workgroup, in thread order.
__device__ __forceinline__ void block_excl_scan2(uint32_t va, uint32_t vb, uint32_t* sa, uint32_t* sb, uint32_t* before_a,
                                                 uint32_t* before_b, uint32_t* total_a, uint32_t* total_b) {
  const uint32_t ia = wave_incl_scan_u32(va), ib = wave_incl_scan_u32(vb);
  const uint32_t wave = threadIdx.x / kWave;
  __syncthreads();
  if (lane_id() == kWave - 1) {
    sa[wave] = ia;
    sb[wave] = ib;
  }
  __syncthreads();
  uint32_t ba = 0, bb = 0, ta = 0, tb = 0;
#pragma unroll
  for (uint32_t w = 0; w < kDecWaves; ++w) {
    const uint32_t xa = sa[w], xb = sb[w];
    if (w < wave) { ba += xa; bb += xb; }
    ta += xa;
    tb += xb;
  }
  *before_a = ba + ia - va;
  *before_b = bb + ib - vb;
  *total_a = ta;
  *total_b = tb;
}

// LDS accesses of one wavefront complete in order; this keeps the compiler from
// moving them across the point where lanes read what other lanes wrote.
__device__ __forceinline__ void wave_lds_fence() { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); }

// SIGNED: the streams' codes hold a sign bit above the level (QSGD).
template <bool SIGNED>
__global__ __launch_bounds__(kDecBlock, 6) void decode_tiles_kernel(const CompactDesc* __restrict__ cdesc,
                                                              const DecodeCtl* __restrict__ ctl,
                                                              const uint32_t* __restrict__ table, float* out,
                                                              uint32_t d, uint32_t n_tiles, uint32_t accumulate,
                                                              uint32_t* status) {
  __shared__ DecodeShared S;
  const uint32_t tid = threadIdx.x, lane = lane_id();
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const uint32_t n_active = ctl->n_active;
  const bool one_batch = n_active <= kListBatch;
  bool bad = false;
  auto load_descs = [&](uint32_t l0, uint32_t nl) {
    const uint4* src = reinterpret_cast<const uint4*>(cdesc + l0);
    for (uint32_t i = tid; i < nl * 2u; i += kDecBlock) (&S.desc[0][0])[i] = src[i];
  };
  if (one_batch) load_descs(0, n_active);
  // the two table entries of this thread's list (first batch) for the next tile, asked for a tile ahead
  auto request_rows = [&](uint32_t tile) {
    uint2 r = make_uint2(0u, 0u);
    if (tile < n_tiles && tid < min(n_active, kListBatch)) {
      const uint32_t* row = table + (size_t)tid * (n_tiles + 1) + tile;
      r.x = row[0];
      r.y = row[1];
    }
    return r;
  };
  // Which tiles a workgroup takes.  Workgroup b runs on XCD b mod 8, and every XCD has an L2 of its own: a
  // tile's slice of a list shares its first and last cache line with the neighbouring tiles', so chunks of
  // kChunkTiles consecutive tiles are decoded at the same time by as many workgroups of one XCD, and the
  // chunks go round the XCDs (whole eighths of the vector per XCD would leave the XCD with the dense layers
  // behind).  Grids that do not divide into such chunks (fewer tiles than the device holds): tile b, b + grid, ...
  const bool chunked = gridDim.x % (8u * kChunkTiles) == 0;
  const uint32_t xcd = blockIdx.x & 7u, seat = blockIdx.x >> 3, chunks_at_once = gridDim.x / (8u * kChunkTiles);
  auto tile_of = [&](uint32_t r) {
    return chunked ? ((seat / kChunkTiles + chunks_at_once * r) * 8u + xcd) * kChunkTiles + seat % kChunkTiles
                   : blockIdx.x + r * gridDim.x;
  };
  uint32_t round = 0;
  uint2 next_rows = request_rows(tile_of(0));
  for (uint32_t tile = tile_of(0); tile < n_tiles; tile = tile_of(++round)) {
    const uint32_t lo = tile * kDecTile;
    const uint2 rows = next_rows;
    next_rows = request_rows(tile_of(round + 1u));
    __syncthreads();  // the tile before is written out; the descriptors are in place
    for (uint32_t i = tid; i < kDecTile; i += kDecBlock) S.acc[i] = 0.0;
    for (uint32_t l0 = 0; l0 < n_active; l0 += kListBatch) {
      const uint32_t nl = min(n_active - l0, kListBatch);
      if (!one_batch) {
        __syncthreads();
        load_descs(l0, nl);
        __syncthreads();
      }
      // this thread's list: its slice [begin, end) from two neighbouring table entries
      uint32_t len = 0, begin = 0;
      if (tid < nl) {
        const uint32_t P = S.desc[tid][1].x;
        uint32_t end;
        if (l0 == 0) {
          begin = rows.x;
          end = rows.y;
        } else {
          const uint32_t* row = table + (size_t)(l0 + tid) * (n_tiles + 1) + tile;
          begin = row[0];
          end = row[1];
        }
        if (begin > P) begin = P;  // table entries of a malformed list may hold anything
        if (end > P) end = P;
        if (end > begin) len = end - begin;
        if (len > kDecTile) {  // positions ascend strictly: a tile holds at most one record per coordinate
          bad = true;
          len = 0;
        }
      }
      uint32_t before, j, total, n_live;
      // (its barriers also separate the writes below from the reads of the batch before)
      block_excl_scan2(len, len ? 1u : 0u, S.scan_a, S.scan_b, &before, &j, &total, &n_live);
      if (len) {
        S.first[j] = before | (tid << kFirstBits);
        S.begin[j] = begin;
      }
      if (tid == 0) S.first[n_live] = total;
      __syncthreads();
      // the wavefront's share of the records, a multiple of 64
      const uint32_t share = ((total + kDecBlock - 1) / kDecBlock) * kWave;
      const uint32_t q_begin = min(wave * share, total), q_end = min(q_begin + share, total);
      if (q_begin < q_end) {  // uniform per wavefront
        // last slice whose first record is at or before the first record of the turns at hand (uniform): the
        // lanes look at all slices of the batch at once (first[] ascends; slice 0 starts at record 0)
        uint32_t cur = 0;
        {
          uint32_t at_or_before = 0;
#pragma unroll
          for (uint32_t k = 0; k < kListBatch / kWave; ++k) {
            const uint32_t i = k * kWave + lane;
            const bool hit = i < n_live && (S.first[min(i, n_live)] & kFirstMask) <= q_begin;
            at_or_before += (uint32_t)__popcll(__ballot(hit));
          }
          cur = __builtin_amdgcn_readfirstlane(at_or_before) - 1u;
        }
        // kDecTurns turns at a time.  First the start masks of all of them; then, turn by turn but without one
        // turn waiting for another, list and record number from LDS; then all record loads together, so that their
        // latencies overlap.  Nothing in this half branches on data (a lane past the end works on the last record
        // again, the words after a record's first are clamped to the record's last), so that no load has to be
        // waited for before the next one is issued.
        unsigned long long* masks = S.turn_mask[wave];
        for (uint32_t q0 = q_begin; q0 < q_end; q0 += kWave * kDecTurns) {
          const uint32_t n_turns = __builtin_amdgcn_readfirstlane(min((q_end - q0 + kWave - 1u) / kWave, kDecTurns));
          // slices after `cur` that start inside the turns: first[] ascends strictly, first[n_live] = total.
          // 64 slices are looked at per round; more start inside the turns only when most hold a few records.
          if (lane < kDecTurns) masks[lane] = 0ull;
          wave_lds_fence();
          for (uint32_t seen = 0;; seen += kWave) {  // uniform
            const uint32_t idx = cur + 1u + seen + lane;
            const uint32_t f = (S.first[min(idx, n_live)] & kFirstMask) - q0;  // >= 0
            if (idx <= n_live && f < kWave * kDecTurns) atomicOr(&masks[f >> 6], 1ull << (f & 63u));
            // done when the last one looked at lies past the turns at hand, or nothing is left to look at
            if (cur + seen + kWave >= n_live || __builtin_amdgcn_readlane(f, kWave - 1) >= kWave * n_turns) break;
          }
          wave_lds_fence();
          uint32_t base_of[kDecTurns], w0[kDecTurns], w1[kDecTurns], w2[kDecTurns], at[kDecTurns];  // at: list | bit inside the first word << 9
          unsigned long long starts[kDecTurns];
#pragma unroll
          for (uint32_t u = 0; u < kDecTurns; ++u) starts[u] = masks[u];
#pragma unroll
          for (uint32_t u = 0; u < kDecTurns; ++u) {
            base_of[u] = cur;
            if (u < n_turns)  // uniform; the sentinel's bit lies in the last turn at hand or past it
              cur += (uint32_t)__popc((uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)starts[u])) +
                     (uint32_t)__popc((uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(starts[u] >> 32)));
          }
          uint32_t x_of[kDecTurns], e_of[kDecTurns];
#pragma unroll
          for (uint32_t u = 0; u < kDecTurns; ++u) {
            x_of[u] = e_of[u] = 0;
            if (u >= n_turns) continue;          // uniform
            const uint32_t qt = q0 + u * kWave;  // the turn's first record (uniform)
            const uint32_t place = min(lane, q_end - 1u - qt);
            const uint32_t a = base_of[u] + (uint32_t)__popcll(starts[u] & ((2ull << place) - 1ull));
            x_of[u] = S.first[a];
            e_of[u] = S.begin[a] + (qt + place);
          }
#pragma unroll
          for (uint32_t u = 0; u < kDecTurns; ++u) {
            w0[u] = w1[u] = w2[u] = at[u] = 0;
            if (u >= n_turns) continue;  // uniform
            const uint32_t li = x_of[u] >> kFirstBits;
            const uint32_t e = e_of[u] - (x_of[u] & kFirstMask);
            const uint2 ptr = *reinterpret_cast<const uint2*>(&S.desc[li][0]);  // payload
            const uint32_t W = S.desc[li][1].y & 0xFFu;
            GlobalConstWordPtr pay = (GlobalConstWordPtr)(((uint64_t)ptr.y << 32) | ptr.x);
            const uint64_t bit = (uint64_t)e * W;
            const uint32_t w = (uint32_t)(bit >> 5), sh = (uint32_t)bit & 31u;  // payloads have fewer than 2^32 words
            const uint32_t w_end = w + ((sh + W - 1u) >> 5);                   // the word that holds the record's last bit
            at[u] = li | (sh << 9);
            w0[u] = pay[w];
            w1[u] = pay[min(w + 1u, w_end)];
            w2[u] = pay[min(w + 2u, w_end)];
          }
#pragma unroll
          for (uint32_t u = 0; u < kDecTurns; ++u) {
            if (u >= n_turns) continue;  // uniform
            if (q0 + u * kWave + lane >= q_end) continue;
            const uint32_t li = at[u] & 511u, sh = at[u] >> 9;
            const uint4 d0 = S.desc[li][0], d1 = S.desc[li][1];
            const uint32_t s = (d1.y >> 8) & 0xFFu, y = (d1.y >> 16) & 0xFFu;
            const double weight = __hiloint2double((int)d0.w, (int)d0.z);
            const uint32_t lo32 = __builtin_amdgcn_alignbit(w1[u], w0[u], sh);  // bits [sh, sh + 32) of the three words
            const uint32_t hi32 = __builtin_amdgcn_alignbit(w2[u], w1[u], sh);  // bits [sh + 32, sh + 64)
            const uint32_t pid = lo32 & (s >= 32 ? 0xFFFFFFFFu : (1u << s) - 1u);
            const uint32_t code_mask = y >= 32 ? 0xFFFFFFFFu : (1u << y) - 1u;
            const uint32_t cid = __builtin_amdgcn_alignbit(hi32, lo32, s & 31u) & code_mask;  // s <= 31
            if (pid - lo >= kDecTile || pid >= d) { bad = true; continue; }  // a position below the tile wraps to a large value
            float xhat;
            if (y == 32) {
              xhat = __uint_as_float(cid);
            } else if (SIGNED) {
              const float mag = __fmaf_rn((float)(cid & ((1u << (y - 1u)) - 1u)), __uint_as_float(d1.w), __uint_as_float(d1.z));
              xhat = __uint_as_float(__float_as_uint(mag) ^ ((cid >> (y - 1u)) << 31));
            } else {
              xhat = __fmaf_rn((float)cid, __uint_as_float(d1.w), __uint_as_float(d1.z));
            }
            atomicAdd(&S.acc[pid - lo], weight * (double)xhat);
          }
        }
      }
    }
    __syncthreads();
    // four pairs of coordinates per thread, neighbouring lanes neighbouring pairs (LDS reads without bank
    // conflicts, 512-byte stores per wavefront): all reads first, then the stores
    static_assert(kDecTile == kDecBlock * 8u, "four pairs of coordinates per thread");
    {
      double2 v[4];
#pragma unroll
      for (uint32_t c = 0; c < 4u; ++c) v[c] = *reinterpret_cast<const double2*>(&S.acc[c * (2u * kDecBlock) + tid * 2u]);
      const bool aligned = (reinterpret_cast<uintptr_t>(out + lo) & 7u) == 0;  // uniform
#pragma unroll
      for (uint32_t c = 0; c < 4u; ++c) {
        const uint32_t j0 = lo + c * (2u * kDecBlock) + tid * 2u;
        if (aligned && j0 + 2u <= d) {
          float2* dst = reinterpret_cast<float2*>(out + j0);
          if (accumulate) {
            const float2 o = *dst;
            v[c].x += (double)o.x;
            v[c].y += (double)o.y;
          }
          *dst = make_float2((float)v[c].x, (float)v[c].y);
        } else {
          if (j0 < d) out[j0] = (float)(accumulate ? v[c].x + (double)out[j0] : v[c].x);
          if (j0 + 1u < d) out[j0 + 1u] = (float)(accumulate ? v[c].y + (double)out[j0 + 1u] : v[c].y);
        }
      }
    }
  }
  if (bad) atomicOr(status, CVLC_DEV_STREAM);
}

// ------------------------------------------------------------------ scratch for callers that cannot allocate
// cvlc_decode_aggregate_static works in this array instead of a caller's
// workspace.  Every device the library runs on holds its own copy at its own
// address; host code never uses the array's name as an address, only what
// hipGetSymbolAddress returned for the current device.
static __device__ __align__(256) unsigned char scratch[CVLC_DECODE_STATIC_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CVLC_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CVLC_ERR_DEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CVLC_OK;
}

__global__ void copy_status_kernel(const uint32_t* __restrict__ status, uint32_t* __restrict__ dst) { *dst = *status; }

}  // namespace
}  // namespace cvlc

extern "C" {

size_t cvlc_decode_workspace_bytes(uint32_t d, uint32_t n_clients) {
  if (d < 1) return 0;
  return cvlc::decode_layout(d, n_clients < 1 ? 1 : n_clients).total;
}

int cvlc_decode_aggregate(uint32_t n, const void* const* d_streams, const size_t* stream_bytes,
                          const float* weights, float* d_out, uint32_t d, uint32_t flags, void* d_workspace,
                          size_t ws_bytes, void* hip_stream) {
  using namespace cvlc;
  if (!d_out || d < 1 || d > 0x7FFFFFFFu || !d_workspace) return CVLC_ERR_ARG;
  if (n > 65535u) return CVLC_ERR_ARG;  // streams index the grid's y dimension
  if (n > 0 && (!d_streams || !stream_bytes)) return CVLC_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(d_workspace) % 256u || reinterpret_cast<uintptr_t>(d_out) % 4u) return CVLC_ERR_ARG;
  uint64_t items_bound = 0;  // tile_table work items are counted in 32 bits: a record takes two bits at least
  for (uint32_t i = 0; i < n; ++i) {
    if (!d_streams[i] || reinterpret_cast<uintptr_t>(d_streams[i]) % 4u) return CVLC_ERR_ARG;
    if (stream_bytes[i] < 4u * kGlobalHeaderWords) return CVLC_ERR_STREAM;
    items_bound += (uint64_t)stream_bytes[i] * 4u / kTabChunk + kListsPerClient;
  }
  if (items_bound > 0xFFFFFFFFull) return CVLC_ERR_ARG;
  if (ws_bytes < cvlc_decode_workspace_bytes(d, n)) return CVLC_ERR_CAPACITY;
  if (flags & ~(CVLC_DECODE_ACCUMULATE | CVLC_DECODE_QSGD)) return CVLC_ERR_ARG;
  const uint32_t quant = (flags & CVLC_DECODE_QSGD) ? CVLC_QUANT_QSGD : CVLC_QUANT_PQ;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const DecodeLayout L = decode_layout(d, n < 1 ? 1 : n);
  char* base = static_cast<char*>(d_workspace);
  uint32_t* status = reinterpret_cast<uint32_t*>(base + L.status);
  uint32_t* stream_bad = reinterpret_cast<uint32_t*>(base + L.stream_bad);
  ListDesc* descs = reinterpret_cast<ListDesc*>(base + L.desc);
  CompactDesc* cdesc = reinterpret_cast<CompactDesc*>(base + L.cdesc);
  uint32_t* item_start = reinterpret_cast<uint32_t*>(base + L.item_start);
  DecodeCtl* ctl = reinterpret_cast<DecodeCtl*>(base + L.ctl);
  uint32_t* table = reinterpret_cast<uint32_t*>(base + L.table);
  const uint32_t n_lists = n * kListsPerClient;

  profile_mark(CVLC_STAGE_DEC_SETUP, true, stream);
  {
    ParseChunk chunk;
    chunk.pad[0] = chunk.pad[1] = 0;
    const bool fused = n > 0 && n <= kParseStreams;  // one launch parses and numbers
    for (uint32_t first = 0; first < n; first += kParseStreams) {
      chunk.first = first;
      chunk.count = (n - first < kParseStreams) ? n - first : kParseStreams;
      for (uint32_t i = 0; i < chunk.count; ++i) {
        StreamArg& sa = chunk.args[i];
        sa.words = static_cast<const uint32_t*>(d_streams[first + i]);
        sa.n_words = stream_bytes[first + i] / 4u;
        sa.weight = weights ? (double)weights[first + i] : 0.0;
        sa.has_weight = weights ? 1u : 0u;
        sa.pad = 0;
      }
      if (fused)
        hipLaunchKernelGGL(setup_kernel, dim3(1), dim3(1024), 0, stream, chunk, descs, d, quant, cdesc, item_start, ctl,
                           stream_bad, status);
      else
        hipLaunchKernelGGL(parse_headers_kernel, dim3(chunk.count), dim3(64), 0, stream, chunk, descs, d, n, stream_bad,
                           quant);
    }
    // also for n = 0: writes the (empty) list counts and the status word
    if (!fused)
      hipLaunchKernelGGL(compact_lists_kernel, dim3(1), dim3(1024), 0, stream, descs, n_lists, cdesc, item_start, ctl,
                         stream_bad, n, status);
  }
  profile_mark(CVLC_STAGE_DEC_SETUP, false, stream);
  if (n > 0) {
    StageScope scope(CVLC_STAGE_DEC_TABLE, stream);
    // the number of work items is only known on the device: 2048 workgroups (eight per CU) walk them
    hipLaunchKernelGGL(tile_table_kernel, dim3(2048), dim3(kBlock), 0, stream, cdesc, item_start, ctl, table, d,
                       L.n_tiles, status);
  }
  {
    StageScope scope(CVLC_STAGE_DEC_TILES, stream);
    const uint32_t g = L.n_tiles < 768u ? L.n_tiles : 768u;  // three workgroups per CU
    auto kernel = quant == CVLC_QUANT_QSGD ? decode_tiles_kernel<true> : decode_tiles_kernel<false>;
    hipLaunchKernelGGL(kernel, dim3(g), dim3(kDecBlock), 0, stream, cdesc, ctl, table, d_out, d, L.n_tiles,
                       flags & CVLC_DECODE_ACCUMULATE, status);
  }
  return hip_check(hipGetLastError());
}

int cvlc_decode_aggregate_static(uint32_t n, const void* const* d_streams, const size_t* stream_bytes,
                                 const float* weights, float* d_out, uint32_t d, uint32_t flags,
                                 uint32_t* d_status_out, void* hip_stream) {
  using namespace cvlc;
  if (d < 1 || d > 0x7FFFFFFFu || n > 65535u) return CVLC_ERR_ARG;
  if (d_status_out && reinterpret_cast<uintptr_t>(d_status_out) % 4u) return CVLC_ERR_ARG;
  if (cvlc_decode_workspace_bytes(d, n) > (size_t)CVLC_DECODE_STATIC_BYTES) return CVLC_ERR_CAPACITY;
  void* ptr = nullptr;
  int rc = static_scratch(&ptr);
  if (rc) return rc;
  // everything the kernels read from the array they have written earlier in the same call, so what the
  // call before left there does not matter
  rc = cvlc_decode_aggregate(n, d_streams, stream_bytes, weights, d_out, d, flags, ptr, CVLC_DECODE_STATIC_BYTES,
                             hip_stream);
  if (rc) return rc;
  if (d_status_out) {
    hipLaunchKernelGGL(copy_status_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint32_t*>(ptr), d_status_out);
    rc = hip_check(hipGetLastError());
  }
  return rc;
}

}  // extern "C"
