// Parameter-server side of libcvlc for gfx950: decode n clients' streams and
// aggregate them into one dense fp32 vector (Sec. III step 3 with the 1/B
// scaling of Sec. IV-B):  out[j] = sum_i w_i * xhat_{i,j}.
//
// Records are stored per (client, group) in ascending position, so every such
// list is sorted.  Each workgroup owns a tile of output coordinates, pulls the
// slice of every list that falls into its tile, accumulates in LDS in fp64 and
// writes the tile once; nothing is scattered into global memory.
//   parse_headers  validate headers, build one descriptor per list
//   tile_table     for every list, the first record of every output tile
//   decode_tiles   fused decode + accumulate + single write of each tile
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>

#include "cvlc_common.h"

namespace cvlc {
namespace {

struct DecodeLayout {
  size_t status, streams, desc, table, total;
  uint32_t n_tiles, n_lists;
};

size_t align256(size_t v) { return (v + 255u) & ~(size_t)255u; }

struct StreamArg {  // per-stream inputs, uploaded through kernel arguments
  const uint32_t* words;
  uint64_t n_words;
  double weight;
  uint32_t has_weight;  // 0: derive 1/(n*B) from the header
  uint32_t pad;
};

DecodeLayout decode_layout(uint32_t d, uint32_t n) {
  DecodeLayout L;
  L.n_tiles = (uint32_t)(((uint64_t)d + kDecTile - 1) / kDecTile);
  L.n_lists = n * CVLC_MAX_CODED;
  size_t off = 0;
  L.status = off; off = align256(off + 256);
  L.streams = off; off = align256(off + (size_t)n * sizeof(StreamArg));
  L.desc = off; off = align256(off + (size_t)L.n_lists * sizeof(ListDesc));
  L.table = off; off = align256(off + (size_t)(L.n_tiles + 1) * L.n_lists * sizeof(uint32_t));
  L.total = off;
  return L;
}

constexpr uint32_t kUploadWords = 960;
struct UploadChunk {
  uint32_t n_words, dst_word;
  uint32_t data[kUploadWords];
};

__global__ void upload_kernel(uint32_t* dst, UploadChunk c) {
  for (uint32_t i = threadIdx.x; i < c.n_words; i += blockDim.x) dst[c.dst_word + i] = c.data[i];
}

// Bits [bit, bit + W) of a little-endian word array, W <= 63.  Reads the three
// words the field can touch; `n_words` bounds the reads.
__device__ __forceinline__ uint64_t read_bits(const uint32_t* __restrict__ words, uint64_t n_words, uint64_t bit,
                                              uint32_t W) {
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
// One workgroup (64 threads) per stream.  A stream that fails any check
// contributes nothing: all its lists are marked empty and the status bit is set.
__global__ __launch_bounds__(64) void parse_headers_kernel(const StreamArg* __restrict__ streams, ListDesc* descs,
                                                           uint32_t d, uint32_t n, uint32_t* status) {
  __shared__ uint32_t s_ok;
  __shared__ uint64_t s_payload[CVLC_MAX_CODED];
  const uint32_t client = blockIdx.x, t = threadIdx.x;
  const StreamArg sa = streams[client];
  const uint32_t* w = sa.words;
  ListDesc* out = descs + (size_t)client * CVLC_MAX_CODED;
  if (t == 0) {
    bool ok = sa.n_words >= kGlobalHeaderWords;
    uint32_t R = 0, s = 0;
    if (ok) {
      R = w[3];
      s = w[4];
      const float B = __uint_as_float(w[5]);
      ok = w[0] == kMagic && w[1] == kVersion && w[2] == d && R <= CVLC_MAX_CODED && s == position_bits(d) &&
           B > 0.0f && fabsf(B) <= 3.4028234664e38f;
    }
    uint64_t pos = kGlobalHeaderWords + (uint64_t)kSegHeaderWords * R;
    ok = ok && sa.n_words >= pos;
    if (ok) {
      uint64_t k = 0;
      for (uint32_t r = 0; r < R; ++r) {
        const uint32_t* h = w + kGlobalHeaderWords + kSegHeaderWords * r;
        const uint32_t y = h[0], P = h[1];
        const float m = __uint_as_float(h[2]), M = __uint_as_float(h[3]);
        ok = ok && code_len_supported(y) && fabsf(m) <= 3.4028234664e38f && fabsf(M) <= 3.4028234664e38f &&
             fabsf(M - m) <= 3.4028234664e38f;
        if (!ok) break;
        k += P;
        s_payload[r] = pos;
        pos += payload_words(P, s + y);
      }
      ok = ok && k <= d && pos == w[7] && sa.n_words >= pos;
    }
    s_ok = ok ? 1u : 0u;
    if (!ok) atomicOr(status, CVLC_DEV_STREAM);
  }
  __syncthreads();
  if (t < CVLC_MAX_CODED) {
    ListDesc ld;
    ld.payload = nullptr; ld.weight = 0.0; ld.P = 0; ld.W = 0; ld.s = 0; ld.y = 0; ld.m = 0.0f; ld.step = 0.0f;
    if (s_ok && t < w[3]) {
      const uint32_t* h = w + kGlobalHeaderWords + kSegHeaderWords * t;
      const uint32_t y = h[0];
      const float m = __uint_as_float(h[2]), M = __uint_as_float(h[3]);
      float step = 0.0f, inv = 0.0f;
      if (y != 32) centroid_spacing(m, M, y, &step, &inv);
      ld.payload = w + s_payload[t];
      ld.weight = sa.has_weight ? sa.weight : 1.0 / ((double)n * (double)__uint_as_float(w[5]));
      ld.P = h[1];
      ld.s = w[4];
      ld.y = y;
      ld.W = w[4] + y;
      ld.m = m;
      ld.step = step;
    }
    out[t] = ld;
  }
}

// ------------------------------------------------------------------ 2. tile table
// table[t][list] = index of the first record of `list` whose position lies in
// output tile t or later; row n_tiles holds the list length.  Thread e compares
// the tiles of records e-1 and e and fills the rows in between.
__global__ __launch_bounds__(kBlock) void tile_table_kernel(const ListDesc* __restrict__ descs, uint32_t* table,
                                                            uint32_t d, uint32_t n_tiles, uint32_t n_lists,
                                                            uint32_t* status) {
  const uint32_t list = blockIdx.y;
  const ListDesc ld = descs[list];
  if (ld.P == 0) return;
  const uint64_t n_words = payload_words(ld.P, ld.W);
  const uint64_t pid_mask = (1ull << ld.s) - 1ull;
  bool bad = false;
  for (uint32_t e = blockIdx.x * kBlock + threadIdx.x; e < ld.P; e += gridDim.x * kBlock) {
    const uint32_t pid = (uint32_t)(read_bits(ld.payload, n_words, (uint64_t)e * ld.W, ld.W) & pid_mask);
    int64_t t_prev = -1;
    if (e > 0) {
      const uint32_t prev = (uint32_t)(read_bits(ld.payload, n_words, (uint64_t)(e - 1) * ld.W, ld.W) & pid_mask);
      bad |= prev >= pid;  // positions must ascend strictly
      t_prev = prev < d ? (int64_t)(prev / kDecTile) : (int64_t)n_tiles;
    }
    bad |= pid >= d;
    const int64_t t_cur = pid < d ? (int64_t)(pid / kDecTile) : (int64_t)n_tiles;
    for (int64_t t = t_prev + 1; t <= t_cur && t <= (int64_t)n_tiles; ++t) table[(size_t)t * n_lists + list] = e;
    if (e == ld.P - 1)
      for (int64_t t = t_cur + 1; t <= (int64_t)n_tiles; ++t) table[(size_t)t * n_lists + list] = ld.P;
  }
  if (bad) atomicOr(status, CVLC_DEV_STREAM);
}

// ------------------------------------------------------------------ 3. fused decode + accumulate
__global__ __launch_bounds__(kBlock) void decode_tiles_kernel(const ListDesc* __restrict__ descs,
                                                              const uint32_t* __restrict__ table, float* out,
                                                              uint32_t d, uint32_t n_tiles, uint32_t n_lists,
                                                              uint32_t accumulate, uint32_t* status) {
  __shared__ double acc[kDecTile];
  const uint32_t tile = blockIdx.x;
  const uint32_t lo = tile * kDecTile;
  for (uint32_t i = threadIdx.x; i < kDecTile; i += kBlock) acc[i] = 0.0;
  __syncthreads();
  bool bad = false;
  for (uint32_t list = threadIdx.x; list < n_lists; list += kBlock) {
    uint32_t begin = table[(size_t)tile * n_lists + list];
    uint32_t end = table[(size_t)(tile + 1) * n_lists + list];
    const ListDesc ld = descs[list];
    if (ld.P == 0) continue;
    if (begin > ld.P) begin = ld.P;  // table rows of a malformed list may hold anything
    if (end > ld.P) end = ld.P;
    if (end <= begin) continue;
    const uint64_t n_words = payload_words(ld.P, ld.W);
    const uint64_t pid_mask = (1ull << ld.s) - 1ull;
    for (uint32_t e = begin; e < end; ++e) {
      const uint64_t rec = read_bits(ld.payload, n_words, (uint64_t)e * ld.W, ld.W);
      const uint32_t pid = (uint32_t)(rec & pid_mask);
      const uint32_t cid = (uint32_t)(rec >> ld.s);
      if (pid < lo || pid - lo >= kDecTile || pid >= d) { bad = true; continue; }
      const float xhat = ld.y == 32 ? __uint_as_float(cid) : __fmaf_rn((float)cid, ld.step, ld.m);
      atomicAdd(&acc[pid - lo], ld.weight * (double)xhat);
    }
  }
  if (bad) atomicOr(status, CVLC_DEV_STREAM);
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < kDecTile; i += kBlock) {
    const uint32_t j = lo + i;
    if (j < d) {
      double v = acc[i];
      if (accumulate) v += (double)out[j];
      out[j] = (float)v;
    }
  }
}

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
  if (n > 0 && (!d_streams || !stream_bytes)) return CVLC_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(d_workspace) % 256u || reinterpret_cast<uintptr_t>(d_out) % 4u) return CVLC_ERR_ARG;
  for (uint32_t i = 0; i < n; ++i) {
    if (!d_streams[i] || reinterpret_cast<uintptr_t>(d_streams[i]) % 4u) return CVLC_ERR_ARG;
    if (stream_bytes[i] < 4u * kGlobalHeaderWords) return CVLC_ERR_STREAM;
  }
  if (ws_bytes < cvlc_decode_workspace_bytes(d, n)) return CVLC_ERR_CAPACITY;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const DecodeLayout L = decode_layout(d, n < 1 ? 1 : n);
  char* base = static_cast<char*>(d_workspace);
  uint32_t* status = reinterpret_cast<uint32_t*>(base + L.status);
  StreamArg* sargs = reinterpret_cast<StreamArg*>(base + L.streams);
  ListDesc* descs = reinterpret_cast<ListDesc*>(base + L.desc);
  uint32_t* table = reinterpret_cast<uint32_t*>(base + L.table);
  const uint32_t n_lists = n * CVLC_MAX_CODED;

  profile_mark(CVLC_STAGE_DEC_SETUP, true, stream);
  int rc = hip_check(hipMemsetAsync(status, 0, 256, stream));
  if (rc) return rc;
  if (n > 0) {
    constexpr uint32_t words_per = sizeof(StreamArg) / 4u;
    const uint32_t per_chunk = kUploadWords / words_per;
    UploadChunk chunk;
    for (uint32_t first = 0; first < n; first += per_chunk) {
      const uint32_t cnt = (n - first < per_chunk) ? n - first : per_chunk;
      chunk.n_words = cnt * words_per;
      chunk.dst_word = first * words_per;
      for (uint32_t i = 0; i < cnt; ++i) {
        StreamArg sa;
        sa.words = static_cast<const uint32_t*>(d_streams[first + i]);
        sa.n_words = stream_bytes[first + i] / 4u;
        sa.weight = weights ? (double)weights[first + i] : 0.0;
        sa.has_weight = weights ? 1u : 0u;
        sa.pad = 0;
        std::memcpy(&chunk.data[i * words_per], &sa, sizeof(sa));
      }
      hipLaunchKernelGGL(upload_kernel, dim3(1), dim3(256), 0, stream, reinterpret_cast<uint32_t*>(sargs), chunk);
    }
    hipLaunchKernelGGL(parse_headers_kernel, dim3(n), dim3(64), 0, stream, sargs, descs, d, n, status);
  }
  profile_mark(CVLC_STAGE_DEC_SETUP, false, stream);
  if (n > 0) {
    StageScope scope(CVLC_STAGE_DEC_TABLE, stream);
    hipLaunchKernelGGL(tile_table_kernel, dim3(8, n_lists), dim3(kBlock), 0, stream, descs, table, d, L.n_tiles,
                       n_lists, status);
  }
  {
    StageScope scope(CVLC_STAGE_DEC_TILES, stream);
    hipLaunchKernelGGL(decode_tiles_kernel, dim3(L.n_tiles), dim3(kBlock), 0, stream, descs, table, d_out, d,
                       L.n_tiles, n_lists, flags & CVLC_DECODE_ACCUMULATE, status);
  }
  return hip_check(hipGetLastError());
}

}  // extern "C"
