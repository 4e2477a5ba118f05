// cvlc_packet.hip -- packets (Sec. IV-C Eq. (3), Sec. IV-D): a client's stream
// is cut into packets of at most mtu bytes, each holding records of one group
// only and a header that lets the parameter server place and decode it on its
// own; the server puts the stream back together from the packets it received.
//
// Packet = little-endian 32-bit words:
//   0 "CVLP"   1 version | quantiser << 16   2 d   3 client   4 bits(B)
//   5 r | R << 8 | y_r << 16 | s << 24        6 P_r
//   7 e0, the number of the packet's first record inside its group
//   8, 9 the group's two centroid words ({min, max} or {norm, 0})
//   then c = min(cap_r, P_r - e0) records of W_r = s + y_r bits from bit 0,
//   zero padded to a word.  cap_r = floor((8 mtu - 320) / W_r) is the largest
//   record count that satisfies Eq. (3) with H = 320 bits.
// Packets are numbered group by group; an empty group sends one packet with no
// records so that its header fields survive.  In memory packets sit at a stride
// of mtu bytes.
#include <hip/hip_runtime.h>

#include "cvlc_common.h"

namespace cvlc {
namespace {

constexpr uint32_t kPktMagic = 0x504C5643u;  // "CVLP"
constexpr uint32_t kPktHeaderWords = CVLC_PACKET_HEADER_WORDS;
constexpr uint32_t kPktBlock = 64;           // one wavefront per packet

typedef const uint32_t __attribute__((address_space(1))) * GlobalConstWordPtr;
typedef uint32_t __attribute__((address_space(1))) * GlobalWordPtr;

__host__ __device__ __forceinline__ bool mtu_supported(uint32_t mtu) {
  return mtu % 4u == 0 && mtu >= 64u && mtu <= 65532u;
}
__host__ __device__ __forceinline__ uint32_t packet_cap(uint32_t mtu, uint32_t W) {
  return (8u * mtu - 32u * kPktHeaderWords) / W;  // W <= 63 and mtu >= 64: at least 3
}
__host__ __device__ __forceinline__ uint32_t group_packets(uint32_t P, uint32_t cap) {
  return P == 0 ? 1u : (P + cap - 1u) / cap;
}

// Bits [32 i - sh, 32 i - sh + 32) of a word array `src` of n_src words whose bits from `nbits` on do not
// count (sh < 32; positions before the array read as 0): what the array, shifted up by sh bits, puts into
// word i of its destination.
__device__ __forceinline__ uint32_t shifted_word(GlobalConstWordPtr src, uint32_t n_src, uint32_t nbits, uint32_t i,
                                                 uint32_t sh) {
  auto word = [&](uint32_t k) -> uint32_t {  // src[k] with the bits beyond nbits cleared; k may be "-1"
    if (k >= n_src) return 0u;
    const uint32_t full = nbits >> 5, rem = nbits & 31u;
    const uint32_t v = src[k];
    return k < full ? v : (k == full ? v & ((1u << rem) - 1u) : 0u);
  };
  const uint32_t hi = word(i), lo = word(i - 1u);  // i = 0: i - 1 wraps and reads as 0
  return sh ? (hi << sh) | (lo >> (32u - sh)) : hi;
}

// ------------------------------------------------------------------ sender
struct PacketPlan {  // what the sender's kernel needs from the plan
  uint32_t R, s, mtu_words;
  uint32_t y[CVLC_MAX_CODED], P[CVLC_MAX_CODED];
};

// One wavefront per packet: finds its (group, number inside the group) from the
// plan, copies the header fields from the stream's headers and moves its records
// down to bit 0 of the packet's payload; the rest of the packet's slot is zeroed.
__global__ __launch_bounds__(kPktBlock) void packetize_kernel(PacketPlan plan, const uint32_t* __restrict__ stream,
                                                              uint32_t* __restrict__ packets) {
  const uint32_t mtu = plan.mtu_words * 4u;
  uint32_t r = 0, first_packet = 0, payload = kGlobalHeaderWords + kSegHeaderWords * plan.R;
  uint32_t W = 0, cap = 1, npk = 0;
  for (; r < plan.R; ++r) {  // uniform: every lane walks the same groups
    W = plan.s + plan.y[r];
    cap = packet_cap(mtu, W);
    npk = group_packets(plan.P[r], cap);
    if (blockIdx.x < first_packet + npk) break;
    first_packet += npk;
    payload += (uint32_t)payload_words(plan.P[r], W);
  }
  if (r >= plan.R) return;  // the grid has exactly one workgroup per packet; never taken
  const uint32_t P = plan.P[r], e0 = (blockIdx.x - first_packet) * cap;
  const uint32_t c = P - e0 < cap ? P - e0 : cap;
  GlobalWordPtr out = (GlobalWordPtr)(packets + (size_t)blockIdx.x * plan.mtu_words);
  const uint32_t lane = threadIdx.x;
  if (lane < kPktHeaderWords) {
    const uint32_t* gh = stream + kGlobalHeaderWords + kSegHeaderWords * r;
    uint32_t v;
    switch (lane) {
      case 0: v = kPktMagic; break;
      case 1: v = stream[1]; break;
      case 2: v = stream[2]; break;
      case 3: v = stream[6]; break;
      case 4: v = stream[5]; break;
      case 5: v = r | (plan.R << 8) | (plan.y[r] << 16) | (plan.s << 24); break;
      case 6: v = P; break;
      case 7: v = e0; break;
      case 8: v = gh[2]; break;
      default: v = gh[3]; break;
    }
    out[lane] = v;
  }
  // the packet's records are bits [e0 W, (e0 + c) W) of the group's payload
  const uint64_t bit0 = (uint64_t)e0 * W;
  const uint32_t group_words = (uint32_t)payload_words(P, W);
  const uint32_t w0 = (uint32_t)(bit0 >> 5), sh = (uint32_t)(bit0 & 31u);
  const uint32_t nbits = c * W, n_out = (nbits + 31u) >> 5;
  GlobalConstWordPtr src = (GlobalConstWordPtr)(stream + payload);
  for (uint32_t i = lane; i < plan.mtu_words - kPktHeaderWords; i += kPktBlock) {
    uint32_t v = 0;
    if (i < n_out) {
      const uint32_t a = src[min(w0 + i, group_words - 1u)];
      const uint32_t b = w0 + i + 1u < group_words ? src[w0 + i + 1u] : 0u;
      v = sh ? (a >> sh) | (b << (32u - sh)) : a;
      if (i == n_out - 1u && (nbits & 31u)) v &= (1u << (nbits & 31u)) - 1u;
    }
    out[kPktHeaderWords + i] = v;
  }
}

// ------------------------------------------------------------------ receiver
struct ReassemblyState {  // at the start of the workspace, after the status word's 256 bytes
  uint32_t valid;         // 1: the second kernel may copy
  uint32_t R, s, pad;
  uint32_t y[32], P[32], payload[32], first_packet[32];
};

constexpr uint32_t kGatherBlock = 1024;

// One workgroup: reads every packet's header, takes each group's fields from
// the packet that holds its record 0, lays the stream out, writes its headers,
// checks every packet against that and that every place is taken exactly once,
// and clears the stream words that two packets share.
__global__ __launch_bounds__(kGatherBlock) void reassemble_headers_kernel(const uint32_t* __restrict__ packets,
                                                                         uint32_t n, uint32_t mtu_words, uint32_t d,
                                                                         uint32_t* __restrict__ stream,
                                                                         uint64_t cap_words, uint32_t* status,
                                                                         ReassemblyState* st,
                                                                         uint32_t* __restrict__ seen) {
  __shared__ uint32_t g_y[32], g_P[32], g_c0[32], g_c1[32], g_have[32], g_payload[33], g_first[33];
  __shared__ uint32_t s_bad;
  const uint32_t tid = threadIdx.x, mtu = mtu_words * 4u;
  if (tid < 32) g_have[tid] = 0;
  if (tid == 0) s_bad = 0;
  for (uint32_t i = tid; i < n; i += kGatherBlock) seen[i] = 0;
  const uint32_t f1 = packets[1], f3 = packets[3], f4 = packets[4], f5 = packets[5];
  const uint32_t R = (f5 >> 8) & 0xFFu, s = f5 >> 24;
  const float B = __uint_as_float(f4);
  const bool global_ok = packets[0] == kPktMagic && (f1 & 0xFFFFu) == kVersion && (f1 >> 16) <= CVLC_QUANT_QSGD &&
                         packets[2] == d && R <= CVLC_MAX_CODED && s == position_bits(d) && B > 0.0f &&
                         fabsf(B) <= 3.4028234664e38f;
  __syncthreads();
  if (global_ok) {
    for (uint32_t p = tid; p < n; p += kGatherBlock) {
      const uint32_t* pk = packets + (size_t)p * mtu_words;
      const uint32_t r = pk[5] & 0xFFu;
      if (pk[0] != kPktMagic || r >= R) {
        atomicOr(&s_bad, 1u);
      } else if (pk[7] == 0) {  // holds the group's record 0: exactly one such packet per group
        if (atomicAdd(&g_have[r], 1u) == 0) {
          g_y[r] = (pk[5] >> 16) & 0xFFu;
          g_P[r] = pk[6];
          g_c0[r] = pk[8];
          g_c1[r] = pk[9];
        } else {
          atomicOr(&s_bad, 1u);
        }
      }
    }
  }
  __syncthreads();
  if (tid == 0) {
    bool ok = global_ok && !s_bad;
    uint64_t first = 0, payload = kGlobalHeaderWords + (uint64_t)kSegHeaderWords * R;
    for (uint32_t r = 0; ok && r < R; ++r) {
      ok = g_have[r] == 1 && code_len_supported(g_y[r]) && g_P[r] <= d;
      if (!ok) break;
      const uint32_t W = s + g_y[r];
      g_first[r] = (uint32_t)first;
      g_payload[r] = (uint32_t)payload;
      first += group_packets(g_P[r], packet_cap(mtu, W));
      payload += payload_words(g_P[r], W);
      ok = first <= n && payload <= 0xFFFFFFFFull;
    }
    ok = ok && first == n && payload <= cap_words;
    if (ok) {
      g_first[R] = (uint32_t)first;
      g_payload[R] = (uint32_t)payload;
      stream[0] = kMagic; stream[1] = f1; stream[2] = d; stream[3] = R; stream[4] = s; stream[5] = f4; stream[6] = f3;
      stream[7] = (uint32_t)payload;
      for (uint32_t r = 0; r < R; ++r) {
        uint32_t* gh = stream + kGlobalHeaderWords + kSegHeaderWords * r;
        gh[0] = g_y[r]; gh[1] = g_P[r]; gh[2] = g_c0[r]; gh[3] = g_c1[r];
      }
    } else {
      s_bad = 1;
    }
  }
  __syncthreads();
  if (!s_bad) {
    for (uint32_t p = tid; p < n; p += kGatherBlock) {
      const uint32_t* pk = packets + (size_t)p * mtu_words;
      const uint32_t r = pk[5] & 0xFFu;  // < R, checked above
      const uint32_t W = s + g_y[r], cap = packet_cap(mtu, W), P = g_P[r], e0 = pk[7];
      bool ok = pk[1] == f1 && pk[2] == d && pk[3] == f3 && pk[4] == f4 &&
                pk[5] == (r | (R << 8) | (g_y[r] << 16) | (s << 24)) && pk[6] == P && pk[8] == g_c0[r] &&
                pk[9] == g_c1[r] && e0 % cap == 0 && (e0 < P || (e0 == 0 && P == 0));
      if (ok) ok = atomicAdd(&seen[g_first[r] + e0 / cap], 1u) == 0;  // n places, n packets, none twice: none missing
      if (!ok) {
        atomicOr(&s_bad, 1u);
        continue;
      }
      const uint32_t c = P - e0 < cap ? P - e0 : cap;
      if (c) {  // the first and the last stream word of the packet's records may be shared with its neighbours
        const uint64_t bit0 = (uint64_t)e0 * W, bit1 = bit0 + (uint64_t)c * W;
        stream[g_payload[r] + (uint32_t)(bit0 >> 5)] = 0;
        stream[g_payload[r] + (uint32_t)((bit1 - 1) >> 5)] = 0;
      }
    }
  }
  __syncthreads();
  if (tid < 32) {
    st->y[tid] = tid < R ? g_y[tid] : 0;
    st->P[tid] = tid < R ? g_P[tid] : 0;
    st->payload[tid] = tid < R ? g_payload[tid] : 0;
    st->first_packet[tid] = tid < R ? g_first[tid] : 0;
  }
  if (tid == 0) {
    st->valid = s_bad ? 0u : 1u;
    st->R = R; st->s = s; st->pad = 0;
    *status = s_bad ? CVLC_DEV_STREAM : 0u;
    if (s_bad) stream[0] = 0;  // what is there is not a stream
  }
}

// One wavefront per packet: its records move up to their place in the group's
// payload.  Words wholly inside the packet's bit range are stored, the first
// and the last are OR-ed into the words the header kernel cleared.
__global__ __launch_bounds__(kPktBlock) void reassemble_payload_kernel(const uint32_t* __restrict__ packets,
                                                                       uint32_t mtu_words,
                                                                       const ReassemblyState* __restrict__ st,
                                                                       uint32_t* __restrict__ stream) {
  if (!st->valid) return;
  const uint32_t* pk = packets + (size_t)blockIdx.x * mtu_words;
  const uint32_t r = pk[5] & 0xFFu, e0 = pk[7];
  const uint32_t W = st->s + st->y[r], cap = packet_cap(mtu_words * 4u, W), P = st->P[r];
  const uint32_t c = P - e0 < cap ? P - e0 : cap;
  if (c == 0) return;
  const uint64_t bit0 = (uint64_t)e0 * W;
  const uint32_t nbits = c * W, sh = (uint32_t)(bit0 & 31u);
  const uint32_t w0 = (uint32_t)(bit0 >> 5), w_last = (uint32_t)((bit0 + nbits - 1u) >> 5);
  GlobalConstWordPtr src = (GlobalConstWordPtr)(pk + kPktHeaderWords);
  GlobalWordPtr dst = (GlobalWordPtr)(stream + st->payload[r] + w0);
  const uint32_t n_src = mtu_words - kPktHeaderWords;
  for (uint32_t i = threadIdx.x; i <= w_last - w0; i += kPktBlock) {
    const uint32_t v = shifted_word(src, n_src, nbits, i, sh);
    if (i == 0 || i == w_last - w0) {
      if (v) atomicOr((uint32_t*)(dst + i), v);
    } else {
      dst[i] = v;
    }
  }
}

size_t align256(size_t v) { return (v + 255u) & ~(size_t)255u; }

bool plan_packets(const cvlc_plan_t* plan, uint32_t mtu, uint64_t* count) {
  if (!plan || cvlc_plan_validate(plan) != CVLC_OK || !mtu_supported(mtu)) return false;
  uint64_t n = 0;
  for (uint32_t r = 0; r < plan->n_coded; ++r)
    n += group_packets(plan->count[r], packet_cap(mtu, plan->s + plan->code_len[r]));
  *count = n;
  return n <= 0xFFFFFFFFull;
}

}  // namespace
}  // namespace cvlc

extern "C" {

uint32_t cvlc_packet_count(const cvlc_plan_t* plan, uint32_t mtu_bytes) {
  uint64_t n = 0;
  return cvlc::plan_packets(plan, mtu_bytes, &n) ? (uint32_t)n : 0u;
}

uint32_t cvlc_packet_size(const cvlc_plan_t* plan, uint32_t mtu_bytes, uint32_t index) {
  using namespace cvlc;
  uint64_t n = 0;
  if (!plan_packets(plan, mtu_bytes, &n) || index >= n) return 0;
  uint32_t first = 0;
  for (uint32_t r = 0; r < plan->n_coded; ++r) {
    const uint32_t W = plan->s + plan->code_len[r], cap = packet_cap(mtu_bytes, W);
    const uint32_t npk = group_packets(plan->count[r], cap);
    if (index < first + npk) {
      const uint32_t e0 = (index - first) * cap;
      const uint32_t c = plan->count[r] - e0 < cap ? plan->count[r] - e0 : cap;
      return 4u * (kPktHeaderWords + (uint32_t)payload_words(c, W));
    }
    first += npk;
  }
  return 0;
}

int cvlc_packetize(const cvlc_plan_t* plan, const void* d_stream, uint32_t mtu_bytes, void* d_packets_out,
                   size_t capacity, void* hip_stream) {
  using namespace cvlc;
  if (!plan || !d_stream || !d_packets_out) return CVLC_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(d_stream) % 4u || reinterpret_cast<uintptr_t>(d_packets_out) % 4u) return CVLC_ERR_ARG;
  if (!mtu_supported(mtu_bytes)) return CVLC_ERR_ARG;
  const int rc = cvlc_plan_validate(plan);
  if (rc) return rc;
  if (plan->total_bits / 32u > 0xFFFFFFFFull) return CVLC_ERR_PLAN;
  uint64_t n = 0;
  if (!plan_packets(plan, mtu_bytes, &n)) return CVLC_ERR_PLAN;
  if (capacity < n * (uint64_t)mtu_bytes) return CVLC_ERR_CAPACITY;
  if (n == 0) return CVLC_OK;  // no coded group: nothing to send
  PacketPlan pp;
  pp.R = plan->n_coded;
  pp.s = plan->s;
  pp.mtu_words = mtu_bytes / 4u;
  for (uint32_t r = 0; r < CVLC_MAX_CODED; ++r) {
    pp.y[r] = r < plan->n_coded ? plan->code_len[r] : 0;
    pp.P[r] = r < plan->n_coded ? plan->count[r] : 0;
  }
  hipLaunchKernelGGL(packetize_kernel, dim3((uint32_t)n), dim3(kPktBlock), 0, static_cast<hipStream_t>(hip_stream), pp,
                     static_cast<const uint32_t*>(d_stream), static_cast<uint32_t*>(d_packets_out));
  return hip_check(hipGetLastError());
}

size_t cvlc_depacketize_workspace_bytes(uint32_t n_packets) {
  return 256u + cvlc::align256(sizeof(cvlc::ReassemblyState)) + cvlc::align256((size_t)n_packets * sizeof(uint32_t));
}

int cvlc_depacketize(const void* d_packets, uint32_t n_packets, uint32_t mtu_bytes, uint32_t d, void* d_stream_out,
                     size_t capacity, void* d_workspace, size_t ws_bytes, void* hip_stream) {
  using namespace cvlc;
  if (!d_packets || !d_stream_out || !d_workspace || n_packets == 0) return CVLC_ERR_ARG;
  if (d < 1 || d > 0x7FFFFFFFu || !mtu_supported(mtu_bytes)) return CVLC_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(d_packets) % 4u || reinterpret_cast<uintptr_t>(d_stream_out) % 4u ||
      reinterpret_cast<uintptr_t>(d_workspace) % 256u)
    return CVLC_ERR_ARG;
  if (capacity < 4u * kGlobalHeaderWords) return CVLC_ERR_CAPACITY;
  if (ws_bytes < cvlc_depacketize_workspace_bytes(n_packets)) return CVLC_ERR_CAPACITY;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* base = static_cast<char*>(d_workspace);
  uint32_t* status = reinterpret_cast<uint32_t*>(base);
  ReassemblyState* st = reinterpret_cast<ReassemblyState*>(base + 256);
  uint32_t* seen = reinterpret_cast<uint32_t*>(base + 256 + align256(sizeof(ReassemblyState)));
  hipLaunchKernelGGL(reassemble_headers_kernel, dim3(1), dim3(kGatherBlock), 0, stream,
                     static_cast<const uint32_t*>(d_packets), n_packets, mtu_bytes / 4u, d,
                     static_cast<uint32_t*>(d_stream_out), (uint64_t)(capacity / 4u), status, st, seen);
  hipLaunchKernelGGL(reassemble_payload_kernel, dim3(n_packets), dim3(kPktBlock), 0, stream,
                     static_cast<const uint32_t*>(d_packets), mtu_bytes / 4u, st, static_cast<uint32_t*>(d_stream_out));
  return hip_check(hipGetLastError());
}

}  // extern "C"
