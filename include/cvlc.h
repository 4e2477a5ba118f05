/*
 * cvlc.h -- C ABI of the MI355X (gfx950) implementation of Fed-CVLC's per-round
 * hot path: compress a client's model-update vector with variable-length codes
 * and, on the parameter server, decode and aggregate many clients' streams.
 *
 * Conventions
 *   - Every function returns CVLC_OK (0) or a negative cvlc_status; none throws
 *     or aborts.  Errors that the host can see (null pointers, plan shape,
 *     capacities, workspace size) are returned before anything is launched.
 *   - "d_" arguments are DEVICE pointers, everything else is HOST memory.  All
 *     buffers are owned by the caller; the library keeps no state between calls
 *     and allocates no device memory.
 *   - GPU entry points only enqueue work on `hip_stream` (a hipStream_t, NULL =
 *     the default stream) and return; results are ready when the stream has
 *     drained.  Conditions only the device can see (a NaN in the update, a
 *     malformed stream) set bits in a status word at the start of the
 *     workspace; read it with cvlc_device_status().
 *   - The library needs a gfx950 device; there is no CPU fallback.
 */
#ifndef CVLC_H
#define CVLC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum cvlc_status {
  CVLC_OK = 0,
  CVLC_ERR_ARG = -1,       /* null pointer, zero size, misaligned buffer          */
  CVLC_ERR_PLAN = -2,      /* plan violates Eq. (3)-(4) or an unsupported length  */
  CVLC_ERR_BUDGET = -3,    /* the bit budget cannot hold even k_min = R updates   */
  CVLC_ERR_CAPACITY = -4,  /* stream buffer or workspace too small                */
  CVLC_ERR_NONFINITE = -5, /* reserved for host-side checks of non-finite input   */
  CVLC_ERR_STREAM = -6,    /* stream shorter than a header                        */
  CVLC_ERR_DEVICE = -7     /* a HIP call failed                                   */
} cvlc_status;

/* bits of the device status word */
#define CVLC_DEV_NONFINITE 1u /* update holds NaN/Inf, or a group's max-min overflows  */
#define CVLC_DEV_STREAM 2u    /* malformed stream: header, code length, PID >= d, order */
#define CVLC_DEV_INTERNAL 4u  /* an internal consistency check failed                   */
#define CVLC_DEV_WORKSPACE 8u /* encode: a vector needs more candidate room than given  */

#define CVLC_MAX_CODED 31u    /* at most 31 coded groups plus the implicit 0-bit tail   */
#define CVLC_STATS_STRIDE 32u /* stats entries per client: groups 1..R, then the tail   */

/* The code-length plan of one client for one round (Algorithm 1's output
 * k*, P_r*, y_r*): coded group r = 1..R takes the P_r updates of ranks
 * (Z_{r-1}, Z_r] by magnitude and spends y_r bits on each; ranks beyond
 * k = P_1+...+P_R are sparsified away (code length 0). */
typedef struct cvlc_plan_t {
  uint32_t d;                        /* number of model updates, 1 .. 2^31-1          */
  uint32_t n_coded;                  /* R                                             */
  uint32_t s;                        /* position-ID width ceil(log2 d) (below Eq. (2)) */
  uint32_t code_len[CVLC_MAX_CODED]; /* y_r, non-increasing, each in 1..16 or 32 (raw) */
  uint32_t count[CVLC_MAX_CODED];    /* P_r, may be 0                                 */
  uint64_t total_bits;               /* exact stream size, headers and padding included */
  float B;                           /* scale factor of Lemma 1, > 0 (1 = no scaling) */
  uint32_t quant;                    /* CVLC_QUANT_PQ or CVLC_QUANT_QSGD (set by the   */
                                     /* caller; the planner's modes leave PQ)          */
} cvlc_plan_t;

/* The two quantisers of Sec. IV-D.
 *   PQ    2^y centroids spread uniformly over the group's [min, max]; the group
 *         header carries {min, max}.
 *   QSGD  the magnitude relative to the group's l2-norm is rounded to one of the
 *         levels 0, 1/s, ..., 1 with s = 2^(y-1) - 1; the code holds the sign in
 *         its top bit and the level below; the group header carries {norm, 0};
 *         needs y >= 2.  The norm is the smallest fp32 value whose square reaches
 *         the exact sum of the group's squares, so the stream does not depend on
 *         the order anything is added in. */
#define CVLC_QUANT_PQ 0u
#define CVLC_QUANT_QSGD 1u

/* Per-group statistics returned by the encoder: entries 0..R-1 are the coded
 * groups, entry R the sparsified tail (min = max = 0 there; its sumsq is the
 * sparsification error energy of Proposition 1's first term).
 * errsq is the error energy of this draw after quantisation and scaling,
 * sum over the group of (xtilde/B - x)^2 with xtilde the centroid value the
 * parameter server will read: the left side of Lemma 1.  It is filled for the
 * coded groups only when CVLC_ENCODE_ERROR_STATS is set (else 0); the tail is
 * dropped whole, so its errsq always equals its sumsq. */
typedef struct cvlc_seg_stats_t {
  float min, max;
  double sumsq;
  uint32_t count;
  uint32_t reserved;
  double errsq;
} cvlc_seg_stats_t;

/* s = ceil(log2 d), at least 1 (Sec. IV-C, below Eq. (2)). */
uint32_t cvlc_position_bits(uint32_t d);

/* CPU.  Builds a plan for a d-dimensional update with n_coded groups.
 *   fractions != NULL (with code_len): group r takes the fraction fractions[r]
 *       of the d coordinates; budget_bits is ignored.
 *   fractions == NULL, code_len != NULL: group sizes from the budget, every
 *       group getting the same bit share b, P_r = floor((b-H)/(s+y_r)), Eq. (3).
 *   both NULL: Algorithm 1 -- enumerate k, sweep the atomic operation of Eq. (6)
 *       over adjacent groups, pick the plan minimising gamma of Eq. (5) for the
 *       power-law exponent alpha of Definition 1 (alpha < 0).
 * The stream layout charges a 256-bit global header and H = 128 bits per group.
 * Returns CVLC_ERR_BUDGET when the budget cannot hold one update per group. */
int cvlc_plan(uint32_t d, uint64_t budget_bits, uint32_t n_coded, const uint32_t* code_len,
              const double* fractions, double alpha, float B, cvlc_plan_t* out);

/* CPU.  Algorithm 1 for either quantiser: as cvlc_plan with both arrays NULL,
 * but the groups are priced with the named quantiser's error model Q(P_r)
 * (appendix case study: PQ P/(2^y-1)^2, QSGD min(P/s^2, sqrt(P)/s)), code
 * lengths stay at or above the quantiser's shortest code (1 bit, QSGD 2) and
 * the plan's `quant` is set. */
int cvlc_plan_algorithm1(uint32_t d, uint64_t budget_bits, uint32_t n_coded, double alpha, float B,
                         uint32_t quant, cvlc_plan_t* out);

/* CPU.  Checks a caller-built plan (sizes, monotone code lengths, total_bits). */
int cvlc_plan_validate(const cvlc_plan_t* plan);

/* CPU.  Exact stream size in bits for the plan's d, code_len and count. */
uint64_t cvlc_plan_total_bits(const cvlc_plan_t* plan);

/* CPU.  gamma of Eq. (5) for the plan under exponent alpha. */
double cvlc_plan_gamma(const cvlc_plan_t* plan, double alpha);

/* CPU.  Scale factor for the next round (footnote to Proposition 1: the exact
 * B is max_r Q(P_r, y_r) + 1, taken from the previous round's plan), with PQ's
 * Q(P, y) = P / (2^y - 1)^2 of the appendix case study; raw 32-bit and empty
 * groups contribute 0.  Returns 1 for a NULL plan. */
double cvlc_plan_next_scale(const cvlc_plan_t* plan);

/* CPU.  ||Uhat - U||^2 / ||U||^2 of one encoded vector, the quantity that
 * Propositions 1 and 2 bound by gamma, from a HOST copy of that client's
 * statistics entries (n_coded groups, then the tail) written by an encode with
 * CVLC_ENCODE_ERROR_STATS.  0 for an all-zero vector. */
double cvlc_stats_gamma(const cvlc_seg_stats_t* stats, uint32_t n_coded);

/* Bytes a stream buffer must hold for this plan (= total_bits / 8). */
size_t cvlc_stream_capacity(const cvlc_plan_t* plan);

/* Scratch bytes cvlc_encode_batch needs for n_clients vectors of length d, and
 * cvlc_decode_aggregate needs for n_clients streams of a d-dimensional model.
 * The encoder's figure is the worst case, enough for any vector and plan. */
size_t cvlc_encode_workspace_bytes(uint32_t d, uint32_t n_clients);
size_t cvlc_decode_workspace_bytes(uint32_t d, uint32_t n_clients);

/* Encoder scratch sized to what is kept (Sec. IV-B keeps k of d updates).  The
 * encoder first drops every coordinate below a sampled magnitude threshold; the
 * survivors ("candidates", somewhat more than k) are what all later steps work
 * on.  cvlc_encode_workspace_bytes_for gives the bytes for at most
 * max_candidates of them per client (1 .. d; d = the worst case above): about
 * 6 bytes per coordinate for the threshold pass plus 8.25 per candidate,
 * against 14.25 per coordinate.  cvlc_encode_batch reads the room off
 * ws_bytes, which must hold at least the largest k of the batch
 * (CVLC_ERR_CAPACITY otherwise).  A vector with more candidates than there is
 * room for (many equal magnitudes, or the rare sample that places the
 * threshold below the k-th magnitude, after which every coordinate is a
 * candidate) sets CVLC_DEV_WORKSPACE in the status word and gets no stream:
 * the first word of its buffer is cleared, its statistics entries are not
 * written, the other clients of the batch are encoded as usual.  Encode it
 * again with more room.
 * cvlc_plan_candidates_hint: CPU; a max_candidates that holds for vectors
 * without heavy ties, from the plan's k and the sampling margins (d for plans
 * that keep too much to sample; 0 for an invalid plan). */
size_t cvlc_encode_workspace_bytes_for(uint32_t d, uint32_t n_clients, uint32_t max_candidates);
uint32_t cvlc_plan_candidates_hint(const cvlc_plan_t* plan);

/* GPU.  Compresses n clients' update vectors (Sec. IV-B sparsification and
 * quantisation, Algorithm 1's final loop, packet format of Sec. IV-D).
 *   plans[i]         host; all plans must share the same d
 *   d_updates[i]     host array of device pointers, each d fp32, 16-byte aligned
 *   seed             key of the counter-based rounding generator
 *   client_ids[i]    host; written to the header and mixed into the generator
 *   d_streams_out[i] host array of device pointers, 4-byte aligned, each at
 *                    least capacities[i] >= cvlc_stream_capacity(&plans[i]) bytes
 *   d_workspace      device, 256-byte aligned, ws_bytes >= cvlc_encode_workspace_bytes(d, n),
 *                    or less as cvlc_encode_workspace_bytes_for describes
 *   d_stats_out      device or NULL: n * CVLC_STATS_STRIDE cvlc_seg_stats_t
 *   flags            CVLC_ENCODE_ERROR_STATS: also measure every coded group's
 *                    error energy (errsq; needs d_stats_out, else CVLC_ERR_ARG);
 *                    the stream does not depend on it
 * All plans of a batch must name the same quantiser.
 * The stream is bit-identical for identical (update, plan, seed, client id).
 * Calls that share a workspace must not overlap in time. */
#define CVLC_ENCODE_ERROR_STATS 1u
int cvlc_encode_batch(uint32_t n, const cvlc_plan_t* plans, const float* const* d_updates,
                      uint64_t seed, const uint32_t* client_ids, void* const* d_streams_out,
                      const size_t* capacities, void* d_workspace, size_t ws_bytes,
                      cvlc_seg_stats_t* d_stats_out, uint32_t flags, void* hip_stream);

/* GPU.  One client; same as cvlc_encode_batch with n = 1. */
int cvlc_encode(const cvlc_plan_t* plan, const float* d_update, uint64_t seed, uint32_t client_id,
                void* d_stream_out, size_t capacity, void* d_workspace, size_t ws_bytes,
                cvlc_seg_stats_t* d_stats_out, uint32_t flags, void* hip_stream);

/* GPU.  Parameter-server side (Sec. III step 3 with the scaling of Sec. IV-B):
 * d_out[j] = sum_i w_i * xhat_{i,j}, xhat the centroid value stored for
 * position j in stream i, 0 where the stream holds nothing.
 *   d_streams[i]    host array of device pointers, 4-byte aligned
 *   stream_bytes[i] host; bytes readable at d_streams[i]
 *   weights         host or NULL; NULL => w_i = 1/(n * B_i), B_i from the header
 *   flags bit 0     0 = overwrite d_out, 1 = add to the values already there
 *   flags bit 1     the quantiser the streams must name: 0 = PQ, 1 = QSGD (a
 *                   federation uses one; a stream that names the other is malformed)
 * Products and sums are carried in fp64 and rounded to fp32 once; the order of
 * the fp64 additions is not fixed, so a coordinate that three or more records
 * meet in may differ by one unit in the last place between two runs.  A
 * malformed stream sets CVLC_DEV_STREAM; its offending records are skipped and
 * nothing is written out of bounds.  Positions must ascend strictly inside a
 * group; a position that two groups of one stream both name (no encoder writes
 * that) is not an error: both records are added. */
#define CVLC_DECODE_ACCUMULATE 1u
#define CVLC_DECODE_QSGD 2u
int cvlc_decode_aggregate(uint32_t n, const void* const* d_streams, const size_t* stream_bytes,
                          const float* weights, float* d_out, uint32_t d, uint32_t flags,
                          void* d_workspace, size_t ws_bytes, void* hip_stream);

/* GPU.  cvlc_decode_aggregate for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same kernels, working in an array of CVLC_DECODE_STATIC_BYTES
 * that the library holds in every device's memory from the moment it is loaded
 * until the process ends, instead of a caller's workspace.  The call allocates
 * nothing.  Arguments as for cvlc_decode_aggregate, except
 *   d_status_out  device or NULL: receives the call's status word (CVLC_DEV_*
 *                 bits) when the stream reaches that point
 * Returns CVLC_ERR_CAPACITY when cvlc_decode_workspace_bytes(d, n) exceeds
 * CVLC_DECODE_STATIC_BYTES (16 MiB: 32 clients of an 11.2 M-dimensional model
 * fit), before anything is launched.  All calls on one device share that
 * device's array: calls that overlap in time on one device race (also on
 * different streams); calls on different devices do not touch each other. */
#define CVLC_DECODE_STATIC_BYTES (16u << 20)
int cvlc_decode_aggregate_static(uint32_t n, const void* const* d_streams, const size_t* stream_bytes,
                                 const float* weights, float* d_out, uint32_t d, uint32_t flags,
                                 uint32_t* d_status_out, void* hip_stream);

/* Ranks at which Definition 1's power law is fitted: 1, 2, 4, ... (powers of two
 * below d) and d itself, ascending.  Writes them to ranks_out (CVLC_FIT_RANKS_MAX
 * entries, may be NULL) and returns how many there are (0 for d = 0). */
#define CVLC_FIT_RANKS_MAX 32u
uint32_t cvlc_fit_ranks(uint32_t d, uint32_t* ranks_out);

/* Scratch bytes for cvlc_fit_alpha.  cvlc_fit_workspace_bytes(n): the least it
 * runs in, independent of d (about 100 KB per client); it then reads the vectors
 * three times.  cvlc_fit_workspace_bytes_for(n, d): with room for the keys the
 * second pass sets aside (4 bytes per coordinate in the worst case, every
 * wavefront owning room for all it reads); given that much, cvlc_fit_alpha reads
 * the vectors twice.  Same results either way.  0 for n = 0 or d outside
 * 1 .. 2^31-1. */
size_t cvlc_fit_workspace_bytes(uint32_t n_clients);
size_t cvlc_fit_workspace_bytes_for(uint32_t n_clients, uint32_t d);

/* GPU.  First step of Algorithm 1: the decay exponent alpha_i of Definition 1
 * for each of n update vectors, |U{l}| ~ phi * l^alpha with U{l} the l-th
 * largest magnitude.  alpha is the ordinary-least-squares slope of ln|U{l}| on
 * ln l over the ranks of cvlc_fit_ranks(d), ranks whose magnitude is zero left
 * out; fewer than two usable ranks give alpha = -1.  The magnitudes are exact
 * order statistics of the whole vector (two or three passes over it, by the
 * size of the workspace).
 *   d_updates[i]  host array of device pointers, each d fp32, 16-byte aligned
 *   d_alpha_out   device, n doubles
 *   d_keys_out    device or NULL: n * CVLC_FIT_RANKS_MAX words; word j of client
 *                 i = fp32 bit pattern (sign cleared) of the magnitude at the
 *                 j-th fitted rank, 0 beyond the last rank
 *   d_workspace   device, 256-byte aligned, ws_bytes >= cvlc_fit_workspace_bytes(n);
 *                 from cvlc_fit_workspace_bytes_for(n, d) on, the faster path runs
 * A NaN or Inf in a vector sets CVLC_DEV_NONFINITE in the workspace's status
 * word (cvlc_device_status); that vector's outputs are then meaningless.
 * Calls that share a workspace must not overlap in time. */
int cvlc_fit_alpha(uint32_t n, const float* const* d_updates, uint32_t d, double* d_alpha_out,
                   uint32_t* d_keys_out, void* d_workspace, size_t ws_bytes, void* hip_stream);

/* Packets (Sec. IV-C Eq. (3), Sec. IV-D).  A stream is cut into packets of at
 * most mtu_bytes (a multiple of 4 in 64..65532; 1500 in the paper), each with
 * records of one group only and a header of CVLC_PACKET_HEADER_WORDS words that
 * lets the parameter server place and decode it on its own:
 *   0 "CVLP"  1 version | quantiser << 16  2 d  3 client  4 bits(B)
 *   5 r | R << 8 | y_r << 16 | s << 24     6 P_r
 *   7 e0 = number of the packet's first record inside its group
 *   8, 9 the group's centroid words ({min, max} or {norm, 0})
 * followed by min(cap_r, P_r - e0) records of s + y_r bits from bit 0, zero
 * padded to a word; cap_r = floor((8 mtu - 320) / (s + y_r)), the largest count
 * Eq. (3) allows with H = 320 bits.  Packets are numbered group by group (an
 * empty group sends one packet without records) and sit at a stride of
 * mtu_bytes in memory, zero filled behind each packet's end. */
#define CVLC_PACKET_HEADER_WORDS 10u

/* CPU.  Number of packets of a stream made with this plan (0: invalid plan or
 * mtu), and the length in bytes of packet `index` (0: out of range). */
uint32_t cvlc_packet_count(const cvlc_plan_t* plan, uint32_t mtu_bytes);
uint32_t cvlc_packet_size(const cvlc_plan_t* plan, uint32_t mtu_bytes, uint32_t index);

/* GPU, sender.  Cuts the stream that cvlc_encode wrote for `plan` into packets.
 *   d_stream       device, the encoded stream (4-byte aligned)
 *   d_packets_out  device, 4-byte aligned, capacity >= cvlc_packet_count * mtu_bytes */
int cvlc_packetize(const cvlc_plan_t* plan, const void* d_stream, uint32_t mtu_bytes, void* d_packets_out,
                   size_t capacity, void* hip_stream);

/* GPU, receiver.  Puts a stream back together from all n_packets packets of one
 * client, given in any order at a stride of mtu_bytes.  Every packet must agree
 * with the others on the global fields and on its group's fields, and every
 * place must be taken exactly once; otherwise CVLC_DEV_STREAM is set in the
 * workspace's status word and d_stream_out does not hold a stream (its first
 * word is cleared).  The result is what cvlc_decode_aggregate takes.
 *   d_stream_out  device, 4-byte aligned, `capacity` bytes (a stream that needs
 *                 more is refused the same way)
 *   d_workspace   device, 256-byte aligned, >= cvlc_depacketize_workspace_bytes(n_packets) */
size_t cvlc_depacketize_workspace_bytes(uint32_t n_packets);
int cvlc_depacketize(const void* d_packets, uint32_t n_packets, uint32_t mtu_bytes, uint32_t d,
                     void* d_stream_out, size_t capacity, void* d_workspace, size_t ws_bytes, void* hip_stream);

/* Waits for hip_stream and copies the workspace's device status word to
 * *status_out (0 = clean, else CVLC_DEV_* bits). */
int cvlc_device_status(const void* d_workspace, void* hip_stream, uint32_t* status_out);

/* Profiling aid (not part of the hot path).  Between cvlc_profile_start and
 * cvlc_profile_stop every cvlc_encode_batch / cvlc_decode_aggregate / cvlc_fit_alpha call of this
 * process brackets the stages selected in stage_mask (bit i = stage i) with a
 * pair of HIP events on the call's stream.  cvlc_profile_stop waits for those
 * events and returns, per stage, the summed elapsed milliseconds and the number
 * of brackets; both arrays hold CVLC_PROFILE_STAGES entries.  Not thread safe. */
enum {
  CVLC_STAGE_ENC_SETUP = 0,    /* clear scratch, upload per-client parameters   */
  CVLC_STAGE_ENC_SAMPLE = 1,   /* sample histogram -> candidate threshold       */
  CVLC_STAGE_ENC_FILTER = 2,   /* the full pass over the update vectors         */
  CVLC_STAGE_ENC_REFILTER = 3, /* prefix of the kept runs, level-1 boundaries;  */
                               /* keep-all second pass if the sample misjudged  */
  CVLC_STAGE_ENC_SELECT = 4,   /* dense candidate list, exact boundary keys, ties */
  CVLC_STAGE_ENC_CLASSIFY = 5, /* group counts and statistics                   */
  CVLC_STAGE_ENC_LAYOUT = 6,   /* prefix sums, headers, statistics block        */
  CVLC_STAGE_ENC_EMIT = 7,     /* quantise + pack                               */
  CVLC_STAGE_DEC_SETUP = 8,    /* header parsing, list numbering                */
  CVLC_STAGE_DEC_TABLE = 9,    /* per-list tile boundaries                      */
  CVLC_STAGE_DEC_TILES = 10,   /* fused decode + accumulate                     */
  CVLC_STAGE_FIT_ALPHA = 11,   /* cvlc_fit_alpha, the whole call                */
  CVLC_PROFILE_STAGES = 12
};
int cvlc_profile_start(uint32_t stage_mask);
int cvlc_profile_stop(float* ms_per_stage, uint32_t* brackets_per_stage);

/* Static description of a status code. */
const char* cvlc_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CVLC_H */
