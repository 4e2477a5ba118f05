"""ctypes binding of libcvlc (include/cvlc.h).  Names mirror the C entry points.

PyTorch is used for device memory and the current HIP stream only.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

MAX_CODED = 31
STATS_STRIDE = 32
DEV_NONFINITE, DEV_STREAM, DEV_INTERNAL, DEV_WORKSPACE = 1, 2, 4, 8
DECODE_ACCUMULATE = 1
DECODE_QSGD = 2
QUANT_PQ, QUANT_QSGD = 0, 1
ENCODE_ERROR_STATS = 1
FIT_RANKS_MAX = 32

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcvlc.so")


class Plan(C.Structure):
    """cvlc_plan_t"""
    _fields_ = [
        ("d", C.c_uint32), ("n_coded", C.c_uint32), ("s", C.c_uint32),
        ("code_len", C.c_uint32 * MAX_CODED), ("count", C.c_uint32 * MAX_CODED),
        ("total_bits", C.c_uint64), ("B", C.c_float), ("quant", C.c_uint32),
    ]

    def code_lens(self) -> List[int]:
        return [int(self.code_len[r]) for r in range(self.n_coded)]

    def counts(self) -> List[int]:
        return [int(self.count[r]) for r in range(self.n_coded)]

    @property
    def k(self) -> int:
        return sum(self.counts())

    @property
    def stream_bytes(self) -> int:
        return int(self.total_bits // 8)


class SegStats(C.Structure):
    """cvlc_seg_stats_t"""
    _fields_ = [("min", C.c_float), ("max", C.c_float), ("sumsq", C.c_double),
                ("count", C.c_uint32), ("reserved", C.c_uint32), ("errsq", C.c_double)]


class CvlcError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {status_string(code)} ({code})")
        self.code = code


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """The loaded libcvlc.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python paper_2402_03770_amd/build.py` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, u32p, szp = C.c_void_p, C.POINTER(C.c_uint32), C.POINTER(C.c_size_t)
        L.cvlc_position_bits.argtypes = [C.c_uint32]
        L.cvlc_position_bits.restype = C.c_uint32
        L.cvlc_plan.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, u32p, C.POINTER(C.c_double), C.c_double,
                                C.c_float, C.POINTER(Plan)]
        L.cvlc_plan_algorithm1.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, C.c_double, C.c_float, C.c_uint32,
                                           C.POINTER(Plan)]
        L.cvlc_plan_validate.argtypes = [C.POINTER(Plan)]
        L.cvlc_plan_total_bits.argtypes = [C.POINTER(Plan)]
        L.cvlc_plan_total_bits.restype = C.c_uint64
        L.cvlc_plan_gamma.argtypes = [C.POINTER(Plan), C.c_double]
        L.cvlc_plan_gamma.restype = C.c_double
        L.cvlc_stream_capacity.argtypes = [C.POINTER(Plan)]
        L.cvlc_stream_capacity.restype = C.c_size_t
        L.cvlc_encode_workspace_bytes.argtypes = [C.c_uint32, C.c_uint32]
        L.cvlc_encode_workspace_bytes.restype = C.c_size_t
        L.cvlc_encode_workspace_bytes_for.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32]
        L.cvlc_encode_workspace_bytes_for.restype = C.c_size_t
        L.cvlc_plan_candidates_hint.argtypes = [C.POINTER(Plan)]
        L.cvlc_plan_candidates_hint.restype = C.c_uint32
        L.cvlc_decode_workspace_bytes.argtypes = [C.c_uint32, C.c_uint32]
        L.cvlc_decode_workspace_bytes.restype = C.c_size_t
        L.cvlc_encode_batch.argtypes = [C.c_uint32, C.POINTER(Plan), C.POINTER(vp), C.c_uint64, u32p, C.POINTER(vp),
                                        szp, vp, C.c_size_t, vp, C.c_uint32, vp]
        L.cvlc_encode.argtypes = [C.POINTER(Plan), vp, C.c_uint64, C.c_uint32, vp, C.c_size_t, vp, C.c_size_t, vp,
                                  C.c_uint32, vp]
        L.cvlc_plan_next_scale.argtypes = [C.POINTER(Plan)]
        L.cvlc_plan_next_scale.restype = C.c_double
        L.cvlc_stats_gamma.argtypes = [C.POINTER(SegStats), C.c_uint32]
        L.cvlc_stats_gamma.restype = C.c_double
        L.cvlc_decode_aggregate.argtypes = [C.c_uint32, C.POINTER(vp), szp, C.POINTER(C.c_float), vp, C.c_uint32,
                                            C.c_uint32, vp, C.c_size_t, vp]
        L.cvlc_decode_aggregate_static.argtypes = [C.c_uint32, C.POINTER(vp), szp, C.POINTER(C.c_float), vp, C.c_uint32,
                                                   C.c_uint32, vp, vp]
        L.cvlc_device_status.argtypes = [vp, vp, u32p]
        L.cvlc_packet_count.argtypes = [C.POINTER(Plan), C.c_uint32]
        L.cvlc_packet_count.restype = C.c_uint32
        L.cvlc_packet_size.argtypes = [C.POINTER(Plan), C.c_uint32, C.c_uint32]
        L.cvlc_packet_size.restype = C.c_uint32
        L.cvlc_packetize.argtypes = [C.POINTER(Plan), vp, C.c_uint32, vp, C.c_size_t, vp]
        L.cvlc_depacketize_workspace_bytes.argtypes = [C.c_uint32]
        L.cvlc_depacketize_workspace_bytes.restype = C.c_size_t
        L.cvlc_depacketize.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_uint32, vp, C.c_size_t, vp, C.c_size_t, vp]
        L.cvlc_fit_ranks.argtypes = [C.c_uint32, u32p]
        L.cvlc_fit_ranks.restype = C.c_uint32
        L.cvlc_fit_workspace_bytes.argtypes = [C.c_uint32]
        L.cvlc_fit_workspace_bytes.restype = C.c_size_t
        L.cvlc_fit_workspace_bytes_for.argtypes = [C.c_uint32, C.c_uint32]
        L.cvlc_fit_workspace_bytes_for.restype = C.c_size_t
        L.cvlc_fit_alpha.argtypes = [C.c_uint32, C.POINTER(vp), C.c_uint32, vp, vp, vp, C.c_size_t, vp]
        L.cvlc_profile_start.argtypes = [C.c_uint32]
        L.cvlc_profile_stop.argtypes = [C.POINTER(C.c_float), u32p]
        L.cvlc_status_string.argtypes = [C.c_int]
        L.cvlc_status_string.restype = C.c_char_p
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().cvlc_status_string(code).decode()


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise CvlcError(rc, what)


def _stream_handle() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


# ----------------------------------------------------------------------------- host side
def position_bits(d: int) -> int:
    return int(lib().cvlc_position_bits(d))


def plan(d: int, budget_bits: int = 0, n_coded: Optional[int] = None, code_len: Optional[Sequence[int]] = None,
         fractions: Optional[Sequence[float]] = None, alpha: float = -0.5, B: float = 1.0) -> Plan:
    """cvlc_plan: fractions+code_len, or budget+code_len, or budget+n_coded (Algorithm 1)."""
    if code_len is not None:
        n_coded = len(code_len)
    assert n_coded is not None
    cl = (C.c_uint32 * max(n_coded, 1))(*code_len) if code_len is not None else None
    fr = (C.c_double * max(n_coded, 1))(*fractions) if fractions is not None else None
    out = Plan()
    _check(lib().cvlc_plan(d, budget_bits, n_coded, cl, fr, alpha, B, C.byref(out)), "cvlc_plan")
    return out


def plan_algorithm1(d: int, budget_bits: int, n_coded: int, alpha: float = -0.5, B: float = 1.0,
                    quant: int = QUANT_PQ) -> Plan:
    """cvlc_plan_algorithm1: Algorithm 1 priced with the named quantiser's error model."""
    out = Plan()
    _check(lib().cvlc_plan_algorithm1(d, budget_bits, n_coded, alpha, B, quant, C.byref(out)), "cvlc_plan_algorithm1")
    return out


def plan_manual(d: int, code_len: Sequence[int], counts: Sequence[int], B: float = 1.0,
                quant: int = QUANT_PQ) -> Plan:
    """A caller-built plan, checked by cvlc_plan_validate."""
    p = Plan()
    p.d, p.n_coded, p.s, p.B, p.quant = d, len(code_len), position_bits(d), B, quant
    for r, (y, P) in enumerate(zip(code_len, counts)):
        p.code_len[r], p.count[r] = y, P
    p.total_bits = lib().cvlc_plan_total_bits(C.byref(p))
    _check(lib().cvlc_plan_validate(C.byref(p)), "cvlc_plan_validate")
    return p


def plan_gamma(p: Plan, alpha: float) -> float:
    return float(lib().cvlc_plan_gamma(C.byref(p), alpha))


def plan_next_scale(p: Plan) -> float:
    """cvlc_plan_next_scale: B for the next round from this round's plan."""
    return float(lib().cvlc_plan_next_scale(C.byref(p)))


def stats_gamma(stats: Sequence[SegStats], n_coded: int) -> float:
    """cvlc_stats_gamma over one client's entries as read_stats returns them."""
    arr = (SegStats * (n_coded + 1))(*stats[: n_coded + 1])
    return float(lib().cvlc_stats_gamma(arr, n_coded))


def stream_capacity(p: Plan) -> int:
    return int(lib().cvlc_stream_capacity(C.byref(p)))


def encode_workspace_bytes(d: int, n_clients: int) -> int:
    return int(lib().cvlc_encode_workspace_bytes(d, n_clients))


def encode_workspace_bytes_for(d: int, n_clients: int, max_candidates: int) -> int:
    return int(lib().cvlc_encode_workspace_bytes_for(d, n_clients, max_candidates))


def plan_candidates_hint(p: Plan) -> int:
    return int(lib().cvlc_plan_candidates_hint(C.byref(p)))


def decode_workspace_bytes(d: int, n_clients: int) -> int:
    return int(lib().cvlc_decode_workspace_bytes(d, n_clients))


def packet_count(p: Plan, mtu: int = 1500) -> int:
    return int(lib().cvlc_packet_count(C.byref(p), mtu))


def packet_size(p: Plan, index: int, mtu: int = 1500) -> int:
    return int(lib().cvlc_packet_size(C.byref(p), mtu, index))


def depacketize_workspace_bytes(n_packets: int) -> int:
    return int(lib().cvlc_depacketize_workspace_bytes(n_packets))


def fit_ranks(d: int) -> List[int]:
    """cvlc_fit_ranks: the ranks at which cvlc_fit_alpha reads the magnitudes."""
    out = (C.c_uint32 * FIT_RANKS_MAX)()
    n = int(lib().cvlc_fit_ranks(d, out))
    return [int(out[j]) for j in range(n)]


def fit_workspace_bytes(n_clients: int) -> int:
    return int(lib().cvlc_fit_workspace_bytes(n_clients))


def fit_workspace_bytes_for(n_clients: int, d: int) -> int:
    return int(lib().cvlc_fit_workspace_bytes_for(n_clients, d))


# ----------------------------------------------------------------------------- device side
def new_workspace(n_bytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(n_bytes), 256), dtype=torch.uint8, device=device)


def new_stream_buffer(p: Plan, device="cuda") -> torch.Tensor:
    return torch.empty(max(p.stream_bytes // 4, 1), dtype=torch.int32, device=device)


def encode_batch(plans: Sequence[Plan], updates: Sequence[torch.Tensor], seed: int, client_ids: Sequence[int],
                 streams_out: Sequence[torch.Tensor], workspace: torch.Tensor,
                 stats_out: Optional[torch.Tensor] = None, error_stats: bool = False) -> None:
    """cvlc_encode_batch on the current stream.  `streams_out[i]` is an int32/uint8 device
    tensor of at least plan.stream_bytes; `stats_out` an optional uint8 device tensor of
    n * STATS_STRIDE * sizeof(SegStats) bytes; `error_stats` sets CVLC_ENCODE_ERROR_STATS."""
    n = len(plans)
    vp = C.c_void_p
    plan_arr = (Plan * n)(*plans)
    upd = (vp * n)(*[u.data_ptr() for u in updates])
    ids = (C.c_uint32 * n)(*client_ids)
    outs = (vp * n)(*[s.data_ptr() for s in streams_out])
    caps = (C.c_size_t * n)(*[s.numel() * s.element_size() for s in streams_out])
    _check(lib().cvlc_encode_batch(n, plan_arr, upd, seed, ids, outs, caps, workspace.data_ptr(),
                                   workspace.numel(), stats_out.data_ptr() if stats_out is not None else None,
                                   ENCODE_ERROR_STATS if error_stats else 0, _stream_handle()), "cvlc_encode_batch")


def encode(p: Plan, update: torch.Tensor, seed: int, client_id: int, stream_out: torch.Tensor,
           workspace: torch.Tensor, stats_out: Optional[torch.Tensor] = None, error_stats: bool = False) -> None:
    """cvlc_encode on the current stream."""
    _check(lib().cvlc_encode(C.byref(p), update.data_ptr(), seed, client_id, stream_out.data_ptr(),
                             stream_out.numel() * stream_out.element_size(), workspace.data_ptr(), workspace.numel(),
                             stats_out.data_ptr() if stats_out is not None else None,
                             ENCODE_ERROR_STATS if error_stats else 0, _stream_handle()), "cvlc_encode")


def decode_aggregate(streams: Sequence[torch.Tensor], out: torch.Tensor, workspace: torch.Tensor,
                     weights: Optional[Sequence[float]] = None, accumulate: bool = False,
                     stream_bytes: Optional[Sequence[int]] = None, quant: int = QUANT_PQ) -> None:
    """cvlc_decode_aggregate on the current stream; `out` is a float32 device tensor of d entries."""
    n = len(streams)
    vp = C.c_void_p
    ptrs = (vp * max(n, 1))(*[s.data_ptr() for s in streams])
    if stream_bytes is None:
        stream_bytes = [s.numel() * s.element_size() for s in streams]
    sizes = (C.c_size_t * max(n, 1))(*stream_bytes)
    w = (C.c_float * max(n, 1))(*weights) if weights is not None else None
    _check(lib().cvlc_decode_aggregate(n, ptrs, sizes, w, out.data_ptr(), out.numel(),
                                       (DECODE_ACCUMULATE if accumulate else 0) | (DECODE_QSGD if quant == QUANT_QSGD else 0),
                                       workspace.data_ptr(),
                                       workspace.numel(), _stream_handle()), "cvlc_decode_aggregate")


DECODE_STATIC_BYTES = 16 << 20


def decode_aggregate_static(streams: Sequence[torch.Tensor], out: torch.Tensor,
                            status_out: Optional[torch.Tensor] = None, weights: Optional[Sequence[float]] = None,
                            accumulate: bool = False, stream_bytes: Optional[Sequence[int]] = None,
                            quant: int = QUANT_PQ) -> None:
    """cvlc_decode_aggregate_static on the current stream: no workspace, no allocation; `status_out` is an
    optional int32 device tensor of one entry that receives the status word."""
    n = len(streams)
    vp = C.c_void_p
    ptrs = (vp * max(n, 1))(*[s.data_ptr() for s in streams])
    if stream_bytes is None:
        stream_bytes = [s.numel() * s.element_size() for s in streams]
    sizes = (C.c_size_t * max(n, 1))(*stream_bytes)
    w = (C.c_float * max(n, 1))(*weights) if weights is not None else None
    _check(lib().cvlc_decode_aggregate_static(n, ptrs, sizes, w, out.data_ptr(), out.numel(),
                                              (DECODE_ACCUMULATE if accumulate else 0) | (DECODE_QSGD if quant == QUANT_QSGD else 0),
                                              status_out.data_ptr() if status_out is not None else None,
                                              _stream_handle()), "cvlc_decode_aggregate_static")


def packetize(p: Plan, stream: torch.Tensor, packets_out: torch.Tensor, mtu: int = 1500) -> None:
    """cvlc_packetize on the current stream; `packets_out` holds packet_count(p, mtu) * mtu bytes."""
    _check(lib().cvlc_packetize(C.byref(p), stream.data_ptr(), mtu, packets_out.data_ptr(),
                                packets_out.numel() * packets_out.element_size(), _stream_handle()), "cvlc_packetize")


def depacketize(packets: torch.Tensor, n_packets: int, d: int, stream_out: torch.Tensor, workspace: torch.Tensor,
                mtu: int = 1500) -> None:
    """cvlc_depacketize on the current stream."""
    _check(lib().cvlc_depacketize(packets.data_ptr(), n_packets, mtu, d, stream_out.data_ptr(),
                                  stream_out.numel() * stream_out.element_size(), workspace.data_ptr(),
                                  workspace.numel(), _stream_handle()), "cvlc_depacketize")


def fit_alpha(updates: Sequence[torch.Tensor], alpha_out: torch.Tensor, workspace: torch.Tensor,
              keys_out: Optional[torch.Tensor] = None) -> None:
    """cvlc_fit_alpha on the current stream.  `alpha_out` is a float64 device tensor of n entries,
    `keys_out` an optional int32 device tensor of n * FIT_RANKS_MAX entries."""
    n = len(updates)
    vp = C.c_void_p
    upd = (vp * max(n, 1))(*[u.data_ptr() for u in updates])
    d = updates[0].numel() if n else 0
    _check(lib().cvlc_fit_alpha(n, upd, d, alpha_out.data_ptr(), keys_out.data_ptr() if keys_out is not None else None,
                                workspace.data_ptr(), workspace.numel(), _stream_handle()), "cvlc_fit_alpha")


def device_status(workspace: torch.Tensor) -> int:
    """cvlc_device_status: waits for the current stream, returns the CVLC_DEV_* bits."""
    st = C.c_uint32(0)
    _check(lib().cvlc_device_status(workspace.data_ptr(), _stream_handle(), C.byref(st)), "cvlc_device_status")
    return int(st.value)


def read_stats(stats_out: torch.Tensor, client: int, n_coded: int) -> List[SegStats]:
    """Host copy of one client's statistics block (n_coded groups, then the tail)."""
    raw = stats_out.cpu().numpy().tobytes()
    size = C.sizeof(SegStats)
    base = client * STATS_STRIDE * size
    return [SegStats.from_buffer_copy(raw[base + r * size: base + (r + 1) * size]) for r in range(n_coded + 1)]


PROFILE_STAGES = ["enc_setup", "enc_sample", "enc_filter", "enc_refilter", "enc_select", "enc_classify",
                  "enc_layout", "enc_emit", "dec_setup", "dec_table", "dec_tiles", "fit_alpha"]


def profile_start(stages: Sequence[str] = tuple(PROFILE_STAGES)) -> None:
    """cvlc_profile_start for the named stages."""
    mask = 0
    for name in stages:
        mask |= 1 << PROFILE_STAGES.index(name)
    _check(lib().cvlc_profile_start(mask), "cvlc_profile_start")


def profile_stop() -> dict:
    """cvlc_profile_stop: {stage: (total_ms, brackets)} for the stages that ran."""
    n = len(PROFILE_STAGES)
    ms = (C.c_float * n)()
    cnt = (C.c_uint32 * n)()
    _check(lib().cvlc_profile_stop(ms, cnt), "cvlc_profile_stop")
    return {PROFILE_STAGES[i]: (float(ms[i]), int(cnt[i])) for i in range(n) if cnt[i]}
