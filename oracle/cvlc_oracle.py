"""ctypes front end of the C oracle (oracle/cvlc_oracle.c).

Test infrastructure: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg only.  Nothing here touches the GPU library.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

MAX_R = 31
OK, ERR_ARG, ERR_PLAN, ERR_BUDGET, ERR_CAPACITY, ERR_NONFINITE, ERR_STREAM = 0, -1, -2, -3, -4, -5, -6


class Plan(C.Structure):
    _fields_ = [
        ("d", C.c_uint32), ("R", C.c_uint32), ("s", C.c_uint32),
        ("y", C.c_uint32 * MAX_R), ("P", C.c_uint32 * MAX_R),
        ("total_bits", C.c_uint64), ("B", C.c_float), ("quant", C.c_uint32),
    ]

    def code_len(self) -> List[int]:
        return [int(self.y[r]) for r in range(self.R)]

    def counts(self) -> List[int]:
        return [int(self.P[r]) for r in range(self.R)]

    @property
    def k(self) -> int:
        return sum(self.counts())

    @property
    def total_words(self) -> int:
        return int(self.total_bits // 32)


class SegStats(C.Structure):
    _fields_ = [("min", C.c_float), ("max", C.c_float), ("sumsq", C.c_double),
                ("count", C.c_uint32), ("pad", C.c_uint32), ("errsq", C.c_double)]


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: oracle status {code}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build(force=False))
        u32p, f32p, u64p = C.POINTER(C.c_uint32), C.POINTER(C.c_float), C.POINTER(C.c_uint64)
        L.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.orc_philox4x32_10.restype = None
        L.orc_u24.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        L.orc_u24.restype = C.c_uint32
        L.orc_s_bits.argtypes = [C.c_uint32]
        L.orc_s_bits.restype = C.c_uint32
        L.orc_plan_total_bits.argtypes = [C.POINTER(Plan)]
        L.orc_plan_total_bits.restype = C.c_uint64
        L.orc_plan_validate.argtypes = [C.POINTER(Plan)]
        L.orc_plan_fractions.argtypes = [C.c_uint32, C.c_uint32, u32p, C.POINTER(C.c_double), C.c_float, C.POINTER(Plan)]
        L.orc_plan_budget.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, u32p, C.c_float, C.POINTER(Plan)]
        L.orc_plan_alg1.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, C.c_double, C.c_float, C.POINTER(Plan)]
        L.orc_plan_alg1_quant.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, C.c_double, C.c_float, C.c_uint32,
                                          C.POINTER(Plan)]
        L.orc_alg1_sweep.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, C.c_double, C.c_float, C.c_uint32, C.c_double,
                                     C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.orc_gamma.argtypes = [C.POINTER(Plan), C.c_double]
        L.orc_gamma.restype = C.c_double
        L.orc_rank.argtypes = [f32p, C.c_uint32, u32p]
        L.orc_segments.argtypes = [f32p, C.POINTER(Plan), u32p]
        L.orc_quantise.argtypes = [C.c_float, C.c_float, C.c_float, C.c_uint32, C.c_uint32]
        L.orc_quantise.restype = C.c_uint32
        L.orc_dequantise.argtypes = [C.c_uint32, C.c_float, C.c_float, C.c_uint32]
        L.orc_dequantise.restype = C.c_float
        L.orc_encode.argtypes = [f32p, C.POINTER(Plan), C.c_uint64, C.c_uint32, u32p, C.c_uint64,
                                 C.POINTER(SegStats), u32p, u32p]
        L.orc_decode_aggregate.argtypes = [C.c_uint32, C.POINTER(u32p), u64p, f32p, C.c_uint32, f32p, C.c_int]
        L.orc_unpack.argtypes = [u32p, C.c_uint64, C.c_uint32, u32p, u32p, u32p]
        L.orc_unpack.restype = C.c_int64
        L.orc_fit_alpha.argtypes = [f32p, C.c_uint32, C.POINTER(C.c_double)]
        L.orc_packet_count.argtypes = [C.POINTER(Plan), C.c_uint32]
        L.orc_packet_count.restype = C.c_int64
        L.orc_packetize.argtypes = [u32p, C.c_uint64, C.c_uint32, C.c_uint32, u32p, C.c_uint64, u32p]
        L.orc_packetize.restype = C.c_int64
        L.orc_depacketize.argtypes = [u32p, C.c_uint32, C.c_uint32, C.c_uint32, u32p, C.c_uint64]
        L.orc_depacketize.restype = C.c_int64
        L.orc_qsgd_norm.argtypes = [f32p, C.c_uint32, C.POINTER(C.c_float)]
        L.orc_quantise_qsgd.argtypes = [C.c_float, C.c_float, C.c_uint32, C.c_uint32]
        L.orc_quantise_qsgd.restype = C.c_uint32
        L.orc_dequantise_qsgd.argtypes = [C.c_uint32, C.c_float, C.c_uint32]
        L.orc_dequantise_qsgd.restype = C.c_float
        L.orc_next_scale.argtypes = [C.POINTER(Plan)]
        L.orc_next_scale.restype = C.c_double
        L.orc_empirical_gamma.argtypes = [C.POINTER(SegStats), C.c_uint32]
        L.orc_empirical_gamma.restype = C.c_double
        L.orc_fit_points.argtypes = [f32p, C.c_uint32, u32p, u32p, u32p]
        _lib = L
    return _lib


def _f32(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _u32(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.uint32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_uint32))


def _check(rc: int, what: str) -> None:
    if rc != OK:
        raise OracleError(rc, what)


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> Tuple[int, int, int, int]:
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return tuple(int(v) for v in o)


def u24(seed: int, client: int, i: int) -> int:
    return int(lib().orc_u24(seed, client, i))


def s_bits(d: int) -> int:
    return int(lib().orc_s_bits(d))


def plan_fractions(d: int, code_len: Sequence[int], fractions: Sequence[float], B: float = 1.0) -> Plan:
    R = len(code_len)
    p = Plan()
    _check(lib().orc_plan_fractions(d, R, (C.c_uint32 * R)(*code_len), (C.c_double * R)(*fractions), B, C.byref(p)),
           "plan_fractions")
    return p


def plan_budget(d: int, budget_bits: int, code_len: Sequence[int], B: float = 1.0) -> Plan:
    R = len(code_len)
    p = Plan()
    _check(lib().orc_plan_budget(d, budget_bits, R, (C.c_uint32 * R)(*code_len), B, C.byref(p)), "plan_budget")
    return p


def plan_alg1(d: int, budget_bits: int, R: int, alpha: float, B: float = 1.0, quant: int = 0) -> Plan:
    p = Plan()
    _check(lib().orc_plan_alg1_quant(d, budget_bits, R, alpha, B, quant, C.byref(p)), "plan_alg1")
    return p


PQ, QSGD = 0, 1


def alg1_sweep(d: int, budget_bits: int, R: int, alpha: float, k: float, B: float = 1.0,
               quant: int = 0) -> Tuple[List[float], float]:
    """Real-valued P_1..P_R the sweep of atomic operations settles on for this k, and gamma there."""
    P = (C.c_double * R)()
    g = C.c_double()
    _check(lib().orc_alg1_sweep(d, budget_bits, R, alpha, B, quant, k, P, C.byref(g)), "alg1_sweep")
    return [float(v) for v in P], float(g.value)


def plan_manual(d: int, code_len: Sequence[int], counts: Sequence[int], B: float = 1.0, quant: int = PQ) -> Plan:
    """A plan with explicit group sizes (validated by the oracle)."""
    p = Plan()
    p.d, p.R, p.s, p.B, p.quant = d, len(code_len), s_bits(d), B, quant
    for r, (y, P) in enumerate(zip(code_len, counts)):
        p.y[r], p.P[r] = y, P
    p.total_bits = lib().orc_plan_total_bits(C.byref(p))
    _check(lib().orc_plan_validate(C.byref(p)), "plan_manual")
    return p


def plan_for(workload, client: int = 0, alpha: float = -0.5, d: Optional[int] = None) -> Plan:
    """Plan of a cvlc_synth.Workload, optionally at a reduced vector length."""
    dd = workload.d if d is None else d
    scale = dd / workload.d
    if workload.mode == "fractions":
        return plan_fractions(dd, workload.code_len, workload.fractions)
    if workload.mode == "budget":
        return plan_budget(dd, int(workload.budget_bits(client) * scale), workload.code_len)
    return plan_alg1(dd, int(workload.budget_bits(client) * scale), workload.n_coded, alpha)


def gamma(plan: Plan, alpha: float) -> float:
    return float(lib().orc_gamma(C.byref(plan), alpha))


def rank(U: np.ndarray) -> np.ndarray:
    order = np.empty(U.size, dtype=np.uint32)
    _check(lib().orc_rank(_f32(U), U.size, _u32(order)), "rank")
    return order


def segments(U: np.ndarray, plan: Plan) -> np.ndarray:
    seg = np.empty(U.size, dtype=np.uint32)
    _check(lib().orc_segments(_f32(U), C.byref(plan), _u32(seg)), "segments")
    return seg


def quantise(x: float, m: float, M: float, y: int, u: int) -> int:
    return int(lib().orc_quantise(x, m, M, y, u))


def dequantise(cid: int, m: float, M: float, y: int) -> float:
    return float(lib().orc_dequantise(cid, m, M, y))


@dataclass
class Encoded:
    words: np.ndarray           # uint32 stream
    stats: List[SegStats]       # R coded groups, then the tail
    seg: Optional[np.ndarray]   # per coordinate group id (0 = dropped)
    cid: Optional[np.ndarray]   # per coordinate CID


def encode(U: np.ndarray, plan: Plan, seed: int, client: int, debug: bool = False,
           cap_words: Optional[int] = None) -> Encoded:
    n = plan.total_words if cap_words is None else cap_words
    words = np.zeros(max(n, 1), dtype=np.uint32)
    stats = (SegStats * (plan.R + 1))()
    seg = np.empty(U.size, dtype=np.uint32) if debug else None
    cid = np.empty(U.size, dtype=np.uint32) if debug else None
    _check(lib().orc_encode(_f32(U), C.byref(plan), seed, client, _u32(words), n, stats, _u32(seg), _u32(cid)),
           "encode")
    return Encoded(words[: plan.total_words], list(stats), seg, cid)


def decode_aggregate(streams: Sequence[np.ndarray], d: int, weights: Optional[Sequence[float]] = None,
                     out: Optional[np.ndarray] = None) -> np.ndarray:
    """Aggregate of the streams; with `out` given, accumulates into it."""
    n = len(streams)
    u32p = C.POINTER(C.c_uint32)
    ptrs = (u32p * max(n, 1))(*[_u32(s) for s in streams])
    nwords = (C.c_uint64 * max(n, 1))(*[s.size for s in streams])
    w = None
    if weights is not None:
        w = (C.c_float * max(n, 1))(*weights)
    accumulate = out is not None
    if out is None:
        out = np.zeros(d, dtype=np.float32)
    _check(lib().orc_decode_aggregate(n, ptrs, nwords, w, d, _f32(out), int(accumulate)), "decode_aggregate")
    return out


def unpack(stream: np.ndarray, d: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    cap = int(stream.size * 32)  # more records than any stream of this size can hold
    cap = min(cap, d)
    pid = np.empty(max(cap, 1), dtype=np.uint32)
    cid = np.empty(max(cap, 1), dtype=np.uint32)
    seg = np.empty(max(cap, 1), dtype=np.uint32)
    k = lib().orc_unpack(_u32(stream), stream.size, d, _u32(pid), _u32(cid), _u32(seg))
    if k < 0:
        raise OracleError(int(k), "unpack")
    return pid[:k], cid[:k], seg[:k]


def packet_count(plan: Plan, mtu: int = 1500) -> int:
    n = int(lib().orc_packet_count(C.byref(plan), mtu))
    if n < 0:
        raise OracleError(n, "packet_count")
    return n


def packetize(stream: np.ndarray, d: int, mtu: int = 1500) -> Tuple[np.ndarray, np.ndarray]:
    """(packets as an (n, mtu/4) uint32 array, zero behind each packet's end; their lengths in bytes)."""
    cap = stream.size // 1 + 64   # never more packets than words
    buf = np.zeros((cap, mtu // 4), dtype=np.uint32)
    sizes = np.zeros(cap, dtype=np.uint32)
    n = int(lib().orc_packetize(_u32(stream), stream.size, d, mtu, _u32(buf), cap, _u32(sizes)))
    if n < 0:
        raise OracleError(n, "packetize")
    return buf[:n].copy(), sizes[:n].copy()


def depacketize(packets: np.ndarray, d: int, mtu: int = 1500, cap_words: Optional[int] = None) -> np.ndarray:
    packets = np.ascontiguousarray(packets, dtype=np.uint32)
    cap = int(cap_words) if cap_words is not None else packets.size + 64
    out = np.zeros(cap, dtype=np.uint32)
    n = int(lib().orc_depacketize(_u32(packets), packets.shape[0], mtu, d, _u32(out), cap))
    if n < 0:
        raise OracleError(n, "depacketize")
    return out[:n].copy()


def qsgd_norm(x: np.ndarray) -> float:
    """The l2-norm QSGD's header carries: smallest fp32 n with n*n >= sum of x_i^2 (exactly)."""
    out = C.c_float()
    _check(lib().orc_qsgd_norm(_f32(x), x.size, C.byref(out)), "qsgd_norm")
    return float(out.value)


def quantise_qsgd(x: float, norm: float, y: int, u: int) -> int:
    return int(lib().orc_quantise_qsgd(x, norm, y, u))


def dequantise_qsgd(cid: int, norm: float, y: int) -> float:
    return float(lib().orc_dequantise_qsgd(cid, norm, y))


def next_scale(plan: Plan) -> float:
    """B for the next round: max_r Q(P_r, y_r) + 1 (footnote to Proposition 1)."""
    return float(lib().orc_next_scale(C.byref(plan)))


def empirical_gamma(stats: Sequence[SegStats], R: int) -> float:
    """||Uhat - U||^2 / ||U||^2 from an encode's statistics block."""
    arr = (SegStats * (R + 1))(*stats[: R + 1])
    return float(lib().orc_empirical_gamma(arr, R))


def fit_points(U: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(ranks, magnitude bit patterns) at which Definition 1's exponent is fitted."""
    ranks = np.zeros(32, dtype=np.uint32)
    keys = np.zeros(32, dtype=np.uint32)
    n = C.c_uint32(0)
    _check(lib().orc_fit_points(_f32(U), U.size, _u32(ranks), _u32(keys), C.byref(n)), "fit_points")
    return ranks[: n.value].copy(), keys[: n.value].copy()


def fit_alpha(U: np.ndarray) -> float:
    a = C.c_double()
    _check(lib().orc_fit_alpha(_f32(U), U.size, C.byref(a)), "fit_alpha")
    return float(a.value)
