"""Seeded synthetic inputs: request traces, request classes, profile tables,
candidate configurations and SLOs.

This module only *produces data*.  It contains none of the evaluator's
arithmetic (no binning of requests into cells, no load, no interpolation, no
percentiles, no selection): both the CPU oracle and the HIP library receive the
arrays made here and each does all of that on its own.

The traces stand in for production invocation traces of the kind the paper
characterises in Section III (a record is: arrival timestamp, number of input
tokens, number of output tokens; inputs of at most 8192 tokens, Table IV; a
diurnal and weekday/weekend load pattern, Section III-B).  No record of any real
trace is reproduced; everything is drawn from the distributions below.

Random numbers come from a counter-based SplitMix64 sequence so that element i of
a stream can be produced independently of every other element and the result is
identical on every machine up to the last-bit behaviour of libm's log/cos/exp.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Tuple

import numpy as np

_MASK = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

# stream identifiers (one independent random stream per purpose)
_S_ARRIVAL_T, _S_ARRIVAL_ACC, _S_IN, _S_OUT, _S_MODEL, _S_PROFILE = 1, 2, 3, 4, 5, 16


def _mix_int(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


def stream_key(seed: int, purpose: int) -> int:
    """64-bit key of the random stream (seed, purpose)."""
    return _mix_int(_mix_int(seed * _GAMMA + 0x1234567) ^ ((purpose + 1) * _GAMMA))


def u64_stream(key: int, start: int, count: int) -> np.ndarray:
    """Elements start .. start+count-1 of the SplitMix64 sequence keyed by `key`."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(key) + idx * np.uint64(_GAMMA)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
        return z ^ (z >> np.uint64(31))


def uniform_stream(key: int, start: int, count: int) -> np.ndarray:
    """53-bit uniforms in [0, 1)."""
    return (u64_stream(key, start, count) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def normal_stream(key: int, start: int, count: int) -> np.ndarray:
    """Standard normals by Box-Muller; element i uses uniforms 2i and 2i+1."""
    u = uniform_stream(key, 2 * start, 2 * count)
    r = np.sqrt(-2.0 * np.log(1.0 - u[0::2]))
    return r * np.cos((2.0 * math.pi) * u[1::2])


@dataclasses.dataclass(frozen=True)
class WorkloadSpec:
    name: str
    seed: int
    n_req: int
    n_window: int
    window_s: float
    rate_shape: str                 # "const" | "hour" | "day" | "week"
    in_edges: Tuple[int, ...]       # interior class edges on input tokens
    out_edges: Tuple[int, ...]
    tp: Tuple[int, ...]
    f_mhz: Tuple[float, ...]
    n_inst_max: int
    n_rho: int
    n_model: int = 1
    model_mix: Tuple[float, ...] = (1.0,)
    idle_cost_weight: float = 0.0
    per_class_exponent: bool = False

    @property
    def n_class(self) -> int:
        return self.n_model * (len(self.in_edges) + 1) * (len(self.out_edges) + 1)

    @property
    def n_config(self) -> int:
        return len(self.tp) * len(self.f_mhz) * self.n_inst_max

    def scaled(self, n_req: int, n_window: int, name: str | None = None) -> "WorkloadSpec":
        """Same shape with fewer requests / windows (for tests)."""
        return dataclasses.replace(self, n_req=n_req, n_window=n_window,
                                   name=name or f"{self.name}-r{n_req}-w{n_window}")


def _freqs(lo: int, hi: int, step: int) -> Tuple[float, ...]:
    return tuple(float(f) for f in range(lo, hi + 1, step))


_EDGES5 = (169, 446, 1176, 3104)   # interior points of 64 * 128**(i/5), i = 0..5, rounded

SPECS: Dict[int, WorkloadSpec] = {
    0: WorkloadSpec("cfg0-tiny", 0, 10_000, 1, 60.0, "const", (256, 2048), (128, 512),
                    (2, 4, 8), _freqs(880, 1980, 220), 4, 16),
    1: WorkloadSpec("cfg1-hour", 1, 1_000_000, 60, 60.0, "hour", (256, 2048), (128, 512),
                    (2, 4, 8), _freqs(880, 1980, 100), 16, 32),
    2: WorkloadSpec("cfg2-day", 2, 10_000_000, 1440, 60.0, "day", _EDGES5, _EDGES5,
                    (2, 4, 8), _freqs(880, 1980, 100), 16, 64),
    3: WorkloadSpec("cfg3-week", 3, 50_000_000, 2016, 300.0, "week", _EDGES5, _EDGES5,
                    (2, 4, 8), _freqs(880, 1980, 100), 32, 64, per_class_exponent=True),
    4: WorkloadSpec("cfg4-multimodel", 4, 100_000_000, 2016, 300.0, "week", _EDGES5, _EDGES5,
                    (1, 2, 4, 8), _freqs(480, 1980, 100), 32, 64, n_model=4,
                    model_mix=(0.4, 0.3, 0.2, 0.1), idle_cost_weight=0.1),
}


def _rate(shape: str, t: np.ndarray) -> np.ndarray:
    """Relative arrival rate (only its shape matters: the request count is fixed)."""
    if shape == "const":
        return np.ones_like(t)
    if shape == "hour":
        return 1.0 + 0.3 * np.sin((2.0 * math.pi / 3600.0) * t)
    day = 1.0 + 0.6 * np.sin((2.0 * math.pi / 86400.0) * (t - 6.0 * 3600.0))
    if shape == "day":
        return day
    if shape == "week":        # t = 0 is Monday 00:00; days 5 and 6 are the weekend
        dow = np.floor(t / 86400.0).astype(np.int64) % 7
        return day * np.where(dow >= 5, 0.6, 1.0)
    raise ValueError(shape)


_RATE_MAX = {"const": 1.0, "hour": 1.3, "day": 1.6, "week": 1.6}
# peak rate / mean rate of each shape over whole periods
_PEAK_OVER_MEAN = {"const": 1.0, "hour": 1.3, "day": 1.6, "week": 1.6 / ((5.0 + 2.0 * 0.6) / 7.0)}


def arrivals(spec: WorkloadSpec) -> np.ndarray:
    """Exactly n_req arrival times on [0, n_window*window_s): a Poisson process with
    the spec's rate shape, conditioned on its count (thinning of uniform candidates
    taken in stream order), sorted ascending."""
    horizon = spec.n_window * spec.window_s
    kt, ka = stream_key(spec.seed, _S_ARRIVAL_T), stream_key(spec.seed, _S_ARRIVAL_ACC)
    rmax = _RATE_MAX[spec.rate_shape]
    out = np.empty(spec.n_req, dtype=np.float64)
    have, pos, chunk = 0, 0, min(1 << 22, max(1 << 12, 2 * spec.n_req))
    while have < spec.n_req:
        t = uniform_stream(kt, pos, chunk) * horizon
        keep = t[uniform_stream(ka, pos, chunk) * rmax <= _rate(spec.rate_shape, t)]
        take = min(keep.size, spec.n_req - have)
        out[have:have + take] = keep[:take]
        have += take
        pos += chunk
    out.sort()
    # a product u*horizon can round up to the horizon itself; keep times strictly inside
    np.minimum(out, np.nextafter(horizon, 0.0), out=out)
    return out


def _tokens(key: int, n: int, median: float, sigma: float) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    chunk = 1 << 22
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        z = normal_stream(key, s, c)
        v = np.rint(np.exp(math.log(median) + sigma * z))
        out[s:s + c] = np.clip(v, 1.0, 8192.0).astype(np.int32)
    return out


def trace(spec: WorkloadSpec) -> Dict[str, np.ndarray]:
    """Request records: t_s (f64, ascending), in_tok, out_tok, model (i32)."""
    n = spec.n_req
    t_s = arrivals(spec)
    in_tok = _tokens(stream_key(spec.seed, _S_IN), n, 1000.0, 1.0)
    out_tok = _tokens(stream_key(spec.seed, _S_OUT), n, 250.0, 0.8)
    if spec.n_model == 1:
        model = np.zeros(n, dtype=np.int32)
    else:
        cum = np.cumsum(np.asarray(spec.model_mix, dtype=np.float64))
        model = np.empty(n, dtype=np.int32)
        km, chunk = stream_key(spec.seed, _S_MODEL), 1 << 22
        for s in range(0, n, chunk):
            c = min(chunk, n - s)
            u = uniform_stream(km, s, c)
            model[s:s + c] = np.minimum((u[:, None] >= cum[None, :-1]).sum(axis=1),
                                        spec.n_model - 1).astype(np.int32)
    return {"t_s": t_s, "in_tok": in_tok, "out_tok": out_tok, "model": model}


def profile(spec: WorkloadSpec) -> Dict[str, np.ndarray]:
    """Synthetic energy-performance profile tables over (class, TP, frequency, load).

    Laws (per class c of model j, TP degree p, frequency f, load-grid point r):
      slow(c,p,f)  = (f_max/f)**a / p**b
      prefill ms/token = k_p[c] * slow            (constant along the load axis)
      TBT ms           = min(k_d[c] * slow / (1 - r), 1000)
      power W          = p * (100 + 600 * (f/f_max)**3 * r)   (whole instance)
      capacity tok/s   = S_j * p * 1000 / (k_d[c] * slow)
    with a ~ U[0.6,1.0], b ~ U[0.6,0.9] per model (a per class ~ U[0.5,1.1] when
    spec.per_class_exponent), k_p ~ U[0.05,0.2], k_d ~ U[15,40] per class, both scaled
    by 2**j for model j.  S_j is fixed from the spec alone (never from the drawn trace):
    it puts a class carrying 1/sqrt(classes per model) of the model's nominal peak token
    rate (2000 tokens per request) at load 0.6 on the largest configuration.
    """
    bi, bo = len(spec.in_edges) + 1, len(spec.out_edges) + 1
    cpm = bi * bo
    g_all = spec.n_model * cpm
    tp = np.asarray(spec.tp, dtype=np.int32)
    f = np.asarray(spec.f_mhz, dtype=np.float64)
    rho = np.linspace(0.0, 0.95, spec.n_rho)
    f_max = float(f[-1])
    shape = (g_all, tp.size, f.size, rho.size)
    pf = np.empty(shape); tb = np.empty(shape); pw = np.empty(shape)
    ml = np.empty(shape[:3])
    horizon = spec.n_window * spec.window_s
    peak_rate = spec.n_req / horizon * _PEAK_OVER_MEAN[spec.rate_shape]
    tpf = tp.astype(np.float64)
    for j in range(spec.n_model):
        u = uniform_stream(stream_key(spec.seed, _S_PROFILE + j), 0, 2 + 3 * cpm)
        a_m = 0.6 + 0.4 * u[0]
        b_m = 0.6 + 0.3 * u[1]
        k_p = (0.05 + 0.15 * u[2:2 + 3 * cpm:3]) * (2.0 ** j)
        k_d = (15.0 + 25.0 * u[3:3 + 3 * cpm:3]) * (2.0 ** j)
        a_c = 0.5 + 0.6 * u[4:4 + 3 * cpm:3] if spec.per_class_exponent else np.full(cpm, a_m)
        l_ref = peak_rate * spec.model_mix[j] * 2000.0 / math.sqrt(cpm)
        cap_unit = np.mean(tpf[-1] * 1000.0 / (k_d / tpf[-1] ** b_m))
        s_j = l_ref / (spec.n_inst_max * 0.6 * cap_unit)
        for c in range(cpm):
            g = j * cpm + c
            slow = (f_max / f)[None, :] ** a_c[c] / (tpf[:, None] ** b_m)       # [tp][f]
            pf[g] = (k_p[c] * slow)[:, :, None] * np.ones_like(rho)[None, None, :]
            tb[g] = np.minimum((k_d[c] * slow)[:, :, None] / (1.0 - rho)[None, None, :], 1000.0)
            pw[g] = tpf[:, None, None] * (100.0 + 600.0 * ((f / f_max) ** 3)[None, :, None]
                                          * rho[None, None, :])
            ml[g] = s_j * tpf[:, None] * 1000.0 / (k_d[c] * slow)
    return {"tp": tp, "f_mhz": f, "rho": rho,
            "prefill_ms_per_tok": np.ascontiguousarray(pf), "tbt_ms": np.ascontiguousarray(tb),
            "power_w": np.ascontiguousarray(pw), "max_load_tps": np.ascontiguousarray(ml)}


def configs(spec: WorkloadSpec) -> Dict[str, np.ndarray]:
    """Candidate (instances, TP, frequency) triples; TP outermost, then frequency,
    instance count fastest.  Candidate frequencies are the profiled ones."""
    n_inst, tp_index, f_mhz = [], [], []
    for ti in range(len(spec.tp)):
        for f in spec.f_mhz:
            for n in range(1, spec.n_inst_max + 1):
                n_inst.append(n); tp_index.append(ti); f_mhz.append(f)
    return {"n_inst": np.asarray(n_inst, np.int32), "tp_index": np.asarray(tp_index, np.int32),
            "f_mhz": np.asarray(f_mhz, np.float64)}


def slos(spec: WorkloadSpec, prof: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    """P99 SLOs in the paper's style (Section III-A: five times the latency of a single
    request on an unloaded system; Table IV: one TTFT SLO per input-length bin, TBT SLO
    100 ms): TTFT SLO of a class = 5 x (largest input of its bin) x unloaded prefill
    ms/token on the fastest configuration (largest TP, highest frequency)."""
    bi, bo = len(spec.in_edges) + 1, len(spec.out_edges) + 1
    upper = list(spec.in_edges) + [8192]
    g_all = spec.n_class
    ttft = np.empty(g_all); tbt = np.full(g_all, 100.0)
    for g in range(g_all):
        ib = (g % (bi * bo)) // bo
        ttft[g] = 5.0 * upper[ib] * prof["prefill_ms_per_tok"][g, -1, -1, 0]
    return {"slo_ttft_ms": ttft, "slo_tbt_ms": tbt}


def class_edges(spec: WorkloadSpec) -> Dict[str, np.ndarray]:
    """Interior bin edges per model, [n_model][bins-1]."""
    return {"in_edge": np.tile(np.asarray(spec.in_edges, np.int32), (spec.n_model, 1)),
            "out_edge": np.tile(np.asarray(spec.out_edges, np.int32), (spec.n_model, 1))}


def make(spec: WorkloadSpec, with_trace: bool = True) -> Dict[str, object]:
    """Everything one evaluation needs, as plain arrays and scalars."""
    prof = profile(spec)
    w = {"spec": spec, "profile": prof, "configs": configs(spec), "slos": slos(spec, prof),
         "edges": class_edges(spec), "pct": (99, 100), "idle_cost_weight": spec.idle_cost_weight,
         "n_window": spec.n_window, "window_s": spec.window_s, "n_class": spec.n_class}
    if with_trace:
        w["trace"] = trace(spec)
    return w


def checksum(a: np.ndarray) -> int:
    """Order-sensitive 64-bit hash of an array's bytes (to prove two runs used the same input)."""
    b = np.frombuffer(np.ascontiguousarray(a).tobytes(), dtype=np.uint8)
    pad = (-b.size) % 8
    if pad:
        b = np.concatenate([b, np.zeros(pad, np.uint8)])
    w = b.view(np.uint64)
    with np.errstate(over="ignore"):
        idx = np.arange(1, w.size + 1, dtype=np.uint64)
        z = w ^ (idx * np.uint64(_GAMMA))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
        z = z ^ (z >> np.uint64(31))
        return int(np.bitwise_xor.reduce(z)) ^ (w.size * _GAMMA & _MASK)
