"""Seeded synthetic inputs for the WindowKV window-selection path.

This module only *draws numbers*: it holds none of the method's arithmetic (no softmax,
pooling, selection or gather).  Both the CPU oracle's callers and the GPU path's callers take
their inputs from here, so the two sides see the same bytes.

Every tensor element is a pure function of ``(seed, stream, linear index)``: a 64-bit
counter is scrambled with the splitmix64 finaliser (Steele, Lea & Flood 2014; Vigna's public
domain constants) and its top 16 bits pick one entry of a 65 536-entry table of standard
normal quantiles.  The same function is written twice, once with numpy (host slices for the
oracle) and once with torch integer ops (whole tensors directly in device memory); integer
arithmetic and a table lookup are bit-identical on every device, which the CPU tests check.

The workloads are the five configurations the benchmark description names: LLaMA-3-8B shaped
tensors (32 query / 8 KV heads, head_dim 128, layer groups of 4), the window / observation
sizes the paper lists in its implementation details (Appendix "Implementation Details") and
sweeps in its window-size figure, and a 12 % budget as in its abstract.  They stand in for
the LongBench and Needle-in-a-Haystack inputs the paper evaluates on (Section 3.1), which
are not available here; the planted spans of ``c4`` play the role of a needle passage.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from functools import lru_cache
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_M64 = (1 << 64) - 1
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_GOLD = 0x9E3779B97F4A7C15


# --------------------------------------------------------------------------------------
# counter-based generator
# --------------------------------------------------------------------------------------
def _mix64_int(x: int) -> int:
    x &= _M64
    x ^= x >> 30
    x = (x * _C1) & _M64
    x ^= x >> 27
    x = (x * _C2) & _M64
    x ^= x >> 31
    return x


def stream_base(seed: int, stream: int) -> int:
    """64-bit starting counter of one named stream of one seed."""
    return _mix64_int(_mix64_int(seed * _GOLD + 1) + stream * _GOLD)


def stream_id(*parts: int) -> int:
    """Fold small non-negative integers (tensor kind, layer, ...) into one stream number."""
    s = 0
    for p in parts:
        s = _mix64_int(s * 1000003 + int(p) + 17)
    return s


def _mix64_np(x: np.ndarray) -> np.ndarray:
    x = x.astype(np.uint64, copy=True)
    x ^= x >> np.uint64(30)
    x *= np.uint64(_C1)
    x ^= x >> np.uint64(27)
    x *= np.uint64(_C2)
    x ^= x >> np.uint64(31)
    return x


@lru_cache(maxsize=None)
def normal_table_f32() -> np.ndarray:
    """65 536 standard-normal quantiles at the bin midpoints, as float32."""
    from scipy.special import ndtri

    u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return ndtri(u).astype(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float64."""
    u = b.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


@lru_cache(maxsize=None)
def normal_table_bf16_bits() -> np.ndarray:
    return f32_to_bf16_bits(normal_table_f32())


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to IEEE half (round to nearest even); returns the uint16 bit patterns."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Widen IEEE half bit patterns (uint16) exactly to float64."""
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float64)


@lru_cache(maxsize=None)
def normal_table_f16_bits() -> np.ndarray:
    """The float32 table rounded to IEEE half: 11 significant bits, so products and sums of these
    values exercise half's mantissa (unlike bf16-valued numbers stored as half)."""
    return f32_to_f16_bits(normal_table_f32())


def table_index_np(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """Table indices (0..65535) of elements ``start .. start+count-1`` of a stream."""
    base = stream_base(seed, stream)
    ctr = (np.arange(start, start + count, dtype=np.uint64) + np.uint64(base))
    return (_mix64_np(ctr) >> np.uint64(48)).astype(np.int64)


def normal_np(seed: int, stream: int, start: int, count: int, dtype: str) -> np.ndarray:
    """Host slice of a stream. ``dtype`` 'f32' -> float32 values, 'bf16' / 'f16' -> uint16 bits."""
    idx = table_index_np(seed, stream, start, count)
    if dtype == "f32":
        return normal_table_f32()[idx]
    if dtype == "bf16":
        return normal_table_bf16_bits()[idx]
    if dtype == "f16":
        return normal_table_f16_bits()[idx]
    raise ValueError(dtype)


def _torch_consts():
    import torch

    def s64(v: int) -> int:  # two's complement view of a 64-bit constant
        return v - (1 << 64) if v >= (1 << 63) else v

    return torch, s64


def _mix64_torch(x):
    """splitmix64 finaliser on an int64 tensor (wrapping multiply, logical shifts)."""
    torch, s64 = _torch_consts()
    x = x ^ ((x >> 30) & ((1 << 34) - 1))
    x = x * s64(_C1)
    x = x ^ ((x >> 27) & ((1 << 37) - 1))
    x = x * s64(_C2)
    x = x ^ ((x >> 31) & ((1 << 33) - 1))
    return x


def normal_torch(seed: int, stream: int, numel: int, dtype: str, device, start: int = 0,
                 chunk: int = 1 << 24):
    """Whole stream (or a slice of it) as a flat torch tensor on ``device``.

    Bit-identical to :func:`normal_np` for the same arguments.
    """
    torch, s64 = _torch_consts()
    base = s64(stream_base(seed, stream))
    if dtype == "f32":
        table = torch.from_numpy(normal_table_f32().copy()).to(device)
        out = torch.empty(numel, dtype=torch.float32, device=device)
    elif dtype == "bf16":
        bits = normal_table_bf16_bits().view(np.int16).copy()
        table = torch.from_numpy(bits).to(device).view(torch.bfloat16)
        out = torch.empty(numel, dtype=torch.bfloat16, device=device)
    elif dtype == "f16":
        bits = normal_table_f16_bits().view(np.int16).copy()
        table = torch.from_numpy(bits).to(device).view(torch.float16)
        out = torch.empty(numel, dtype=torch.float16, device=device)
    else:
        raise ValueError(dtype)
    for lo in range(0, numel, chunk):
        n = min(chunk, numel - lo)
        ctr = torch.arange(start + lo, start + lo + n, dtype=torch.int64, device=device) + base
        idx = (_mix64_torch(ctr) >> 48) & 0xFFFF
        out[lo:lo + n] = table[idx]
    return out


def uniform_ints(seed: int, stream: int, count: int, lo: int, hi: int) -> List[int]:
    """``count`` integers in ``[lo, hi]`` (inclusive) from a stream (modulo reduction)."""
    base = stream_base(seed, stream)
    return [lo + _mix64_int(base + i) % (hi - lo + 1) for i in range(count)]


# --------------------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------------------
KIND_Q, KIND_K, KIND_V, KIND_META, KIND_SPAN = 1, 2, 3, 4, 5


@dataclass
class Workload:
    """One synthetic workload: shapes, per-sequence parameters, and how to draw tensors.

    Tensor layouts (all contiguous): ``q_obs [B, Hq, w_obs, d]`` per layer group (the last
    ``w_obs`` query vectors of the group's first layer), ``K, V [B, Hkv, Lmax, d]`` per
    layer.  Sequence ``b`` occupies token rows ``0 .. seq_len[b]-1``; rows beyond are
    filler noise that no result may depend on.
    """

    name: str
    seed: int
    dtype: str                      # 'f32' | 'bf16' | 'f16'
    n_groups: int
    gamma: int                      # layers per group
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    w_obs: int
    seq_len: List[int]
    win: List[int]
    top_p: List[int]
    k_windows: List[int]
    outlier_channels: int = 0       # per (layer, kv head): channels scaled by 8
    planted_spans: int = 0          # aligned-key spans of 64 tokens in scoring layers
    span_len: int = 64
    span_cos: float = 0.9
    _cache: Dict = field(default_factory=dict, repr=False)

    # ---- shapes -------------------------------------------------------------------
    @property
    def batch(self) -> int:
        return len(self.seq_len)

    @property
    def max_seq_len(self) -> int:
        return max(self.seq_len)

    @property
    def n_layers(self) -> int:
        return self.n_groups * self.gamma

    @property
    def q_per_kv(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def n_windows(self, b: int) -> int:
        return -(-(self.seq_len[b] - self.w_obs) // self.win[b])

    @property
    def nkeep_max(self) -> int:
        return max(k * w for k, w in zip(self.k_windows, self.win)) + self.w_obs

    @property
    def total_tokens(self) -> int:
        return sum(self.seq_len)

    def kv_shape(self) -> Tuple[int, int, int, int]:
        return (self.batch, self.n_kv_heads, self.max_seq_len, self.head_dim)

    def q_shape(self) -> Tuple[int, int, int, int]:
        return (self.batch, self.n_q_heads, self.w_obs, self.head_dim)

    # ---- per (layer, head) structure ------------------------------------------------
    def outlier_channel_ids(self, layer: int, kind: int, h: int) -> List[int]:
        """Channels of KV head ``h`` of ``layer`` (kind K or V) that are scaled by 8."""
        if not self.outlier_channels:
            return []
        st = stream_id(KIND_META, layer, kind, h)
        base = stream_base(self.seed, st)
        picked: List[int] = []
        i = 0
        while len(picked) < self.outlier_channels:
            c = _mix64_int(base + i) % self.head_dim
            if c not in picked:
                picked.append(c)
            i += 1
        return sorted(picked)

    def span_starts(self) -> List[List[int]]:
        """Per sequence: start tokens of the planted spans (multiples of span_len,
        distinct, inside the review context; the same in every layer group)."""
        if "spans" in self._cache:
            return self._cache["spans"]
        out = []
        for b in range(self.batch):
            n_slots = (self.seq_len[b] - self.w_obs) // self.span_len
            base = stream_base(self.seed, stream_id(KIND_SPAN, b))
            picked: List[int] = []
            i = 0
            while len(picked) < self.planted_spans:
                s = _mix64_int(base + i) % n_slots
                if s not in picked:
                    picked.append(s)
                i += 1
            out.append(sorted(s * self.span_len for s in picked))
        self._cache["spans"] = out
        return out

    # ---- host slices (what the oracle is fed) -----------------------------------------
    def _raw_np(self, kind: int, which: int, start: int, count: int) -> np.ndarray:
        return normal_np(self.seed, stream_id(kind, which), start, count, self.dtype)

    def q_obs_np(self, group: int) -> np.ndarray:
        """``[B, Hq, w_obs, d]`` of one group; float32 values or bf16 bit patterns."""
        n = int(np.prod(self.q_shape()))
        return self._raw_np(KIND_Q, group, 0, n).reshape(self.q_shape())

    def kv_np(self, kind: int, layer: int, b: int, h: int, rows: Optional[np.ndarray] = None
              ) -> np.ndarray:
        """Rows of K (kind=KIND_K) or V of ``layer`` for sequence ``b``, KV head ``h``:
        ``[n_rows, d]``.  ``rows`` defaults to all ``seq_len[b]`` rows."""
        B, H, Lm, d = self.kv_shape()
        if rows is None:
            start = ((b * H + h) * Lm) * d
            x = self._raw_np(kind, layer, start, self.seq_len[b] * d).reshape(-1, d)
            rows_arr = np.arange(self.seq_len[b])
        else:
            rows_arr = np.asarray(rows, dtype=np.int64)
            x = np.empty((len(rows_arr), d), dtype=np.float32 if self.dtype == "f32" else np.uint16)
            for i, r in enumerate(rows_arr):
                start = ((b * H + h) * Lm + int(r)) * d
                x[i] = self._raw_np(kind, layer, start, d)
        x = self._apply_outliers_np(x, layer, kind, h)
        if kind == KIND_K and self.planted_spans and layer % self.gamma == 0:
            x = self._apply_spans_np(x, layer // self.gamma, b, h, rows_arr)
        return x

    def _apply_outliers_np(self, x: np.ndarray, layer: int, kind: int, h: int) -> np.ndarray:
        ch = self.outlier_channel_ids(layer, kind, h)
        if not ch:
            return x
        x = x.copy()
        if self.dtype == "f32":
            x[:, ch] *= np.float32(8.0)
        elif self.dtype == "bf16":  # widening, scaling by a power of two and narrowing again are all exact
            v = bf16_bits_to_f64(x[:, ch]) * 8.0
            x[:, ch] = f32_to_bf16_bits(v.astype(np.float32))
        else:                       # half: |value| * 8 < 64, far inside its range, so exact as well
            v = f16_bits_to_f64(x[:, ch]) * 8.0
            x[:, ch] = f32_to_f16_bits(v.astype(np.float32))
        return x

    def span_rows_np(self, group: int, b: int, h: int) -> np.ndarray:
        """The planted key rows of scoring layer ``group*gamma`` for (b, h):
        ``[planted_spans*span_len, d]`` in the workload dtype, in span order.

        Each row is ``|k| * (c*qhat + sqrt(1-c^2)*uhat)`` with ``qhat`` the unit mean of the
        head's ``G*w_obs`` observation queries, ``uhat`` a unit vector orthogonal to it drawn
        from the seed, ``|k| = sqrt(d)`` and ``c = span_cos``.  This is input construction,
        not part of the method.
        """
        key = ("spanrows", group, b, h)
        if key in self._cache:
            return self._cache[key]
        d, G = self.head_dim, self.q_per_kv
        q = self.q_obs_np(group)[b, h * G:(h + 1) * G]
        qf = self.to_f64(q)
        qhat = qf.reshape(-1, d).mean(0)
        qhat /= np.linalg.norm(qhat)
        n = self.planted_spans * self.span_len
        st = stream_id(KIND_SPAN, 100 + group, b, h)
        u = normal_np(self.seed, st, 0, n * d, "f32").astype(np.float64).reshape(n, d)
        u -= np.outer(u @ qhat, qhat)
        u /= np.linalg.norm(u, axis=1, keepdims=True)
        c = self.span_cos
        rows = math.sqrt(d) * (c * qhat[None, :] + math.sqrt(1.0 - c * c) * u)
        rows = rows.astype(np.float32)
        out = rows if self.dtype == "f32" else (f32_to_bf16_bits(rows) if self.dtype == "bf16" else f32_to_f16_bits(rows))
        self._cache[key] = out
        return out

    def _apply_spans_np(self, x, group, b, h, rows_arr):
        starts = self.span_starts()[b]
        planted = self.span_rows_np(group, b, h)
        x = x.copy()
        for si, s0 in enumerate(starts):
            m = (rows_arr >= s0) & (rows_arr < s0 + self.span_len)
            if m.any():
                x[m] = planted[si * self.span_len + (rows_arr[m] - s0)]
        return x

    # ---- device tensors (what the GPU path is fed) -------------------------------------
    def _torch_dtype(self):
        import torch
        return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[self.dtype]

    def _np_to_torch(self, x: np.ndarray, device):
        import torch
        if self.dtype == "f32":
            return torch.from_numpy(np.ascontiguousarray(x)).to(device)
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).to(device).view(self._torch_dtype())

    def q_obs_torch(self, group: int, device):
        n = int(np.prod(self.q_shape()))
        t = normal_torch(self.seed, stream_id(KIND_Q, group), n, self.dtype, device)
        return t.view(self.q_shape())

    def kv_torch(self, kind: int, layer: int, device):
        """Whole ``[B, Hkv, Lmax, d]`` tensor of one layer, generated in device memory."""
        n = int(np.prod(self.kv_shape()))
        t = normal_torch(self.seed, stream_id(kind, layer), n, self.dtype, device).view(self.kv_shape())
        if self.outlier_channels:
            for h in range(self.n_kv_heads):
                ch = self.outlier_channel_ids(layer, kind, h)
                t[:, h, :, ch] = t[:, h, :, ch] * 8.0   # exact: power of two
        if kind == KIND_K and self.planted_spans and layer % self.gamma == 0:
            g = layer // self.gamma
            for b in range(self.batch):
                for h in range(self.n_kv_heads):
                    planted = self._np_to_torch(self.span_rows_np(g, b, h), device)
                    for si, s0 in enumerate(self.span_starts()[b]):
                        t[b, h, s0:s0 + self.span_len] = planted[si * self.span_len:(si + 1) * self.span_len]
        return t

    # ---- conversions ---------------------------------------------------------------------
    def to_f64(self, x: np.ndarray) -> np.ndarray:
        """Widen a host slice in the workload dtype exactly to float64."""
        if self.dtype == "bf16":
            return bf16_bits_to_f64(x)
        return f16_bits_to_f64(x) if self.dtype == "f16" else x.astype(np.float64)


def _llama(name, seed, seq_len, win, top_p, k, n_groups, **kw) -> Workload:
    return Workload(name=name, seed=seed, dtype="bf16", n_groups=n_groups, gamma=4,
                    n_q_heads=32, n_kv_heads=8, head_dim=128, w_obs=32,
                    seq_len=list(seq_len), win=list(win), top_p=list(top_p),
                    k_windows=list(k), **kw)


def make_workload(name: str) -> Workload:
    """The named configurations.  Budgets count review tokens; the observation window is kept
    on top of them.  ``top_p`` is the window size in localisation mode (window mean) and half
    of it in aggregation mode (the paper gives no value for p)."""
    if name == "c1":      # tiny fp32 case
        return Workload(name="c1", seed=1001, dtype="f32", n_groups=1, gamma=2, n_q_heads=4,
                        n_kv_heads=2, head_dim=64, w_obs=8, seq_len=[512], win=[8], top_p=[8],
                        k_windows=[8])
    if name == "c2":      # one LLaMA-3-8B shaped group, outlier channels
        return _llama("c2", 1002, [4096], [8], [8], [64], 1, outlier_channels=4)
    if name == "c3a":     # long prefix, localisation mode
        return _llama("c3a", 1003, [16384], [8], [8], [256], 1)
    if name == "c3b":     # same tensors, aggregation mode
        return _llama("c3b", 1003, [16384], [32], [16], [64], 1)
    if name == "c4":      # full-model prefill compression with planted spans
        return _llama("c4", 1004, [32768], [16], [8], [256], 8, planted_spans=3)
    if name == "c5":      # batched mixed lengths and task modes
        lens = uniform_ints(1005, stream_id(KIND_META, 1), 8, 4096, 32768)
        modes = uniform_ints(1005, stream_id(KIND_META, 2), 8, 0, 1)
        win = [8 if m == 0 else 32 for m in modes]
        top_p = [8 if m == 0 else 16 for m in modes]
        k = [int(0.12 * L) // w for L, w in zip(lens, win)]
        return _llama("c5", 1005, lens, win, top_p, k, 8)
    raise KeyError(name)


def scaled_workload(base: Workload, **overrides) -> Workload:
    """A copy of a workload with some fields replaced (smaller test shapes)."""
    d = {f: getattr(base, f) for f in base.__dataclass_fields__ if f != "_cache"}
    d.update(overrides)
    return Workload(**d)


WORKLOAD_NAMES = ("c1", "c2", "c3a", "c3b", "c4", "c5")
