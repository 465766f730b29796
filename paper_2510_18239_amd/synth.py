"""Seeded synthetic inputs shaped like the paper's latency workloads.

This module only draws random numbers and rounds them to the storage type; it
holds none of the method's arithmetic, so that the tests can hand the very
same bytes to the HIP library and to the CPU oracle.

Recipe (Section 4 latency study, Appendix C hyper-parameters for the shapes):
every tensor is iid Gaussian.  Weights W_Q, W_K, W_V have variance 1/d (W_V times ``value_gain``^2 where a test sizes its outputs).
Embeddings E, T, L have standard deviation ``gain * d**-0.5``: ``gain = 1`` is
the benchmark distribution; a larger gain sharpens the attention logits so that
the softmaxes are far from uniform (used by the parity tests, since at gain 1
every output is O(1e-3) and an absolute tolerance alone would prove little).
Stream for tensor k of workload w: Philox(seed = 20251018 + 1000*w + k).
Ragged lengths are integers uniform on a closed interval.
"""

from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20251018
_TENSOR_INDEX = {"E": 0, "T": 1, "L": 2, "Wq": 3, "Wk": 4, "Wv": 5, "lens": 6, "LCu": 7,
                 "bwdQS": 10, "bwdKS": 11, "bwdVS": 12, "bwddOS": 13, "bwdQT": 14, "bwdKT": 15, "bwdVT": 16, "bwddOT": 17,
                 "bwdlens": 18, "scoring": 30}


def _rng(workload: int, name: str) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(BASE_SEED + 1000 * workload + _TENSOR_INDEX[name]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = np.isnan(x)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    rounded = np.where(nan, np.uint32(0x7FC0), rounded)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Values of x after storage in ``dtype`` ("fp32" or "bf16"), as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp32":
        return x
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    raise ValueError(dtype)


@dataclass
class Workload:
    """One seeded problem instance; every array holds storage-rounded float32 values."""

    B: int
    N: int
    C: int
    d: int
    h: int
    m: int
    dtype: str
    E: np.ndarray  # [B, N, d]
    T: np.ndarray  # [B, C, d]
    L: np.ndarray  # [m, d]
    Wq: np.ndarray  # [d, d]
    Wk: np.ndarray
    Wv: np.ndarray
    lens: np.ndarray | None  # [B] int32 or None (= all N)
    meta: dict = field(default_factory=dict)

    @property
    def softmax_scale(self) -> float:
        return float((self.d // self.h) ** -0.5)


def make_workload(workload: int, B: int, N: int, C: int, d: int, h: int, m: int, dtype: str = "bf16",
                  gain: float = 1.0, len_range: tuple[int, int] | None = None,
                  pad_value: float | None = None, value_gain: float = 1.0) -> Workload:
    """Draw one workload.  ``len_range = (lo, hi)`` draws ragged lengths uniform on
    [lo, hi]; history rows at or beyond a user's length are then overwritten with
    ``pad_value`` (NaN in the mask tests, 0 for timing) when it is given.
    ``value_gain`` multiplies the standard deviation of W_V only: it sizes the outputs
    without touching any logit (the parity tests keep the sharpened outputs below one,
    where the absolute error bar applies as stated)."""
    sd = gain * d ** -0.5

    def normal(name, shape, std):
        return round_to(_rng(workload, name).standard_normal(shape, dtype=np.float32) * np.float32(std), dtype)

    E = normal("E", (B, N, d), sd)
    T = normal("T", (B, C, d), sd)
    L = normal("L", (m, d), sd)
    Wq = normal("Wq", (d, d), d ** -0.5)
    Wk = normal("Wk", (d, d), d ** -0.5)
    Wv = normal("Wv", (d, d), value_gain * d ** -0.5)
    lens = None
    if len_range is not None:
        lo, hi = len_range
        lens = _rng(workload, "lens").integers(lo, hi, size=B, endpoint=True).astype(np.int32)
        if pad_value is not None:
            for b in range(B):
                E[b, lens[b]:] = pad_value
    return Workload(B, N, C, d, h, m, dtype, E, T, L, Wq, Wk, Wv, lens,
                    {"workload": workload, "gain": gain, "len_range": len_range, "value_gain": value_gain})


def per_user_links(workload: int, B: int, m: int, d: int, dtype: str, gain: float = 1.0) -> np.ndarray:
    """Per-user contextualised links L^C [B, m, d] (stand-in for the output of Eq. 2)."""
    x = _rng(workload, "LCu").standard_normal((B, m, d), dtype=np.float32) * np.float32(gain * d ** -0.5)
    return round_to(x, dtype)


def backward_inputs(workload: int, B: int, N: int, m: int, d: int, h: int, dtype: str, logit_std: float = 1.0,
                    len_range=None, pad_value: float = 0.0, value_std: float = 1.0, grad_std: float = 1.0) -> dict:
    """Inputs of the XORA backward pass: projected history rows QS, KS, VS [B, N, d], projected per-user links
    QT, KT, VT [B, m, d] and upstream gradients dOS, dOT of the same shapes, all ~N(0, std^2) and rounded to the
    storage type.  Queries and keys have the standard deviation that gives un-scaled logits <q_head, k_head> a
    standard deviation of ``logit_std`` (the trained layer runs with logits of order one); values and upstream
    gradients have standard deviations ``value_std`` and ``grad_std`` (one for timing; the parity tests size them so
    that the gradients, which are linear in both, stay below one, where the absolute error bar applies as stated).  ``lens`` as in make_workload; rows at or past lens[b] of the history tensors hold ``pad_value``."""
    dh = d // h
    qk_std = float((logit_std / np.sqrt(dh)) ** 0.5)
    t = {}
    for name, rows, std in (("QS", N, qk_std), ("KS", N, qk_std), ("VS", N, value_std), ("dOS", N, grad_std),
                            ("QT", m, qk_std), ("KT", m, qk_std), ("VT", m, value_std), ("dOT", m, grad_std)):
        x = _rng(workload, "bwd" + name).standard_normal((B, rows, d), dtype=np.float32) * np.float32(std)
        t[name] = round_to(x, dtype)
    if len_range is None:
        t["lens"] = None
    else:
        lens = _rng(workload, "bwdlens").integers(len_range[0], len_range[1] + 1, size=B).astype(np.int32)
        t["lens"] = lens
        for b in range(B):
            for name in ("QS", "KS", "VS", "dOS"):
                t[name][b, lens[b]:] = pad_value
    return t


def scoring_params(workload: int, B: int, m: int, d: int, dc: int, dhid: int, widths, dtype: str,
                   value_gain: float = 0.25) -> dict:
    """Parameters of the scoring pipeline around the attention stages, all seeded Gaussians rounded to the storage type:
    user context vectors EC [B, dc] ~ N(0, 1); Eq. 2's MLP ctx = (W1 [d + dc, dhid] ~ N(0, 2/(d + dc)), b1 ~ N(0, 0.1^2),
    W2 [dhid, d] ~ N(0, 1/dhid), b2 ~ N(0, 0.1^2)); five layer normalisations ln_* = (gamma ~ 1 + N(0, 0.2^2),
    beta ~ N(0, 0.2^2)); two weight sets hist, cand = (Wq, Wk, Wv) ~ N(0, 1/d) with W_V times ``value_gain`` (normalised
    rows have unit entries, so the logits of a head have standard deviation about sqrt(d/h) before the scale and the
    outputs stay below one); the interaction network mlp = (weights, biases) with He-scaled weights ~ N(0, 2/d_in),
    biases ~ N(0, 0.1^2), ``widths`` the hidden widths followed by 1."""
    r = _rng(workload, "scoring")

    def normal(shape, std, mean=0.0):
        return round_to(r.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean), dtype)

    p = {"EC": normal((B, dc), 1.0),
         "ctx": (normal((d + dc, dhid), (2.0 / (d + dc)) ** 0.5), normal((dhid,), 0.1), normal((dhid, d), dhid ** -0.5), normal((d,), 0.1))}
    for name in ("ln_hist_q", "ln_hist_kv", "ln_cand_q", "ln_cand_k", "ln_cand_v"):
        p[name] = (normal((d,), 0.2, 1.0), normal((d,), 0.2))
    for name in ("hist", "cand"):
        p[name] = (normal((d, d), d ** -0.5), normal((d, d), d ** -0.5), normal((d, d), value_gain * d ** -0.5))
    dims = [d] + list(widths)
    p["mlp"] = ([normal((dims[i], dims[i + 1]), (2.0 / dims[i]) ** 0.5) for i in range(len(widths))],
                [normal((dims[i + 1],), 0.1) for i in range(len(widths))])
    return p


# W_V gain of the sharpened parity inputs: at logit standard deviation 2 a softmax picks out single rows, so an
# output is about as large as a projected value, gain * value_gain * d^-1/2 * sqrt(d) = 1.4 * value_gain per
# standard deviation with the softmax scale; a quarter keeps the largest output entry below one.
SHARP_VALUE_GAIN = 0.25


def sharp_gain(d: int, h: int, scale: float, logit_std: float = 2.0) -> float:
    """Embedding gain g such that scale * <q_head, k_head> has about ``logit_std``
    standard deviation when both sides are projections of gain-g embeddings."""
    dh = d // h
    # projected entries have variance g^2/d; a head's dot product of dh such pairs
    # has standard deviation sqrt(dh) * g^2 / d.
    return float(np.sqrt(logit_std * d / (scale * np.sqrt(dh))))


# The five workload families the benchmark and the parity tests use.
CONFIGS = {
    1: dict(B=1, N=128, C=64, d=64, h=1, m=16, dtype="fp32"),
    2: dict(B=32, N=1024, C=1024, d=128, h=4, m=64, dtype="bf16", len_range=(512, 1024)),
    3: dict(B=1, N=2048, C=32768, d=256, h=4, m=64, dtype="bf16"),
    4: dict(B=8, N=16384, C=512, d=128, h=4, m=64, dtype="bf16"),
    5: dict(B=16, N=4096, C=8192, d=256, h=4, m=128, dtype="bf16", len_range=(2048, 4096)),
}
