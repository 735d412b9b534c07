"""Seeded synthetic inputs for the VFA / VSA attention forward path.

This module is the only thing the GPU path's callers and the CPU checker have in
common: it produces Q, K, V as bf16 bit patterns (numpy uint16) from a seed, so that
both sides read the same numbers.  It holds none of the method's arithmetic (no
softmax, no block summaries, no visit order); it only shapes the *scores* Q K^T so
that they look like what the paper's data analysis describes: a few "sink" keys at
the start that almost every query scores highly, a diagonal "local" band, a mild
heavy tail with distance, and (for the m-initialisation stress case) a planted
maximum in a random middle block.

Recipe "sinklocal" (per KV head, softmax scale 1/sqrt(d)):
  a           unit vector, zero in the 2F positional dimensions
  Q[r]        g_r + beta * a,               g_r ~ N(0, I)
  K[c]        h_c ~ N(0, I);  K[0] = kappa * sqrt(d) * a
              => background logits ~ N(0, ~1), sink logit ~ kappa * (beta + N(0,1))
  positional  the last 2F dimensions of Q[p] and K[p] are gamma*[cos(w_f p), sin(w_f p)],
              w_f = (pi / W) * theta**(-f / F), gamma**2 = bump / (scale * F)
              => logit bump(delta) = (bump / F) * sum_f cos(w_f * delta): +bump nats at
              distance 0, main lobe about W wide, slow decay beyond
  V           N(0, I)

All random numbers come from numpy's counter-based Philox generator keyed by
(seed, tensor id), so each tensor is reproducible on its own.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

DEFAULT_SEED = 20260412


# ----------------------------------------------------------------------------- bf16 <-> fp32
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r[nan] = 0x7FC0
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32, exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- workload description
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    N: int
    d: int
    block_m: int
    block_n: int
    causal: bool
    n_sink: int = 1
    n_local: int = 1
    skip_threshold_nats: float = 8.0
    # generator constants
    kind: str = "sinklocal"  # "sinklocal" | "planted" | "sink_meanq"
    beta: float = 2.0
    kappa: float = 4.0
    F: int = 8
    W: float = 256.0
    theta: float = 64.0
    bump: float = 4.0
    planted_boost: float = 6.0

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def Tr(self) -> int:
        return -(-self.N // self.block_m)

    @property
    def Tc(self) -> int:
        return -(-self.N // self.block_n)

    def dense_flop(self) -> float:
        """FlashAttention convention: 4*B*Hq*N^2*d, halved when causal."""
        f = 4.0 * self.B * self.Hq * float(self.N) ** 2 * self.d
        return f / 2 if self.causal else f


CONFIGS = {
    # tiny causal prefill (parity + every oracle self-check)
    "cfg1": Workload("cfg1", 1, 1, 1, 512, 64, 64, 64, True, kind="sink_meanq", beta=1.0, F=0),
    # causal prefill bf16
    "cfg2": Workload("cfg2", 1, 32, 32, 4096, 128, 128, 64, True),
    # GQA causal prefill bf16 (headline)
    "cfg3": Workload("cfg3", 2, 32, 8, 16384, 128, 128, 64, True),
    # non-causal m-init stress: planted maximum in a random middle block
    "cfg4": Workload("cfg4", 1, 16, 16, 32768, 128, 128, 64, False, kind="planted", F=0),
    # block-sparse causal: stronger sink and a wide positional spectrum whose logit bonus decays roughly
    # with the log of the distance, so that the 8-nat skip test removes a graded share of far tiles
    "cfg5": Workload("cfg5", 1, 8, 8, 65536, 128, 128, 64, True, beta=6.0, kappa=3.0, F=16, theta=4096.0, bump=12.0),
}


def small(w: Workload, **kw) -> Workload:
    """A reduced copy of a workload (same generator constants, other sizes)."""
    return dataclasses.replace(w, **kw)


# ----------------------------------------------------------------------------- generators
def _rng(seed: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed) & 0xFFFFFFFFFFFFFFFF, tensor_id]))


def _normal(seed: int, tensor_id: int, shape) -> np.ndarray:
    return _rng(seed, tensor_id).standard_normal(shape, dtype=np.float32)


def _positional(w: Workload) -> np.ndarray | None:
    """[N, 2F] float32 block gamma*[cos, sin](w_f * p), or None when F == 0."""
    if w.F <= 0:
        return None
    f = np.arange(w.F, dtype=np.float64)
    omega = (math.pi / w.W) * w.theta ** (-f / w.F)
    gamma = math.sqrt(w.bump / (w.scale * w.F))
    p = np.arange(w.N, dtype=np.float64)[:, None]
    ang = p * omega[None, :]
    return (gamma * np.concatenate([np.cos(ang), np.sin(ang)], axis=1)).astype(np.float32)


def generate(w: Workload, seed: int = DEFAULT_SEED) -> dict:
    """Return {"Q","K","V"}: uint16 bf16 bit patterns, shapes [B,Hq,N,d] / [B,Hkv,N,d]."""
    B, Hq, Hkv, N, d = w.B, w.Hq, w.Hkv, w.N, w.d
    g = Hq // Hkv
    Q = _normal(seed, 1, (B, Hq, N, d))
    K = _normal(seed, 2, (B, Hkv, N, d))
    V = _normal(seed, 3, (B, Hkv, N, d))
    nd = d - 2 * max(w.F, 0)

    if w.kind in ("sinklocal", "sink_meanq"):
        a = _normal(seed, 4, (B, Hkv, d)).astype(np.float64)
        a[..., nd:] = 0.0
        a /= np.linalg.norm(a, axis=-1, keepdims=True)
        a32 = a.astype(np.float32)
        for h in range(Hq):
            Q[:, h] += np.float32(w.beta) * a32[:, h // g][:, None, :]
        if w.kind == "sinklocal":
            K[:, :, 0, :] = np.float32(w.kappa * math.sqrt(d)) * a32
        else:
            # key 0 scaled x kappa along the mean query direction (one KV head per query head here)
            qbar = Q.reshape(B, Hkv, g * N, d).mean(axis=2, dtype=np.float64)
            u = qbar / np.linalg.norm(qbar, axis=-1, keepdims=True)
            k0n = np.linalg.norm(K[:, :, 0, :].astype(np.float64), axis=-1, keepdims=True)
            K[:, :, 0, :] = (w.kappa * k0n * u).astype(np.float32)
        pos = _positional(w)
        if pos is not None:
            Q[..., nd:] = pos[None, None]
            K[..., nd:] = pos[None, None]
    elif w.kind == "planted":
        # per query row one target key, drawn uniformly from key blocks that are neither the
        # first n_sink blocks nor overlap the row's own query block; Q[r] += boost*sqrt(d)*K[t]/|K[t]|^2
        rng = _rng(seed, 5)
        Tc = w.Tc
        for b in range(B):
            for h in range(Hq):
                rows = np.arange(N)
                i = rows // w.block_m
                a_lo = (i * w.block_m) // w.block_n
                a_hi = (np.minimum((i + 1) * w.block_m, N) - 1) // w.block_n
                n_excl = w.n_sink + (a_hi - a_lo + 1)
                pick = rng.integers(0, np.maximum(Tc - n_excl, 1), size=N)
                blk = pick + w.n_sink                      # skip the sink blocks
                blk = np.where(blk >= a_lo, blk + (a_hi - a_lo + 1), blk)  # skip the aligned span
                blk = np.minimum(blk, Tc - 1)
                t = np.minimum(blk * w.block_n + rng.integers(0, w.block_n, size=N), N - 1)
                kt = K[b, h // g, t, :].astype(np.float64)
                Q[b, h] += (w.planted_boost * math.sqrt(d) * kt / (kt * kt).sum(-1, keepdims=True)).astype(np.float32)
    else:
        raise ValueError(w.kind)
    return {"Q": f32_to_bf16_bits(Q), "K": f32_to_bf16_bits(K), "V": f32_to_bf16_bits(V)}


def generate_decode(w: Workload, n_keys: int, seed: int = DEFAULT_SEED) -> dict:
    """Decode-step inputs in the "sinklocal" recipe: {"q" [B,Hq,d], "K","V" [B,Hkv,N,d]} as bf16 bits.
    K and V are the cache (w.N = its capacity; rows >= n_keys are filled too but are never to be read),
    q is the query of the token at position n_keys - 1 (same sink direction, same positional dims)."""
    assert w.kind == "sinklocal" and 1 <= n_keys <= w.N
    B, Hq, Hkv, N, d = w.B, w.Hq, w.Hkv, w.N, w.d
    g = Hq // Hkv
    q = _normal(seed, 6, (B, Hq, d))
    K = _normal(seed, 2, (B, Hkv, N, d))
    V = _normal(seed, 3, (B, Hkv, N, d))
    nd = d - 2 * max(w.F, 0)
    a = _normal(seed, 4, (B, Hkv, d)).astype(np.float64)
    a[..., nd:] = 0.0
    a /= np.linalg.norm(a, axis=-1, keepdims=True)
    a32 = a.astype(np.float32)
    for h in range(Hq):
        q[:, h] += np.float32(w.beta) * a32[:, h // g]
    K[:, :, 0, :] = np.float32(w.kappa * math.sqrt(d)) * a32
    pos = _positional(w)
    if pos is not None:
        q[..., nd:] = pos[n_keys - 1][None, None]
        K[..., nd:] = pos[None, None]
    return {"q": f32_to_bf16_bits(q), "K": f32_to_bf16_bits(K), "V": f32_to_bf16_bits(V)}


# decode step timed by bench.py beside the prefill headline: 32 query heads over 8 KV heads, 32K cached keys
DECODE = Workload("decode32k", 4, 32, 8, 32768, 128, 128, 64, True)
DECODE_SPLITS = 16


def sample_blocks(w: Workload, n_random: int, seed: int = DEFAULT_SEED) -> np.ndarray:
    """Query blocks (b, h, i) used where a full-size CPU check is too slow: for the first
    and last (b, h) the first, last and quarter-point blocks, plus n_random drawn uniformly."""
    Tr = w.Tr
    fixed = sorted({0, Tr // 4, Tr // 2, (3 * Tr) // 4, Tr - 1})
    out = [(b, h, i) for (b, h) in {(0, 0), (w.B - 1, w.Hq - 1)} for i in fixed]
    rng = _rng(seed, 99)
    for _ in range(n_random):
        out.append((int(rng.integers(w.B)), int(rng.integers(w.Hq)), int(rng.integers(Tr))))
    return np.array(sorted(set(out)), dtype=np.int32)


def all_blocks(w: Workload) -> np.ndarray:
    return np.array([(b, h, i) for b in range(w.B) for h in range(w.Hq) for i in range(w.Tr)], dtype=np.int32)
