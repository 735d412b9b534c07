"""ctypes loader for the float64 CPU checker in vfa_oracle.c.

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the benchmark's cpu_baseline
leg may import this; the GPU library and its Python binding never do.  Nothing here
imports the GPU package.  The wrappers below only marshal numpy arrays; every step of
the arithmetic is in the C file, which cites the passages it follows.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vfa_oracle.c")
_LIB = os.path.join(_HERE, "libvfa_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile vfa_oracle.c with gcc (plain C, -O2, OpenMP over query blocks)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def brute(Q, K, V, causal: bool, scale: float | None = None):
    """One head, whole N x N matrix. Q,K,V [N,d]. Returns (P [N,N], O [N,d], LSE [N])."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    N, d = Q.shape
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    P = np.empty((N, N)); O = np.empty((N, d)); L = np.empty(N)
    rc = _load().oracle_brute(_p(Q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float),
                              N, d, int(causal), ctypes.c_double(scale),
                              _p(P, ctypes.c_double), _p(O, ctypes.c_double), _p(L, ctypes.c_double))
    assert rc == 0
    return P, O, L


def _dims(Q, K):
    B, Hq, N, d = Q.shape
    Hkv = K.shape[1]
    assert K.shape == (B, Hkv, N, d) and Hq % Hkv == 0
    return B, Hq, Hkv, N, d


def exact(Q, K, V, block_m: int, causal: bool, blocks, scale: float | None = None):
    """Exact attention rows of the listed query blocks. Returns (O, LSE, M)."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    B, Hq, Hkv, N, d = _dims(Q, K)
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    blocks = np.ascontiguousarray(blocks, dtype=np.int32)
    n = len(blocks)
    O = np.full((n, block_m, d), np.nan); L = np.full((n, block_m), np.nan); M = np.full((n, block_m), np.nan)
    rc = _load().oracle_exact(_p(Q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float),
                              B, Hq, Hkv, N, d, block_m, int(causal), ctypes.c_double(scale), n,
                              _p(blocks, ctypes.c_int), _p(O, ctypes.c_double), _p(L, ctypes.c_double),
                              _p(M, ctypes.c_double))
    assert rc == 0
    return O, L, M


def sabsmax(K, block_n: int, repr_mode: int = 0):
    """Key-block summaries [B,Hkv,Tc,d] (float64). repr_mode 0 is the method's sabsmax."""
    K = _f32(K)
    B, Hkv, N, d = K.shape
    Tc = -(-N // block_n)
    out = np.empty((B, Hkv, Tc, d))
    rc = _load().oracle_sabsmax(_p(K, ctypes.c_float), B, Hkv, N, d, block_n, repr_mode, _p(out, ctypes.c_double))
    assert rc == 0
    return out


def visit_list(N, block_m, block_n, causal, i, n_sink, n_local, reorder=True):
    Tc = -(-N // block_n)
    j = np.zeros(Tc, dtype=np.int32); s = np.zeros(Tc, dtype=np.int32)
    n = _load().oracle_visit_list(N, block_m, block_n, int(causal), i, n_sink, n_local, int(reorder),
                                  _p(j, ctypes.c_int), _p(s, ctypes.c_int))
    return j[:n].copy(), s[:n].copy()


def blocks(Q, K, V, block_m, block_n, causal, blocks, *, n_sink=1, n_local=1, use_minit=True,
           reorder=True, freeze=True, vsa=False, skip_threshold_nats=None, scale=None,
           krepr=None, qrepr=None, m_override=None, want_traj=False):
    """Alg. 1 (default), Alg. 2 (vsa=True) or online softmax on every block
    (use_minit=False, reorder=False, freeze=False) for the listed query blocks.
    qrepr [B,Hq,Tr,d] (e.g. sabsmax(Q, block_m, mode)) switches the m-initialisation to the block-wise
    score of the ablation study: one summary vector per query block, one seed for all its rows.
    Returns a dict: O, LSE, m_init, m_final, mask, margin, counters[, traj]."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    B, Hq, Hkv, N, d = _dims(Q, K)
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    Tc = -(-N // block_n)
    blk = np.ascontiguousarray(blocks, dtype=np.int32)
    n = len(blk)
    if use_minit and krepr is None:
        krepr = sabsmax(K, block_n)
    if krepr is not None:
        krepr = np.ascontiguousarray(krepr, dtype=np.float64)
    if qrepr is not None:
        qrepr = np.ascontiguousarray(qrepr, dtype=np.float64)
        assert qrepr.shape == (B, Hq, -(-N // block_m), d)
    if m_override is not None:
        m_override = np.ascontiguousarray(m_override, dtype=np.float64)
        assert m_override.shape == (n, block_m)
    ln_lambda = -float(skip_threshold_nats) if vsa else 0.0
    if vsa:
        assert skip_threshold_nats is not None and skip_threshold_nats > 0
    O = np.full((n, block_m, d), np.nan); L = np.full((n, block_m), np.nan)
    mi = np.full((n, block_m), np.nan); mf = np.full((n, block_m), np.nan)
    mask = np.zeros((n, Tc), dtype=np.uint8); margin = np.empty((n, Tc))
    cnt = np.zeros((n, 4), dtype=np.int64)
    traj = np.full((n, Tc, block_m, 2), np.nan) if want_traj else None
    rc = _load().oracle_blocks_qrepr(
        _p(Q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float), B, Hq, Hkv, N, d,
        block_m, block_n, int(causal), ctypes.c_double(scale), _p(krepr, ctypes.c_double),
        _p(qrepr, ctypes.c_double), n_sink, n_local, int(use_minit), int(reorder), int(freeze), int(vsa), ctypes.c_double(ln_lambda),
        n, _p(blk, ctypes.c_int), _p(m_override, ctypes.c_double), _p(O, ctypes.c_double), _p(L, ctypes.c_double),
        _p(mi, ctypes.c_double), _p(mf, ctypes.c_double), _p(mask, ctypes.c_uint8), _p(margin, ctypes.c_double),
        _p(cnt, ctypes.c_int64), _p(traj, ctypes.c_double))
    assert rc == 0
    out = dict(O=O, LSE=L, m_init=mi, m_final=mf, mask=mask, margin=margin, counters=cnt)
    if want_traj:
        out["traj"] = traj
    return out


def fa_lazy(Q, K, V, block_m, block_n, causal, blocks_, tau, scale=None):
    """Online softmax whose rows keep their old max while it grows by at most tau*ln2 (the
    rescale-skip stage of the Blasst_FA4 variant).  Returns dict O, LSE, counters
    (tiles visited, rowmax executions, tiles whose rescale ran, 0)."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    B, Hq, Hkv, N, d = _dims(Q, K)
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    blk = np.ascontiguousarray(blocks_, dtype=np.int32)
    n = len(blk)
    O = np.full((n, block_m, d), np.nan); L = np.full((n, block_m), np.nan)
    cnt = np.zeros((n, 4), dtype=np.int64)
    rc = _load().oracle_fa_lazy(
        _p(Q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float), B, Hq, Hkv, N, d,
        block_m, block_n, int(causal), ctypes.c_double(scale), ctypes.c_double(float(tau)), n,
        _p(blk, ctypes.c_int), _p(O, ctypes.c_double), _p(L, ctypes.c_double), _p(cnt, ctypes.c_int64))
    assert rc == 0
    return dict(O=O, LSE=L, counters=cnt)


def blasst_variant(Q, K, V, block_m, block_n, causal, blocks_, skip_threshold_nats, *, rowskip=False, lazy_tau=None,
                   scale=None):
    """Blasst_Rowskip (rowskip=True) or Blasst_FA4 (lazy_tau >= 0) of the appendix; with neither, vanilla BLASST.
    Returns dict O, LSE, mask, margin, counters."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    B, Hq, Hkv, N, d = _dims(Q, K)
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    Tc = -(-N // block_n)
    blk = np.ascontiguousarray(blocks_, dtype=np.int32)
    n = len(blk)
    O = np.full((n, block_m, d), np.nan); L = np.full((n, block_m), np.nan)
    mask = np.zeros((n, Tc), dtype=np.uint8); margin = np.empty((n, Tc)); cnt = np.zeros((n, 4), dtype=np.int64)
    rc = _load().oracle_blasst_variant(
        _p(Q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float), B, Hq, Hkv, N, d, block_m, block_n,
        int(causal), ctypes.c_double(scale), ctypes.c_double(-float(skip_threshold_nats)), int(bool(rowskip)),
        ctypes.c_double(-1.0 if lazy_tau is None else float(lazy_tau)), n, _p(blk, ctypes.c_int), _p(O, ctypes.c_double),
        _p(L, ctypes.c_double), _p(mask, ctypes.c_uint8), _p(margin, ctypes.c_double), _p(cnt, ctypes.c_int64))
    assert rc == 0
    return dict(O=O, LSE=L, mask=mask, margin=margin, counters=cnt)


def e4m3_quantize(x, inv_scale: float):
    """OCP E4M3 codes (uint8) of float32 x * inv_scale: round to nearest even, saturating at +-448."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.empty(x.shape, dtype=np.uint8)
    rc = _load().oracle_e4m3_quantize(_p(x, ctypes.c_float), ctypes.c_longlong(x.size), ctypes.c_float(inv_scale),
                                      _p(codes, ctypes.c_uint8))
    assert rc == 0
    return codes


def e4m3_dequantize(codes, scale: float = 1.0):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, dtype=np.float64)
    rc = _load().oracle_e4m3_dequantize(_p(codes, ctypes.c_uint8), ctypes.c_longlong(codes.size), ctypes.c_double(scale),
                                        _p(out, ctypes.c_double))
    assert rc == 0
    return out


def mx_quantize(x, fmt: int = 0, pre_scale: float = 1.0):
    """MX block quantisation along the last axis (32 elements per E8M0 scale): fmt 0 = E2M1 nibbles
    (MXFP4, codes [..., d/2]), fmt 1 = E5M2 bytes (codes [..., d]); returns (codes, scales [..., d/32])."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    d = x.shape[-1]
    rows = x.size // d
    codes = np.zeros(x.shape[:-1] + ((d // 2) if fmt == 0 else d,), dtype=np.uint8)
    scales = np.zeros(x.shape[:-1] + (d // 32,), dtype=np.uint8)
    rc = _load().oracle_mx_quantize(_p(x, ctypes.c_float), ctypes.c_longlong(rows), d, ctypes.c_float(pre_scale), fmt,
                                    _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8))
    assert rc == 0
    return codes, scales


def mx_dequantize(codes, scales, fmt: int = 0):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    d = scales.shape[-1] * 32
    out = np.empty(scales.shape[:-1] + (d,), dtype=np.float64)
    rc = _load().oracle_mx_dequantize(_p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint8),
                                      ctypes.c_longlong(out.size // d), d, fmt, _p(out, ctypes.c_double))
    assert rc == 0
    return out


def decode(q, K, V, n_keys, block_n, *, n_sink=1, n_local=1, use_minit=True, n_parts=1, scale=None):
    """One query token per head against the first n_keys rows of a K/V cache [B,Hkv,n_cap,d].
    Returns dict O [B,Hq,d], LSE, m_init, m_final [B,Hq], l_parts [B,Hq,n_parts]."""
    q = np.ascontiguousarray(q, dtype=np.float32)
    K, V = _f32(K), _f32(V)
    B, Hq, d = q.shape
    Hkv, n_cap = K.shape[1], K.shape[2]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    krepr = np.ascontiguousarray(sabsmax(K[:, :, :n_keys], block_n), dtype=np.float64) if use_minit else None
    O = np.full((B, Hq, d), np.nan); L = np.full((B, Hq), np.nan)
    mi = np.full((B, Hq), np.nan); mf = np.full((B, Hq), np.nan); lp = np.full((B, Hq, n_parts), np.nan)
    rc = _load().oracle_decode(
        _p(q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float), B, Hq, Hkv, n_cap, int(n_keys), d,
        block_n, ctypes.c_double(scale), n_sink, n_local, _p(krepr, ctypes.c_double), n_parts, _p(O, ctypes.c_double),
        _p(L, ctypes.c_double), _p(mi, ctypes.c_double), _p(mf, ctypes.c_double), _p(lp, ctypes.c_double))
    assert rc == 0
    return dict(O=O, LSE=L, m_init=mi, m_final=mf, l_parts=lp)


def fa2(Q, K, V, block_m, block_n, causal, blocks_, scale=None, want_traj=False):
    """FA column of Table 1: ascending order, exact-max update on every block."""
    return blocks(Q, K, V, block_m, block_n, causal, blocks_, n_sink=0, n_local=0, use_minit=False,
                  reorder=False, freeze=False, scale=scale, want_traj=want_traj)


def stabilisation_index(Q, K, V, block_m, block_n, causal, blocks_, scale=None):
    """Where the running maximum stabilises (attention-statistics section, the stabilisation-position equation): for
    every row of the listed query blocks, the first key block j of the default ascending scan at which the
    online-softmax running maximum m^(j) equals its final value m^(T_c).  Taken from the trajectory of the FA column
    of Table 1 (fa2), block by block, as the equation reads.  Returns int64 [n, block_m]; -1 for rows past the end of
    the sequence."""
    r = fa2(Q, K, V, block_m, block_n, causal, blocks_, scale=scale, want_traj=True)
    m = r["traj"][..., 0]                       # [n, Tc, block_m]: m after the k-th block (NaN: block not visited)
    final = r["m_final"]                        # [n, block_m]
    n, Tc, Br = m.shape
    hit = m == final[:, None, :]                # NaN compares unequal: unvisited blocks and absent rows never hit
    first = np.argmax(hit, axis=1)              # index of the first block that hits (0 where none does)
    return np.where(hit.any(axis=1), first, -1).astype(np.int64)

