"""Thin Python binding of libvfa.so (the C ABI declared in include/vfa.h).

Argument marshalling only: every step of the attention path runs in the HIP kernels behind
the C entry points.  torch is used for device memory and streams.  There is no fallback: if
the library is missing, or a call returns an error code, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvfa.so")
_lib = None

EXPORTS = ("vfa_workspace_bytes", "vfa_kblock_summary", "vfa_kblock_summary_mode", "fa_baseline_fwd",
           "fa_lazy_rescale_fwd", "fa_lazy_rescale_softexp_fwd", "vfa_attn_fwd", "vsa_attn_fwd", "vfa_variant_fwd", "vfa_kblock_summary_append",
           "vfa_decode_workspace_bytes", "vfa_decode_fwd", "vfa_decode_noalloc_fwd", "vfa_kblock_summary_append_varlen", "vfa_decode_varlen_fwd", "vfa_fp8_quantize", "vfa_fp8_v_bytes", "vfa_fp8_pack_v",
           "vfa_fp8_attn_fwd", "vfa_fp8_attn_noexp_fwd", "vfa_mxfp4_quantize", "vfa_mxfp4_workspace_bytes", "vfa_mxfp4_attn_fwd", "vfa_mxfp4_attn_noexp_fwd", "vfa_strerror")


class VfaError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} (code {code})")
        self.code = code


def lib() -> ctypes.CDLL:
    """Load libvfa.so (built in-tree by build.py / __graft_entry__.build()); never falls back."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_12798_amd.build`")
        # torch first: it brings its own copy of the HIP runtime, and this library must bind to that one.  Loaded the
        # other way round, the process holds two runtimes, the tensors live in one, this library's kernels are
        # registered with the other, and every launch from here fails
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        L.vfa_workspace_bytes.restype = sz
        L.vfa_workspace_bytes.argtypes = [i, i, i, i, i]
        L.vfa_kblock_summary.restype = i
        L.vfa_kblock_summary.argtypes = [vp, vp, i, i, i, i, i, vp]
        L.vfa_kblock_summary_mode.restype = i
        L.vfa_kblock_summary_mode.argtypes = [vp, vp, i, i, i, i, i, i, vp]
        L.vfa_variant_fwd.restype = i
        L.vfa_variant_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, i, i, i, i, i, f, f, f, vp, vp, sz, vp]
        L.vfa_kblock_summary_append.restype = i
        L.vfa_kblock_summary_append.argtypes = [vp, vp, i, i, i, i, i, i, i, vp]
        L.vfa_decode_workspace_bytes.restype = sz
        L.vfa_decode_workspace_bytes.argtypes = [i, i, i, i]
        L.vfa_decode_fwd.restype = i
        L.vfa_decode_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, f, vp, sz, vp]
        L.vfa_decode_noalloc_fwd.restype = i
        L.vfa_decode_noalloc_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, f, vp]
        L.vfa_kblock_summary_append_varlen.restype = i
        L.vfa_kblock_summary_append_varlen.argtypes = [vp, vp, i, i, i, vp, vp, i, i, vp]
        L.vfa_decode_varlen_fwd.restype = i
        L.vfa_decode_varlen_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp, i, i, i, i, i, i, f, vp, sz, vp]
        L.vfa_fp8_quantize.restype = i
        L.vfa_fp8_quantize.argtypes = [vp, vp, ctypes.c_longlong, f, vp]
        L.vfa_fp8_v_bytes.restype = sz
        L.vfa_fp8_v_bytes.argtypes = [i, i, i]
        L.vfa_fp8_pack_v.restype = i
        L.vfa_fp8_pack_v.argtypes = [vp, vp, i, i, i, i, f, vp]
        L.vfa_fp8_attn_noexp_fwd.restype = i
        L.vfa_fp8_attn_noexp_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, f, f, f, f, vp, sz, vp]
        L.vfa_mxfp4_quantize.restype = i
        L.vfa_mxfp4_quantize.argtypes = [vp, vp, vp, ctypes.c_longlong, f, vp]
        L.vfa_mxfp4_workspace_bytes.restype = sz
        L.vfa_mxfp4_workspace_bytes.argtypes = [i, i, i]
        L.vfa_mxfp4_attn_fwd.restype = i
        L.vfa_mxfp4_attn_fwd.argtypes = [i, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, f, f, vp, sz, vp]
        L.vfa_mxfp4_attn_noexp_fwd.restype = i
        L.vfa_mxfp4_attn_noexp_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, f, f, vp, sz, vp]
        L.vfa_fp8_attn_fwd.restype = i
        L.vfa_fp8_attn_fwd.argtypes = [i, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, f, f, f, f, vp, sz, vp]
        L.fa_baseline_fwd.restype = i
        L.fa_baseline_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, f, vp]
        L.fa_lazy_rescale_fwd.restype = i
        L.fa_lazy_rescale_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, f, f, vp]
        L.fa_lazy_rescale_softexp_fwd.restype = i
        L.fa_lazy_rescale_softexp_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, f, f, vp]
        L.vfa_attn_fwd.restype = i
        L.vfa_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, f, vp, sz, vp]
        L.vsa_attn_fwd.restype = i
        L.vsa_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, i, i, f, f, vp, vp, sz, vp]
        L.vfa_strerror.restype = ctypes.c_char_p
        L.vfa_strerror.argtypes = [i]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().vfa_strerror(int(code)).decode()


def workspace_bytes(B: int, Hkv: int, N: int, d: int, block_n: int) -> int:
    return int(lib().vfa_workspace_bytes(B, Hkv, N, d, block_n))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check_qkv(Q, K, V):
    import torch
    for t in (Q, K, V):
        if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.dim() == 4):
            raise ValueError("Q, K, V must be contiguous 4-d bf16 tensors on the GPU")
    B, Hq, N, d = Q.shape
    if K.shape != V.shape or K.shape[0] != B or K.shape[2] != N or K.shape[3] != d:
        raise ValueError("K, V must be [B, Hkv, N, d] matching Q [B, Hq, N, d]")
    return B, Hq, K.shape[1], N, d


def _outputs(Q, out, lse, want_lse):
    import torch
    B, Hq, N, d = Q.shape
    O = torch.empty_like(Q) if out is None else out
    L = lse
    if L is None and want_lse:
        L = torch.empty((B, Hq, N), dtype=torch.float32, device=Q.device)
    return O, L


def kblock_summary(K, block_n: int = 64, out=None, stream=None, repr_mode: int = 0):
    """Key-block summaries Krepr [B, Hkv, ceil(N/block_n), d] (bf16) of K [B, Hkv, N, d].
    repr_mode 0 = sabsmax (the method); 1 / 2 / 3 = per-dimension max / mean / unsigned absmax."""
    import torch
    B, Hkv, N, d = K.shape
    Tc = -(-N // block_n)
    R = torch.empty((B, Hkv, Tc, d), dtype=torch.bfloat16, device=K.device) if out is None else out
    if repr_mode == 0:
        rc = lib().vfa_kblock_summary(_ptr(K), _ptr(R), B, Hkv, N, d, block_n, _stream(stream))
    else:
        rc = lib().vfa_kblock_summary_mode(_ptr(K), _ptr(R), B, Hkv, N, d, block_n, int(repr_mode), _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_kblock_summary")
    return R


def fa_baseline_fwd(Q, K, V, *, block_m=128, block_n=64, causal=True, softmax_scale=0.0, out=None, lse=None,
                    want_lse=True, stream=None):
    B, Hq, Hkv, N, d = _check_qkv(Q, K, V)
    O, L = _outputs(Q, out, lse, want_lse)
    rc = lib().fa_baseline_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(L), B, Hq, Hkv, N, d, block_m, block_n,
                               int(bool(causal)), float(softmax_scale), _stream(stream))
    if rc != 0:
        raise VfaError(rc, "fa_baseline_fwd")
    return O, L


def fa_lazy_rescale_fwd(Q, K, V, *, block_m=128, block_n=64, causal=True, softmax_scale=0.0, rescale_tau=8.0, out=None,
                        lse=None, want_lse=True, stream=None):
    B, Hq, Hkv, N, d = _check_qkv(Q, K, V)
    O, L = _outputs(Q, out, lse, want_lse)
    rc = lib().fa_lazy_rescale_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(L), B, Hq, Hkv, N, d, block_m, block_n,
                                   int(bool(causal)), float(softmax_scale), float(rescale_tau), _stream(stream))
    if rc != 0:
        raise VfaError(rc, "fa_lazy_rescale_fwd")
    return O, L


def fa_lazy_rescale_softexp_fwd(Q, K, V, *, block_m=128, block_n=64, causal=True, softmax_scale=0.0, rescale_tau=8.0,
                                out=None, lse=None, want_lse=True, stream=None):
    B, Hq, Hkv, N, d = _check_qkv(Q, K, V)
    O, L = _outputs(Q, out, lse, want_lse)
    rc = lib().fa_lazy_rescale_softexp_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(L), B, Hq, Hkv, N, d, block_m,
                                           block_n, int(bool(causal)), float(softmax_scale), float(rescale_tau),
                                           _stream(stream))
    if rc != 0:
        raise VfaError(rc, "fa_lazy_rescale_softexp_fwd")
    return O, L


def _workspace(Q, K, block_n, workspace):
    import torch
    B, Hkv, N, d = K.shape
    need = workspace_bytes(B, Hkv, N, d, block_n)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Q.device)
    return workspace, workspace.numel() * workspace.element_size()


def vfa_attn_fwd(Q, K, V, *, block_m=128, block_n=64, causal=True, n_sink=1, n_local=1, use_minit=True,
                 softmax_scale=0.0, workspace=None, out=None, lse=None, want_lse=True, stream=None):
    B, Hq, Hkv, N, d = _check_qkv(Q, K, V)
    O, L = _outputs(Q, out, lse, want_lse)
    ws, ws_bytes = _workspace(Q, K, block_n, workspace)
    rc = lib().vfa_attn_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(L), B, Hq, Hkv, N, d, block_m, block_n,
                            int(bool(causal)), int(n_sink), int(n_local), int(use_minit), float(softmax_scale),
                            _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_attn_fwd")
    return O, L


def vsa_attn_fwd(Q, K, V, *, block_m=128, block_n=64, causal=True, n_sink=1, n_local=1, use_minit=True,
                 softmax_scale=0.0, skip_threshold_nats=8.0, skip_mask=None, want_mask=True, workspace=None,
                 out=None, lse=None, want_lse=True, stream=None):
    import torch
    B, Hq, Hkv, N, d = _check_qkv(Q, K, V)
    O, L = _outputs(Q, out, lse, want_lse)
    ws, ws_bytes = _workspace(Q, K, block_n, workspace)
    M = skip_mask
    if M is None and want_mask:
        M = torch.empty((B, Hq, -(-N // block_m), -(-N // block_n)), dtype=torch.uint8, device=Q.device)
    rc = lib().vsa_attn_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(L), B, Hq, Hkv, N, d, block_m, block_n,
                            int(bool(causal)), int(n_sink), int(n_local), int(use_minit), float(softmax_scale),
                            float(skip_threshold_nats), _ptr(M), _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vsa_attn_fwd")
    return O, L, M


def vfa_variant_fwd(Q, K, V, *, block_m=128, block_n=64, causal=True, n_sink=1, n_local=1, use_minit=True, repr_mode=0,
                    q_repr_mode=0, reorder=True, freeze=True, rowskip=False, lazy_rescale_tau=-1.0, softmax_scale=0.0,
                    skip_threshold_nats=0.0, skip_mask=None,
                    workspace=None, out=None, lse=None, want_lse=True, stream=None):
    """VFA / VSA with the ablation switches; returns (O, LSE, mask) with mask None when nothing is skipped."""
    import torch
    B, Hq, Hkv, N, d = _check_qkv(Q, K, V)
    O, L = _outputs(Q, out, lse, want_lse)
    if workspace is None and q_repr_mode:   # query-block summaries behind the key-block summaries
        need = workspace_bytes(B, Hkv, N, d, block_n) + workspace_bytes(B, Hq, N, d, block_m)
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    ws, ws_bytes = _workspace(Q, K, block_n, workspace)
    M = skip_mask
    if M is None and skip_threshold_nats != 0.0:
        M = torch.empty((B, Hq, -(-N // block_m), -(-N // block_n)), dtype=torch.uint8, device=Q.device)
    rc = lib().vfa_variant_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(L), B, Hq, Hkv, N, d, block_m, block_n,
                               int(bool(causal)), int(n_sink), int(n_local), int(use_minit), int(repr_mode),
                               int(q_repr_mode), int(bool(reorder)), int(bool(freeze)), int(bool(rowskip)), float(lazy_rescale_tau),
                               float(softmax_scale), float(skip_threshold_nats),
                               _ptr(M), _ptr(ws), ws_bytes, _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_variant_fwd")
    return O, L, M


def kblock_summary_append(K, Krepr, n_old: int, n_new: int, block_n: int = 64, stream=None):
    """Refresh, in place, the summaries of the blocks of cache K [B, Hkv, n_cap, d] that hold rows [n_old, n_new)."""
    B, Hkv, n_cap, d = K.shape
    rc = lib().vfa_kblock_summary_append(_ptr(K), _ptr(Krepr), B, Hkv, n_cap, int(n_old), int(n_new), d, block_n,
                                         _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_kblock_summary_append")
    return Krepr


def kblock_summary_append_varlen(K, Krepr, old_lens, new_lens, block_n: int = 64, stream=None):
    """As kblock_summary_append with per-sequence lengths (int32 device tensors of B entries)."""
    B, Hkv, n_cap, d = K.shape
    rc = lib().vfa_kblock_summary_append_varlen(_ptr(K), _ptr(Krepr), B, Hkv, n_cap, _ptr(old_lens), _ptr(new_lens), d,
                                                block_n, _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_kblock_summary_append_varlen")
    return Krepr


def decode_varlen_fwd(q, K, V, seq_lens, *, krepr=None, block_n=64, n_sink=1, n_local=1, use_minit=True, n_splits=8,
                      softmax_scale=0.0, workspace=None, out=None, lse=None, want_lse=True, stream=None):
    """As decode_fwd with per-sequence lengths (int32 device tensor of B entries)."""
    import torch
    B, Hq, d = q.shape
    Hkv, n_cap = K.shape[1], K.shape[2]
    assert seq_lens.is_cuda and seq_lens.dtype == torch.int32 and seq_lens.numel() == B
    O = torch.empty_like(q) if out is None else out
    L = lse if (lse is not None or not want_lse) else torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    need = decode_workspace_bytes(B, Hq, d, n_splits)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device) if workspace is None else workspace
    rc = lib().vfa_decode_varlen_fwd(_ptr(q), _ptr(K), _ptr(V), _ptr(krepr), _ptr(O), _ptr(L), B, Hq, Hkv, n_cap,
                                     _ptr(seq_lens), d, block_n, int(n_sink), int(n_local), int(bool(use_minit)),
                                     int(n_splits), float(softmax_scale), _ptr(ws), ws.numel() * ws.element_size(),
                                     _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_decode_varlen_fwd")
    return O, L


def decode_workspace_bytes(B: int, Hq: int, d: int, n_splits: int) -> int:
    return int(lib().vfa_decode_workspace_bytes(B, Hq, d, n_splits))


def decode_fwd(q, K, V, n_keys: int, *, krepr=None, block_n=64, n_sink=1, n_local=1, use_minit=True, n_splits=8,
               softmax_scale=0.0, workspace=None, out=None, lse=None, want_lse=True, stream=None):
    """One query token per head, q [B, Hq, d], against the first n_keys rows of the cache K, V [B, Hkv, n_cap, d]."""
    import torch
    B, Hq, d = q.shape
    Hkv, n_cap = K.shape[1], K.shape[2]
    for t in (q, K, V):
        if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()):
            raise ValueError("q, K, V must be contiguous bf16 tensors on the GPU")
    O = torch.empty_like(q) if out is None else out
    L = lse if (lse is not None or not want_lse) else torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    need = decode_workspace_bytes(B, Hq, d, n_splits)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device) if workspace is None else workspace
    rc = lib().vfa_decode_fwd(_ptr(q), _ptr(K), _ptr(V), _ptr(krepr), _ptr(O), _ptr(L), B, Hq, Hkv, n_cap, int(n_keys), d,
                              block_n, int(n_sink), int(n_local), int(bool(use_minit)), int(n_splits), float(softmax_scale),
                              _ptr(ws), ws.numel() * ws.element_size(), _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_decode_fwd")
    return O, L


DECODE_NOALLOC_MAX_BYTES = 4 << 20   # VFA_DECODE_NOALLOC_MAX_BYTES of vfa.h


def decode_noalloc_fwd(q, K, V, n_keys: int, out, lse=None, *, krepr=None, block_n=64, n_sink=1, n_local=1, use_minit=True,
                       n_splits=8, softmax_scale=0.0, stream=None):
    """vfa_decode_noalloc_fwd: as decode_fwd, but neither the library nor this wrapper allocates: the caller passes
    the output tensors (lse may be None) and the partial sums live in the library's fixed device array."""
    B, Hq, d = q.shape
    Hkv, n_cap = K.shape[1], K.shape[2]
    rc = lib().vfa_decode_noalloc_fwd(_ptr(q), _ptr(K), _ptr(V), _ptr(krepr), _ptr(out), _ptr(lse), B, Hq, Hkv, n_cap,
                                      int(n_keys), d, block_n, int(n_sink), int(n_local), int(bool(use_minit)),
                                      int(n_splits), float(softmax_scale), _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_decode_noalloc_fwd")
    return out, lse


def fp8_quantize(X, inv_scale: float, stream=None):
    """bf16 tensor -> uint8 tensor of E4M3 codes of X * inv_scale (same shape)."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous()
    Y = torch.empty(X.shape, dtype=torch.uint8, device=X.device)
    rc = lib().vfa_fp8_quantize(_ptr(X), _ptr(Y), X.numel(), float(inv_scale), _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_fp8_quantize")
    return Y


def fp8_pack_v(V, inv_scale: float, stream=None):
    """V [B, Hkv, N, 128] bf16 -> [B, Hkv, ceil(N/64), 128, 64] uint8 (transposed, key-permuted E4M3 tiles)."""
    import torch
    B, Hkv, N, d = V.shape
    Vt = torch.empty((B, Hkv, -(-N // 64), 128, 64), dtype=torch.uint8, device=V.device)
    rc = lib().vfa_fp8_pack_v(_ptr(V), _ptr(Vt), B, Hkv, N, d, float(inv_scale), _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_fp8_pack_v")
    return Vt


def fp8_attn_fwd(Q8, K8, Vt8, *, descale_q, descale_k, descale_v, frozen=True, block_m=128, block_n=64, causal=True,
                 n_sink=1, n_local=1, use_minit=True, softmax_scale=0.0, workspace=None, out=None, lse=None,
                 want_lse=True, stream=None, noexp=False):
    """E4M3 attention; noexp=True calls vfa_fp8_attn_noexp_fwd (Alg. 1 with the weights' codes taken from the scores)."""
    import torch
    B, Hq, N, d = Q8.shape
    Hkv = K8.shape[1]
    O = torch.empty((B, Hq, N, d), dtype=torch.bfloat16, device=Q8.device) if out is None else out
    L = lse if (lse is not None or not want_lse) else torch.empty((B, Hq, N), dtype=torch.float32, device=Q8.device)
    need = B * Hkv * (-(-N // block_n)) * 128
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=Q8.device) if workspace is None else workspace
    tail = (B, Hq, Hkv, N, d, block_m, block_n, int(bool(causal)), int(n_sink), int(n_local), int(use_minit),
            float(softmax_scale), float(descale_q), float(descale_k), float(descale_v), _ptr(ws),
            ws.numel() * ws.element_size(), _stream(stream))
    if noexp:
        rc = lib().vfa_fp8_attn_noexp_fwd(_ptr(Q8), _ptr(K8), _ptr(Vt8), _ptr(O), _ptr(L), *tail)
    else:
        rc = lib().vfa_fp8_attn_fwd(int(bool(frozen)), _ptr(Q8), _ptr(K8), _ptr(Vt8), _ptr(O), _ptr(L), *tail)
    if rc != 0:
        raise VfaError(rc, "vfa_fp8_attn_noexp_fwd" if noexp else "vfa_fp8_attn_fwd")
    return O, L


def mxfp4_quantize(X, pre_scale: float = 1.0, stream=None):
    """bf16 tensor [..., d] (d a multiple of 32) -> (uint8 [..., d/2] E2M1 pairs, uint8 [..., d/32] E8M0 scales) of X * pre_scale."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.is_contiguous() and X.shape[-1] % 32 == 0
    d = X.shape[-1]
    X4 = torch.empty(X.shape[:-1] + (d // 2,), dtype=torch.uint8, device=X.device)
    XS = torch.empty(X.shape[:-1] + (d // 32,), dtype=torch.uint8, device=X.device)
    rc = lib().vfa_mxfp4_quantize(_ptr(X), _ptr(X4), _ptr(XS), X.numel(), float(pre_scale), _stream(stream))
    if rc != 0:
        raise VfaError(rc, "vfa_mxfp4_quantize")
    return X4, XS


def mxfp4_workspace_bytes(B, Hkv, N) -> int:
    return int(lib().vfa_mxfp4_workspace_bytes(B, Hkv, N))


def mxfp4_attn_fwd(Q4, QS, K4, KS, Vt8, *, descale_v, frozen=True, block_m=128, block_n=64, causal=True, n_sink=1,
                   n_local=1, use_minit=True, softmax_scale=0.0, workspace=None, out=None, lse=None, want_lse=True,
                   stream=None, noexp=False):
    """Attention with MXFP4 scores (Q4/QS, K4/KS from mxfp4_quantize) and 8-bit P.V (Vt8 from fp8_pack_v);
    noexp=True calls vfa_mxfp4_attn_noexp_fwd."""
    import torch
    B, Hq, N, dh = Q4.shape
    d, Hkv = 2 * dh, K4.shape[1]
    O = torch.empty((B, Hq, N, d), dtype=torch.bfloat16, device=Q4.device) if out is None else out
    L = lse if (lse is not None or not want_lse) else torch.empty((B, Hq, N), dtype=torch.float32, device=Q4.device)
    need = mxfp4_workspace_bytes(B, Hkv, N)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=Q4.device) if workspace is None else workspace
    tail = (B, Hq, Hkv, N, d, block_m, block_n, int(bool(causal)), int(n_sink), int(n_local), int(use_minit),
            float(softmax_scale), float(descale_v), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream))
    ops = (_ptr(Q4), _ptr(QS), _ptr(K4), _ptr(KS), _ptr(Vt8), _ptr(O), _ptr(L))
    rc = lib().vfa_mxfp4_attn_noexp_fwd(*ops, *tail) if noexp else lib().vfa_mxfp4_attn_fwd(int(bool(frozen)), *ops, *tail)
    if rc != 0:
        raise VfaError(rc, "vfa_mxfp4_attn_noexp_fwd" if noexp else "vfa_mxfp4_attn_fwd")
    return O, L, ws
