"""vfa_decode_noalloc_fwd (the decode step for callers that cannot allocate: its partial sums live in a fixed
device array of the library) against vfa_decode_fwd (caller-supplied workspace), through the C ABI.  Same
kernels on a different scratch address, so the bar is equality bit for bit; the oracle bars of the decode
tests are checked on top.  Two calls in a row, the second on a smaller problem, so that what the first call
left in the array would show if any of it were read; then the size limit."""
import ctypes

import numpy as np
import pytest

from paper_2604_12798_amd import workloads as wl

from gpu_util import LSE_ABS, O_MAX_ABS, O_MEAN_ABS, to_gpu

pytestmark = pytest.mark.gpu


def _problem(B, Hq, Hkv, n_cap, d):
    w = wl.small(wl.CONFIGS["cfg2"], B=B, Hq=Hq, Hkv=Hkv, N=n_cap, d=d)
    return wl.generate(w, wl.DEFAULT_SEED)


def _run_both(vfa, oracle, t, n_keys, n_splits):
    import torch
    L = vfa.lib()
    Qb = np.ascontiguousarray(t["Q"][:, :, n_keys - 1])
    q, K, V = to_gpu(Qb), to_gpu(t["K"]), to_gpu(t["V"])
    B, Hq, d = q.shape
    Hkv, n_cap = K.shape[1], K.shape[2]
    R = torch.zeros((B, Hkv, -(-n_cap // 64), d), dtype=torch.bfloat16, device="cuda")
    vfa.kblock_summary_append(K, R, 0, n_keys)
    need = vfa.decode_workspace_bytes(B, Hq, d, n_splits)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    O_ref = torch.full((B, Hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    L_ref = torch.full((B, Hq), float("nan"), dtype=torch.float32, device="cuda")
    O_new, L_new = O_ref.clone(), L_ref.clone()
    torch.cuda.synchronize()
    vp = lambda x: ctypes.c_void_p(x.data_ptr())
    common = (B, Hq, Hkv, n_cap, n_keys, d, 64, 1, 1, 1, n_splits, 0.0)
    print(f"noalloc: B={B} Hq={Hq} Hkv={Hkv} n_keys={n_keys} n_splits={n_splits} scratch {need} B", flush=True)
    rc = L.vfa_decode_fwd(vp(q), vp(K), vp(V), vp(R), vp(O_ref), vp(L_ref), *common, vp(ws), need, None)
    assert rc == 0, vfa.strerror(rc)
    rc = L.vfa_decode_noalloc_fwd(vp(q), vp(K), vp(V), vp(R), vp(O_new), vp(L_new), *common, None)
    assert rc == 0, vfa.strerror(rc)
    torch.cuda.synchronize()
    assert not torch.isnan(O_new.float()).any() and not torch.isnan(L_new).any()
    assert torch.equal(O_new, O_ref) and torch.equal(L_new, L_ref), "differs from vfa_decode_fwd"
    ref = oracle.decode(wl.bf16_bits_to_f32(Qb), wl.bf16_bits_to_f32(t["K"]), wl.bf16_bits_to_f32(t["V"]), n_keys, 64)
    err = np.abs(O_new.float().cpu().numpy().astype(np.float64) - ref["O"])
    lerr = np.abs(L_new.cpu().numpy().astype(np.float64) - ref["LSE"]).max()
    assert err.max() <= O_MAX_ABS and err.mean() <= O_MEAN_ABS and lerr <= LSE_ABS, (err.max(), err.mean(), lerr)
    return float(err.max()), float(lerr)


def test_noalloc_decode_equals_workspace_decode_twice(oracle):
    import torch
    assert torch.cuda.is_available()
    import paper_2604_12798_amd as vfa
    vfa.lib()
    big = _problem(B=2, Hq=16, Hkv=4, n_cap=4096, d=128)
    print("first call", _run_both(vfa, oracle, big, 4000, 16), flush=True)
    small = _problem(B=1, Hq=4, Hkv=2, n_cap=1024, d=128)
    print("second, smaller call", _run_both(vfa, oracle, small, 700, 3), flush=True)


def test_noalloc_decode_rejects_what_does_not_fit():
    import torch
    import paper_2604_12798_amd as vfa
    L = vfa.lib()
    B, Hq, Hkv, d, n_cap = 2, 64, 8, 128, 256
    q = torch.zeros((B, Hq, d), dtype=torch.bfloat16, device="cuda")
    K = torch.zeros((B, Hkv, n_cap, d), dtype=torch.bfloat16, device="cuda")
    R = torch.zeros((B, Hkv, n_cap // 64, d), dtype=torch.bfloat16, device="cuda")
    O = torch.full_like(q, 3.0)
    vp = lambda x: ctypes.c_void_p(x.data_ptr())
    # 2 * 64 * n_splits * 130 * 4 bytes: 63 ranges fit in 4 MiB, 64 do not
    assert vfa.decode_workspace_bytes(B, Hq, d, 63) <= vfa.DECODE_NOALLOC_MAX_BYTES < vfa.decode_workspace_bytes(B, Hq, d, 64)
    rc = L.vfa_decode_noalloc_fwd(vp(q), vp(K), vp(K), vp(R), vp(O), None, B, Hq, Hkv, n_cap, n_cap, d, 64, 1, 1, 1, 64, 0.0, None)
    assert rc == -4 and "scratch" in vfa.strerror(rc)
    torch.cuda.synchronize()
    assert bool((O.float() == 3.0).all()), "a rejected call must not launch anything"
    rc = L.vfa_decode_noalloc_fwd(vp(q), vp(K), vp(K), vp(R), vp(O), None, B, Hq, Hkv, n_cap, n_cap, d, 64, 1, 1, 1, 63, 0.0, None)
    assert rc == 0
    torch.cuda.synchronize()
    assert bool((O.float() == 0.0).all())      # all-zero V
