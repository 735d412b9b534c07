"""The entry points under HIP graph capture.  The library allocates nothing, records no memset and launches plain
kernels on the caller's stream, so a prefill call and a decode step can be captured once and replayed; every replay,
with the program's own eager work and synchronisations in between, must reproduce the eager result bit for bit."""
import numpy as np
import pytest

from paper_2604_12798_amd import workloads as wl

from gpu_util import gpu_inputs, to_gpu

pytestmark = pytest.mark.gpu


def test_prefill_and_decode_replay_from_a_graph():
    import torch
    import paper_2604_12798_amd as vfa
    vfa.lib()
    w = wl.small(wl.CONFIGS["cfg3"], B=1, Hq=4, Hkv=2, N=2048)
    Q, K, V = gpu_inputs(wl.generate(w, 1))
    dev = Q.device
    kw = dict(block_m=w.block_m, block_n=w.block_n, causal=w.causal, n_sink=w.n_sink, n_local=w.n_local)
    ws = torch.empty(vfa.workspace_bytes(w.B, w.Hkv, w.N, w.d, w.block_n), dtype=torch.uint8, device=dev)
    O, L = torch.empty_like(Q), torch.empty((w.B, w.Hq, w.N), dtype=torch.float32, device=dev)
    Os, Ls = torch.empty_like(Q), torch.empty_like(L)
    M = torch.empty((w.B, w.Hq, w.Tr, w.Tc), dtype=torch.uint8, device=dev)
    q1 = Q[:, :, -1].contiguous()                      # decode: the last token against the whole cache
    n_splits = 4
    R = torch.empty((w.B, w.Hkv, w.Tc, w.d), dtype=torch.bfloat16, device=dev)
    dws = torch.empty(vfa.decode_workspace_bytes(w.B, w.Hq, w.d, n_splits), dtype=torch.uint8, device=dev)
    Od, Ld = torch.empty_like(q1), torch.empty((w.B, w.Hq), dtype=torch.float32, device=dev)

    def step(o, l, os_, ls_, m, od, ld):
        vfa.vfa_attn_fwd(Q, K, V, out=o, lse=l, workspace=ws, **kw)
        vfa.vsa_attn_fwd(Q, K, V, out=os_, lse=ls_, skip_mask=m, workspace=ws, skip_threshold_nats=1.0, **kw)
        vfa.kblock_summary_append(K, R, 0, w.N, w.block_n)
        vfa.decode_fwd(q1, K, V, w.N, krepr=R, n_splits=n_splits, workspace=dws, out=od, lse=ld,
                       n_sink=w.n_sink, n_local=w.n_local)

    step(O, L, Os, Ls, M, Od, Ld)                      # eager once: one-time attribute calls happen outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(O, L, Os, Ls, M, Od, Ld)
    eo, el = torch.empty_like(O), torch.empty_like(L)
    eos, els, em = torch.empty_like(Os), torch.empty_like(Ls), torch.empty_like(M)
    eod, eld = torch.empty_like(Od), torch.empty_like(Ld)
    for rnd in range(3):
        t = wl.generate(w, 10 + rnd)                   # new inputs into the captured buffers, by ordinary eager copies
        Q.copy_(to_gpu(t["Q"])); K.copy_(to_gpu(t["K"])); V.copy_(to_gpu(t["V"]))
        q1.copy_(Q[:, :, -1])
        for x in (O, L, Os, Ls, Od, Ld):
            x.fill_(float("nan"))
        M.fill_(7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        step(eo, el, eos, els, em, eod, eld)           # the same step eagerly, into other outputs
        torch.cuda.synchronize()
        for name, a, b in (("O", O, eo), ("LSE", L, el), ("VSA O", Os, eos), ("VSA LSE", Ls, els), ("mask", M, em),
                           ("decode O", Od, eod), ("decode LSE", Ld, eld)):
            assert torch.equal(a, b), (rnd, name)
        assert int((M == 1).sum().item()) > 0 and not torch.isnan(O.float()).any()
