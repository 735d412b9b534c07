"""GPU parity where the ping-pong kernel runs as persistent workgroups (more work items than CUs) in the
forms the workload list does not reach: one item list for the whole chip (B * Hkv not a multiple of 8),
and a last round that only some workgroups take part in, for head pairs and for block pairs.
Besides the sampled oracle check, every output row must have been written exactly as the other entry
points write it: the two baselines and Alg. 1 compute the same attention, so their outputs have to agree
to rounding everywhere, which a work item that was dropped, done twice or decoded wrongly would break."""
import numpy as np
import pytest

from paper_2604_12798_amd import workloads as wl

from gpu_util import check_o_lse, gpu_inputs, host_f32

pytestmark = pytest.mark.gpu

# (name, base config, overrides): items = B * Hq/2 * Tr (head pairs) or B * Hq * ceil(Tr/2) (block pairs)
CASES = [
    ("chip_list_head_pairs", "cfg3", dict(B=3, Hq=4, Hkv=2, N=5632)),    # B*Hkv = 6: 264 items in one list
    ("xcd_lists_block_pairs", "cfg2", dict(B=1, Hq=8, Hkv=8, N=8448)),   # 8 lists of 33 items: partial round
    ("xcd_lists_head_pairs", "cfg3", dict(B=1, Hq=16, Hkv=8, N=4480)),   # 8 lists of 35 items: partial round
    ("chip_list_ragged", "cfg3", dict(B=1, Hq=6, Hkv=3, N=11300)),       # 267 items, ragged last block
]


@pytest.mark.parametrize("name,base,over", CASES, ids=[c[0] for c in CASES])
def test_persistent_workgroups(oracle, name, base, over):
    import torch
    import paper_2604_12798_amd as vfa
    vfa.lib()
    w = wl.small(wl.CONFIGS[base], **over)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    g = w.Hq // w.Hkv
    items = w.B * (w.Hq // 2) * w.Tr if g % 2 == 0 else w.B * w.Hq * ((w.Tr + 1) // 2)
    assert items > n_cu, "shape no longer exceeds the CU count: the persistent path is not exercised"
    print(f"{name}: {items} items on {n_cu} CUs", flush=True)
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    kw = dict(block_m=w.block_m, block_n=w.block_n, causal=w.causal)
    vkw = dict(n_sink=w.n_sink, n_local=w.n_local, **kw)
    blocks = wl.sample_blocks(w, 6)
    Oe, Le, _ = oracle.exact(Qh, Kh, Vh, w.block_m, w.causal, blocks)
    ref = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, n_sink=w.n_sink, n_local=w.n_local)

    def run(fn, **kws):
        O = torch.full_like(Q, float("nan"))
        L = torch.full((w.B, w.Hq, w.N), float("nan"), dtype=torch.float32, device=Q.device)
        fn(Q, K, V, out=O, lse=L, **kws)
        torch.cuda.synchronize()
        assert not torch.isnan(O.float()).any() and not torch.isnan(L).any(), name + ": rows left unwritten"
        return O, L

    O_fa, L_fa = run(vfa.fa_baseline_fwd, **kw)
    print(name, "fa", check_o_lse(O_fa, L_fa, Oe, Le, blocks, w.block_m, w.N, "fa_baseline_fwd vs exact"), flush=True)
    O_v, L_v = run(vfa.vfa_attn_fwd, **vkw)
    print(name, "vfa", check_o_lse(O_v, L_v, ref["O"], ref["LSE"], blocks, w.block_m, w.N, "vfa_attn_fwd vs oracle"), flush=True)
    O_l, L_l = run(vfa.fa_lazy_rescale_fwd, rescale_tau=8.0, **kw)
    # every row, against each other (bf16 outputs of the same attention: a few ulps of bf16 apart at most)
    for what, (Oa, La) in {"vfa": (O_v, L_v), "fa_lazy": (O_l, L_l)}.items():
        do = (Oa.float() - O_fa.float()).abs().max().item()
        dl = (La - L_fa).abs().max().item()
        print(name, what, "vs fa over all rows: max |dO| %.4f max |dLSE| %.2e" % (do, dl), flush=True)
        assert do <= 4e-2 and dl <= 2e-3, (name, what, do, dl)
    # VSA with a threshold nothing reaches: the same attention again, every visited tile kept
    O_s, L_s, M = vfa.vsa_attn_fwd(Q, K, V, skip_threshold_nats=1e4, **vkw)
    torch.cuda.synchronize()
    assert int((M == 1).sum().item()) == 0
    assert (O_s.float() - O_v.float()).abs().max().item() <= 4e-2 and (L_s - L_v).abs().max().item() <= 2e-3
