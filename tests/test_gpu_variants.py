"""GPU parity of the ablation / variant switches (vfa_variant_fwd, vfa_kblock_summary_mode) against
the float64 oracle run with the same switches.  Bars as in test_gpu_parity.py."""
import numpy as np
import pytest

from paper_2604_12798_amd import workloads as wl

from gpu_util import MASK_GUARD_NATS, check_o_lse, gpu_inputs, host_f32, to_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vfa():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2604_12798_amd as pkg
    pkg.lib()
    return pkg


def W(base="cfg2", **kw):
    return wl.small(wl.CONFIGS[base], **kw)


SHAPES = [
    ("gqa_causal", W(B=2, Hq=4, Hkv=2, N=1024)),
    ("noncausal", W(B=1, Hq=2, Hkv=2, N=768, causal=False)),
    ("ragged_d64", W(B=1, Hq=2, Hkv=1, N=1000, d=64, F=4, block_m=64)),
]


@pytest.mark.parametrize("name,w", SHAPES, ids=[s[0] for s in SHAPES])
@pytest.mark.parametrize("mode", [1, 2, 3])
def test_ablated_block_representations(vfa, oracle, name, w, mode):
    import torch
    t = wl.generate(w)
    R = vfa.kblock_summary(to_gpu(t["K"]), w.block_n, repr_mode=mode)
    torch.cuda.synchronize()
    got = R.float().cpu().numpy().astype(np.float64)
    want = oracle.sabsmax(wl.bf16_bits_to_f32(t["K"]), w.block_n, mode)
    if mode == 2:   # a mean is not an element of K: fp32 sum, one rounding to bf16
        assert np.abs(got - want).max() <= 2.0 ** -8 * np.abs(want).max() + 1e-6
        assert np.abs(got - want).mean() <= 2.0 ** -9 * np.abs(want).mean() + 1e-6
    else:
        assert np.array_equal(got, want)


# (repr_mode, reorder, freeze, use_minit)
SWITCHES = [(1, True, True, True), (2, True, True, True), (3, True, True, True), (0, False, True, True),
            (0, False, True, False), (0, True, False, True), (0, False, False, False)]


@pytest.mark.parametrize("name,w", SHAPES, ids=[s[0] for s in SHAPES])
def test_variants_without_skipping_are_exact_attention(vfa, oracle, name, w):
    import torch
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    blocks = wl.all_blocks(w)
    Oe, Le, Me = oracle.exact(Qh, Kh, Vh, w.block_m, w.causal, blocks)
    for mode, reorder, freeze, minit in SWITCHES:
        O, L, M = vfa.vfa_variant_fwd(Q, K, V, block_m=w.block_m, block_n=w.block_n, causal=w.causal, n_sink=w.n_sink,
                                      n_local=w.n_local, use_minit=minit, repr_mode=mode, reorder=reorder, freeze=freeze)
        torch.cuda.synchronize()
        assert M is None
        ref = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, n_sink=w.n_sink, n_local=w.n_local,
                            use_minit=minit, reorder=reorder, freeze=freeze,
                            krepr=oracle.sabsmax(Kh, w.block_n, mode) if minit else None)
        tag = "variant repr=%d reorder=%d freeze=%d minit=%d" % (mode, reorder, freeze, minit)
        stats = check_o_lse(O, L, ref["O"], ref["LSE"], blocks, w.block_m, w.N, tag + " vs oracle")
        check_o_lse(O, L, Oe, Le, blocks, w.block_m, w.N, tag + " vs exact")
        gap = (Me - ref["m_final"])[~np.isnan(Me)]
        print(name, tag, stats, "true max minus final max (nats): max %.2f" % gap.max(), flush=True)


SKIP_CASES = [
    ("blasst", dict(use_minit=False, reorder=False, freeze=False)),          # vanilla BLASST
    ("blasst_swa", dict(use_minit=False, reorder=True, freeze=False)),       # BLASST in sink, local, rest order
    ("vsa_no_reorder", dict(use_minit=True, reorder=False, freeze=True)),    # Alg. 2 without the reordering
    ("vsa_kmax", dict(use_minit=True, reorder=True, freeze=True, repr_mode=1)),
]
SKIP_SHAPES = [
    ("causal_thr4", W(B=1, Hq=4, Hkv=2, N=2048, beta=6.0, kappa=3.0), 4.0),
    ("noncausal_thr5", W(B=1, Hq=2, Hkv=2, N=1024, beta=6.0, kappa=3.0, causal=False), 5.0),
]


@pytest.mark.parametrize("sname,w,thr", SKIP_SHAPES, ids=[s[0] for s in SKIP_SHAPES])
@pytest.mark.parametrize("vname,sw", SKIP_CASES, ids=[c[0] for c in SKIP_CASES])
def test_skipping_variants_mask_bit_exact(vfa, oracle, sname, w, thr, vname, sw):
    import torch
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    blocks = wl.all_blocks(w)
    mode = sw.get("repr_mode", 0)
    O, L, M = vfa.vfa_variant_fwd(Q, K, V, block_m=w.block_m, block_n=w.block_n, causal=w.causal, n_sink=w.n_sink,
                                  n_local=w.n_local, skip_threshold_nats=thr, **sw)
    torch.cuda.synchronize()
    ref = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, n_sink=w.n_sink, n_local=w.n_local,
                        use_minit=sw["use_minit"], reorder=sw["reorder"], freeze=sw["freeze"], vsa=True,
                        skip_threshold_nats=thr, krepr=oracle.sabsmax(Kh, w.block_n, mode) if sw["use_minit"] else None)
    got = M.cpu().numpy().reshape(len(blocks), w.Tc)
    near = np.abs(ref["margin"]) < MASK_GUARD_NATS
    cmp = ~near
    assert near.sum() <= 2, "too many tiles on the threshold: pick another seed"
    assert np.array_equal(got[cmp], ref["mask"][cmp]), (vname, int((got[cmp] != ref["mask"][cmp]).sum()))
    sparsity = (ref["mask"] == 1).sum() / max(1, (ref["mask"] != 2).sum())
    if near.sum() == 0:
        stats = check_o_lse(O, L, ref["O"], ref["LSE"], blocks, w.block_m, w.N, vname + " vs oracle")
    else:
        stats = "output not compared: %d tile(s) within the guard band" % near.sum()
    print(sname, vname, "sparsity %.3f" % sparsity, stats, flush=True)


@pytest.mark.parametrize("sname,w,thr", SKIP_SHAPES, ids=[s[0] for s in SKIP_SHAPES])
@pytest.mark.parametrize("vname,okw", [("rowskip", dict(rowskip=True)), ("fa4_tau1.5", dict(lazy_tau=1.5))],
                         ids=["rowskip", "fa4"])
def test_rowskip_and_fa4_variants(vfa, oracle, sname, w, thr, vname, okw):
    import torch
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    blocks = wl.all_blocks(w)
    gkw = dict(rowskip=True) if "rowskip" in okw else dict(lazy_rescale_tau=okw["lazy_tau"])
    O, L, M = vfa.vfa_variant_fwd(Q, K, V, block_m=w.block_m, block_n=w.block_n, causal=w.causal, n_sink=0, n_local=0,
                                  use_minit=False, reorder=False, freeze=False, skip_threshold_nats=thr, **gkw)
    torch.cuda.synchronize()
    ref = oracle.blasst_variant(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, thr, **okw)
    got = M.cpu().numpy().reshape(len(blocks), w.Tc)
    near = np.abs(ref["margin"]) < MASK_GUARD_NATS
    assert near.sum() <= 2
    assert np.array_equal(got[~near], ref["mask"][~near])
    # (row-level decisions sit on the same threshold: rows within the guard band of it may differ, so the output
    # is compared at the ordinary bars, which a single flipped row of a tile that carries < lambda of the mass meets)
    stats = check_o_lse(O, L, ref["O"], ref["LSE"], blocks, w.block_m, w.N, vname + " vs oracle")
    print(sname, vname, stats, "counter %d of %d" % (ref["counters"][:, 2].sum(), ref["counters"][:, 0].sum()), flush=True)


# ------------------------------------------------------------------ block-wise q_repr ablation
# q_repr_mode of the library -> reduction of the oracle's summary routine (1 absmax without sign, 2 sabsmax, 3 mean)
Q_SUMMARY = {1: 3, 2: 0, 3: 2}


def _q_summaries(oracle, Qh, block_m, q_mode):
    """Query-block summaries as the kernel holds them: elements of Q are exact in bf16, a mean is rounded once."""
    qr = oracle.sabsmax(Qh, block_m, Q_SUMMARY[q_mode])
    if q_mode == 3:
        qr = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(qr.astype(np.float32))).astype(np.float64)
    return qr


@pytest.mark.parametrize("name,w", SHAPES, ids=[s[0] for s in SHAPES])
@pytest.mark.parametrize("q_mode", [1, 2, 3])
def test_blockwise_q_repr_is_exact_attention(vfa, oracle, name, w, q_mode):
    import torch
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    blocks = wl.all_blocks(w)
    Oe, Le, Me = oracle.exact(Qh, Kh, Vh, w.block_m, w.causal, blocks)
    O, L, M = vfa.vfa_variant_fwd(Q, K, V, block_m=w.block_m, block_n=w.block_n, causal=w.causal, n_sink=w.n_sink,
                                  n_local=w.n_local, q_repr_mode=q_mode)
    torch.cuda.synchronize()
    assert M is None
    ref = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, n_sink=w.n_sink, n_local=w.n_local,
                        qrepr=_q_summaries(oracle, Qh, w.block_m, q_mode))
    tag = "q_repr_mode=%d" % q_mode
    stats = check_o_lse(O, L, ref["O"], ref["LSE"], blocks, w.block_m, w.N, tag + " vs oracle")
    check_o_lse(O, L, Oe, Le, blocks, w.block_m, w.N, tag + " vs exact")
    gap = (Me - ref["m_final"])[~np.isnan(Me)]
    print(name, tag, stats, "true max minus final max (nats): min %.2f max %.2f" % (gap.min(), gap.max()), flush=True)


@pytest.mark.parametrize("sname,w,thr", SKIP_SHAPES, ids=[s[0] for s in SKIP_SHAPES])
@pytest.mark.parametrize("q_mode", [1, 2, 3])
@pytest.mark.parametrize("specials", [True, False], ids=["sink_local", "seed_only"])
def test_blockwise_q_repr_skip_mask_bit_exact(vfa, oracle, sname, w, thr, q_mode, specials):
    """The skip decisions depend on the frozen max, hence on the seed: the masks agree with the oracle's only if the
    kernel seeds every row of a block with the block-wise score (and they differ from the row-wise method's).
    Without sink and local blocks the seed alone is the frozen max, so every decision hangs on it."""
    import torch
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    blocks = wl.all_blocks(w)
    n_sink, n_local = (w.n_sink, w.n_local) if specials else (0, 0)
    kw = dict(block_m=w.block_m, block_n=w.block_n, causal=w.causal, n_sink=n_sink, n_local=n_local,
              skip_threshold_nats=thr)
    O, L, M = vfa.vfa_variant_fwd(Q, K, V, q_repr_mode=q_mode, **kw)
    torch.cuda.synchronize()
    okw = dict(n_sink=n_sink, n_local=n_local, vsa=True, skip_threshold_nats=thr)
    ref = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks,
                        qrepr=_q_summaries(oracle, Qh, w.block_m, q_mode), **okw)
    got = M.cpu().numpy().reshape(len(blocks), w.Tc)
    near = np.abs(ref["margin"]) < MASK_GUARD_NATS
    assert near.sum() <= 2, "too many tiles on the threshold: pick another seed"
    assert np.array_equal(got[~near], ref["mask"][~near]), (q_mode, int((got[~near] != ref["mask"][~near]).sum()))
    rowwise = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, **okw)
    differ = int((rowwise["mask"] != ref["mask"]).sum())
    if near.sum() == 0:
        stats = check_o_lse(O, L, ref["O"], ref["LSE"], blocks, w.block_m, w.N, "q_repr skip vs oracle")
    else:
        stats = "output not compared: %d tile(s) within the guard band" % near.sum()
    sparsity = (ref["mask"] == 1).sum() / max(1, (ref["mask"] != 2).sum())
    print(sname, "q_repr_mode", q_mode, "specials", specials, "sparsity %.3f" % sparsity, "tiles decided differently from the row-wise seed:",
          differ, stats, flush=True)
