"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle on the same
seeded inputs.  Bars: O max-abs <= 2e-2 and mean-abs <= 2e-3, LSE <= 1e-3, skip masks bit-exact
(outside a 1e-3-nat guard band around the threshold), key-block summaries bit-exact."""
import dataclasses

import numpy as np
import pytest

from paper_2604_12798_amd import workloads as wl

from gpu_util import MASK_GUARD_NATS, check_o_lse, gather_blocks, gpu_inputs, host_f32, to_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vfa():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2604_12798_amd as pkg
    pkg.lib()   # raises if libvfa.so is missing: no fallback
    return pkg


def W(base="cfg2", **kw):
    return wl.small(wl.CONFIGS[base], **kw)


SMALL = [
    ("cfg1", wl.CONFIGS["cfg1"]),
    ("cfg2_small_gqa", W(B=2, Hq=4, Hkv=2, N=1024)),
    ("cfg2_small_noncausal", W(B=1, Hq=2, Hkv=2, N=768, causal=False)),
    ("ragged_1000", W(B=1, Hq=2, Hkv=1, N=1000)),
    ("ragged_77_noncausal", W(B=1, Hq=1, Hkv=1, N=77, causal=False)),
    ("one_key", W(B=1, Hq=1, Hkv=1, N=1)),
    ("d64_128x64", W(B=1, Hq=2, Hkv=1, N=640, d=64, F=4)),
    ("d128_64x64", W(B=1, Hq=2, Hkv=2, N=576, block_m=64)),
    ("sink2_local3", W(B=1, Hq=2, Hkv=1, N=1024, n_sink=2, n_local=3)),
    ("sink0_local2_noncausal", W(B=1, Hq=1, Hkv=1, N=896, n_sink=0, n_local=2, causal=False)),
    ("sink1_local0", W(B=1, Hq=1, Hkv=1, N=768, n_sink=1, n_local=0)),
    ("planted_noncausal", W("cfg4", B=1, Hq=2, Hkv=2, N=2048)),
    # odd number of query heads per KV head: the ping-pong kernel pairs adjacent query blocks (odd block count, ragged)
    ("gqa3_ragged_1100", W(B=1, Hq=3, Hkv=1, N=1100)),
    ("mha_causal_1280_sink2_local2", W(B=2, Hq=2, Hkv=2, N=1280, n_sink=2, n_local=2)),
]


def _run_all(vfa, w, t, blocks, oracle, use_minit=True):
    import torch
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    kw = dict(block_m=w.block_m, block_n=w.block_n, causal=w.causal)
    res = {}
    Oe, Le, Me = oracle.exact(Qh, Kh, Vh, w.block_m, w.causal, blocks)
    O, L = vfa.fa_baseline_fwd(Q, K, V, **kw)
    torch.cuda.synchronize()
    res["fa"] = check_o_lse(O, L, Oe, Le, blocks, w.block_m, w.N, "fa_baseline_fwd vs exact")
    ref = oracle.fa2(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks)
    check_o_lse(O, L, ref["O"], ref["LSE"], blocks, w.block_m, w.N, "fa_baseline_fwd vs oracle FA")
    for tau in (0.0, 8.0):   # conditional rescale: same exact attention for any tau (0: every new max is adopted)
        O, L = vfa.fa_lazy_rescale_fwd(Q, K, V, rescale_tau=tau, **kw)
        torch.cuda.synchronize()
        res["fa_lazy%g" % tau] = check_o_lse(O, L, Oe, Le, blocks, w.block_m, w.N, "fa_lazy_rescale_fwd vs exact")
    O, L = vfa.fa_lazy_rescale_softexp_fwd(Q, K, V, rescale_tau=8.0, **kw)   # half of the exponentials in software
    torch.cuda.synchronize()
    res["fa_softexp"] = check_o_lse(O, L, Oe, Le, blocks, w.block_m, w.N, "fa_lazy_rescale_softexp_fwd vs exact")
    O, L = vfa.vfa_attn_fwd(Q, K, V, n_sink=w.n_sink, n_local=w.n_local, use_minit=use_minit, **kw)
    torch.cuda.synchronize()
    ref = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, n_sink=w.n_sink, n_local=w.n_local,
                        use_minit=use_minit)
    res["vfa"] = check_o_lse(O, L, ref["O"], ref["LSE"], blocks, w.block_m, w.N, "vfa_attn_fwd vs oracle VFA")
    check_o_lse(O, L, Oe, Le, blocks, w.block_m, w.N, "vfa_attn_fwd vs exact")
    return res


@pytest.mark.parametrize("name,w", SMALL, ids=[n for n, _ in SMALL])
def test_fa_and_vfa_match_oracle(vfa, oracle, name, w):
    t = wl.generate(w)
    print(name, _run_all(vfa, w, t, wl.all_blocks(w), oracle), flush=True)


@pytest.mark.parametrize("name,w", [SMALL[1], SMALL[8]], ids=[SMALL[1][0], SMALL[8][0]])
def test_vfa_without_minit(vfa, oracle, name, w):
    t = wl.generate(w)
    print(name, _run_all(vfa, w, t, wl.all_blocks(w), oracle, use_minit=False), flush=True)


@pytest.mark.parametrize("name,w", SMALL[:5] + SMALL[6:9], ids=[n for n, _ in SMALL[:5] + SMALL[6:9]])
def test_kblock_summary_bit_exact(vfa, oracle, name, w):
    import torch
    t = wl.generate(w)
    K = to_gpu(t["K"])
    R = vfa.kblock_summary(K, w.block_n)
    torch.cuda.synchronize()
    got = R.float().cpu().numpy().astype(np.float64)
    want = oracle.sabsmax(wl.bf16_bits_to_f32(t["K"]), w.block_n)
    assert got.shape == want.shape and np.array_equal(got, want)


def test_kblock_summary_tie_takes_positive(vfa, oracle):
    import torch
    K = np.zeros((1, 1, 128, 64), np.float32)
    K[0, 0, 3, :] = -2.0
    K[0, 0, 40, :32] = 2.0          # tie in the first 32 dims: +2 wins
    K[0, 0, 70, 5] = -0.5
    bits = wl.f32_to_bf16_bits(K)
    R = vfa.kblock_summary(to_gpu(bits), 64).float().cpu().numpy().astype(np.float64)
    assert np.array_equal(R, oracle.sabsmax(K, 64))
    assert np.all(R[0, 0, 0, :32] == 2.0) and np.all(R[0, 0, 0, 32:] == -2.0) and R[0, 0, 1, 5] == -0.5


VSA_CASES = [
    ("cfg1_thr3", wl.small(wl.CONFIGS["cfg1"], beta=4.0), 3.0),
    ("small_thr4", W(B=1, Hq=4, Hkv=2, N=2048, beta=6.0, kappa=3.0), 4.0),
    ("small_thr8", W(B=1, Hq=2, Hkv=1, N=2048, beta=6.0, kappa=3.0), 8.0),
    ("noncausal_thr5", W(B=1, Hq=2, Hkv=2, N=1024, beta=6.0, kappa=3.0, causal=False), 5.0),
    ("ragged_thr4", W(B=1, Hq=2, Hkv=1, N=1000, beta=6.0, kappa=3.0), 4.0),
    ("d64_64x64_thr4", W(B=1, Hq=2, Hkv=1, N=1024, d=64, F=4, block_m=64, beta=6.0, kappa=3.0), 4.0),
    # one query head per KV head, causal: two adjacent query blocks share a workgroup (odd block count: one is alone)
    ("mha_causal_thr4_17blocks", W(B=1, Hq=2, Hkv=2, N=2176, beta=6.0, kappa=3.0), 4.0),
    ("gqa3_causal_thr6_ragged", W(B=1, Hq=3, Hkv=1, N=1900, beta=6.0, kappa=3.0), 6.0),
    ("mha_causal_thr4_no_local", W(B=1, Hq=2, Hkv=2, N=1024, beta=6.0, kappa=3.0, n_local=0), 4.0),
    ("mha_causal_thr4_local2_generic", W(B=1, Hq=2, Hkv=2, N=1024, beta=6.0, kappa=3.0, n_local=2), 4.0),
]


@pytest.mark.parametrize("name,w,thr", VSA_CASES, ids=[c[0] for c in VSA_CASES])
def test_vsa_mask_bit_exact_and_output(vfa, oracle, name, w, thr):
    import torch
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    blocks = wl.all_blocks(w)
    O, L, M = vfa.vsa_attn_fwd(Q, K, V, block_m=w.block_m, block_n=w.block_n, causal=w.causal, n_sink=w.n_sink,
                               n_local=w.n_local, skip_threshold_nats=thr)
    torch.cuda.synchronize()
    ref = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, n_sink=w.n_sink, n_local=w.n_local,
                        vsa=True, skip_threshold_nats=thr)
    got = M.cpu().numpy().reshape(len(blocks), w.Tc)
    near = np.abs(ref["margin"]) < MASK_GUARD_NATS            # NaN (not visited) compares False
    assert near.sum() == 0, "pick another seed: a tile sits on the threshold"
    assert np.array_equal(got, ref["mask"]), (name, int((got != ref["mask"]).sum()))
    sparsity = (ref["mask"] == 1).sum() / max(1, (ref["mask"] != 2).sum())
    stats = check_o_lse(O, L, ref["O"], ref["LSE"], blocks, w.block_m, w.N, "vsa_attn_fwd vs oracle VSA")
    print(name, "sparsity %.3f" % sparsity, stats, flush=True)
    assert sparsity > 0.02


# The VSA ping-pong kernel runs a step in a general or in a fast form, chosen per step from the visit list's shape
# (sink / local visits at the head, masked or ragged tiles at the tail, five visits of look-ahead).  Non-causal lengths
# put the same visit count on every query block, so a sweep over lengths walks the switch points one by one: no fast
# step at all, a single pair, a ragged last tile that shortens the fast range, sinks / locals that move its start.
STEP_FORM_CASES = [
    ("pairs_tc9", W(B=1, Hq=4, Hkv=2, N=576, beta=6.0, kappa=3.0, causal=False), 5.0),
    ("pairs_tc11", W(B=1, Hq=4, Hkv=2, N=704, beta=6.0, kappa=3.0, causal=False), 5.0),
    ("pairs_tc13_ragged", W(B=1, Hq=4, Hkv=2, N=801, beta=6.0, kappa=3.0, causal=False), 5.0),
    ("pairs_tc14", W(B=1, Hq=4, Hkv=2, N=896, beta=6.0, kappa=3.0, causal=False), 9.0),
    ("pairs_tc19_sink2", W(B=1, Hq=4, Hkv=2, N=1216, beta=6.0, kappa=3.0, causal=False, n_sink=2), 5.0),
    ("blocks_tc12", W(B=1, Hq=2, Hkv=2, N=768, beta=6.0, kappa=3.0, causal=False), 9.0),
    ("blocks_tc15_ragged", W(B=1, Hq=2, Hkv=2, N=930, beta=6.0, kappa=3.0, causal=False), 5.0),
    ("blocks_tc20_causal_ragged", W(B=1, Hq=2, Hkv=2, N=1250, beta=6.0, kappa=3.0), 4.0),
    ("pairs_tc24_causal_no_sink", W(B=1, Hq=4, Hkv=2, N=1536, beta=6.0, kappa=3.0, n_sink=0), 4.0),
]


@pytest.mark.parametrize("name,w,thr", STEP_FORM_CASES, ids=[c[0] for c in STEP_FORM_CASES])
def test_vsa_step_forms_switch_points(vfa, oracle, name, w, thr):
    import torch
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    blocks = wl.all_blocks(w)
    O, L, M = vfa.vsa_attn_fwd(Q, K, V, block_m=w.block_m, block_n=w.block_n, causal=w.causal, n_sink=w.n_sink,
                               n_local=w.n_local, skip_threshold_nats=thr)
    torch.cuda.synchronize()
    ref = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, n_sink=w.n_sink, n_local=w.n_local,
                        vsa=True, skip_threshold_nats=thr)
    got = M.cpu().numpy().reshape(len(blocks), w.Tc)
    near = np.abs(ref["margin"]) < MASK_GUARD_NATS
    assert near.sum() <= 2, "too many tiles sit on the threshold"
    assert np.array_equal(got[~near], ref["mask"][~near]), (name, int((got[~near] != ref["mask"][~near]).sum()))
    clean = ~near.any(axis=1)
    stats = check_o_lse(O, L, ref["O"][clean], ref["LSE"][clean], np.asarray(blocks)[clean], w.block_m, w.N,
                        "vsa_attn_fwd vs oracle VSA")
    kept = (ref["mask"] == 0).sum()
    skipped = (ref["mask"] == 1).sum()
    print(name, "kept %d skipped %d" % (kept, skipped), stats, flush=True)
    assert kept > 0 and skipped > 0, "the case should mix kept and skipped tiles"


def _random_shapes(n, seed):
    """Seeded shapes inside the library's domain: d, block_m, heads per KV head (even, odd, one), causal or not, 0-2 sink
    and 0-3 local blocks, lengths from a fraction of a tile to about 30 tiles, mostly ragged."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        d = int(rng.choice([64, 128], p=[0.3, 0.7]))
        g = int(rng.choice([1, 2, 3, 4]))
        Hkv = int(rng.choice([1, 2]))
        kw = dict(B=int(rng.choice([1, 2])), Hq=g * Hkv, Hkv=Hkv, N=int(rng.integers(40, 2000)), d=d,
                  block_m=int(rng.choice([64, 128], p=[0.3, 0.7])), causal=bool(rng.integers(0, 2)),
                  n_sink=int(rng.integers(0, 3)), n_local=int(rng.integers(0, 4)), beta=6.0, kappa=3.0)
        if kw["n_sink"] + kw["n_local"] == 0:
            kw["n_sink"] = 1
        if d == 64:
            kw["F"] = 4
        name = "r%d_d%d_bm%d_g%d_N%d_%s_s%dl%d" % (i, d, kw["block_m"], g, kw["N"], "c" if kw["causal"] else "nc",
                                                   kw["n_sink"], kw["n_local"])
        out.append((name, W(**kw), float(rng.choice([3.0, 4.0, 6.0]))))
    return out


RANDOM_SHAPES = _random_shapes(20, 20260412)


@pytest.mark.parametrize("name,w,thr", RANDOM_SHAPES, ids=[c[0] for c in RANDOM_SHAPES])
def test_random_shapes(vfa, oracle, name, w, thr):
    """Every forward entry point on shapes nobody picked by hand: the dense paths against exact attention and their own
    recurrences, Alg. 2 with the mask compared outside the guard band around the threshold."""
    import torch
    t = wl.generate(w)
    blocks = wl.all_blocks(w)
    print(name, _run_all(vfa, w, t, blocks, oracle), flush=True)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    O, L, M = vfa.vsa_attn_fwd(Q, K, V, block_m=w.block_m, block_n=w.block_n, causal=w.causal, n_sink=w.n_sink,
                               n_local=w.n_local, skip_threshold_nats=thr)
    torch.cuda.synchronize()
    ref = oracle.blocks(Qh, Kh, Vh, w.block_m, w.block_n, w.causal, blocks, n_sink=w.n_sink, n_local=w.n_local,
                        vsa=True, skip_threshold_nats=thr)
    got = M.cpu().numpy().reshape(len(blocks), w.Tc)
    near = np.abs(ref["margin"]) < MASK_GUARD_NATS
    assert near.sum() <= 2, "too many tiles sit on the threshold"
    assert np.array_equal(got[~near], ref["mask"][~near]), (name, int((got[~near] != ref["mask"][~near]).sum()))
    clean = ~near.any(axis=1)
    stats = check_o_lse(O, L, ref["O"][clean], ref["LSE"][clean], np.asarray(blocks)[clean], w.block_m, w.N,
                        "vsa_attn_fwd vs oracle VSA")
    print(name, "vsa kept %d skipped %d" % ((ref["mask"] == 0).sum(), (ref["mask"] == 1).sum()), stats, flush=True)


def test_vsa_huge_threshold_equals_vfa(vfa):
    """With a threshold nothing reaches Alg. 2 is Alg. 1.  The two kernels add a tile's row sum into l in a
    different order (Alg. 2 commits each tile's sum as one number once the block's decision is known), so
    the results agree to fp32 rounding of l, not bit for bit: one bf16 ulp in O, 1e-5 in LSE."""
    import torch
    w = W(B=1, Hq=2, Hkv=1, N=1024)
    Q, K, V = gpu_inputs(wl.generate(w))
    O1, L1 = vfa.vfa_attn_fwd(Q, K, V)
    O2, L2, M = vfa.vsa_attn_fwd(Q, K, V, skip_threshold_nats=1e4)
    torch.cuda.synchronize()
    o1, o2 = O1.float(), O2.float()
    assert ((o1 - o2).abs() <= 2.0 ** -7 * torch.maximum(o1.abs(), o2.abs()) + 1e-30).all()  # <= 1 ulp of bf16
    assert (o1 != o2).float().mean().item() < 0.02
    assert (L1 - L2).abs().max().item() <= 1e-5
    assert int((M == 1).sum()) == 0


def test_all_tiles_skipped_rows_are_zero(vfa, oracle):
    """Caller-supplied summaries (use_minit=2) far above every real score make m_init huge, so
    every tile of every row is skipped: O = 0, LSE = -inf, mask all ones."""
    import torch
    w = W(B=1, Hq=2, Hkv=1, N=512, causal=False, n_sink=0, n_local=0)
    t = wl.generate(w)
    t["Q"] = t["Q"] & np.uint16(0x7FFF)                       # |Q|: every query has positive entries only
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    blocks = wl.all_blocks(w)
    planted = np.full((1, 1, w.Tc, w.d), 4.0, np.float32)   # m_init ~ 35-45 nats above the real scores
    ws = torch.zeros(vfa.workspace_bytes(1, 1, w.N, w.d, 64), dtype=torch.uint8, device="cuda")
    ws.view(torch.bfloat16)[: planted.size] = to_gpu(wl.f32_to_bf16_bits(planted)).flatten()
    kw = dict(block_m=128, block_n=64, causal=False, n_sink=0, n_local=0, skip_threshold_nats=8.0)
    O, L, M = vfa.vsa_attn_fwd(Q, K, V, use_minit=2, workspace=ws, **kw)
    torch.cuda.synchronize()
    ref = oracle.blocks(Qh, Kh, Vh, 128, 64, False, blocks, n_sink=0, n_local=0, vsa=True, skip_threshold_nats=8.0,
                        krepr=planted.astype(np.float64))
    assert np.all(ref["mask"] == 1) and np.all(ref["O"] == 0) and np.all(np.isneginf(ref["LSE"]))
    assert int((M != 1).sum()) == 0
    assert float(O.float().abs().max()) == 0.0 and bool(torch.isneginf(L).all())
    # the same summaries through VFA (no skipping): m is far too high, the result is still exact attention
    O, L = vfa.vfa_attn_fwd(Q, K, V, use_minit=2, workspace=ws, block_m=128, block_n=64, causal=False, n_sink=0, n_local=0)
    torch.cuda.synchronize()
    Oe, Le, _ = oracle.exact(Qh, Kh, Vh, 128, False, blocks)
    check_o_lse(O, L, Oe, Le, blocks, 128, w.N, "vfa with an over-estimated frozen max")


def test_deterministic(vfa):
    import torch
    w = W(B=1, Hq=4, Hkv=2, N=2048, beta=6.0, kappa=3.0)
    Q, K, V = gpu_inputs(wl.generate(w))
    a = vfa.vfa_attn_fwd(Q, K, V)
    b = vfa.vfa_attn_fwd(Q, K, V)
    c = vfa.vsa_attn_fwd(Q, K, V, skip_threshold_nats=4.0)
    d = vfa.vsa_attn_fwd(Q, K, V, skip_threshold_nats=4.0)
    e = vfa.fa_baseline_fwd(Q, K, V)
    f = vfa.fa_baseline_fwd(Q, K, V)
    torch.cuda.synchronize()
    for x, y in zip(a + c + e, b + d + f):
        assert torch.equal(x, y)


def test_custom_scale_and_no_lse(vfa, oracle):
    import torch
    w = W(B=1, Hq=2, Hkv=1, N=512)
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    blocks = wl.all_blocks(w)
    O, L = vfa.vfa_attn_fwd(Q, K, V, softmax_scale=0.05)
    O2, L2 = vfa.vfa_attn_fwd(Q, K, V, softmax_scale=0.05, want_lse=False)
    torch.cuda.synchronize()
    assert L2 is None and torch.equal(O, O2)
    ref = oracle.blocks(Qh, Kh, Vh, 128, 64, True, blocks, scale=0.05)
    check_o_lse(O, L, ref["O"], ref["LSE"], blocks, 128, 512, "custom scale")


def test_graph_capture_and_side_stream(vfa, oracle):
    """The entry points only enqueue kernels on the given stream (no allocation, no synchronisation), so
    they can be captured into a HIP graph and replayed, and run on a stream other than the default one."""
    import torch
    w = W(B=1, Hq=4, Hkv=2, N=1024)
    t = wl.generate(w)
    Q, K, V = gpu_inputs(t)
    kw = dict(block_m=w.block_m, block_n=w.block_n, causal=w.causal)
    ws = torch.empty(vfa.workspace_bytes(w.B, w.Hkv, w.N, w.d, w.block_n), dtype=torch.uint8, device="cuda")
    O0, L0 = vfa.vfa_attn_fwd(Q, K, V, workspace=ws, **kw)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    O1, L1 = torch.empty_like(O0), torch.empty_like(L0)
    with torch.cuda.stream(side):
        vfa.vfa_attn_fwd(Q, K, V, workspace=ws, out=O1, lse=L1, **kw)
    side.synchronize()
    assert torch.equal(O0, O1) and torch.equal(L0, L1)
    O2, L2 = torch.empty_like(O0), torch.empty_like(L0)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        vfa.vfa_attn_fwd(Q, K, V, workspace=ws, out=O2, lse=L2, **kw)
    for rep in range(3):
        O2.zero_(); L2.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(O0, O2) and torch.equal(L0, L2), rep
