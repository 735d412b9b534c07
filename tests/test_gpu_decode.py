"""GPU parity of the decode path (vfa_kblock_summary_append, vfa_decode_fwd) against the float64
oracle.  Bars: O max-abs <= 2e-2, mean-abs <= 2e-3, LSE <= 1e-3 (as for prefill); summaries bit-exact."""
import numpy as np
import pytest

from paper_2604_12798_amd import workloads as wl

from gpu_util import LSE_ABS, O_MAX_ABS, O_MEAN_ABS, to_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vfa():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2604_12798_amd as pkg
    pkg.lib()
    return pkg


def _cache(B, Hq, Hkv, n_cap, d, seed=wl.DEFAULT_SEED, **kw):
    """A prefill-shaped seeded problem: K, V serve as the cache, row n-1 of Q as the query after n keys."""
    w = wl.small(wl.CONFIGS["cfg2"], B=B, Hq=Hq, Hkv=Hkv, N=n_cap, d=d, **kw)
    return wl.generate(w, seed)


def _check(vfa, oracle, t, n_keys, **kw):
    import torch
    Qb = np.ascontiguousarray(t["Q"][:, :, n_keys - 1])
    q, K, V = to_gpu(Qb), to_gpu(t["K"]), to_gpu(t["V"])
    B, Hkv, n_cap, d = K.shape
    R = torch.zeros((B, Hkv, -(-n_cap // 64), d), dtype=torch.bfloat16, device="cuda")
    vfa.kblock_summary_append(K, R, 0, n_keys)
    O, L = vfa.decode_fwd(q, K, V, n_keys, krepr=R, **kw)
    torch.cuda.synchronize()
    okw = {k: v for k, v in kw.items() if k in ("n_sink", "n_local", "use_minit")}
    ref = oracle.decode(wl.bf16_bits_to_f32(Qb), wl.bf16_bits_to_f32(t["K"]), wl.bf16_bits_to_f32(t["V"]), n_keys, 64, **okw)
    err = np.abs(O.float().cpu().numpy().astype(np.float64) - ref["O"])
    lerr = np.abs(L.cpu().numpy().astype(np.float64) - ref["LSE"]).max()
    stats = dict(max_abs=float(err.max()), mean_abs=float(err.mean()), lse=float(lerr))
    assert stats["max_abs"] <= O_MAX_ABS and stats["mean_abs"] <= O_MEAN_ABS and stats["lse"] <= LSE_ABS, stats
    return stats, (O, L)


CASES = [
    ("gqa4_1000keys_3splits", dict(B=2, Hq=8, Hkv=2, n_cap=1024, d=128), 1000, dict(n_splits=3)),
    ("gqa4_full_8splits", dict(B=1, Hq=8, Hkv=2, n_cap=2048, d=128), 2048, dict(n_splits=8)),
    ("mha_1key", dict(B=1, Hq=2, Hkv=2, n_cap=256, d=128), 1, dict(n_splits=4)),
    ("mha_65keys_more_splits_than_tiles", dict(B=1, Hq=2, Hkv=2, n_cap=256, d=128), 65, dict(n_splits=5)),
    ("gqa32_d64", dict(B=1, Hq=32, Hkv=1, n_cap=1024, d=64, F=4), 777, dict(n_splits=2)),
    ("no_minit", dict(B=1, Hq=4, Hkv=1, n_cap=1024, d=128), 900, dict(n_splits=4, use_minit=False)),
    ("sink2_local3_one_split", dict(B=1, Hq=4, Hkv=2, n_cap=1024, d=128), 1024, dict(n_splits=1, n_sink=2, n_local=3)),
    ("minit_only", dict(B=1, Hq=4, Hkv=2, n_cap=1024, d=128), 1024, dict(n_splits=4, n_sink=0, n_local=0)),
]


@pytest.mark.parametrize("name,shape,n_keys,kw", CASES, ids=[c[0] for c in CASES])
def test_decode_matches_oracle(vfa, oracle, name, shape, n_keys, kw):
    t = _cache(**shape)
    stats, _ = _check(vfa, oracle, t, n_keys, **kw)
    print(name, stats, flush=True)


def _random_decode_cases(n, seed):
    """Seeded decode shapes: heads per KV head from 1 to 32, d, cache capacity and fill, 1 to 24 key ranges (also more
    ranges than tiles), 0-2 sink and 0-3 local blocks, with and without the summary estimate."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        d = int(rng.choice([64, 128], p=[0.3, 0.7]))
        g = int(rng.choice([1, 2, 3, 4, 8, 32]))
        Hkv = int(rng.choice([1, 2])) if g < 32 else 1
        n_cap = int(rng.choice([320, 1024, 1536, 2500]))
        n_keys = int(rng.integers(1, n_cap + 1))
        kw = dict(n_splits=int(rng.integers(1, 25)), n_sink=int(rng.integers(0, 3)), n_local=int(rng.integers(0, 4)))
        if rng.integers(0, 4) == 0 and kw["n_sink"] + kw["n_local"] > 0:
            kw["use_minit"] = False
        shape = dict(B=int(rng.choice([1, 2, 3])), Hq=g * Hkv, Hkv=Hkv, n_cap=n_cap, d=d)
        if d == 64:
            shape["F"] = 4
        name = "r%d_d%d_g%d_%dof%d_s%d_sink%d_local%d%s" % (i, d, g, n_keys, n_cap, kw["n_splits"], kw["n_sink"], kw["n_local"],
                                                          "" if kw.get("use_minit", True) else "_noest")
        out.append((name, shape, n_keys, kw))
    return out


RANDOM_CASES = _random_decode_cases(16, 20260412)


@pytest.mark.parametrize("name,shape,n_keys,kw", RANDOM_CASES, ids=[c[0] for c in RANDOM_CASES])
def test_decode_random_shapes(vfa, oracle, name, shape, n_keys, kw):
    t = _cache(**shape)
    stats, _ = _check(vfa, oracle, t, n_keys, **kw)
    print(name, stats, flush=True)


def test_summary_append_equals_full_recompute(vfa, oracle):
    import torch
    t = _cache(B=2, Hq=2, Hkv=2, n_cap=1024, d=128)
    K = to_gpu(t["K"])
    Kh = wl.bf16_bits_to_f32(t["K"])
    R = torch.full((2, 2, 16, 128), 7.0, dtype=torch.bfloat16, device="cuda")   # stale contents must be overwritten
    n = 0
    for step in (1, 62, 1, 1, 200, 63, 400, 296):        # crosses block boundaries, fills partial blocks
        vfa.kblock_summary_append(K, R, n, n + step)
        n += step
        torch.cuda.synchronize()
        got = R.float().cpu().numpy().astype(np.float64)
        Tc = -(-n // 64)
        assert np.array_equal(got[:, :, :Tc], oracle.sabsmax(Kh[:, :, :n], 64)), n
        assert (got[:, :, Tc:] == 7.0).all()              # blocks without keys are not touched
    assert n == 1024
    full = vfa.kblock_summary(K, 64)
    torch.cuda.synchronize()
    assert torch.equal(full, R)


def test_decode_is_deterministic_and_split_count_only_changes_rounding(vfa, oracle):
    import torch
    t = _cache(B=1, Hq=8, Hkv=2, n_cap=4096, d=128)
    (_, (O1, L1)) = _check(vfa, oracle, t, 4000, n_splits=7)
    (_, (O2, L2)) = _check(vfa, oracle, t, 4000, n_splits=7)
    assert torch.equal(O1, O2) and torch.equal(L1, L2)
    (_, (O3, L3)) = _check(vfa, oracle, t, 4000, n_splits=1)
    assert (O1.float() - O3.float()).abs().max().item() <= 2e-2 and (L1 - L3).abs().max().item() <= 1e-5


def test_decode_growing_cache(vfa, oracle):
    """Token by token: append one key, refresh the summaries of its block, decode."""
    import torch
    t = _cache(B=1, Hq=4, Hkv=1, n_cap=256, d=128)
    K, V = to_gpu(t["K"]), to_gpu(t["V"])
    Kh, Vh = wl.bf16_bits_to_f32(t["K"]), wl.bf16_bits_to_f32(t["V"])
    R = torch.zeros((1, 1, 4, 128), dtype=torch.bfloat16, device="cuda")
    for n in range(1, 200, 13):
        vfa.kblock_summary_append(K, R, max(0, n - 13), n)
        Qb = np.ascontiguousarray(t["Q"][:, :, n - 1])
        O, L = vfa.decode_fwd(to_gpu(Qb), K, V, n, krepr=R, n_splits=2)
        torch.cuda.synchronize()
        ref = oracle.decode(wl.bf16_bits_to_f32(Qb), Kh, Vh, n, 64)
        assert np.abs(O.float().cpu().numpy() - ref["O"]).max() <= O_MAX_ABS
        assert np.abs(L.cpu().numpy() - ref["LSE"]).max() <= LSE_ABS


def test_decode_full_size_in_bench_configuration(vfa, oracle):
    """The decode workload and split count bench.py times, every query head checked."""
    import torch
    w, ns = wl.DECODE, wl.DECODE_SPLITS
    t = wl.generate_decode(w, w.N)
    q, K, V = to_gpu(t["q"]), to_gpu(t["K"]), to_gpu(t["V"])
    R = torch.empty((w.B, w.Hkv, w.Tc, w.d), dtype=torch.bfloat16, device="cuda")
    vfa.kblock_summary_append(K, R, 0, w.N)
    O, L = vfa.decode_fwd(q, K, V, w.N, krepr=R, n_splits=ns)
    torch.cuda.synchronize()
    ref = oracle.decode(wl.bf16_bits_to_f32(t["q"]), wl.bf16_bits_to_f32(t["K"]), wl.bf16_bits_to_f32(t["V"]), w.N, 64)
    err = np.abs(O.float().cpu().numpy().astype(np.float64) - ref["O"])
    lerr = np.abs(L.cpu().numpy().astype(np.float64) - ref["LSE"]).max()
    gap = ref["m_final"] - (ref["LSE"] - np.log(np.exp(ref["LSE"] - ref["m_final"])))  # = 0 by construction; kept finite check
    print("decode32k", dict(max_abs=float(err.max()), mean_abs=float(err.mean()), lse=float(lerr)),
          "fixed max minus m_init (nats): max %.2f" % float((ref["m_final"] - ref["m_init"]).max()), flush=True)
    assert np.isfinite(gap).all()
    assert err.max() <= O_MAX_ABS and err.mean() <= O_MEAN_ABS and lerr <= LSE_ABS


def _random_varlen_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = [("hand_picked", dict(B=4, Hq=8, Hkv=2, n_cap=1024, d=128), [1, 777, 1024, 130], 5)]
    for i in range(n):
        d = int(rng.choice([64, 128], p=[0.3, 0.7]))
        g, Hkv, B = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2])), int(rng.integers(2, 6))
        n_cap = int(rng.choice([256, 1024, 1984]))
        lens = [int(x) for x in rng.integers(1, n_cap + 1, size=B)]
        shape = dict(B=B, Hq=g * Hkv, Hkv=Hkv, n_cap=n_cap, d=d)
        if d == 64:
            shape["F"] = 4
        out.append(("r%d_d%d_g%d_cap%d_%s" % (i, d, g, n_cap, "_".join(map(str, lens))), shape, lens, int(rng.integers(1, 20))))
    return out


VARLEN_CASES = _random_varlen_cases(6, 20260412)


@pytest.mark.parametrize("name,shape,lens,n_splits", VARLEN_CASES, ids=[c[0] for c in VARLEN_CASES])
def test_decode_with_per_sequence_lengths(vfa, oracle, name, shape, lens, n_splits):
    """A batch of sequences of different lengths: summaries appended per sequence, one decode call;
    every sequence must equal the single-sequence oracle at its own length."""
    import torch
    B, Hq, Hkv, n_cap, d = shape["B"], shape["Hq"], shape["Hkv"], shape["n_cap"], shape["d"]
    t = _cache(**shape)
    K, V = to_gpu(t["K"]), to_gpu(t["V"])
    Kh, Vh = wl.bf16_bits_to_f32(t["K"]), wl.bf16_bits_to_f32(t["V"])
    lens = np.array(lens, np.int32)
    R = torch.full((B, Hkv, n_cap // 64, d), 3.0, dtype=torch.bfloat16, device="cuda")
    half = torch.from_numpy(lens // 2).cuda()
    full = torch.from_numpy(lens).cuda()
    vfa.kblock_summary_append_varlen(K, R, torch.zeros(B, dtype=torch.int32, device="cuda"), half)
    vfa.kblock_summary_append_varlen(K, R, half, full)                  # grow each sequence to its length
    Qb = np.stack([t["Q"][b, :, lens[b] - 1] for b in range(B)])         # [B, Hq, d]: each sequence's newest token
    O, L = vfa.decode_varlen_fwd(to_gpu(np.ascontiguousarray(Qb)), K, V, full, krepr=R, n_splits=n_splits)
    torch.cuda.synchronize()
    got_R = R.float().cpu().numpy().astype(np.float64)
    for b in range(B):
        n = int(lens[b])
        Tc = -(-n // 64)
        assert np.array_equal(got_R[b, :, :Tc], oracle.sabsmax(Kh[b:b + 1, :, :n], 64)[0])
        assert (got_R[b, :, Tc:] == 3.0).all()
        ref = oracle.decode(wl.bf16_bits_to_f32(Qb[b:b + 1]), Kh[b:b + 1], Vh[b:b + 1], n, 64)
        err = np.abs(O[b].float().cpu().numpy().astype(np.float64) - ref["O"][0])
        lerr = np.abs(L[b].cpu().numpy().astype(np.float64) - ref["LSE"][0]).max()
        assert err.max() <= O_MAX_ABS and err.mean() <= O_MEAN_ABS and lerr <= LSE_ABS, (b, n, err.max(), lerr)
