"""GPU parity of the FP8 (E4M3) path.  The pre-passes (quantise, pack V, summaries) are byte-exact against
the oracle's codec; the attention call is compared with the float64 oracle run on the DEQUANTISED
operands, so the only error left is the rounding of exp(S - m) to E4M3 (3 mantissa bits: relative
error <= 2^-4 per entry, which bounds |O_gpu - O| by 2^-4 * max|V| row by row) plus the bf16 output."""
import math

import numpy as np
import pytest

from paper_2604_12798_amd import workloads as wl

from gpu_util import LSE_ABS, gather_blocks, gpu_inputs, host_f32

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


def pow2_scale(x):
    """Per-tensor scale 2^k with max|x| / scale <= 448 (a power of two keeps the dequantised values exact in float32)."""
    return 2.0 ** math.ceil(math.log2(float(np.abs(x).max()) / 448.0))


def folding_scale(x, sk, d):
    """Scale for Q that makes descale_q * descale_k * softmax_scale * log2(e) a power of two (the smallest
    such scale that still keeps max|x| / scale <= 448): the library then moves that factor into the MFMA."""
    rest = sk * (1.0 / math.sqrt(d)) * math.log2(math.e)
    e = math.ceil(math.log2(float(np.abs(x).max()) / 448.0 * rest))
    return float(np.float32(2.0 ** e / rest))


def quantised_problem(vfa, oracle, w, seed=wl.DEFAULT_SEED, fold=False):
    import torch
    t = wl.generate(w, seed)
    Q, K, V = gpu_inputs(t)
    Qh, Kh, Vh = host_f32(t)
    sq, sk, sv = pow2_scale(Qh), pow2_scale(Kh), pow2_scale(Vh)
    if fold:
        sq = folding_scale(Qh, sk, w.d)
    Q8, K8 = vfa.fp8_quantize(Q, 1 / sq), vfa.fp8_quantize(K, 1 / sk)
    Vt8 = vfa.fp8_pack_v(V, 1 / sv)
    torch.cuda.synchronize()
    cq, ck, cv = (oracle.e4m3_quantize(x, 1 / s) for x, s in ((Qh, sq), (Kh, sk), (Vh, sv)))
    return dict(Q8=Q8, K8=K8, Vt8=Vt8, sq=sq, sk=sk, sv=sv, cq=cq, ck=ck, cv=cv,
                Qd=oracle.e4m3_dequantize(cq, sq).astype(np.float32), Kd=oracle.e4m3_dequantize(ck, sk).astype(np.float32),
                Vd=oracle.e4m3_dequantize(cv, sv).astype(np.float32))


SHAPES = [
    ("gqa_causal_1024", W(B=2, Hq=4, Hkv=2, N=1024)),
    ("mha_noncausal_768", W(B=1, Hq=2, Hkv=2, N=768, causal=False)),
    ("ragged_1000", W(B=1, Hq=2, Hkv=1, N=1000)),
    ("sink2_local2", W(B=1, Hq=2, Hkv=2, N=1280, n_sink=2, n_local=2)),
    ("two_tiles_65", W(B=1, Hq=2, Hkv=1, N=65)),
    ("one_key", W(B=2, Hq=2, Hkv=2, N=1)),
]


def _random_shapes(n, seed):
    """Seeded shapes inside this path's domain (d = 128, 128 x 64 blocks): batch, heads per KV head, causal or not,
    1-2 sink and 1-3 local blocks, lengths from a fraction of a tile to about 30 tiles, mostly ragged.  Sink and local
    blocks are always visited: 8-bit weights are capped at 1, so a frozen max more than the headroom (2.77 nats) below
    the true one changes the result, and on this data the summary estimate alone is up to 4.7 nats low without the exact
    visit of the sink tile and 2.5 (E4M3 operands) to 3 nats (MXFP4) low without that of the diagonal (the capped regime
    has its own test: finite, not NaN)."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        g, Hkv = int(rng.choice([1, 2, 3, 4])), int(rng.choice([1, 2]))
        kw = dict(B=int(rng.choice([1, 2])), Hq=g * Hkv, Hkv=Hkv, N=int(rng.integers(30, 2000)), causal=bool(rng.integers(0, 2)),
                  n_sink=int(rng.integers(1, 3)), n_local=int(rng.integers(1, 4)))
        out.append(("r%d_g%d_N%d_%s_s%dl%d" % (i, g, kw["N"], "c" if kw["causal"] else "nc", kw["n_sink"], kw["n_local"]), W(**kw)))
    return out


RANDOM_SHAPES = _random_shapes(8, 20260412)


@pytest.mark.parametrize("name,w", SHAPES[:3], ids=[s[0] for s in SHAPES[:3]])
def test_prepasses_are_byte_exact(vfa, oracle, name, w):
    pr = quantised_problem(vfa, oracle, w)
    assert np.array_equal(pr["Q8"].cpu().numpy(), pr["cq"]) and np.array_equal(pr["K8"].cpu().numpy(), pr["ck"])
    # V: per 64-key tile, [feature][byte 32 h + j] = code of key 32 (j // 16) + 8 ((j % 16) // 4) + 4 h + j % 4, zero past N
    B, Hkv, N, d = pr["cv"].shape
    Tc = -(-N // 64)
    pad = np.zeros((B, Hkv, Tc * 64, d), np.uint8)
    pad[:, :, :N] = pr["cv"]
    j = np.arange(32)
    order = np.concatenate([32 * (j // 16) + 8 * ((j % 16) // 4) + 4 * h + j % 4 for h in (0, 1)])
    assert sorted(order) == list(range(64))
    want = pad.reshape(B, Hkv, Tc, 64, d)[:, :, :, order, :].transpose(0, 1, 2, 4, 3)
    assert np.array_equal(pr["Vt8"].cpu().numpy(), want)


@pytest.mark.parametrize("name,w", SHAPES[:3] + SHAPES[4:], ids=[s[0] for s in SHAPES[:3] + SHAPES[4:]])
def test_fp8_summaries_are_byte_exact(vfa, oracle, name, w):
    """Summary of a key block = sabsmax of its dequantised keys = again an E4M3 code of that block (per-tensor scale)."""
    import torch
    pr = quantised_problem(vfa, oracle, w)
    ws = torch.zeros(max(256, w.B * w.Hkv * w.Tc * 128), dtype=torch.uint8, device=pr["Q8"].device)
    vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], frozen=True, descale_q=pr["sq"], descale_k=pr["sk"], descale_v=pr["sv"],
                     causal=w.causal, n_sink=w.n_sink, n_local=w.n_local, workspace=ws)
    torch.cuda.synchronize()
    got = ws.cpu().numpy()[:w.B * w.Hkv * w.Tc * 128].reshape(w.B, w.Hkv, w.Tc, 128)
    want = oracle.e4m3_quantize(oracle.sabsmax(pr["Kd"], w.block_n).astype(np.float32), 1 / pr["sk"])
    zero = lambda c: np.where(c == 0x80, 0, c)       # a column of zeros may carry either sign
    assert np.array_equal(zero(got), zero(want))


@pytest.mark.parametrize("name,w", SHAPES + RANDOM_SHAPES, ids=[s[0] for s in SHAPES + RANDOM_SHAPES])
def test_fp8_attention_matches_oracle_on_dequantised_operands(vfa, oracle, name, w):
    import torch
    pr = quantised_problem(vfa, oracle, w)
    blocks = wl.all_blocks(w)
    Oe, Le, Me = oracle.exact(pr["Qd"], pr["Kd"], pr["Vd"], w.block_m, w.causal, blocks)
    vmax = float(np.abs(pr["Vd"]).max())
    kw = dict(descale_q=pr["sq"], descale_k=pr["sk"], descale_v=pr["sv"], block_m=w.block_m, block_n=w.block_n, causal=w.causal)
    for frozen in (False, True):
        O, L = vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], frozen=frozen, n_sink=w.n_sink, n_local=w.n_local, **kw)
        torch.cuda.synchronize()
        got_O, got_L = gather_blocks(O, blocks, w.block_m, w.N), gather_blocks(L, blocks, w.block_m, w.N)
        valid = ~np.isnan(Le)
        assert not np.isnan(got_O[valid]).any()
        err = np.abs(got_O[valid] - Oe[valid])
        lerr = np.abs(got_L[valid] - Le[valid]).max()
        print(name, "frozen" if frozen else "online", "max_abs %.4f mean_abs %.5f lse %.2e (bound %.3f)" % (err.max(), err.mean(), lerr, vmax / 16), flush=True)
        # 2^-4 |V|max is the hard bound of the E4M3 rounding of P; bf16 output rounding and entries below 2^-9 add a little
        assert err.max() <= vmax / 16 * 1.05 + 2e-2
        assert err.mean() <= vmax / 16 / 8
        assert lerr <= LSE_ABS
    if w.causal:   # the frozen run really froze: its summaries are the sabsmax of the codes
        ref = oracle.blocks(pr["Qd"], pr["Kd"], pr["Vd"], w.block_m, w.block_n, True, blocks, n_sink=w.n_sink, n_local=w.n_local)
        gap = (Me - ref["m_final"])[~np.isnan(Me)]
        print(name, "true max above frozen max (nats): max %.2f (headroom 2.77)" % gap.max(), flush=True)
        assert gap.max() < 2.77


@pytest.mark.parametrize("name,w", SHAPES + RANDOM_SHAPES, ids=[s[0] for s in SHAPES + RANDOM_SHAPES])
def test_fp8_folded_scale_matches_oracle(vfa, oracle, name, w):
    """Alg. 1 with Q quantised so that the factor between code products and log2-domain scores is a power of
    two: the library then applies it inside the MFMA and starts the accumulators of frozen tiles at -(m + H).
    Same bars as the unfolded path, against the oracle on these (differently scaled) dequantised operands; and
    the two paths must agree with each other on the SAME operands when the fold is defeated by one ulp."""
    import torch
    pr = quantised_problem(vfa, oracle, w, fold=True)
    assert np.array_equal(pr["Q8"].cpu().numpy(), pr["cq"])
    blocks = wl.all_blocks(w)
    Oe, Le, Me = oracle.exact(pr["Qd"], pr["Kd"], pr["Vd"], w.block_m, w.causal, blocks)
    vmax = float(np.abs(pr["Vd"]).max())
    kw = dict(descale_k=pr["sk"], descale_v=pr["sv"], block_m=w.block_m, block_n=w.block_n, causal=w.causal,
              frozen=True, n_sink=w.n_sink, n_local=w.n_local)
    O, L = vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], descale_q=pr["sq"], **kw)
    torch.cuda.synchronize()
    got_O, got_L = gather_blocks(O, blocks, w.block_m, w.N), gather_blocks(L, blocks, w.block_m, w.N)
    valid = ~np.isnan(Le)
    assert not np.isnan(got_O[valid]).any()
    err = np.abs(got_O[valid] - Oe[valid])
    lerr = np.abs(got_L[valid] - Le[valid]).max()
    print(name, "folded max_abs %.4f mean_abs %.5f lse %.2e (bound %.3f)" % (err.max(), err.mean(), lerr, vmax / 16), flush=True)
    assert err.max() <= vmax / 16 * 1.05 + 2e-2 and err.mean() <= vmax / 16 / 8 and lerr <= LSE_ABS
    # descale_q off by 2^-12: no power of two any more, so the ordinary path runs, on scores 2^-12 (relative) apart
    O2, L2 = vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], descale_q=pr["sq"] * (1 + 2.0 ** -12), **kw)
    torch.cuda.synchronize()
    dO = (O.float() - O2.float()).abs().max().item()
    dO_mean = (O.float() - O2.float()).abs().mean().item()
    dL = (L - L2).abs().max().item()
    print(name, "folded vs unfolded: max |dO| %.4f mean %.5f max |dLSE| %.2e" % (dO, dO_mean, dL), flush=True)
    # each path is within vmax / 16 (+ rounding) of the exact result, so two of them are within twice that of each
    # other; the hand-picked shapes stay at the single bound they have always met.  A one-step flip of an E4M3 weight
    # code (6 % of the weight) under a 2^-12 change of the scores is what separates the paths, so the mean is tiny
    hand_picked = any(name == n for n, _ in SHAPES)
    assert dO <= (1 if hand_picked else 2) * (vmax / 16 * 1.05 + 2e-2) and dO_mean <= vmax / 16 / 8 and dL <= 2e-2


def test_fp8_frozen_max_far_too_low_is_capped_not_nan(vfa, oracle):
    """No m-init and a single local block: rows whose maximum lies in a far (frozen) tile exceed the 4-binade
    headroom; the result is then not exact, but it must stay finite and normalised (|O| <= max|V|)."""
    import torch
    w = W("cfg4", B=1, Hq=2, Hkv=2, N=2048)
    pr = quantised_problem(vfa, oracle, w)
    O, L = vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], frozen=True, use_minit=False, n_sink=1, n_local=1,
                            descale_q=pr["sq"], descale_k=pr["sk"], descale_v=pr["sv"], causal=False)
    torch.cuda.synchronize()
    o = O.float().cpu().numpy()
    assert np.isfinite(o).all() and np.isfinite(L.cpu().numpy()).all()
    assert np.abs(o).max() <= float(np.abs(pr["Vd"]).max()) * 1.01


def test_fp8_noexp_full_size_sampled_blocks(vfa, oracle):
    """cfg3 in the launch configuration bench.py times, checked on a sample of query blocks."""
    import torch
    w = wl.CONFIGS["cfg3"]
    pr = quantised_problem(vfa, oracle, w, fold=True)
    blocks = wl.sample_blocks(w, 6)
    Oe, Le, Me = oracle.exact(pr["Qd"], pr["Kd"], pr["Vd"], w.block_m, w.causal, blocks)
    vmax = float(np.abs(pr["Vd"]).max())
    O, L = vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], noexp=True, n_sink=w.n_sink, n_local=w.n_local, descale_q=pr["sq"],
                            descale_k=pr["sk"], descale_v=pr["sv"], block_m=w.block_m, block_n=w.block_n, causal=w.causal)
    torch.cuda.synchronize()
    got_O, got_L = gather_blocks(O, blocks, w.block_m, w.N), gather_blocks(L, blocks, w.block_m, w.N)
    err = np.abs(got_O - Oe)
    lerr = np.abs(got_L - Le).max()
    print("cfg3 fp8 no exp max_abs %.4f mean_abs %.5f lse %.3f" % (err.max(), err.mean(), lerr), flush=True)
    assert not np.isnan(got_O).any()
    assert err.max() <= vmax / 8 * 1.05 + 2e-2 and err.mean() <= vmax / 8 / 8 and lerr <= 0.12


def test_fp8_full_size_sampled_blocks(vfa, oracle):
    """cfg3 in the launch configuration bench.py times, checked on a sample of query blocks."""
    import torch
    w = wl.CONFIGS["cfg3"]
    pr = quantised_problem(vfa, oracle, w)
    blocks = wl.sample_blocks(w, 6)
    Oe, Le, Me = oracle.exact(pr["Qd"], pr["Kd"], pr["Vd"], w.block_m, w.causal, blocks)
    vmax = float(np.abs(pr["Vd"]).max())
    kw = dict(descale_q=pr["sq"], descale_k=pr["sk"], descale_v=pr["sv"], block_m=w.block_m, block_n=w.block_n, causal=w.causal)
    for frozen in (False, True):
        O, L = vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], frozen=frozen, n_sink=w.n_sink, n_local=w.n_local, **kw)
        torch.cuda.synchronize()
        got_O, got_L = gather_blocks(O, blocks, w.block_m, w.N), gather_blocks(L, blocks, w.block_m, w.N)
        err = np.abs(got_O - Oe)
        lerr = np.abs(got_L - Le).max()
        print("cfg3 fp8", "frozen" if frozen else "online", "max_abs %.4f mean_abs %.5f lse %.2e" % (err.max(), err.mean(), lerr), flush=True)
        assert not np.isnan(got_O).any()
        assert err.max() <= vmax / 16 * 1.05 + 2e-2 and err.mean() <= vmax / 16 / 8 and lerr <= LSE_ABS


@pytest.mark.parametrize("name,w", SHAPES, ids=[s[0] for s in SHAPES])
def test_fp8_noexp_matches_oracle_within_the_code_error(vfa, oracle, name, w):
    """Alg. 1 with the weights' E5M2 codes taken straight from the scores (no exponential): every weight is within
    [0.89, 1.12] of the exact one and the row sum uses the same weights, so with eps = 0.12
    |O - O_exact| <= 2 eps / (1 - eps) max|V| in the worst case (two keys with opposite V and opposite errors; plus the
    bf16 output) and |LSE - LSE_exact| <= -ln 0.89 = 0.117; typical rows average the errors out."""
    import torch
    pr = quantised_problem(vfa, oracle, w, fold=True)
    blocks = wl.all_blocks(w)
    Oe, Le, Me = oracle.exact(pr["Qd"], pr["Kd"], pr["Vd"], w.block_m, w.causal, blocks)
    vmax = float(np.abs(pr["Vd"]).max())
    kw = dict(descale_k=pr["sk"], descale_v=pr["sv"], block_m=w.block_m, block_n=w.block_n, causal=w.causal,
              n_sink=w.n_sink, n_local=w.n_local)
    O, L = vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], descale_q=pr["sq"], noexp=True, **kw)
    torch.cuda.synchronize()
    got_O, got_L = gather_blocks(O, blocks, w.block_m, w.N), gather_blocks(L, blocks, w.block_m, w.N)
    valid = ~np.isnan(Le)
    assert not np.isnan(got_O[valid]).any()
    err = np.abs(got_O[valid] - Oe[valid])
    lerr = got_L[valid] - Le[valid]
    eps = 0.12
    print(name, "noexp max_abs %.4f mean_abs %.5f lse err min %.4f max %.4f mean |.| %.4f (worst-case bound %.3f)" %
          (err.max(), err.mean(), lerr.min(), lerr.max(), np.abs(lerr).mean(), 2 * eps / (1 - eps) * vmax), flush=True)
    assert err.max() <= vmax / 8 * 1.05 + 2e-2             # in practice inside the bar of properly rounded E5M2 weights
    assert err.mean() <= vmax / 8 / 8
    assert -0.12 <= lerr.min() and lerr.max() <= 0.12
    # a scale that is not a power of two cannot be folded into the matrix instruction: refused, not approximated
    with pytest.raises(vfa.VfaError):
        vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], descale_q=pr["sq"] * 1.01, noexp=True, **kw)


def test_fp8_noexp_frozen_max_far_too_low_is_capped_not_nan(vfa, oracle):
    """No m-init and a single local block: rows whose maximum lies in a far (frozen) tile exceed the headroom; their
    codes are clamped to the largest finite one, so the result is not exact but stays finite and normalised."""
    import torch
    w = W("cfg4", B=1, Hq=2, Hkv=2, N=2048)
    pr = quantised_problem(vfa, oracle, w, fold=True)
    O, L = vfa.fp8_attn_fwd(pr["Q8"], pr["K8"], pr["Vt8"], noexp=True, use_minit=False, n_sink=1, n_local=1,
                            descale_q=pr["sq"], descale_k=pr["sk"], descale_v=pr["sv"], causal=False)
    torch.cuda.synchronize()
    o = O.float().cpu().numpy()
    assert np.isfinite(o).all() and np.isfinite(L.cpu().numpy()).all()
    assert np.abs(o).max() <= float(np.abs(pr["Vd"]).max()) * 1.01
