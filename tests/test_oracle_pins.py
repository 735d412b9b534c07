"""Pins for the CPU oracle: each test ties one part of it to something the paper or the
mathematics fixes (a library routine, a closed form, an invariant, a hand-worked value),
so that a dropped term, wrong sign, wrong index or transposed operand fails somewhere."""
import math
import os

import numpy as np
import pytest
import scipy.special

from paper_2604_12798_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def lib_attention(Q, K, V, causal, scale):
    """Whole-matrix softmax attention from library routines (numpy matmul, scipy softmax)."""
    S = scale * (Q.astype(np.float64) @ K.astype(np.float64).T)
    if causal:
        S = np.where(np.tril(np.ones_like(S, dtype=bool)), S, -np.inf)
    P = scipy.special.softmax(S, axis=1)
    return P, P @ V.astype(np.float64), scipy.special.logsumexp(S, axis=1), S


# ------------------------------------------------------------------ brute force and exact rows
@pytest.mark.parametrize("N,d,causal", [(7, 3, False), (7, 3, True), (33, 16, True), (64, 8, False)])
def test_brute_matches_library_softmax(oracle, N, d, causal):
    Q, K, V = rnd(1, N, d), rnd(2, N, d), rnd(3, N, d)
    scale = 0.37
    P, O, L = oracle.brute(Q, K, V, causal, scale)
    Pl, Ol, Ll, _ = lib_attention(Q, K, V, causal, scale)
    assert np.abs(P - Pl).max() < 1e-14
    assert np.abs(O - Ol).max() < 1e-13
    assert np.abs(L - Ll).max() < 1e-13
    assert np.abs(P.sum(1) - 1).max() < 1e-13                      # rows of P sum to one
    if causal:
        assert np.all(np.triu(P, 1) == 0)                          # no weight on future keys


def test_hand_worked_two_keys(oracle):
    # s = q*k with scale 1: scores (0, ln 2) -> P = (1/3, 2/3); V = (3, 6) -> O = 5, LSE = ln 3
    Q = np.array([[1.0], [1.0]], np.float32)
    K = np.array([[0.0], [math.log(2.0)]], np.float32)
    V = np.array([[3.0], [6.0]], np.float32)
    P, O, L = oracle.brute(Q, K, V, False, 1.0)
    k1 = float(K[1, 0])
    p1 = math.exp(k1) / (1 + math.exp(k1))
    assert abs(P[1, 1] - p1) < 1e-15 and abs(O[1, 0] - (3 + 3 * p1)) < 1e-14
    assert abs(O[1, 0] - 5.0) < 1e-6 and abs(L[1] - math.log(3.0)) < 1e-6
    P, O, L = oracle.brute(Q, K, V, True, 1.0)
    assert O[0, 0] == 3.0 and L[0] == 0.0                          # causal: row 0 sees key 0 only


def test_uniform_keys_closed_form(oracle):
    # identical keys => uniform P => O = (prefix) mean of V, LSE = s + ln(n)
    N, d = 40, 8
    Q, V = rnd(4, 1, 2, N, d), rnd(5, 1, 1, N, d)
    K = np.tile(rnd(6, 1, 1, 1, d), (1, 1, N, 1))
    blocks = np.array([(0, h, i) for h in range(2) for i in range(3)], np.int32)
    O, L, M = oracle.exact(Q, K, V, 16, True, blocks)
    for n, (b, h, i) in enumerate(blocks):
        for rr in range(16):
            r = i * 16 + rr
            if r >= N:
                assert np.isnan(O[n, rr]).all()
                continue
            s = float(Q[0, h, r].astype(np.float64) @ K[0, 0, 0].astype(np.float64)) / math.sqrt(d)
            assert np.abs(O[n, rr] - V[0, 0, : r + 1].astype(np.float64).mean(0)).max() < 1e-13
            assert abs(L[n, rr] - (s + math.log(r + 1))) < 1e-12 and abs(M[n, rr] - s) < 1e-12


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("g", [1, 2, 4])
def test_exact_rows_match_brute_gqa(oracle, causal, g):
    B, Hkv, N, d, bm = 2, 2, 50, 12, 16
    Hq = Hkv * g
    Q, K, V = rnd(7, B, Hq, N, d), rnd(8, B, Hkv, N, d), rnd(9, B, Hkv, N, d)
    blocks = np.array([(b, h, i) for b in range(B) for h in range(Hq) for i in range(4)], np.int32)
    O, L, M = oracle.exact(Q, K, V, bm, causal, blocks)
    for n, (b, h, i) in enumerate(blocks):
        _, Ob, Lb, S = lib_attention(Q[b, h], K[b, h // g], V[b, h // g], causal, 1 / math.sqrt(d))
        rows = slice(i * bm, min(N, (i + 1) * bm))
        nr = rows.stop - rows.start
        assert np.abs(O[n, :nr] - Ob[rows]).max() < 1e-13
        assert np.abs(L[n, :nr] - Lb[rows]).max() < 1e-13
        assert np.abs(M[n, :nr] - S[rows].max(1)).max() < 1e-13


# ------------------------------------------------------------------ sabsmax
def test_sabsmax_golden(oracle):
    for line in open(os.path.join(GOLDEN, "sabsmax_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        lhs, rhs = line.split("=>")
        block = np.array([[float(x) for x in row.split()] for row in lhs.split(";")], np.float32)
        want = np.array([float(x) for x in rhs.split()])
        got = oracle.sabsmax(block[None, None], block.shape[0])[0, 0, 0]
        assert np.array_equal(got, want), (block, got, want)


def test_sabsmax_properties(oracle):
    K = rnd(10, 2, 3, 70, 5)
    for bn in (16, 32):
        R = oracle.sabsmax(K, bn)
        Tc = -(-70 // bn)
        assert R.shape == (2, 3, Tc, 5)
        for j in range(Tc):
            blk = K[:, :, j * bn: min(70, (j + 1) * bn)].astype(np.float64)
            assert np.array_equal(np.abs(R[:, :, j]), np.abs(blk).max(2))          # magnitude = absmax
            assert np.all((blk == R[:, :, j][:, :, None, :]).any(2))               # an element of the block
    # order of keys inside a block is irrelevant
    perm = np.random.default_rng(0).permutation(16)
    K2 = K[:, :, :64].copy().reshape(2, 3, 4, 16, 5)[:, :, :, perm].reshape(2, 3, 64, 5)
    assert np.array_equal(oracle.sabsmax(K[:, :, :64], 16), oracle.sabsmax(K2, 16))


def test_alternative_block_representations_hand_worked(oracle):
    """The ablated summaries (Experiments, ablation of the k_repr construction) on the block
    [[1,-3],[-2,2]], worked by hand: per-dimension max [1, 2], mean [-0.5, -0.5], magnitude
    without sign [2, 3]; the method's signed extreme is [-2, -3]."""
    blk = np.array([[1, -3], [-2, 2]], np.float32)[None, None]
    for mode, want in ((0, [-2.0, -3.0]), (1, [1.0, 2.0]), (2, [-0.5, -0.5]), (3, [2.0, 3.0])):
        assert np.array_equal(oracle.sabsmax(blk, 2, mode)[0, 0, 0], want), mode
    # an all-negative column: the maximum is the element closest to zero, not the extreme
    neg = np.array([[-1, 4], [-5, -4], [-3, 0]], np.float32)[None, None]
    assert np.array_equal(oracle.sabsmax(neg, 3, 1)[0, 0, 0], [-1.0, 4.0])
    assert np.array_equal(oracle.sabsmax(neg, 3, 3)[0, 0, 0], [5.0, 4.0])
    assert np.array_equal(oracle.sabsmax(neg, 3, 2)[0, 0, 0], [-3.0, 0.0])


@pytest.mark.parametrize("bn", [8, 16, 32])
def test_alternative_block_representations_match_library_reductions(oracle, bn):
    """Modes 1, 2, 3 over key blocks against numpy's max / mean / abs-max, block by block, with a
    ragged last block (70 keys) reduced over its valid rows only."""
    N = 70
    K = rnd(17, 2, 3, N, 5)
    K[0, 1, 3:9] -= 6.0           # a block whose entries are all negative in every dimension
    lib = {1: lambda x: x.max(2), 2: lambda x: x.mean(2), 3: lambda x: np.abs(x).max(2)}
    Tc = -(-N // bn)
    for mode, f in lib.items():
        R = oracle.sabsmax(K, bn, mode)
        assert R.shape == (2, 3, Tc, 5)
        for j in range(Tc):
            blk = K[:, :, j * bn: min(N, (j + 1) * bn)].astype(np.float64)
            want = f(blk)
            if mode == 2:
                assert np.abs(R[:, :, j] - want).max() < 1e-15, (mode, j)
            else:
                assert np.array_equal(R[:, :, j], want), (mode, j)
    # orderings that separate the four summaries from one another on generic data
    R0, R1, R2, R3 = (oracle.sabsmax(K, bn, m) for m in range(4))
    assert np.all(R1 <= R3) and np.all(np.abs(R0) == R3) and np.all(R2 <= R1)
    assert (R1 < R3).any() and (R0 != R1).any()


# ------------------------------------------------------------------ visit order
def test_visit_order_golden(oracle):
    for line in open(os.path.join(GOLDEN, "visit_order.txt")):
        if line.startswith("#") or not line.strip():
            continue
        lhs, rhs = line.split(":")
        Tc, i = (int(x) for x in lhs.split())
        want = [int(x) - 1 for x in rhs.split()]
        j, s = oracle.visit_list(Tc * 8, 8, 8, False, i - 1, 1, 1)
        assert list(j) == want
        assert [int(x) for x in s] == [1 if (b == 0 or b == i - 1) else 0 for b in want]


@pytest.mark.parametrize("bm,bn", [(8, 8), (16, 8), (8, 16), (24, 8)])
@pytest.mark.parametrize("causal", [False, True])
def test_visit_list_is_a_permutation_of_visible_blocks(oracle, bm, bn, causal):
    N = 100
    Tc = -(-N // bn)
    for n_sink, n_local in [(0, 0), (1, 1), (2, 1), (1, 3), (0, 2), (3, 0)]:
        for i in range(-(-N // bm)):
            j, s = oracle.visit_list(N, bm, bn, causal, i, n_sink, n_local)
            last_row = min(N, (i + 1) * bm) - 1
            j_hi = last_row // bn if causal else Tc - 1
            assert sorted(j) == list(range(j_hi + 1))                               # each visible block once
            a_lo, a_hi = (i * bm) // bn, last_row // bn
            special = {b for b in range(min(n_sink, j_hi + 1))}
            if n_local > 0:
                special |= set(range(max(0, a_lo - (n_local - 1)), min(a_hi, j_hi) + 1))
            assert {int(b) for b, f in zip(j, s) if f} == special
            k = len(special)
            assert set(int(b) for b in j[:k]) == special                            # special blocks come first
            assert list(j[k:]) == sorted(j[k:])                                      # the rest ascending
            j0, s0 = oracle.visit_list(N, bm, bn, causal, i, n_sink, n_local, reorder=False)
            assert list(j0) == list(range(j_hi + 1))                                 # "w/o reorder": ascending
            assert {int(b) for b, f in zip(j0, s0) if f} == special


# ------------------------------------------------------------------ m-initialisation
def test_m_init_is_max_of_q_dot_summaries(oracle):
    B, Hq, Hkv, N, d, bm, bn = 1, 4, 2, 96, 8, 16, 8
    Q, K, V = rnd(11, B, Hq, N, d), rnd(12, B, Hkv, N, d), rnd(13, B, Hkv, N, d)
    R = oracle.sabsmax(K, bn)
    blocks = np.array([(0, h, i) for h in range(Hq) for i in range(N // bm)], np.int32)
    for causal in (False, True):
        out = oracle.blocks(Q, K, V, bm, bn, causal, blocks)
        for n, (b, h, i) in enumerate(blocks):
            j_hi = ((i + 1) * bm - 1) // bn if causal else N // bn - 1
            approx = (Q[0, h, i * bm:(i + 1) * bm].astype(np.float64) @ R[0, h // 2, : j_hi + 1].T) / math.sqrt(d)
            assert np.abs(out["m_init"][n] - approx.max(1)).max() < 1e-13


# ------------------------------------------------------------------ block-wise q_repr ablation
def test_blockwise_q_repr_hand_worked(oracle):
    """One query block [[1,-2],[-3,1]], one key block holding [2,1] twice, scale 1 (values worked by hand):
    absmax(Q) = [3,2], sabsmax(Q) = [-3,-2], mean(Q) = [-1,-0.5]; k_repr = [2,1];
    seeds 8, -8, -2.5 for both rows, where the row-wise method gives 0 and -5."""
    Q = np.array([[1, -2], [-3, 1]], np.float32).reshape(1, 1, 2, 2)
    K = np.array([[2, 1], [2, 1]], np.float32).reshape(1, 1, 2, 2)   # the key twice, as one block
    V = np.array([[1, 0], [0, 1]], np.float32).reshape(1, 1, 2, 2)
    blocks = np.array([(0, 0, 0)], np.int32)
    kw = dict(n_sink=0, n_local=0, scale=1.0)
    assert np.array_equal(oracle.blocks(Q, K, V, 2, 2, False, blocks, **kw)["m_init"][0], [0.0, -5.0])
    for mode, seed in ((3, 8.0), (0, -8.0), (2, -2.5)):
        qr = oracle.sabsmax(Q, 2, mode)
        out = oracle.blocks(Q, K, V, 2, 2, False, blocks, qrepr=qr, **kw)
        assert np.array_equal(out["m_init"][0], [seed, seed]), (mode, out["m_init"])
        # both keys equal: O is the mean of V's rows whatever the seed, LSE = s + ln 2
        assert np.abs(out["O"][0] - 0.5).max() < 1e-15
        assert np.abs(out["LSE"][0] - (np.array([0.0, -5.0]) + math.log(2))).max() < 1e-14


def test_blockwise_q_repr_reduces_to_rowwise_for_constant_blocks(oracle):
    """If all rows of a query block are the same vector, its signed-absmax and its mean are that vector,
    so the block-wise seed equals the row-wise one; the unsigned summary agrees where Q >= 0."""
    B, Hq, Hkv, N, d, bm, bn = 1, 2, 1, 64, 6, 16, 8
    rows = rnd(70, B, Hq, N // bm, 1, d)
    Q = np.broadcast_to(rows, (B, Hq, N // bm, bm, d)).reshape(B, Hq, N, d).copy()
    K, V = rnd(71, B, Hkv, N, d), rnd(72, B, Hkv, N, d)
    blocks = np.array([(0, h, i) for h in range(Hq) for i in range(N // bm)], np.int32)
    for causal in (False, True):
        row = oracle.blocks(Q, K, V, bm, bn, causal, blocks)
        for mode in (0, 2):
            blk = oracle.blocks(Q, K, V, bm, bn, causal, blocks, qrepr=oracle.sabsmax(Q, bm, mode))
            assert np.abs(blk["m_init"] - row["m_init"]).max() < 1e-13
            assert np.abs(blk["O"] - row["O"]).max() < 1e-13
        Qp = np.abs(Q)
        rowp = oracle.blocks(Qp, K, V, bm, bn, causal, blocks)
        blkp = oracle.blocks(Qp, K, V, bm, bn, causal, blocks, qrepr=oracle.sabsmax(Qp, bm, 3))
        assert np.abs(blkp["m_init"] - rowp["m_init"]).max() < 1e-13


@pytest.mark.parametrize("causal", [False, True])
def test_blockwise_q_repr_seed_is_broadcast_and_result_stays_exact(oracle, causal):
    """The seed is one scalar per (query block, visible key blocks): recomputed here from library
    reductions over the block; rows of a block share it; a ragged last block summarises its valid
    rows only; and the attention output is still the exact one (the seed cancels in O / l)."""
    B, Hq, Hkv, N, d, bm, bn = 1, 4, 2, 90, 8, 16, 8
    Q, K, V = rnd(73, B, Hq, N, d), rnd(74, B, Hkv, N, d), rnd(75, B, Hkv, N, d)
    Tr = -(-N // bm)
    blocks = np.array([(0, h, i) for h in range(Hq) for i in range(Tr)], np.int32)
    R = oracle.sabsmax(K, bn)
    Oe, Le, _ = oracle.exact(Q, K, V, bm, causal, blocks)
    reduce = {3: lambda x: np.abs(x).max(0), 2: lambda x: x.mean(0),
              0: lambda x: x[np.abs(x).argmax(0), np.arange(x.shape[1])]}
    for mode in (0, 2, 3):
        out = oracle.blocks(Q, K, V, bm, bn, causal, blocks, qrepr=oracle.sabsmax(Q, bm, mode))
        for n, (b, h, i) in enumerate(blocks):
            nr = min(bm, N - i * bm)
            qs = reduce[mode](Q[0, h, i * bm:i * bm + nr].astype(np.float64))
            j_hi = (i * bm + nr - 1) // bn if causal else -(-N // bn) - 1
            seed = (R[0, h // 2, :j_hi + 1] @ qs).max() / math.sqrt(d)
            assert np.abs(out["m_init"][n][:nr] - seed).max() < 1e-13
            assert np.abs(out["O"][n][:nr] - Oe[n][:nr]).max() < 1e-12
            assert np.abs(out["LSE"][n][:nr] - Le[n][:nr]).max() < 1e-12


# ------------------------------------------------------------------ exactness identity
CASES = [
    dict(N=96, d=8, bm=16, bn=16, causal=True, n_sink=1, n_local=1),
    dict(N=96, d=8, bm=16, bn=16, causal=False, n_sink=1, n_local=1),
    dict(N=100, d=5, bm=32, bn=8, causal=True, n_sink=2, n_local=2),     # ragged, B_r > B_c
    dict(N=100, d=5, bm=8, bn=32, causal=True, n_sink=1, n_local=1),     # B_r < B_c
    dict(N=77, d=16, bm=16, bn=16, causal=False, n_sink=0, n_local=3),
    dict(N=64, d=4, bm=64, bn=8, causal=True, n_sink=3, n_local=0),
]


@pytest.mark.parametrize("c", CASES)
@pytest.mark.parametrize("g", [1, 2])
def test_vfa_equals_exact_for_any_seeded_max(oracle, c, g):
    """m cancels between O and l, so Alg. 1 gives exact attention whatever value the max was
    seeded with; in particular whenever the seed bounds the true row max."""
    B, Hkv = 2, 2
    Hq = Hkv * g
    N, d, bm, bn = c["N"], c["d"], c["bm"], c["bn"]
    Q, K, V = rnd(14, B, Hq, N, d), rnd(15, B, Hkv, N, d), rnd(16, B, Hkv, N, d)
    K[:, :, 0] *= 3.0
    blocks = np.array([(b, h, i) for b in range(B) for h in range(Hq) for i in range(-(-N // bm))], np.int32)
    Oe, Le, Me = oracle.exact(Q, K, V, bm, c["causal"], blocks)
    valid = ~np.isnan(Le)
    kw = dict(n_sink=c["n_sink"], n_local=c["n_local"])
    # (a) the method's own m-init
    out = oracle.blocks(Q, K, V, bm, bn, c["causal"], blocks, **kw)
    assert np.abs(out["O"][valid] - Oe[valid]).max() < 1e-12
    assert np.abs(out["LSE"][valid] - Le[valid]).max() < 1e-12
    # (b) arbitrary seeds in [M-30, M+30]
    junk = np.where(valid, Me, 0.0) + np.random.default_rng(5).uniform(-30, 30, Me.shape)
    out = oracle.blocks(Q, K, V, bm, bn, c["causal"], blocks, m_override=junk, **kw)
    assert np.abs(out["O"][valid] - Oe[valid]).max() < 1e-10
    assert np.abs(out["LSE"][valid] - Le[valid]).max() < 1e-10
    # (c) seeds that bound the true max: every exponent is <= 0 and the frozen m stays the seed
    bound = np.where(valid, Me, 0.0) + 1.5
    out = oracle.blocks(Q, K, V, bm, bn, c["causal"], blocks, m_override=bound, **kw)
    assert np.abs(out["O"][valid] - Oe[valid]).max() < 1e-12
    assert np.array_equal(out["m_final"][valid], bound[valid])
    # (d) no m-init at all (allowed when a special block exists)
    if c["n_sink"] + c["n_local"] > 0:
        out = oracle.blocks(Q, K, V, bm, bn, c["causal"], blocks, use_minit=False, **kw)
        assert np.abs(out["O"][valid] - Oe[valid]).max() < 1e-10


def test_causal_rows_ignore_future_keys(oracle):
    B, H, N, d, bm, bn = 1, 1, 64, 8, 16, 16
    Q, K, V = rnd(17, B, H, N, d), rnd(18, B, H, N, d), rnd(19, B, H, N, d)
    blocks = np.array([(0, 0, 1)], np.int32)                     # rows 16..31
    a = oracle.blocks(Q, K, V, bm, bn, True, blocks)
    K2, V2 = K.copy(), V.copy()
    K2[:, :, 32:] = 100.0
    V2[:, :, 32:] = -7.0
    b = oracle.blocks(Q, K2, V2, bm, bn, True, blocks)
    assert np.array_equal(a["O"], b["O"]) and np.array_equal(a["LSE"], b["LSE"])
    # keys inside the diagonal block but after the row are masked too
    K3 = K.copy(); K3[:, :, 31] = 50.0
    c = oracle.blocks(Q, K3, V, bm, bn, True, blocks)
    # (the block summary, hence m_init, sees key 31, so agreement is to rounding, not bitwise)
    assert np.abs(a["O"][0, :15] - c["O"][0, :15]).max() < 1e-13 and np.abs(a["O"][0, 15] - c["O"][0, 15]).max() > 1e-3
    a0 = oracle.blocks(Q, K, V, bm, bn, True, blocks, use_minit=False)
    c0 = oracle.blocks(Q, K3, V, bm, bn, True, blocks, use_minit=False)
    assert np.array_equal(a0["O"][0, :15], c0["O"][0, :15])


# ------------------------------------------------------------------ online-softmax state, step by step
def test_fa_trajectory_is_running_max_and_sum(oracle):
    """FA column of Table 1 = online softmax: after k blocks m is the max and l the sum of
    exp(s - m) over the keys seen so far (definitions, evaluated on the whole score matrix)."""
    N, d, bm, bn = 80, 6, 16, 16
    Q, K, V = rnd(20, 1, 1, N, d), rnd(21, 1, 1, N, d), rnd(22, 1, 1, N, d)
    blocks = np.array([(0, 0, i) for i in range(N // bm)], np.int32)
    for causal in (False, True):
        out = oracle.fa2(Q, K, V, bm, bn, causal, blocks, want_traj=True)
        _, _, _, S = lib_attention(Q[0, 0], K[0, 0], V[0, 0], causal, 1 / math.sqrt(d))
        for n, (_, _, i) in enumerate(blocks):
            nvis = (i + 1) if causal else N // bn
            for k in range(nvis):
                seen = S[i * bm:(i + 1) * bm, : (k + 1) * bn]
                m = seen.max(1)
                l = np.exp(seen - m[:, None]).sum(1)
                assert np.abs(out["traj"][n, k, :, 0] - m).max() < 1e-14
                assert np.abs(out["traj"][n, k, :, 1] - l).max() < 1e-12
        # same switches spelled out on the VFA entry: all blocks special, ascending, no m-init
        same = oracle.blocks(Q, K, V, bm, bn, causal, blocks, n_sink=0, n_local=0, use_minit=False,
                             reorder=False, freeze=False)
        assert np.array_equal(same["O"], out["O"])


def test_vfa_trajectory_freezes_after_special_blocks(oracle):
    N, d, bm, bn = 96, 6, 16, 16
    Q, K, V = rnd(23, 1, 1, N, d), rnd(24, 1, 1, N, d), rnd(25, 1, 1, N, d)
    blocks = np.array([(0, 0, 4)], np.int32)
    out = oracle.blocks(Q, K, V, bm, bn, False, blocks, want_traj=True)
    _, _, _, S = lib_attention(Q[0, 0], K[0, 0], V[0, 0], False, 1 / math.sqrt(d))
    rows = S[4 * bm:5 * bm]
    m_after_special = np.maximum(out["m_init"][0], np.maximum(rows[:, 0:16].max(1), rows[:, 64:80].max(1)))
    order = [0, 4, 1, 2, 3, 5]
    seen = []
    for k, j in enumerate(order):
        seen.append(rows[:, j * bn:(j + 1) * bn])
        if k >= 1:
            assert np.array_equal(out["traj"][0, k, :, 0], m_after_special)          # frozen
            l = np.exp(np.concatenate(seen, 1) - m_after_special[:, None]).sum(1)    # no rescale factor needed
            assert np.abs(out["traj"][0, k, :, 1] - l).max() < 1e-11


def test_table1_op_counts(oracle):
    """Table 1: FA runs rowmax and the rescale on every tile; VFA only on the special tiles."""
    N, d, bm, bn = 128, 4, 16, 16
    Q, K, V = rnd(26, 1, 1, N, d), rnd(27, 1, 1, N, d), rnd(28, 1, 1, N, d)
    blocks = np.array([(0, 0, i) for i in range(N // bm)], np.int32)
    fa = oracle.fa2(Q, K, V, bm, bn, True, blocks)["counters"]
    vfa = oracle.blocks(Q, K, V, bm, bn, True, blocks)["counters"]
    for i in range(N // bm):
        assert fa[i, 0] == fa[i, 1] == fa[i, 2] == i + 1
        assert vfa[i, 0] == i + 1 and vfa[i, 1] == vfa[i, 2] == min(2, i + 1)
    vfa = oracle.blocks(Q, K, V, bm, bn, False, blocks, n_sink=2, n_local=3)["counters"]
    for i in range(N // bm):
        n_special = len(set(range(2)) | set(range(max(0, i - 2), i + 1)))
        assert vfa[i, 0] == N // bn and vfa[i, 1] == vfa[i, 2] == n_special


def test_lazy_rescale_is_exact_and_runs_the_rescale_less_often(oracle):
    """Conditional rescale (appendix, Blasst_FA4 variant, second stage): any tau >= 0 gives the
    exact output (the max cancels in O / l); tau = 0 is the FA column itself; the number of tiles
    whose rescale chain runs falls as tau grows and is 1 once tau exceeds every score gap."""
    N, d, bm, bn = 160, 6, 32, 16
    Q, K, V = 3.0 * rnd(40, 1, 2, N, d), rnd(41, 1, 1, N, d), rnd(42, 1, 1, N, d)
    blocks = np.array([(0, h, i) for h in range(2) for i in range(N // bm)], np.int32)
    for causal in (False, True):
        fa = oracle.fa2(Q, K, V, bm, bn, causal, blocks)
        ex_O, ex_L, _ = oracle.exact(Q, K, V, bm, causal, blocks)
        prev = None
        for tau in (0.0, 0.5, 2.0, 8.0, 1e6):
            out = oracle.fa_lazy(Q, K, V, bm, bn, causal, blocks, tau)
            assert np.abs(out["O"] - ex_O).max() < 1e-12 and np.abs(out["LSE"] - ex_L).max() < 1e-12
            c = out["counters"]
            assert np.array_equal(c[:, 0], fa["counters"][:, 0]) and np.array_equal(c[:, 1], c[:, 0])
            if tau == 0.0:
                assert np.array_equal(out["O"], fa["O"]) and np.array_equal(out["LSE"], fa["LSE"])
            if prev is not None:
                assert (c[:, 2] <= prev).all()
            prev = c[:, 2]
        assert (prev == 1).all()   # only the first tile, where the max leaves -inf
    # the rule itself, row by row on the full score matrix: which tiles change some row's max
    tau = 2.0
    for causal in (False, True):
        got = oracle.fa_lazy(Q, K, V, bm, bn, causal, blocks, tau)["counters"][:, 2]
        for n, (_, h, i) in enumerate(blocks):
            S = (Q[0, h].astype(np.float64) @ K[0, 0].astype(np.float64).T) / math.sqrt(d)
            if causal:
                S = np.where(np.arange(N)[None, :] > np.arange(N)[:, None], -np.inf, S)
            m = np.full(bm, -np.inf)
            changed = 0
            for j in range((i * bm + bm - 1) // bn + 1 if causal else N // bn):
                mt = np.maximum(m, S[i * bm:(i + 1) * bm, j * bn:(j + 1) * bn].max(1))
                adopt = (m == -np.inf) | (mt - m > tau * math.log(2))
                new_m = np.where(adopt, mt, m)
                changed += int((new_m != m).any())
                m = new_m
            assert got[n] == changed


def test_decode_step_is_last_row_of_causal_prefill_and_parts_add(oracle):
    """A decode step over n keys is the last row of causal attention over n tokens (library softmax
    here, and the pinned prefill oracle); with the max fixed after the sink / local blocks the
    per-range sums of exp(s - m) simply add up (Step 3: no rescale, hence no max in the merge)."""
    B, Hq, Hkv, n_cap, d, bn = 2, 4, 2, 200, 8, 16
    K, V = rnd(50, B, Hkv, n_cap, d), rnd(51, B, Hkv, n_cap, d)
    Qfull = 2.0 * rnd(52, B, Hq, n_cap, d)
    for n_keys in (1, 16, 17, 150, 200):
        q = np.ascontiguousarray(Qfull[:, :, n_keys - 1])
        out = oracle.decode(q, K, V, n_keys, bn, n_sink=1, n_local=2, n_parts=3)
        for b in range(B):
            for h in range(Hq):
                s = (K[b, h // 2, :n_keys].astype(np.float64) @ q[b, h].astype(np.float64)) / math.sqrt(d)
                p = scipy.special.softmax(s)
                assert np.abs(out["O"][b, h] - p @ V[b, h // 2, :n_keys].astype(np.float64)).max() < 1e-12
                assert abs(out["LSE"][b, h] - scipy.special.logsumexp(s)) < 1e-12
                Tc = -(-n_keys // bn)
                special = [c for c in range(n_keys) if c // bn < 1 or c // bn >= Tc - 2]
                assert out["m_final"][b, h] >= out["m_init"][b, h]
                assert abs(out["m_final"][b, h] - max(out["m_init"][b, h], s[special].max())) < 1e-12
                assert abs(out["l_parts"][b, h].sum() - math.exp(out["LSE"][b, h] - out["m_final"][b, h])) < 1e-9 * out["l_parts"][b, h].sum()
        if n_keys == n_cap:   # the prefill oracle's last causal row
            blocks = np.array([(b, h, (n_keys - 1) // 8) for b in range(B) for h in range(Hq)], np.int32)
            Oe, Le, _ = oracle.exact(Qfull, K, V, 8, True, blocks)
            assert np.abs(Oe[:, (n_keys - 1) % 8].reshape(B, Hq, d) - out["O"]).max() < 1e-12
    # m_init is the max of q . summary over the cache's blocks (sabsmax pinned elsewhere)
    n_keys = 150
    q = np.ascontiguousarray(Qfull[:, :, 0])
    out = oracle.decode(q, K, V, n_keys, bn)
    R = oracle.sabsmax(K[:, :, :n_keys], bn)
    for b in range(B):
        for h in range(Hq):
            assert abs(out["m_init"][b, h] - (R[b, h // 2] @ q[b, h].astype(np.float64)).max() / math.sqrt(d)) < 1e-12
    assert np.isneginf(oracle.decode(q, K, V, n_keys, bn, use_minit=False, n_sink=0, n_local=0)["m_final"]).all()


# ------------------------------------------------------------------ VSA
def _vsa_problem(seed=30, N=256, d=8, causal=True):
    w = wl.small(wl.CONFIGS["cfg2"], B=1, Hq=2, Hkv=1, N=N, d=d, block_m=32, block_n=16, F=1, W=16.0, theta=4.0,
                 beta=6.0, kappa=3.0)
    t = wl.generate(w, seed)
    Q, K, V = (wl.bf16_bits_to_f32(t[k]) for k in "QKV")
    return w, Q, K, V


@pytest.mark.parametrize("causal", [True, False])
def test_vsa_no_skip_limit_equals_vfa(oracle, causal):
    w, Q, K, V = _vsa_problem(causal=causal)
    blocks = wl.all_blocks(w)
    a = oracle.blocks(Q, K, V, 32, 16, causal, blocks)
    b = oracle.blocks(Q, K, V, 32, 16, causal, blocks, vsa=True, skip_threshold_nats=1e4)   # lambda -> 0
    assert np.array_equal(a["O"], b["O"]) and np.array_equal(a["LSE"], b["LSE"])
    assert not (b["mask"] == 1).any()
    for n, (_, _, i) in enumerate(blocks):
        j_hi = ((i + 1) * 32 - 1) // 16 if causal else w.N // 16 - 1
        assert np.all(b["mask"][n, : j_hi + 1] == 0) and np.all(b["mask"][n, j_hi + 1:] == 2)
        assert b["counters"][n, 1] == j_hi + 1              # rowmax on every visited tile in Alg. 2


@pytest.mark.parametrize("thr", [2.0, 5.0, 7.0])
def test_vsa_is_exact_attention_over_kept_tiles_and_loss_is_bounded(oracle, thr):
    w, Q, K, V = _vsa_problem()
    blocks = wl.all_blocks(w)
    out = oracle.blocks(Q, K, V, 32, 16, True, blocks, vsa=True, skip_threshold_nats=thr)
    Oe, Le, Me = oracle.exact(Q, K, V, 32, True, blocks)
    lam = math.exp(-thr)
    assert (out["mask"] == 1).sum() > 0
    skipped_frac = (out["mask"] == 1).sum() / (out["mask"] != 2).sum()
    assert out["counters"][:, 3].sum() == (out["mask"] == 1).sum()
    for n, (b, h, i) in enumerate(blocks):
        _, _, _, S = lib_attention(Q[b, h], K[b, 0], V[b, 0], True, w.scale)
        rows = S[i * 32:(i + 1) * 32]
        keep = np.repeat(out["mask"][n] == 0, 16)
        Sk = np.where(keep[None, :], rows, -np.inf)
        # (1) O, LSE = softmax restricted to the kept tiles (the frozen m cancels)
        P = scipy.special.softmax(Sk, axis=1)
        assert np.abs(out["O"][n] - P @ V[b, 0].astype(np.float64)).max() < 1e-12
        assert np.abs(out["LSE"][n] - scipy.special.logsumexp(Sk, axis=1)).max() < 1e-12
        # (2) every skipped score lies more than thr below the max in use => bounded lost mass
        skip_keys = np.repeat(out["mask"][n] == 1, 16)
        if skip_keys.any():
            smax = np.where(skip_keys[None, :], rows, -np.inf).max(1)
            assert np.all(smax < out["m_final"][n] - thr)
        delta = np.minimum(1.0, skip_keys.sum() * lam * np.exp(out["m_final"][n] - Le[n]))
        assert np.all(np.abs(out["O"][n] - Oe[n]).max(1) <= 2 * delta * np.abs(V).max() + 1e-12)
        assert np.all(Le[n] - out["LSE"][n] >= -1e-12)
        # (3) margin sign is the decision
        vis = out["mask"][n] != 2
        assert np.array_equal(out["margin"][n][vis] < 0, out["mask"][n][vis] == 1)
    assert 0.01 < skipped_frac < 0.98


def test_blasst_vanilla_mask_from_score_matrix(oracle):
    """All blocks special, ascending order, no m-init: the running max before block j is the
    true max over the earlier keys, so the mask follows from the score matrix alone."""
    w, Q, K, V = _vsa_problem(seed=31, causal=False)
    thr = 3.0
    blocks = wl.all_blocks(w)
    out = oracle.blocks(Q, K, V, 32, 16, False, blocks, n_sink=0, n_local=0, use_minit=False, reorder=False,
                        freeze=False, vsa=True, skip_threshold_nats=thr)
    for n, (b, h, i) in enumerate(blocks):
        _, _, _, S = lib_attention(Q[b, h], K[b, 0], V[b, 0], False, w.scale)
        tile_max = S[i * 32:(i + 1) * 32].reshape(32, -1, 16).max(2)              # [rows, Tc]
        run = np.maximum.accumulate(tile_max, axis=1)
        prev = np.concatenate([np.full((32, 1), -np.inf), run[:, :-1]], 1)
        want = np.all(tile_max - np.maximum(prev, tile_max) < -thr, axis=0)
        assert np.array_equal(out["mask"][n] == 1, want)
    assert (out["mask"] == 1).any() and (out["mask"] == 0).any()


@pytest.mark.parametrize("causal", [False, True])
def test_rowskip_and_fa4_skip_variants(oracle, causal):
    """Appendix variants Blasst_Rowskip and Blasst_FA4.  The decision rules are replayed on the full
    score matrix; what the variants then compute must be library softmax over exactly the entries
    they kept (for any choice of max), and the counters must count what the paper reports for them."""
    w, Q, K, V = _vsa_problem(seed=33, causal=causal)
    thr, tau, bm, bn = 3.0, 1.5, 32, 16
    blocks = wl.all_blocks(w)
    vanilla = oracle.blasst_variant(Q, K, V, bm, bn, causal, blocks, thr)
    same = oracle.blocks(Q, K, V, bm, bn, causal, blocks, n_sink=0, n_local=0, use_minit=False, reorder=False,
                         freeze=False, vsa=True, skip_threshold_nats=thr)
    assert np.array_equal(vanilla["O"], same["O"]) and np.array_equal(vanilla["mask"], same["mask"])
    rs = oracle.blasst_variant(Q, K, V, bm, bn, causal, blocks, thr, rowskip=True)
    f4 = oracle.blasst_variant(Q, K, V, bm, bn, causal, blocks, thr, lazy_tau=tau)
    suppressed_any = rescales_saved = 0
    for n, (b, h, i) in enumerate(blocks):
        _, _, _, S = lib_attention(Q[b, h], K[b, 0], V[b, 0], causal, w.scale)
        rows = S[i * bm:(i + 1) * bm]
        Vd = V[b, 0].astype(np.float64)
        n_tiles = ((i * bm + bm - 1) // bn + 1) if causal else w.Tc
        # --- row skip
        m = np.full(bm, -np.inf); keep_entry = np.zeros_like(rows, dtype=bool); mask = np.full(w.Tc, 2); supp = 0
        for j in range(n_tiles):
            mt = rows[:, j * bn:(j + 1) * bn].max(1)
            with np.errstate(invalid="ignore"):
                ok = np.where(np.isneginf(mt), False, mt - np.maximum(m, mt) >= -thr)
            mask[j] = 0 if ok.any() else 1
            supp += int((~ok).sum())
            if ok.any():
                keep_entry[ok, j * bn:(j + 1) * bn] = True
                m = np.where(ok, np.maximum(m, mt), m)
        assert np.array_equal(rs["mask"][n], mask) and rs["counters"][n, 2] == supp
        for r in range(bm):
            sel = keep_entry[r] & np.isfinite(rows[r])
            want = scipy.special.softmax(rows[r, sel]) @ Vd[sel]
            assert np.abs(rs["O"][n, r] - want).max() < 1e-12
            assert abs(rs["LSE"][n, r] - scipy.special.logsumexp(rows[r, sel])) < 1e-12
        suppressed_any += supp
        # --- block skip, then conditional rescale against the lagging max
        m = np.full(bm, -np.inf); kept_tiles = []; mask = np.full(w.Tc, 2); ran = 0
        for j in range(n_tiles):
            mt = rows[:, j * bn:(j + 1) * bn].max(1)
            with np.errstate(invalid="ignore"):
                ok = np.where(np.isneginf(mt), False, mt - np.maximum(m, mt) >= -thr)
            mask[j] = 0 if ok.any() else 1
            if ok.any():
                kept_tiles.append(j)
                new = np.maximum(m, mt)
                with np.errstate(invalid="ignore"):
                    lag = (~np.isneginf(m)) & (new - m <= tau * math.log(2))
                new = np.where(lag, m, new)
                ran += int((new != m).any())
                m = new
        assert np.array_equal(f4["mask"][n], mask) and f4["counters"][n, 2] == ran
        cols = np.concatenate([np.arange(j * bn, (j + 1) * bn) for j in kept_tiles])
        for r in range(bm):
            sel = cols[np.isfinite(rows[r, cols])]
            assert np.abs(f4["O"][n, r] - scipy.special.softmax(rows[r, sel]) @ Vd[sel]).max() < 1e-12
        rescales_saved += len(kept_tiles) - ran
    assert suppressed_any > 0 and rescales_saved > 0 and (rs["mask"] == 1).any()


def test_vsa_mask_uses_frozen_max(oracle):
    """Alg. 2 with freeze: on non-special tiles the test compares against
    m = max(m_init, rowmax of the special tiles that were kept)."""
    w, Q, K, V = _vsa_problem(seed=32, causal=False)
    thr = 4.0
    blocks = wl.all_blocks(w)
    out = oracle.blocks(Q, K, V, 32, 16, False, blocks, vsa=True, skip_threshold_nats=thr)
    for n, (b, h, i) in enumerate(blocks):
        _, _, _, S = lib_attention(Q[b, h], K[b, 0], V[b, 0], False, w.scale)
        tile_max = S[i * 32:(i + 1) * 32].reshape(32, -1, 16).max(2)
        m = out["m_init"][n].copy()
        special = [0] + [j for j in (2 * i, 2 * i + 1) if j != 0]
        for j in special:
            skip = np.all(tile_max[:, j] - np.maximum(m, tile_max[:, j]) < -thr)
            assert (out["mask"][n, j] == 1) == skip
            if not skip:
                m = np.maximum(m, tile_max[:, j])
        assert np.array_equal(m, out["m_final"][n])
        for j in range(w.N // 16):
            if j not in special:
                assert (out["mask"][n, j] == 1) == bool(np.all(tile_max[:, j] < m - thr))


def test_all_blocks_skipped_gives_zero_row(oracle):
    w, Q, K, V = _vsa_problem(seed=33)
    blocks = wl.all_blocks(w)[:2]
    huge = np.full((2, 32), 1e3)
    out = oracle.blocks(Q, K, V, 32, 16, True, blocks, vsa=True, skip_threshold_nats=8.0, m_override=huge)
    assert np.all(out["O"] == 0) and np.all(np.isneginf(out["LSE"]))
    assert np.all(out["mask"][out["mask"] != 2] == 1)


# ------------------------------------------------------------------ generators
def test_generators_are_seeded_and_structured(oracle):
    w = wl.small(wl.CONFIGS["cfg2"], Hq=2, Hkv=1, N=1024)
    a, b = wl.generate(w, 7), wl.generate(w, 7)
    assert all(np.array_equal(a[k], b[k]) for k in "QKV")
    assert not np.array_equal(a["Q"], wl.generate(w, 8)["Q"])
    Q, K, V = (wl.bf16_bits_to_f32(a[k]) for k in "QKV")
    assert np.array_equal(wl.f32_to_bf16_bits(Q), a["Q"])                          # round trip is exact
    blocks = np.array([(0, 0, 7), (0, 1, 5)], np.int32)
    P, _, _, S = lib_attention(Q[0, 0], K[0, 0], V[0, 0], True, w.scale)
    # sink: key 0 takes a large share; local: the diagonal band beats the far background
    assert P[512:, 0].mean() > 0.3
    near = np.mean([S[r, r - 8:r + 1].mean() for r in range(600, 1000)])
    far = np.mean([S[r, 100:r - 400].mean() for r in range(600, 1000)])
    assert near > far + 2.0
    # planted maxima (m-init stress): the planted key is the row argmax outside sink/local blocks
    w4 = wl.small(wl.CONFIGS["cfg4"], Hq=1, Hkv=1, N=2048)
    t = wl.generate(w4, 3)
    Q, K = wl.bf16_bits_to_f32(t["Q"])[0, 0], wl.bf16_bits_to_f32(t["K"])[0, 0]
    S = (Q.astype(np.float64) @ K.astype(np.float64).T) * w4.scale
    arg = S.argmax(1)
    blk = arg // w4.block_n
    own = (np.arange(2048) // w4.block_m)[:, None] * 2 + np.arange(2)[None, :]
    middle = (blk >= w4.n_sink) & ~(blk[:, None] == own).any(1)
    assert middle.mean() > 0.95 and np.median(S.max(1)) > 5.0


def test_decode_generator_shares_the_cache_of_the_prefill_recipe():
    w = wl.small(wl.DECODE, B=1, N=512)
    a, b = wl.generate_decode(w, 300), wl.generate_decode(w, 300)
    assert all(np.array_equal(a[k], b[k]) for k in a) and a["q"].shape == (1, 32, 128)
    full = wl.generate(w)
    assert np.array_equal(full["K"], a["K"]) and np.array_equal(full["V"], a["V"])
    q, K = wl.bf16_bits_to_f32(a["q"]), wl.bf16_bits_to_f32(a["K"])
    s = np.einsum("bhd,bhnd->bhn", q.reshape(1, 8, 4, 128)[:, :, 0], K[:, :, :300]) / math.sqrt(128)
    assert (s[..., 0] > s[..., 1:250].max(-1)).mean() > 0.5      # the sink key usually carries the largest far logit
    assert s[..., 299].mean() > s[..., 100:200].mean() + 0.5     # and the token's own position gets the local bonus


def test_e4m3_codec_against_the_format_definition():
    """OCP FP8 E4M3 (finite only): sign, 4 exponent bits with bias 7, 3 mantissa bits; exponent 0 is
    the subnormal grid m * 2^-9; S.1111.111 is NaN; largest finite 448.  The table is built here from
    that definition; the encoder must invert it, round ties to even, and saturate."""
    import oracle as orc
    table = []
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        v = float("nan") if (e == 15 and m == 7) else ((m * 2.0 ** -9) if e == 0 else (1 + m / 8) * 2.0 ** (e - 7))
        table.append(-v if s else v)
    table = np.array(table)
    dec = orc.e4m3_dequantize(np.arange(256, dtype=np.uint8))
    assert np.array_equal(np.isnan(dec), np.isnan(table)) and np.array_equal(dec[~np.isnan(table)], table[~np.isnan(table)])
    assert table[0x7E] == 448.0 and table[0x08] == 2.0 ** -6 and table[0x01] == 2.0 ** -9 and table[0x38] == 1.0
    fin = np.array([c for c in range(256) if not np.isnan(table[c]) and c != 0x80], dtype=np.uint8)
    assert np.array_equal(orc.e4m3_quantize(table[fin].astype(np.float32), 1.0), fin)         # every value encodes to itself
    pos = table[:0x7F]                                                                         # codes 0x00..0x7E ascend
    assert np.all(np.diff(pos) > 0)
    mid = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)                                        # exact in float32
    codes = orc.e4m3_quantize(mid, 1.0)
    lo, hi = orc.e4m3_quantize(pos[:-1].astype(np.float32), 1.0), orc.e4m3_quantize(pos[1:].astype(np.float32), 1.0)
    assert np.all((codes == lo) | (codes == hi)) and np.all(codes % 2 == 0)                    # ties go to the even code
    assert np.array_equal(orc.e4m3_quantize(np.array([1e9, 449.0, 464.1, -1e9], np.float32), 1.0), [0x7E, 0x7E, 0x7E, 0xFE])
    assert np.array_equal(orc.e4m3_quantize(np.array([447.9, 2.0 ** -11, 2.0 ** -10, 3 * 2.0 ** -10], np.float32), 1.0),
                          [0x7E, 0x00, 0x00, 0x02])
    x = rnd(60, 4096).astype(np.float32) * 3
    q = orc.e4m3_dequantize(orc.e4m3_quantize(x, 16.0), 1 / 16.0)
    big = np.abs(x) >= 2.0 ** -6 / 16
    assert np.all(np.abs(q - x)[big] <= np.abs(x)[big] * 2.0 ** -4) and np.all(np.abs(q - x)[~big] <= 2.0 ** -10 / 16)
    assert np.all(np.diff(orc.e4m3_dequantize(orc.e4m3_quantize(np.sort(x), 16.0))) >= 0)      # monotone


E2M1_VALUES = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]    # the format's table, codes 0..7; 8..15 are their negatives


def _nearest_on_grid(y, grid):
    """Index of the grid value nearest to y; of two equally near ones, the even index (the codes of a
    small float are consecutive integers, so an even code is an even mantissa); beyond the grid: its end."""
    grid = np.asarray(grid)
    dist = np.abs(grid[None, :] - np.abs(y)[:, None])
    best = dist.min(1)
    out = np.empty(len(y), int)
    for n in range(len(y)):
        cand = np.flatnonzero(dist[n] == best[n])
        out[n] = cand[0] if len(cand) == 1 else [c for c in cand if c % 2 == 0][0]
    return out


def test_mx_codecs_against_the_format_definitions(oracle):
    """E2M1 decode = the published table; E5M2 decode = the top byte of an IEEE half (library: numpy float16);
    encode = nearest table entry, ties to the even code, checked by brute force over the decoded tables on
    random values, on every midpoint between neighbours and beyond the largest finite value."""
    one = np.full((1, 1), 127, np.uint8)                       # scale 2^0
    nib = np.zeros((16, 16), np.uint8)
    nib[:, 0] = np.arange(16)                                  # code c in element 0 of row c, zeros elsewhere
    dec = oracle.mx_dequantize(nib, np.repeat(one, 16, 0), fmt=0)
    assert np.array_equal(dec[:, 0], E2M1_VALUES + [-v for v in E2M1_VALUES]) and np.all(dec[:, 1:] == 0)
    hi = np.zeros((16, 16), np.uint8)
    hi[:, 3] = np.arange(16) << 4                              # high nibble of byte 3 is element 7
    assert np.array_equal(oracle.mx_dequantize(hi, np.repeat(one, 16, 0), fmt=0)[:, 7], dec[:, 0])
    finite = np.array([c for c in range(256) if (c & 0x7C) != 0x7C], np.uint8)
    rows = np.zeros((len(finite), 32), np.uint8)
    rows[:, 5] = finite
    dec5 = oracle.mx_dequantize(rows, np.repeat(one, len(finite), 0), fmt=1)[:, 5]
    half = (finite.astype(np.uint16) << 8).view(np.float16).astype(np.float64)
    assert np.array_equal(dec5, half)
    rng = np.random.default_rng(90)
    for fmt, grid in ((0, np.array(E2M1_VALUES)), (1, half[:len(half) // 2])):   # non-negative half of each table
        assert np.all(np.diff(grid) > 0)
        mids = (grid[1:] + grid[:-1]) / 2
        top = grid[-1]
        # keep the block maximum in [top/2 .. top] * (1 + something < 1) so that the shared scale is 2^0:
        # element 0 of every row carries `top`, the value under test sits in element 1
        ys = np.concatenate([mids, grid, rng.uniform(0, top * 1.3, 400), [top * 1.01, top * 1.29]])
        ys = ys[ys < top * 4 / 3] if fmt == 0 else ys[ys < 65536]
        x = np.zeros((len(ys), 32), np.float32)
        x[:, 0] = top
        x[:, 1] = ys * np.where(np.arange(len(ys)) % 2 == 0, 1, -1)
        ys = np.abs(x[:, 1].astype(np.float64))                 # what float32 kept of them
        codes, scales = oracle.mx_quantize(x, fmt)
        assert np.all(scales == 127)
        got = (codes[:, 0] >> 4) if fmt == 0 else codes[:, 1]
        sign = got & (0x8 if fmt == 0 else 0x80)
        assert np.array_equal(sign != 0, np.signbit(x[:, 1]))      # -0 keeps its sign bit
        assert np.array_equal(got & (0x7 if fmt == 0 else 0x7F), _nearest_on_grid(ys, grid))


def test_mx_shared_scale_rule_hand_values(oracle):
    """byte = floor(log2(max|x|)) - emax + 127: E2M1 (emax 2): max 6 -> 127, 7.9 -> 127 (7.9 saturates to 6),
    8 -> 128 (8 / 2 = 4), 0.3 -> 123 (0.3 * 16 = 4.8 -> 4); E5M2 (emax 15): max 6 -> 114; zeros -> byte 0."""
    x = np.zeros((6, 64), np.float32)
    x[0, 0], x[1, 1], x[2, 2], x[3, 3] = 6.0, -7.9, 8.0, 0.3
    x[4, 40] = 6.0                                             # second block of the row; its first block is all zero
    x[0, 1], x[2, 3] = 1.2, 3.1                                # 1.2 -> 1.0;  3.1 / 2 = 1.55 -> 1.5
    codes, scales = oracle.mx_quantize(x, 0)
    assert scales.tolist() == [[127, 0], [127, 0], [128, 0], [123, 0], [0, 127], [0, 0]]
    back = oracle.mx_dequantize(codes, scales, 0)
    want = np.zeros((6, 64))
    want[0, 0], want[1, 1], want[2, 2], want[3, 3], want[4, 40] = 6.0, -6.0, 8.0, 0.25, 6.0
    want[0, 1], want[2, 3] = 1.0, 3.0
    assert np.array_equal(back, want)
    codes5, scales5 = oracle.mx_quantize(x, 1)
    assert scales5[0, 0] == 114 and scales5[3, 0] == 110 and scales5[5].tolist() == [0, 0]
    back5 = oracle.mx_dequantize(codes5, scales5, 1)
    # two mantissa bits: the top binade of a block holds 4, 5, 6, 7 (times its scale), so a block maximum of 7.9
    # saturates to 7; 1.2 -> 1.25 and 3.1 -> 3 are ordinary roundings
    assert back5[0, 0] == 6.0 and back5[1, 1] == -7.0 and back5[2, 2] == 8.0 and back5[0, 1] == 1.25 and back5[2, 3] == 3.0
    # pre_scale multiplies in float32 before anything else
    c2, s2 = oracle.mx_quantize(x, 0, pre_scale=0.5)
    assert np.array_equal(oracle.mx_dequantize(c2, s2, 0), oracle.mx_dequantize(*oracle.mx_quantize(x * np.float32(0.5), 0), 0))
    assert s2[2, 0] == 127


def test_mx_round_trip_properties(oracle):
    """Values already on a block's grid survive the round trip; any value moves by at most a quarter of the block
    maximum (E2M1: half a step of 2 at the top binade, or the saturation of [6, 8) to 6)."""
    rng = np.random.default_rng(91)
    x = (rng.standard_normal((50, 128)) * np.exp(rng.standard_normal((50, 1)) * 3)).astype(np.float32)
    codes, scales = oracle.mx_quantize(x, 0)
    back = oracle.mx_dequantize(codes, scales, 0)
    amax = np.abs(x.astype(np.float64)).reshape(50, 4, 32).max(2, keepdims=True)
    assert np.all(np.abs(back.reshape(50, 4, 32) - x.reshape(50, 4, 32)) <= amax / 4 * (1 + 1e-12))
    c2, s2 = oracle.mx_quantize(back.astype(np.float32), 0)
    assert np.array_equal(oracle.mx_dequantize(c2, s2, 0), back)
    # E5M2 summaries of E2M1-valued vectors whose entries come from different scales are exact over 29 binades
    mixed = back.reshape(50, 4, 32) * np.exp2(rng.integers(-12, 1, (50, 4, 32)))
    mixed = mixed.reshape(50, 128).astype(np.float32)
    c5, s5 = oracle.mx_quantize(mixed, 1)
    assert np.array_equal(oracle.mx_dequantize(c5, s5, 1), mixed.astype(np.float64))


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.4e38, 1e-40, 0.0], np.float32)
    bits = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 is a tie -> even (1 + 2^-6)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -1.0
    assert np.isinf(back[4]) and back[6] == 0.0
    import torch
    y = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 37
    t = torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wl.f32_to_bf16_bits(y), t)


# ---- where the running maximum stabilises (attention-statistics section, stabilisation-position equation)
def test_stabilisation_index_is_the_block_of_a_planted_maximum(oracle):
    """One key per row made the unique largest score by construction: j* is that key's block, for every row."""
    rng = np.random.default_rng(7)
    N, d, bm, bn = 320, 16, 64, 32
    Q = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    K = (0.01 * rng.standard_normal((1, 1, N, d))).astype(np.float32)
    V = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    planted = 5 * bn + 3                      # key 163, block 5
    K[0, 0, planted] = 0.0
    Q[..., 0] = 4.0                           # every query has a large first coordinate ...
    K[0, 0, planted, 0] = 8.0                 # ... and only the planted key answers it
    blocks = np.array([[0, 0, i] for i in range(N // bm)], dtype=np.int32)
    js = oracle.stabilisation_index(Q, K, V, bm, bn, False, blocks)
    assert js.shape == (N // bm, bm) and np.all(js == 5)
    # causal: rows before the planted key cannot see it; rows from the planted key on stabilise in its block
    jc = oracle.stabilisation_index(Q, K, V, bm, bn, True, blocks)
    rows = np.arange(N).reshape(N // bm, bm)
    assert np.all(jc[rows >= planted] == 5)
    assert np.all(jc[rows < planted] <= rows[rows < planted] // bn)


def test_stabilisation_index_against_brute_force_argmax(oracle):
    """The running maximum reaches its final value in the block that holds the first occurrence of the row's largest
    score: brute force over a full score matrix, ragged length, causal and not."""
    rng = np.random.default_rng(11)
    N, d, bm, bn = 150, 8, 32, 16
    Q = rng.standard_normal((1, 2, N, d)).astype(np.float32)
    K = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    V = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    Tr = -(-N // bm)
    blocks = np.array([[0, h, i] for h in range(2) for i in range(Tr)], dtype=np.int32)
    for causal in (False, True):
        js = oracle.stabilisation_index(Q, K, V, bm, bn, causal, blocks)
        for a, (_, h, i) in enumerate(blocks):
            for rr in range(bm):
                row = i * bm + rr
                if row >= N:
                    assert js[a, rr] == -1
                    continue
                s = Q[0, h, row].astype(np.float64) @ K[0, 0].astype(np.float64).T
                if causal:
                    s = s[: row + 1]
                assert js[a, rr] == int(np.argmax(s)) // bn
