"""Pins for the CPU oracle: closed forms, invariants, library special cases, brute force.

The paper prints no numeric worked example for the scoring path, so the oracle
is pinned to what its equations and plain mathematics fix.  Each test names the
mistake it would catch.  None of these tests touches the HIP library.
"""
import math

import numpy as np
import pytest
import torch

import workloads
from helpers import to_oracle_array


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def _score(oracle, q, k, Hq, G, d, w, n, **kw):
    return oracle.score_layer(q, k, Hq, G, d, w, [n], **kw)


# ------------------------------------------------------------------ Eq. 1 (softmax rows)

def test_two_key_closed_form(oracle):
    # q = (2,0,0,0), k0 = 0, k1 = (ln 3, 0,0,0), d = 4 -> scale 1/2 -> logits (0, ln 3) -> a = (1/4, 3/4)
    # catches: missing 1/sqrt(d), wrong softmax axis, wrong sign
    q = np.zeros((1, 1, 1, 4), np.float32); q[0, 0, 0, 0] = 2.0
    k = np.zeros((1, 2, 4), np.float32); k[0, 1, 0] = math.log(3.0)
    D, ent, ent_h, p = _score(oracle, q, k, 1, 1, 4, 1, 2, want_probs=True)
    ln3 = float(np.float32(math.log(3.0)))       # the stored key is the fp32 rounding of ln 3
    a1 = math.exp(ln3) / (1 + math.exp(ln3))
    assert p[0][0, 0] == pytest.approx([1 - a1, a1], rel=1e-14)
    assert D == pytest.approx([1 - a1, a1], rel=1e-14)
    h = -((1 - a1) * math.log(1 - a1) + a1 * math.log(a1))
    assert ent[0] == pytest.approx(h, rel=1e-13)
    assert abs(a1 - 0.75) < 1e-7


def test_rows_sum_to_one_and_bounds(oracle):
    Hq, G, d, w, n = 8, 2, 64, 16, 700
    q, k = _rand((1, Hq, w, d), 1), _rand((G, n, d), 2)
    D, ent, ent_h, p = _score(oracle, q, k, Hq, G, d, w, n, want_probs=True)
    P = p[0]
    assert np.all(P >= 0) and np.all(P <= 1)
    assert np.abs(P.sum(-1) - 1).max() < 1e-12
    # Eq. 2 summed over j: every row contributes exactly one unit of attention mass
    assert D.sum() == pytest.approx(w * Hq, rel=1e-12)
    assert np.abs(P.sum((0, 1)) - D).max() < 1e-12
    assert 0.0 <= ent[0] <= math.log(n)
    assert ent[0] == pytest.approx(ent_h[0].mean(), rel=1e-13)


def test_single_row_is_library_softmax(oracle):
    # Hq = w = 1 reduces to a textbook softmax of K q / sqrt(d): compare with torch.softmax
    d, n = 32, 257
    q, k = _rand((1, 1, 1, d), 3), _rand((1, n, d), 4)
    D, ent, _, _ = _score(oracle, q, k, 1, 1, d, 1, n)
    logits = torch.tensor(k[0], dtype=torch.float64) @ torch.tensor(q[0, 0, 0], dtype=torch.float64) / math.sqrt(d)
    ref = torch.softmax(logits, 0)
    assert np.abs(ref.numpy() - D).max() < 1e-15
    assert ent[0] == pytest.approx(float(torch.distributions.Categorical(probs=ref).entropy()), rel=1e-12)


def test_brute_force_tiny_python_loops(oracle):
    # pure-Python evaluation of Eq. 1, 2, 4 with GQA head->group mapping; catches transposed
    # operands, a wrong head->group map, a wrong window/row index
    Hq, G, d, w, n = 4, 2, 3, 2, 5
    q, k = _rand((1, Hq, w, d), 5), _rand((G, n, d), 6)
    D, ent, ent_h, _ = _score(oracle, q, k, Hq, G, d, w, n)
    gs = Hq // G
    Dref = [0.0] * n
    eh = []
    for h in range(Hq):
        g = h // gs
        acc_e = 0.0
        for i in range(w):
            s = [sum(float(q[0, h, i, c]) * float(k[g, j, c]) for c in range(d)) / math.sqrt(d) for j in range(n)]
            m = max(s)
            e = [math.exp(x - m) for x in s]
            Z = sum(e)
            a = [x / Z for x in e]
            for j in range(n):
                Dref[j] += a[j]
            acc_e += -sum(x * math.log(x) for x in a)
        eh.append(acc_e / w)
    assert D == pytest.approx(Dref, rel=1e-13)
    assert ent_h[0] == pytest.approx(eh, rel=1e-13)
    assert ent[0] == pytest.approx(sum(eh) / Hq, rel=1e-13)


def test_brute_force_causal_python_loops(oracle):
    # the causal reading (window row i, at position n-w+i, sees keys j <= n-w+i) in pure Python on random data,
    # GQA, w > 1, n not a multiple of anything; catches an off-by-one in the visible range, a mask applied per
    # head instead of per window row, masked keys that still receive mass
    Hq, G, d, w, n = 6, 3, 4, 3, 7
    q, k = _rand((1, Hq, w, d), 15), _rand((G, n, d), 16)
    D, ent, ent_h, p = _score(oracle, q, k, Hq, G, d, w, n, causal=True, want_probs=True)
    gs = Hq // G
    Dref = [0.0] * n
    eh = []
    for h in range(Hq):
        g = h // gs
        acc_e = 0.0
        for i in range(w):
            vis = n - w + i + 1                       # keys 0 .. n-w+i
            s = [sum(float(q[0, h, i, c]) * float(k[g, j, c]) for c in range(d)) / math.sqrt(d) for j in range(vis)]
            m = max(s)
            e = [math.exp(x - m) for x in s]
            Z = sum(e)
            a = [x / Z for x in e]
            for j in range(vis):
                Dref[j] += a[j]
            assert p[0][h, i, :vis] == pytest.approx(a, rel=1e-13)
            assert np.all(p[0][h, i, vis:] == 0.0)
            acc_e += -sum(x * math.log(x) for x in a)
        eh.append(acc_e / w)
    assert D == pytest.approx(Dref, rel=1e-13)
    assert ent_h[0] == pytest.approx(eh, rel=1e-13)
    assert ent[0] == pytest.approx(sum(eh) / Hq, rel=1e-13)
    assert sum(Dref) == pytest.approx(w * Hq, rel=1e-13)      # every visible row still sums to 1
    # the last key is seen by the last window row only: its in-degree is at most H_q
    assert D[n - 1] <= Hq


def test_explicit_scale_and_default(oracle):
    Hq, G, d, w, n = 2, 1, 16, 4, 50
    q, k = _rand((1, Hq, w, d), 7), _rand((G, n, d), 8)
    D0, e0, _, _ = _score(oracle, q, k, Hq, G, d, w, n)
    D1, e1, _, _ = _score(oracle, q, k, Hq, G, d, w, n, scale=1.0 / math.sqrt(d))
    D2, e2, _, _ = _score(oracle, q, 2 * k, Hq, G, d, w, n, scale=0.5 / math.sqrt(d))
    assert np.array_equal(D0, D1) and e0 == e1
    assert D2 == pytest.approx(D0, rel=1e-12) and e2[0] == pytest.approx(e0[0], rel=1e-12)


# ------------------------------------------------------------------ uniform / one-hot limits

def test_uniform_attention_entropy_is_log_n(oracle):
    Hq, G, d, w, n = 4, 2, 8, 4, 333
    q = _rand((1, Hq, w, d), 9)
    k = np.tile(_rand((G, 1, d), 10), (1, n, 1))          # all keys identical
    D, ent, ent_h, _ = _score(oracle, q, k, Hq, G, d, w, n)
    assert D == pytest.approx(np.full(n, w * Hq / n), rel=1e-12)
    assert ent[0] == pytest.approx(math.log(n), rel=1e-13)
    # Q = 0 is the other uniform case
    D, ent, _, _ = _score(oracle, np.zeros_like(q), _rand((G, n, d), 11), Hq, G, d, w, n)
    assert D == pytest.approx(np.full(n, w * Hq / n), rel=1e-12)
    assert ent[0] == pytest.approx(math.log(n), rel=1e-13)


def test_uniform_causal_entropy(oracle):
    Hq, G, d, w, n = 2, 1, 8, 4, 20
    q = _rand((1, Hq, w, d), 12)
    k = np.zeros((G, n, d), np.float32)
    D, ent, _, p = _score(oracle, q, k, Hq, G, d, w, n, causal=True, want_probs=True)
    expect = sum(math.log(n - w + i + 1) for i in range(w)) / w
    assert ent[0] == pytest.approx(expect, rel=1e-13)
    # row i sees keys 0 .. n-w+i; the masked ones carry exactly zero
    for i in range(w):
        assert np.all(p[0][:, i, n - w + i + 1:] == 0.0)
        assert p[0][:, i, :n - w + i + 1] == pytest.approx(1.0 / (n - w + i + 1), rel=1e-13)
    Dref = np.zeros(n)
    for i in range(w):
        Dref[:n - w + i + 1] += Hq / (n - w + i + 1)
    assert D == pytest.approx(Dref, rel=1e-12)


def test_one_hot_and_two_hot_limits(oracle):
    Hq, G, d, w, n = 2, 1, 4, 2, 64
    q = np.ones((1, Hq, w, d), np.float32)
    k = np.zeros((G, n, d), np.float32)
    k[0, 17] = 100.0                                      # one key with a huge logit
    D, ent, _, _ = _score(oracle, q, k, Hq, G, d, w, n)
    assert D[17] == pytest.approx(w * Hq, rel=1e-12) and ent[0] < 1e-60
    k[0, 40] = 100.0                                      # two equal dominant keys
    D, ent, _, _ = _score(oracle, q, k, Hq, G, d, w, n)
    assert D[17] == pytest.approx(w * Hq / 2, rel=1e-12) and D[40] == pytest.approx(w * Hq / 2, rel=1e-12)
    assert ent[0] == pytest.approx(math.log(2.0), rel=1e-12)


# ------------------------------------------------------------------ metamorphic relations

def test_key_permutation_permutes_indegree(oracle):
    Hq, G, d, w, n = 4, 2, 16, 4, 101
    q, k = _rand((1, Hq, w, d), 13), _rand((G, n, d), 14)
    perm = np.random.default_rng(15).permutation(n)
    D, e, _, _ = _score(oracle, q, k, Hq, G, d, w, n)
    Dp, ep, _, _ = _score(oracle, q, np.ascontiguousarray(k[:, perm]), Hq, G, d, w, n)
    assert Dp == pytest.approx(D[perm], rel=1e-12)
    assert ep[0] == pytest.approx(e[0], rel=1e-12)


def test_constant_key_shift_invariance_large(oracle):
    # adding one vector c to every key shifts each row's logits by a constant: softmax unchanged.
    # With |c| large this fails unless the row maximum is subtracted before exponentiation.
    Hq, G, d, w, n = 2, 1, 8, 2, 40
    q = np.round(_rand((1, Hq, w, d), 16) * 4) / 4        # dyadic values: products stay exact
    k = np.round(_rand((G, n, d), 17) * 4) / 4
    c = np.full((1, 1, d), 300.0, np.float32)
    D, e, _, _ = _score(oracle, q, k, Hq, G, d, w, n)
    Ds, es, _, _ = _score(oracle, q, k + c, Hq, G, d, w, n)
    assert np.all(np.isfinite(Ds))
    assert Ds == pytest.approx(D, rel=1e-9)
    assert es[0] == pytest.approx(e[0], rel=1e-9)


def test_gqa_equals_mha_with_repeated_kv(oracle):
    Hq, G, d, w, n = 8, 2, 16, 4, 90
    q, k = _rand((1, Hq, w, d), 18), _rand((G, n, d), 19)
    D, e, eh, _ = _score(oracle, q, k, Hq, G, d, w, n)
    k_rep = np.ascontiguousarray(np.repeat(k, Hq // G, axis=0))
    D2, e2, eh2, _ = _score(oracle, q, k_rep, Hq, Hq, d, w, n)
    assert D2 == pytest.approx(D, rel=1e-12)
    assert eh2[0] == pytest.approx(eh[0], rel=1e-12)


def test_entropy_identity_lse_minus_expected_logit(oracle):
    # H_row = logsumexp(s) - sum_j a_j s_j : a second formula for Eq. 4, evaluated with numpy
    Hq, G, d, w, n = 4, 2, 16, 4, 120
    q, k = _rand((1, Hq, w, d), 20, 1.5), _rand((G, n, d), 21, 1.5)
    _, ent, _, p = _score(oracle, q, k, Hq, G, d, w, n, want_probs=True)
    kk = np.repeat(k.astype(np.float64), Hq // G, axis=0)
    s = np.einsum("hwd,hnd->hwn", q[0].astype(np.float64), kk) / math.sqrt(d)
    lse = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
    h = lse - (p[0] * s).sum(-1)
    assert ent[0] == pytest.approx(h.mean(), rel=1e-12)


def test_bf16_inputs_are_widened_exactly(oracle):
    Hq, G, d, w, n = 4, 2, 16, 4, 77
    qb = torch.tensor(_rand((1, Hq, w, d), 22)).to(torch.bfloat16)
    kb = torch.tensor(_rand((G, n, d), 23)).to(torch.bfloat16)
    D16, e16, _, _ = _score(oracle, to_oracle_array(qb), to_oracle_array(kb), Hq, G, d, w, n)
    D32, e32, _, _ = _score(oracle, qb.float().numpy(), kb.float().numpy(), Hq, G, d, w, n)
    assert np.array_equal(D16, D32) and e16 == e32


def test_ragged_batch_is_per_sequence(oracle):
    Hq, G, d, w = 4, 2, 16, 4
    lens = [30, 0, 7, 55]
    q = _rand((4, Hq, w, d), 24)
    k = _rand((G, sum(lens), d), 25)
    D, e, eh, _ = oracle.score_layer(q, k, Hq, G, d, w, lens)
    off = 0
    for b, n in enumerate(lens):
        if n == 0:
            continue
        Db, eb, _, _ = oracle.score_layer(q[b:b + 1], np.ascontiguousarray(k[:, off:off + n]), Hq, G, d, w, [n])
        assert np.array_equal(Db, D[off:off + n]) and eb[0] == e[b]
        assert D[off:off + n].sum() == pytest.approx(w * Hq, rel=1e-12)
        off += n


# ------------------------------------------------------------------ Eq. 3 / Alg. 1 line 6

def test_recurrence_matches_closed_form_and_mass(oracle):
    rng = np.random.default_rng(26)
    L, n, Hq, w = 7, 50, 8, 4
    # per-layer D with total mass w*Hq, as Eq. 2 guarantees
    Ds = rng.random((L, n))
    Ds *= (w * Hq) / Ds.sum(1, keepdims=True)
    for lam in (0.5, 0.9, 1.0):
        C = np.zeros(n)
        for l in range(L):
            oracle.accumulate(C, np.ascontiguousarray(Ds[l]), lam, 1.0 / w)
        closed = oracle.centrality_closed_form(Ds / w, lam)
        assert C == pytest.approx(closed, rel=1e-12)
        mass = Hq * L if lam == 1.0 else Hq * (1 - lam ** L) / (1 - lam)
        assert C.sum() == pytest.approx(mass, rel=1e-12)
    C = np.zeros(n)
    for l in range(L):
        oracle.accumulate(C, np.ascontiguousarray(Ds[l]), 1e-12, 1.0 / w)
    assert C == pytest.approx(Ds[-1] / w, rel=1e-8)          # lambda -> 0 keeps only the newest layer


def test_accumulate_hand_values(oracle):
    C = np.array([1.0, 2.0, 0.0])
    oracle.accumulate(C, np.array([8.0, 0.0, 4.0]), 0.5, 0.25)
    assert C.tolist() == [2.5, 1.0, 1.0]


# ------------------------------------------------------------------ Eq. 10 / Eq. 13 (selection)

def test_topk_matches_stable_argsort(oracle):
    rng = np.random.default_rng(27)
    for n, k, tail in ((1000, 100, 32), (257, 1, 0), (64, 32, 32), (50, 50, 0), (10, 0, 3)):
        s = rng.standard_normal(n)
        s[rng.integers(0, n, n // 3)] = 0.5                  # many exact ties
        got = oracle.select_topk(s, [n], [k], tail)[0]
        m = n - tail
        order = np.argsort(-s[:m], kind="stable")[:k]
        ref = np.concatenate([np.sort(order), np.arange(m, n)]).astype(np.int32)
        assert np.array_equal(got, ref)
        assert np.all(np.diff(got) > 0)


def test_topk_brute_force_and_degenerate(oracle):
    s = np.array([0.1, 0.7, 0.7, 0.2, 0.7, 0.0, 0.9, 0.3])
    # top-3 of the first 6: 0.7@1, 0.7@2, 0.7@4 (ties -> lower index first, all three fit); tail = 6, 7
    assert oracle.select_topk(s, [8], [3], 2)[0].tolist() == [1, 2, 4, 6, 7]
    assert oracle.select_topk(s, [8], [2], 2)[0].tolist() == [1, 2, 6, 7]
    assert oracle.select_topk(s, [8], [2], 0)[0].tolist() == [1, 6]
    assert oracle.select_topk(np.ones(9), [9], [4], 2)[0].tolist() == [0, 1, 2, 3, 7, 8]   # all equal
    assert oracle.select_topk(s, [8], [6], 2)[0].tolist() == list(range(8))                # k = n - tail
    with pytest.raises(ValueError):
        oracle.select_topk(s, [8], [7], 2)
    # negative scores and signed zeros order like real numbers
    t = np.array([-1.0, -0.0, 0.0, -3.0, 2.0])
    assert oracle.select_topk(t, [5], [3], 0)[0].tolist() == [1, 2, 4]


def test_topk_ragged(oracle):
    rng = np.random.default_rng(28)
    lens, ks = [40, 9, 100], [5, 1, 20]
    s = rng.standard_normal(sum(lens))
    got = oracle.select_topk(s, lens, ks, 4)
    off = 0
    for n, k, g in zip(lens, ks, got):
        seg = s[off:off + n]
        ref = np.concatenate([np.sort(np.argsort(-seg[:n - 4], kind="stable")[:k]), np.arange(n - 4, n)])
        assert np.array_equal(g, ref)
        off += n


# ------------------------------------------------------------------ Alg. 1 line 17 (gather)

def test_gather_identity_and_fancy_index(oracle):
    rng = np.random.default_rng(29)
    src = rng.integers(0, 2 ** 16, (3, 20, 8), dtype=np.uint16)
    ident = oracle.gather_kv(src, [np.arange(20, dtype=np.int32)], [20])
    assert np.array_equal(ident, src)
    lens = [12, 8]
    idx = [np.array([0, 3, 11], np.int32), np.array([1, 7], np.int32)]
    out = oracle.gather_kv(src, idx, lens)
    ref = np.concatenate([src[:, idx[0]], src[:, 12 + idx[1]]], axis=1)
    assert np.array_equal(out, ref)
    src32 = rng.standard_normal((2, 9, 4)).astype(np.float32)
    out = oracle.gather_kv(src32, [np.array([8, 0], np.int32)], [9])
    assert np.array_equal(out, src32[:, [8, 0]])


# ------------------------------------------------------------------ the method's claim on planted structure

def test_truncate_hidden_hand_values_and_identity(oracle):
    # Eq. 11-12: rows and positions at the kept indices; two sequences, second offset by the first's length
    h = (np.arange(7 * 3, dtype=np.float32).reshape(7, 3) * 0.5)
    idx = [np.array([0, 2], np.int32), np.array([1, 3], np.int32)]
    h2, p2 = oracle.truncate_hidden(h, None, idx, [3, 4])
    assert np.array_equal(h2, h[[0, 2, 4, 6]]) and p2.tolist() == [0, 2, 1, 3]
    pos = np.array([10, 11, 12, 100, 101, 102, 103], np.int64)
    h3, p3 = oracle.truncate_hidden(h.view(np.uint32), pos, idx, [3, 4])
    assert np.array_equal(h3.view(np.float32), h2) and p3.tolist() == [10, 12, 101, 103]
    full = [np.arange(3, dtype=np.int32), np.arange(4, dtype=np.int32)]
    h4, p4 = oracle.truncate_hidden(h, pos, full, [3, 4])
    assert np.array_equal(h4, h) and np.array_equal(p4, pos)          # keeping everything changes nothing
    bf = np.arange(5 * 6, dtype=np.uint16).reshape(5, 6)                # 2-byte elements, order reversed
    h5, _ = oracle.truncate_hidden(bf, None, [np.array([4, 0], np.int32)], [5])
    assert np.array_equal(h5, bf[[4, 0]])


def test_block_scores_hand_values_and_invariants(oracle):
    # Sec. 4.1 block-level aggregation: partial last block, per-sequence restart, mass conservation
    s = np.array([1.0, 2.0, 4.0, 8.0, 16.0, 32.0, 64.0, 0.5, 0.25])
    out = oracle.block_scores(s, [7, 2], 3)
    assert out[0].tolist() == [7.0, 56.0, 64.0] and out[1].tolist() == [0.75]
    rng = np.random.default_rng(5)
    x = rng.random(1000)
    for block in (1, 16, 64, 1000, 5000):
        o = oracle.block_scores(x, [1000], block)[0]
        assert len(o) == -(-1000 // block)
        assert o.sum() == pytest.approx(x.sum(), rel=1e-13)
        if block == 1:
            assert np.array_equal(o, x)
        if 1000 % block == 0:
            assert np.allclose(o, x.reshape(-1, block).sum(1), rtol=1e-14, atol=0)
    assert [len(o) for o in oracle.block_scores(np.zeros(5), [0, 5, 0], 4)] == [0, 2, 0]


def test_pivot_metrics_closed_forms(oracle):
    # Eq. 5-6 on hand-made attention rows (probs [Hq][w][n])
    n, w = 40, 2
    uni = np.full((3, w, n), 1.0 / n)
    rho, var = oracle.pivot_metrics([uni])
    assert rho[0] == pytest.approx(4 / n, rel=1e-14) and var[0] == pytest.approx(0.0, abs=1e-30)   # k = ceil(0.1 n) = 4
    one_hot = np.zeros((1, w, n)); one_hot[0, :, 7] = 1.0
    rho, var = oracle.pivot_metrics([one_hot])
    assert rho[0] == pytest.approx(1.0) and var[0] == pytest.approx((1 - 1 / n) / n, rel=1e-13)   # mean of (a-1/n)^2
    # two rows that differ: the pooled vector is their mean; top-4 of n = 40
    a = np.zeros((1, 2, n)); a[0, 0, :4] = 0.25; a[0, 1, 2:6] = 0.25
    pooled = a[0].mean(0)
    rho, var = oracle.pivot_metrics([a])
    assert rho[0] == pytest.approx(np.sort(pooled)[::-1][:4].sum()) == pytest.approx(0.75)
    assert var[0] == pytest.approx(pooled.var(), rel=1e-13)
    # averaged over heads; ceil(0.1 n) with n = 41 is 5; an empty sequence gives zeros
    both = np.concatenate([uni[:1], one_hot], axis=0)
    rho, var = oracle.pivot_metrics([both, np.zeros((2, w, 0))])
    assert rho[0] == pytest.approx((4 / n + 1.0) / 2) and rho[1] == 0.0 and var[1] == 0.0
    u41 = np.full((1, 1, 41), 1 / 41)
    assert oracle.pivot_metrics([u41])[0][0] == pytest.approx(5 / 41)
    # from real rows: matches numpy on the oracle's own probabilities
    wl = workloads.S_F32_W8
    x = workloads.make_layer(wl, 0)
    _, _, _, probs = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads, wl.n_kv_heads,
                                        wl.head_dim, wl.window, wl.seq_lens, want_probs=True)
    rho, var = oracle.pivot_metrics(probs)
    pooled = probs[0].mean(1)
    k = math.ceil(0.1 * pooled.shape[1])
    assert rho[0] == pytest.approx(np.mean([np.sort(r)[::-1][:k].sum() for r in pooled]), rel=1e-12)
    assert var[0] == pytest.approx(pooled.var(axis=1).mean(), rel=1e-12)


def test_transition_scores_hand_values(oracle):
    # Eq. 7-9: a sharp entropy drop with a rise in sparsity and variance between layers 2 and 3
    H = [5.0, 4.9, 4.8, 2.0, 1.9]
    rho = [0.2, 0.2, 0.25, 0.8, 0.8]
    V = [1.0, 1.0, 1.5, 6.0, 6.5]
    T, ls = oracle.transition_scores(H, rho, V, (0.2, 0.3, 0.5))
    # differences: -H: .1 .1 2.8 .1 -> 0 0 1 0 ; rho: 0 .05 .55 0 -> 0 1/11 1 0 ; V: 0 .5 4.5 .5 -> 0 1/9 1 1/9
    assert T.tolist() == pytest.approx([0.0, 0.0, 0.3 / 11 + 0.5 / 9, 1.0, 0.5 / 9])
    assert ls == 4                                                     # argmax_l T_l + 1
    T, ls = oracle.transition_scores([3.0, 3.0, 3.0], [0.1, 0.1, 0.1], [2.0, 2.0, 2.0])
    assert T.tolist() == [0.0, 0.0, 0.0] and ls == 2                   # nothing moves: first candidate
    T, ls = oracle.transition_scores([3.0, 2.0, 1.0], [0.125, 0.25, 0.375], [1.0, 2.0, 3.0])
    assert T.tolist() == [0.0, 0.0, 0.0] and ls == 2                   # equal steps normalise to 0
    T, ls = oracle.transition_scores([1.0, 0.5], [0.1, 0.4], [1.0, 1.0], (1.0, 1.0, 1.0))
    assert ls == 2 and T.tolist() == [0.0, 0.0]                        # a single difference: max == min
    assert oracle.transition_scores([1.0], [0.1], [1.0])[1] == 1
    # weights only scale their own term
    T, _ = oracle.transition_scores(H, rho, V, (1.0, 0.0, 0.0))
    assert T.tolist() == pytest.approx([0.0, 0.0, 0.0, 1.0, 0.0])
    # a second case worked by hand, other weights, entropy that also rises, variance that mostly FALLS:
    #   -dH : -.5  1   .5  -.25  -> (x + .5)/1.5     = 0    1   2/3  1/6
    #   drho: -.125 .5 -.125 .5  -> (x + .125)/.625  = 0    1   0    1
    #   dV  : -2   1  -4   -1    -> (x + 4)/5        = 2/5  1   0    3/5
    #   T = .5 a + .25 b + .25 c = .1, 1, 1/3, 1/12 + 1/4 + 3/20;  argmax at l = 2 -> L* = 3
    # catches: a sign flipped on one metric, min-max taken over the raw metric instead of its differences,
    # weights applied to the wrong metric, L* off by one
    T, ls = oracle.transition_scores([4.0, 4.5, 3.5, 3.0, 3.25], [0.25, 0.125, 0.625, 0.5, 1.0],
                                     [8.0, 6.0, 7.0, 3.0, 2.0], (0.5, 0.25, 0.25))
    assert T.tolist() == pytest.approx([0.0, 0.1, 1.0, 1.0 / 3, 1.0 / 12 + 0.25 + 0.15], rel=1e-14)
    assert ls == 3
    # equal maxima: the lowest layer wins
    T, ls = oracle.transition_scores([2.0, 1.0, 1.0, 0.0], [0.5] * 4, [1.0] * 4, (1.0, 0.0, 0.0))
    assert T.tolist() == [0.0, 1.0, 0.0, 1.0] and ls == 2


def test_golden_rational_sweep(oracle):
    # tests/golden/rational_sweep.json: a four-layer sweep whose every value is an exact rational that follows from
    # integer weights through Eq. 1-10 (written without the oracle).  The fp32 rounding of ln a_j moves a
    # probability by about 1e-7 relative, hence the 2e-6 below.
    # catches: a wrong softmax axis or GQA mapping, a missing 1/w or lambda, pooling over the wrong axis,
    # a wrong difference sign or normalisation in the transition score, a tie broken the wrong way
    from helpers import load_rational_sweep
    doc, qs, ks = load_rational_sweep()
    sh = doc["shape"]
    n, w = sh["n"], sh["window"]
    C = np.zeros(n)
    H, R, V = [], [], []
    for layer, q, k in zip(doc["layers"], qs, ks):
        assert layer["probs"].sum(1) == pytest.approx(1.0, abs=1e-15)        # the fixture itself is consistent
        D, ent, _, probs = oracle.score_layer(q, k, sh["n_q_heads"], sh["n_kv_heads"], sh["head_dim"], w, [n],
                                              scale=sh["scale"], want_probs=True)
        assert probs[0].reshape(-1, n) == pytest.approx(layer["probs"], rel=2e-6)
        assert D == pytest.approx(layer["indegree"], rel=2e-6)
        assert ent[0] == pytest.approx(layer["entropy"], rel=2e-6)
        oracle.accumulate(C, D, doc["lambda"], 1.0 / w)
        assert C == pytest.approx(layer["centrality_after"], rel=2e-6)
        rho, var = oracle.pivot_metrics(probs, doc["top_frac"])
        assert rho[0] == pytest.approx(layer["sparsity"], rel=2e-6)
        assert var[0] == pytest.approx(layer["variance"], rel=1e-5)
        H.append(layer["entropy"]); R.append(layer["sparsity"]); V.append(layer["variance"])
    assert oracle.select_topk(C, [n], [2], 0)[0].tolist() == doc["selection"]["top2"]
    assert oracle.select_topk(C, [n], [1], w)[0].tolist() == doc["selection"]["top1_of_earlier_plus_window"]
    T, ls = oracle.transition_scores(H, R, V, doc["transition_weights"])
    assert T.tolist() == pytest.approx(doc["transition"]["T"], abs=1e-12)
    assert ls == doc["transition"]["pivot_layer"]


def test_golden_fixture_is_reproducible(tmp_path):
    # the committed generator rewrites exactly the committed fixture (no oracle, no GPU involved)
    import importlib.util, os, shutil
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    shutil.copy(os.path.join(here, "make_rational_sweep.py"), tmp_path / "make_rational_sweep.py")
    spec = importlib.util.spec_from_file_location("make_rational_sweep", tmp_path / "make_rational_sweep.py")
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.main()
    assert (tmp_path / "rational_sweep.json").read_text() == open(os.path.join(here, "rational_sweep.json")).read()


def test_planted_hubs_selected_by_centrality(oracle):
    # hubs that are dormant in half of the layers are missed by single-layer scores but kept by C
    wl = workloads.S_BF16
    n, w, k = wl.seq_lens[0], wl.window, wl.k_per_seq[0]
    hubs = workloads.hub_positions(wl)[0]
    C = np.zeros(n)
    total = 0.0
    missed_dormant = 0
    n_dormant = 0
    for l in range(wl.n_layers):
        x = workloads.make_layer(wl, l)
        D, ent, _, _ = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads,
                                          wl.n_kv_heads, wl.head_dim, w, wl.seq_lens)
        total += D.sum()
        oracle.accumulate(C, D, wl.lam, 1.0 / w)
        sel = set(oracle.select_topk(D, [n], [k], w)[0].tolist())
        for p, a in zip(hubs, workloads.hub_active(wl, l)[0]):
            if a:
                assert p in sel, "active hub missed at layer %d" % l
            else:
                n_dormant += 1
                missed_dormant += p not in sel
    assert total == pytest.approx(w * wl.n_q_heads * wl.n_layers, rel=1e-12)   # in-degree totals w*Hq*L
    assert n_dormant > 0 and missed_dormant >= 0.7 * n_dormant
    ever_active = [p for i, p in enumerate(hubs)
                   if any(workloads.hub_active(wl, l)[0][i] for l in range(wl.n_layers))]
    selC = set(oracle.select_topk(C, [n], [k], w)[0].tolist())
    assert ever_active and all(p in selC for p in ever_active)


def test_tiny_config_sweep(oracle):
    wl = workloads.C1_TINY
    n, w = wl.seq_lens[0], wl.window
    hubs = workloads.hub_positions(wl)[0]
    assert len(hubs) == 4 and len(set(hubs)) == 4 and max(hubs) < n - w
    C = np.zeros(n)
    for l in range(wl.n_layers):
        x = workloads.make_layer(wl, l)
        D, ent, _, _ = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads,
                                          wl.n_kv_heads, wl.head_dim, w, wl.seq_lens)
        assert D.sum() == pytest.approx(w * wl.n_q_heads, rel=1e-12)
        assert 0 < ent[0] < math.log(n)
        oracle.accumulate(C, D, wl.lam, 1.0 / w)
    sel = oracle.select_topk(C, [n], [wl.k_per_seq[0]], w)[0]
    assert len(sel) == wl.k_per_seq[0] + w and set(hubs) <= set(sel.tolist())
    assert sel[-w:].tolist() == list(range(n - w, n))
