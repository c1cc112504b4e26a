"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element.

Tolerances (bf16 inputs are exact in both paths; the HIP path accumulates in fp32, whose rounding over
a 128-term dot product and a softmax row of up to 1e6 keys stays below 1e-4 relative):
  in-degree D, centrality C : |gpu - ref| <= 1e-3 * max(|ref|, 1e-6 * mean|ref|)
  entropy                   : rel 1e-3 (abs 1e-4 below 0.1)
  fp32 inputs               : the same checks at 1e-5
  top-k on identical fp32 scores, gather : bit-exact
"""
import math

import numpy as np
import pytest
import torch

import workloads
from helpers import (to_oracle_array, _tol, assert_close_floor, assert_entropy, make_sweep, oracle_layer,
                     sweep_against_oracle)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2604_06746_amd import binding
    return binding


@pytest.fixture(scope="module")
def sweep_mod():
    from paper_2604_06746_amd import sweep
    return sweep


SMALL = ["s_bf16_gqa4", "s_bf16_w64", "s_bf16_d64", "s_bf16_ragged", "s_bf16_r192", "s_bf16_r160", "s_bf16_r512",
         "s_bf16_d64_r256", "s_bf16_w8", "s_bf16_r64", "s_bf16_r96", "s_bf16_r120", "s_bf16_r192_w32", "s_f32_w8", "s_f32_ragged", "c1_tiny"]


# ------------------------------------------------------------------ attention rows (MFMA lane layout)

@pytest.mark.parametrize("name", ["s_bf16_gqa4", "s_bf16_w64", "s_bf16_d64", "s_f32_w8"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("force_simt", [False, True])
def test_attention_rows_match_oracle(B, oracle, name, causal, force_simt):
    wl = workloads.WORKLOADS[name]
    n = wl.seq_lens[0]
    x = workloads.make_layer(wl, 0, "cuda")
    code = B.STRUCTKV_DTYPE_F32 if wl.dtype == "f32" else B.STRUCTKV_DTYPE_BF16
    shape = B.make_shape(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, code, causal)
    ws = torch.empty(B.structkv_workspace_bytes(shape, 1, n) + 4 * n + 1024, dtype=torch.uint8, device="cuda")
    probs = torch.full((wl.n_q_heads, wl.window, n), -1.0, dtype=torch.float32, device="cuda")
    B.structkv_debug_probs(shape, x.q_win, x.k, n, probs, ws, force_simt=force_simt)
    torch.cuda.synchronize()
    _, _, _, p_ref = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads,
                                        wl.n_kv_heads, wl.head_dim, wl.window, [n], causal=causal,
                                        want_probs=True)
    got = probs.cpu().numpy().astype(np.float64)
    assert np.abs(got.sum(-1) - 1.0).max() < 1e-4          # every softmax row sums to 1
    tol = _tol(wl)
    assert np.abs(got - p_ref[0]).max() <= tol * max(p_ref[0].max(), 1e-3)
    assert_close_floor(got, p_ref[0], 5 * tol, "probs")
    if causal:
        w = wl.window
        for i in range(w):
            assert np.all(got[:, i, n - w + i + 1:] == 0.0)


# ------------------------------------------------------------------ score_layer (Eq. 1, 2, 4)

@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("force_simt", [False, True])
def test_score_layer_matches_oracle(B, sweep_mod, oracle, name, causal, force_simt):
    wl = workloads.WORKLOADS[name]
    if causal and min(wl.seq_lens) < wl.window:
        pytest.skip("causal needs n >= w")
    sw = make_sweep(sweep_mod, wl, causal)
    for layer in range(min(wl.n_layers, 2)):
        x = workloads.make_layer(wl, layer, "cuda")
        sw.indeg.fill_(-7.0)
        if force_simt:       # all four kernels of the scoring call, SIMT variants
            B.structkv_debug_score_steps(sw.shape, x.q_win, x.k, sw.cu, sw.indeg, sw.entropy, sw.entropy_per_head,
                                         sw.workspace, 15, force_simt=True)
        else:
            sw.score(x.q_win, x.k)
        torch.cuda.synchronize()
        D, ent, ent_h, _ = oracle_layer(oracle, wl, x, causal)
        got = sw.indeg.cpu().numpy()
        assert_close_floor(got, D, _tol(wl), "indeg layer %d" % layer)
        off = 0
        for n in wl.seq_lens:                       # in-degree total per sequence is w * H_q
            assert abs(got[off:off + n].astype(np.float64).sum() - wl.window * wl.n_q_heads) < 1e-4 * wl.window * wl.n_q_heads
            off += n
        assert_entropy(sw.entropy.cpu().numpy()[:wl.batch], ent, _tol(wl))
        assert_entropy(sw.entropy_per_head.cpu().numpy()[:wl.batch], ent_h, _tol(wl))


@pytest.mark.parametrize("name", ["s_bf16_w64", "s_bf16_gqa4", "s_bf16_r192", "s_f32_ragged"])
def test_per_kv_head_indegree(B, sweep_mod, oracle, name):
    # Eq. 2's inner sum only: per KV head, from the oracle's attention rows
    wl = workloads.WORKLOADS[name]
    sw = make_sweep(sweep_mod, wl)
    x = workloads.make_layer(wl, 0, "cuda")
    G, gs = wl.n_kv_heads, wl.n_q_heads // wl.n_kv_heads
    groups = torch.full((G, wl.total_tokens), -3.0, dtype=torch.float32, device="cuda")
    B.structkv_score_layer_groups(sw.shape, x.q_win, x.k, sw.cu, sw.indeg, groups, sw.entropy, sw.entropy_per_head,
                                  sw.workspace)
    torch.cuda.synchronize()
    D, ent, _, probs = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads, G,
                                          wl.head_dim, wl.window, wl.seq_lens, want_probs=True)
    ref = np.concatenate([p.reshape(G, gs * wl.window, -1).sum(1) for p in probs], axis=1)
    got = groups.cpu().numpy()
    for g in range(G):
        assert_close_floor(got[g], ref[g], _tol(wl), "group %d" % g)
    assert_close_floor(sw.indeg.cpu().numpy(), D, _tol(wl), "indeg")
    assert np.allclose(got.astype(np.float64).sum(0), sw.indeg.cpu().numpy(), rtol=1e-5, atol=1e-7)
    # same call without the extra output: identical in-degree
    keep = sw.indeg.clone()
    sw.score(x.q_win, x.k)
    torch.cuda.synchronize()
    assert torch.equal(keep, sw.indeg)


def test_score_layer_is_deterministic(sweep_mod):
    wl = workloads.S_BF16_RAGGED
    sw = make_sweep(sweep_mod, wl)
    x = workloads.make_layer(wl, 1, "cuda")
    sw.score(x.q_win, x.k)
    a, ea = sw.indeg.clone(), sw.entropy.clone()
    sw.workspace.fill_(0xAB)                               # the workspace needs no particular contents
    sw.score(x.q_win, x.k)
    torch.cuda.synchronize()
    assert torch.equal(a, sw.indeg) and torch.equal(ea, sw.entropy)


def test_score_layer_strided_k_and_explicit_scale(B, sweep_mod, oracle):
    # K stored [total, G, d] (token-major): head stride d, token stride G*d
    wl = workloads.S_BF16
    x = workloads.make_layer(wl, 0, "cuda")
    k_tok_major = x.k.permute(1, 0, 2).contiguous()
    k_view = k_tok_major.permute(1, 0, 2)
    assert k_view.stride() == (wl.head_dim, wl.n_kv_heads * wl.head_dim, 1)
    sw = sweep_mod.LayerSweep(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.torch_dtype, wl.seq_lens,
                              wl.k_per_seq, scale=0.05)
    sw.score(x.q_win, k_view)
    torch.cuda.synchronize()
    D, ent, _, _ = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads,
                                      wl.n_kv_heads, wl.head_dim, wl.window, wl.seq_lens, scale=0.05)
    assert_close_floor(sw.indeg.cpu().numpy(), D, 1e-3, "indeg strided")
    assert_entropy(sw.entropy.cpu().numpy(), ent, 1e-3)


@pytest.mark.parametrize("name", ["s_bf16_w64", "s_bf16_gqa4", "s_bf16_r64"])
def test_late_dominant_keys_rerun_with_running_maximum(sweep_mod, oracle, name):
    # Pass 1 keeps the reference its chunk's FIRST tile set; keys far above it later in the chunk push the sums
    # towards overflow, which the kernel must notice and answer with a rerun under the running maximum.
    # Here every key from 40 % of the sequence on is 24 x larger (logits up to a few hundred above the early ones).
    wl = workloads.WORKLOADS[name]
    x = workloads.make_layer(wl, 0, "cuda")
    n = wl.seq_lens[0]
    k = x.k.clone()
    k[:, int(0.4 * n):, :] *= 24.0
    sw = make_sweep(sweep_mod, wl)
    sw.score(x.q_win, k)
    torch.cuda.synchronize()
    D, ent, ent_h, _ = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(k), wl.n_q_heads, wl.n_kv_heads,
                                          wl.head_dim, wl.window, wl.seq_lens)
    got = sw.indeg.cpu().numpy()
    assert np.isfinite(got).all() and abs(got.sum() - wl.window * wl.n_q_heads) < 1e-2
    assert_close_floor(got, D, 1e-3, "in-degree with late dominant keys")
    assert_entropy(sw.entropy.cpu().numpy(), ent, 1e-3)
    assert_entropy(sw.entropy_per_head.cpu().numpy().ravel(), ent_h.ravel(), 1e-3)


def test_uniform_attention_entropy_is_log_n(sweep_mod):
    # all keys identical -> every row is uniform: D_j = w*H_q/n and entropy = ln n
    n, Hq, G, d, w = 1500, 8, 2, 128, 32
    q = torch.randn(1, Hq, w, d, device="cuda").to(torch.bfloat16)
    k = torch.randn(G, 1, d, device="cuda").to(torch.bfloat16).expand(G, n, d).contiguous()
    sw = sweep_mod.LayerSweep(Hq, G, d, w, torch.bfloat16, [n], [10])
    sw.score(q, k)
    torch.cuda.synchronize()
    assert abs(float(sw.entropy[0]) - math.log(n)) < 1e-3 * math.log(n)
    assert_close_floor(sw.indeg.cpu().numpy(), np.full(n, w * Hq / n), 1e-3, "uniform indeg")


def test_large_logits_do_not_overflow(sweep_mod, oracle):
    # a constant offset on every key shifts each row's logits by up to ~hundreds: needs the running max
    wl = workloads.S_BF16
    x = workloads.make_layer(wl, 0, "cuda")
    k = (x.k.float() + 30.0).to(torch.bfloat16)
    sw = make_sweep(sweep_mod, wl)
    sw.score(x.q_win, k)
    torch.cuda.synchronize()
    D, ent, _, _ = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(k), wl.n_q_heads, wl.n_kv_heads,
                                      wl.head_dim, wl.window, wl.seq_lens)
    got = sw.indeg.cpu().numpy()
    assert np.all(np.isfinite(got))
    assert_close_floor(got, D, 1e-3, "indeg shifted keys")
    assert_entropy(sw.entropy.cpu().numpy(), ent, 1e-3)


def test_empty_sequences_in_batch(sweep_mod, oracle):
    Hq, G, d, w = 8, 2, 128, 32
    lens = [0, 200, 0, 65, 0]
    q = torch.randn(len(lens), Hq, w, d, device="cuda").to(torch.bfloat16)
    k = torch.randn(G, sum(lens), d, device="cuda").to(torch.bfloat16)
    v = torch.randn(G, sum(lens), d, device="cuda").to(torch.bfloat16)
    ks = [0, 20, 0, 5, 0]
    sw = sweep_mod.LayerSweep(Hq, G, d, w, torch.bfloat16, lens, ks)
    sw.keep_tail = 0
    sw.rows_per_seq = ks
    sw.layer(q, k, v)
    torch.cuda.synchronize()
    D, ent, _, _ = oracle.score_layer(to_oracle_array(q), to_oracle_array(k), Hq, G, d, w, lens)
    assert_close_floor(sw.indeg.cpu().numpy(), D, 1e-3, "indeg")
    assert_entropy(sw.entropy.cpu().numpy(), ent, 1e-3)
    got_d = sw.indeg.cpu().numpy()
    ref_idx = oracle.select_topk(got_d, lens, ks, 0)
    got_idx = sw.idx_kv.cpu().numpy()[:sum(ks)]
    assert np.array_equal(got_idx, np.concatenate(ref_idx))
    ref_k = oracle.gather_kv(to_oracle_array(k), ref_idx, lens)
    assert np.array_equal(to_oracle_array(sw.k_cache[0][:, :sum(ks)]), ref_k)


# ------------------------------------------------------------------ accumulate (Eq. 3 / Alg. 1 line 6)

def test_accumulate_matches_oracle(B, oracle):
    rng = np.random.default_rng(5)
    for n in (1, 7, 1024, 4099):
        for lam in (0.5, 0.9, 1.0):
            C = rng.random(n).astype(np.float32)
            D = (rng.random(n) * 50).astype(np.float32)
            c = torch.tensor(C, device="cuda")
            d = torch.tensor(D, device="cuda")
            B.structkv_accumulate_centrality(c, d, lam, 1.0 / 32)
            ref = C.astype(np.float64)
            oracle.accumulate(ref, D.astype(np.float64), float(np.float32(lam)), 1.0 / 32)
            assert np.abs(c.cpu().numpy() - ref).max() <= 2e-7 * np.abs(ref).max()
    # unaligned views take the scalar path
    c = torch.zeros(1001, device="cuda")[1:]
    d = torch.ones(1001, device="cuda")[1:]
    B.structkv_accumulate_centrality(c, d, 0.9, 0.25)
    assert torch.all(c == 0.25)


# ------------------------------------------------------------------ top-k (Eq. 10 / Eq. 13)

def _topk_gpu(B, scores, lens, ks, tail):
    cu = np.concatenate([[0], np.cumsum(lens)]).tolist()
    s = torch.tensor(scores, dtype=torch.float32, device="cuda")
    out = torch.full((max(sum(ks) + tail * len(lens), 1),), -5, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(B.structkv_workspace_bytes(None, len(lens), int(sum(lens))), 256), dtype=torch.uint8,
                     device="cuda")
    ws.fill_(0x5A)
    B.structkv_select_topk(s, cu, ks, tail, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()[:sum(ks) + tail * len(lens)]


@pytest.mark.parametrize("n,k,tail", [(1000, 100, 32), (257, 1, 0), (64, 32, 32), (50, 50, 0), (10, 0, 3),
                                      (4096, 4000, 64), (4097, 17, 1), (20000, 2048, 32), (300000, 16384, 64),
                                      (1, 1, 0), (33, 0, 33),
                                      (2200000, 50000, 64)])      # > 1024 workgroups' worth: shares grow
def test_topk_bit_identical_to_oracle(B, oracle, n, k, tail):
    rng = np.random.default_rng(n * 31 + k)
    for variant in ("normal", "ties", "all_equal", "tiny_range", "signed"):
        if variant == "normal":
            s = rng.standard_normal(n)
        elif variant == "ties":
            s = rng.integers(0, 5, n).astype(np.float64) * 0.25
        elif variant == "all_equal":
            s = np.full(n, 0.125)
        elif variant == "tiny_range":
            s = 1.0 + rng.integers(0, 40, n) * 2.0 ** -23      # neighbours differ in the last mantissa bits
        else:
            s = rng.standard_normal(n) * 10.0 ** rng.integers(-30, 30, n)
            s[rng.integers(0, n, max(1, n // 10))] = 0.0
            s[rng.integers(0, n, max(1, n // 10))] = -0.0
        s32 = s.astype(np.float32)
        got = _topk_gpu(B, s32, [n], [k], tail)
        ref = oracle.select_topk(s32, [n], [k], tail)[0]
        assert np.array_equal(got, ref), variant


def test_topk_ragged_batch(B, oracle):
    rng = np.random.default_rng(77)
    lens = [5000, 0, 33, 12289, 4096, 1]
    ks = [250, 0, 1, 600, 4000, 0]
    tail = 0
    s = rng.standard_normal(sum(lens)).astype(np.float32)
    s[rng.integers(0, sum(lens), 3000)] = 0.5
    got = _topk_gpu(B, s, lens, ks, tail)
    ref = np.concatenate(oracle.select_topk(s, lens, ks, tail))
    assert np.array_equal(got, ref)
    lens, ks, tail = [5000, 40, 12289], [250, 3, 600], 32
    s = rng.standard_normal(sum(lens)).astype(np.float32)
    got = _topk_gpu(B, s, lens, ks, tail)
    ref = np.concatenate(oracle.select_topk(s, lens, ks, tail))
    assert np.array_equal(got, ref)


# ------------------------------------------------------------------ gather (Alg. 1 line 17)

@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64), (torch.bfloat16, 72),
                                     (torch.bfloat16, 3)])
def test_gather_bit_exact(B, oracle, dtype, d):
    rng = np.random.default_rng(9)
    G = 3
    lens = [100, 7, 300]
    rows = [10, 7, 33]
    total = sum(lens)
    k = torch.randn(G, total, d, device="cuda").to(dtype)
    v = torch.randn(G, total, d, device="cuda").to(dtype)
    idx_list = [np.sort(rng.choice(n, r, replace=False)).astype(np.int32) for n, r in zip(lens, rows)]
    idx = torch.tensor(np.concatenate(idx_list), device="cuda")
    cu = [0, 100, 107, 407]
    kd = torch.zeros(G, sum(rows), d, dtype=dtype, device="cuda")
    vd = torch.zeros_like(kd)
    B.structkv_gather_kv(k, v, kd, vd, cu, rows, idx)
    torch.cuda.synchronize()
    assert np.array_equal(to_oracle_array(kd), oracle.gather_kv(to_oracle_array(k), idx_list, lens))
    assert np.array_equal(to_oracle_array(vd), oracle.gather_kv(to_oracle_array(v), idx_list, lens))
    # identity gather, K only
    ident = torch.arange(total, dtype=torch.int32, device="cuda")
    ident_local = torch.cat([torch.arange(n, dtype=torch.int32) for n in lens]).cuda()
    kd2 = torch.zeros_like(k)
    B.structkv_gather_kv(k, None, kd2, None, cu, lens, ident_local)
    torch.cuda.synchronize()
    assert torch.equal(kd2, k) and ident.numel() == total


def test_gather_strided_and_offset_views(B, oracle):
    # token-major source, destination with padding between rows, both at odd element offsets
    G, n, d, r = 2, 50, 128, 9
    base = torch.randn(n, G, d + 8, device="cuda").to(torch.bfloat16)
    src = base[:, :, 3:3 + d].permute(1, 0, 2)              # [G, n, d], misaligned by 6 bytes
    dbase = torch.zeros(G, r, d + 2, dtype=torch.bfloat16, device="cuda")
    dst = dbase[:, :, 1:1 + d]
    idx_np = np.array([0, 5, 6, 7, 20, 33, 41, 48, 49], np.int32)
    B.structkv_gather_kv(src, None, dst, None, [0, n], [r], torch.tensor(idx_np, device="cuda"))
    torch.cuda.synchronize()
    ref = oracle.gather_kv(to_oracle_array(src.contiguous()), [idx_np], [n])
    assert np.array_equal(to_oracle_array(dst.contiguous()), ref)
    assert torch.all(dbase[:, :, 0] == 0) and torch.all(dbase[:, :, -1] == 0)


def test_gather_out_of_range_index_is_contained(B):
    G, n, d = 1, 10, 128
    k = torch.randn(G, n, d, device="cuda").to(torch.bfloat16)
    kd = torch.zeros(G, 3, d, dtype=torch.bfloat16, device="cuda")
    B.structkv_gather_kv(k, None, kd, None, [0, n], [3], torch.tensor([2, 10, -1], dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert torch.equal(kd[0, 0], k[0, 2]) and torch.equal(kd[0, 1], k[0, 0]) and torch.equal(kd[0, 2], k[0, 0])


# ------------------------------------------------------------------ structural truncation (Eq. 11-12)

@pytest.mark.parametrize("dtype,hidden", [(torch.bfloat16, 4096), (torch.float32, 520), (torch.bfloat16, 100)])
def test_truncate_hidden_bit_exact(B, oracle, dtype, hidden):
    rng = np.random.default_rng(hidden)
    lens, ks = [700, 0, 1500], [60, 0, 333]
    total = sum(lens)
    h = torch.randn(total, hidden, device="cuda").to(dtype)
    pos = torch.tensor(np.concatenate([rng.permutation(n) + 1000 * b for b, n in enumerate(lens)]),
                       dtype=torch.int64, device="cuda")
    idx = [np.sort(rng.choice(n, k, replace=False)).astype(np.int32) for n, k in zip(lens, ks)]
    idx_d = torch.tensor(np.concatenate(idx), dtype=torch.int32, device="cuda")
    cu = np.concatenate([[0], np.cumsum(lens)]).tolist()
    rows = sum(ks)
    h_ref, p_ref = oracle.truncate_hidden(to_oracle_array(h), pos.cpu().numpy(), idx, lens)
    h_out = torch.zeros(rows, hidden, dtype=dtype, device="cuda")
    p_out = torch.full((rows,), -1, dtype=torch.int64, device="cuda")
    B.structkv_truncate_hidden(h, h_out, pos, p_out, cu, ks, idx_d)
    torch.cuda.synchronize()
    assert np.array_equal(to_oracle_array(h_out), h_ref) and np.array_equal(p_out.cpu().numpy(), p_ref)
    # identity positions: P' is the index list itself
    _, p_ref0 = oracle.truncate_hidden(to_oracle_array(h), None, idx, lens)
    p_out.fill_(-1)
    B.structkv_truncate_hidden(None, None, None, p_out, cu, ks, idx_d)
    torch.cuda.synchronize()
    assert np.array_equal(p_out.cpu().numpy(), p_ref0) and np.array_equal(p_ref0, np.concatenate(idx))
    # a strided destination (rows of a wider buffer)
    wide = torch.zeros(rows, hidden + 24, dtype=dtype, device="cuda")
    B.structkv_truncate_hidden(h, wide[:, 8:8 + hidden], None, None, cu, ks, idx_d)
    torch.cuda.synchronize()
    assert np.array_equal(to_oracle_array(wide[:, 8:8 + hidden].contiguous()), h_ref)
    assert float(wide[:, :8].abs().sum()) == 0.0 and float(wide[:, 8 + hidden:].abs().sum()) == 0.0


# ------------------------------------------------------------------ block-level aggregation (Sec. 4.1)

@pytest.mark.parametrize("block", [1, 16, 100, 256])
def test_block_scores_match_oracle(B, oracle, block):
    rng = np.random.default_rng(block)
    lens = [5000, 0, 37, 12288]
    s = (rng.random(sum(lens)) ** 4).astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(lens)]).tolist()
    ref = np.concatenate(oracle.block_scores(s, lens, block))
    out = torch.full((len(ref),), -1.0, dtype=torch.float32, device="cuda")
    B.structkv_block_scores(torch.tensor(s, device="cuda"), cu, block, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    # fp32 left-to-right sum of `block` non-negative terms: relative error below block * 2^-24
    assert np.all(np.abs(got - ref) <= block * 2.0 ** -24 * ref + 1e-45)


def test_block_selection_and_block_gather_compose(B, oracle):
    # paged-cache eviction from block scores: keep the best blocks + the blocks of the window, move whole blocks
    rng = np.random.default_rng(11)
    G, n, d, bs = 2, 4096, 64, 16
    nb, keep, tail = n // bs, 40, 2
    c = (rng.random(n) ** 6).astype(np.float32)
    k = torch.randn(G, n, d, device="cuda").to(torch.bfloat16)
    sb = torch.empty(nb, dtype=torch.float32, device="cuda")
    B.structkv_block_scores(torch.tensor(c, device="cuda"), [0, n], bs, sb)
    idx = torch.empty(keep + tail, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.structkv_workspace_bytes(None, 1, nb), dtype=torch.uint8, device="cuda")
    B.structkv_select_topk(sb, [0, nb], [keep], tail, idx, ws)
    kd = torch.empty(G, keep + tail, bs * d, dtype=torch.bfloat16, device="cuda")
    B.structkv_gather_kv(k.view(G, nb, bs * d), None, kd, None, [0, nb], [keep + tail], idx)
    torch.cuda.synchronize()
    ref_blocks = oracle.select_topk(sb.cpu().numpy(), [nb], [keep], tail)[0]
    assert np.array_equal(idx.cpu().numpy(), ref_blocks)
    tokens = (ref_blocks[:, None].astype(np.int64) * bs + np.arange(bs)[None, :]).reshape(-1).astype(np.int32)
    ref_k = oracle.gather_kv(to_oracle_array(k), [tokens], [n])
    assert np.array_equal(to_oracle_array(kd.view(G, (keep + tail) * bs, d)), ref_k)


# ------------------------------------------------------------------ pivot metrics (Eq. 5-6)

# shapes whose metrics come out of the hot path's own scoring (one column-sum plane per query head: a wave's 64 rows
# are one head's window, or its two 32-row blocks are two heads', or its 32 rows are; 1 and 4 waves per workgroup, an
# idle wave, two workgroups per key chunk, d = 64) and shapes that are re-scored head by head (windows of 8 and 24
# rows, which are no whole row block; fp32)
@pytest.mark.parametrize("name,causal", [("s_bf16_w64", False), ("s_bf16_w64", True), ("s_bf16_ragged", False),
                                         ("s_bf16_ragged", True), ("s_bf16_d64", False), ("s_bf16_d64_r256", False),
                                         ("s_bf16_r512", False), ("s_bf16_r192", False), ("s_bf16_gqa4", False),
                                         ("s_bf16_r64", False), ("s_bf16_r192_w32", False), ("s_bf16_r96", False),
                                         ("s_bf16_r120", False),
                                         ("s_bf16_w8", False), ("s_f32_ragged", False), ("c1_tiny", False)])
def test_pivot_metrics_match_oracle(B, sweep_mod, oracle, name, causal):
    wl = workloads.WORKLOADS[name]
    sw = make_sweep(sweep_mod, wl, causal)
    x = workloads.make_layer(wl, 1 % wl.n_layers, "cuda")
    ws = torch.empty(B.structkv_pivot_workspace_bytes(sw.shape, max(wl.seq_lens)), dtype=torch.uint8, device="cuda")
    ws.fill_(0x77)
    rho = torch.full((wl.batch,), -1.0, device="cuda")
    var = torch.full((wl.batch,), -1.0, device="cuda")
    B.structkv_pivot_metrics(sw.shape, x.q_win, x.k, sw.cu, 0.1, rho, var, ws)
    torch.cuda.synchronize()
    _, _, _, probs = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads, wl.n_kv_heads,
                                        wl.head_dim, wl.window, wl.seq_lens, causal=causal, want_probs=True)
    rho_ref, var_ref = oracle.pivot_metrics(probs, 0.1)
    tol = _tol(wl)
    assert np.all(np.abs(rho.cpu().numpy() - rho_ref) <= tol * rho_ref)
    n = np.array(wl.seq_lens, dtype=np.float64)
    # the variance of a near-uniform head is a small difference of squares: floor at 1e-4 of (1/n)^2
    assert np.all(np.abs(var.cpu().numpy() - var_ref) <= 2 * tol * var_ref + 1e-4 / n ** 2)
    assert np.all((rho.cpu().numpy() >= 0.1 - 1e-6) & (rho.cpu().numpy() <= 1 + 1e-6))
    # a different fraction, and the calls leave nothing behind that changes a repeat
    B.structkv_pivot_metrics(sw.shape, x.q_win, x.k, sw.cu, 0.25, rho, var, ws)
    torch.cuda.synchronize()
    rho_ref25, _ = oracle.pivot_metrics(probs, 0.25)
    assert np.all(np.abs(rho.cpu().numpy() - rho_ref25) <= tol * rho_ref25)


@pytest.mark.parametrize("name,causal", [("s_bf16_w64", False), ("s_bf16_ragged", True), ("s_f32_ragged", False)])
def test_score_layer_pivot_equals_the_two_calls(sweep_mod, oracle, name, causal):
    # one per-head scoring yields the layer's scores AND the pivot metrics
    wl = workloads.WORKLOADS[name]
    sw = make_sweep(sweep_mod, wl, causal)
    x = workloads.make_layer(wl, 0, "cuda")
    sw.score(x.q_win, x.k)
    rho, var = sw.pivot_metrics(x.q_win, x.k)
    torch.cuda.synchronize()
    D, ent, ent_h = sw.indeg.clone(), sw.entropy.clone(), sw.entropy_per_head.clone()
    rho, var = rho.clone(), var.clone()
    sw.indeg.fill_(-1.0); sw.entropy.fill_(-1.0); sw.entropy_per_head.fill_(-1.0)
    sw.sparsity.fill_(-1.0); sw.variance.fill_(-1.0)
    r2, v2 = sw.score_pivot(x.q_win, x.k)
    torch.cuda.synchronize()
    assert torch.equal(r2, rho) and torch.equal(v2, var)                     # the same kernels on the same data
    assert_close_floor(sw.indeg.cpu().numpy(), D.cpu().numpy(), 1e-5, "in-degree from the per-head scoring")
    assert torch.allclose(sw.entropy, ent, rtol=1e-5, atol=1e-6)
    assert torch.allclose(sw.entropy_per_head, ent_h, rtol=1e-5, atol=1e-6)
    Dref, eref, _, _ = oracle_layer(oracle, wl, x, causal)
    assert_close_floor(sw.indeg.cpu().numpy(), Dref, _tol(wl), "in-degree vs oracle")
    assert_entropy(sw.entropy.cpu().numpy()[:wl.batch], eref, _tol(wl))


def test_pivot_metrics_uniform_and_empty(B, sweep_mod):
    # zero queries: every head is uniform, so sparsity = ceil(0.1 n)/n and variance = 0; an empty sequence gives 0
    lens = [500, 0, 77]
    sw = sweep_mod.LayerSweep(4, 2, 128, 32, torch.bfloat16, lens, [0, 0, 0])
    q = torch.zeros(3, 4, 32, 128, dtype=torch.bfloat16, device="cuda")
    k = torch.randn(2, sum(lens), 128, device="cuda").to(torch.bfloat16)
    ws = torch.empty(B.structkv_pivot_workspace_bytes(sw.shape, max(lens)), dtype=torch.uint8, device="cuda")
    rho = torch.full((3,), -1.0, device="cuda")
    var = torch.full((3,), -1.0, device="cuda")
    B.structkv_pivot_metrics(sw.shape, q, k, sw.cu, 0.1, rho, var, ws)
    torch.cuda.synchronize()
    r, v = rho.cpu().numpy(), var.cpu().numpy()
    assert abs(r[0] - 50 / 500) < 1e-5 and abs(r[2] - 8 / 77) < 1e-5 and r[1] == 0.0
    assert abs(v[0]) < 1e-12 and abs(v[2]) < 1e-10 and v[1] == 0.0


def test_pivot_layer_of_a_sweep_matches_oracle(B, sweep_mod, oracle):
    # Eq. 4-9 end to end on a small model: per-layer metrics from the GPU, transition score and L* from the library
    wl = workloads.S_BF16_W64
    L = 6
    sw = make_sweep(sweep_mod, wl)
    Hg, Rg, Vg, Ho, Ro, Vo = [], [], [], [], [], []
    for l in range(L):
        x = workloads.make_layer(wl, l % wl.n_layers, "cuda")
        if l >= 3:                       # later layers: sharper queries, so the metrics move
            x.q_win.mul_(1.0 + l)
        sw.score(x.q_win, x.k)
        rho, var = sw.pivot_metrics(x.q_win, x.k)
        torch.cuda.synchronize()
        Hg.append(float(sw.entropy[0])); Rg.append(float(rho[0])); Vg.append(float(var[0]))
        _, ent, _, probs = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads,
                                              wl.n_kv_heads, wl.head_dim, wl.window, wl.seq_lens, want_probs=True)
        r, v = oracle.pivot_metrics(probs)
        Ho.append(ent[0]); Ro.append(r[0]); Vo.append(v[0])
    Tg, lg = B.structkv_transition_scores(Hg, Rg, Vg)
    To, lo = oracle.transition_scores(Ho, Ro, Vo)
    assert lg == lo and lg == 4                                   # the jump is between layers 2 and 3
    assert np.allclose(Tg, To, rtol=0, atol=5e-3)


def test_golden_rational_sweep_on_gpu(B, sweep_mod):
    # the worked example of tests/golden/rational_sweep.json (exact rationals, written without oracle or GPU),
    # through the C ABI in fp32: scoring, recurrence, pivot metrics, both selections, transition score
    from helpers import load_rational_sweep
    doc, qs, ks = load_rational_sweep()
    sh = doc["shape"]
    n, w = sh["n"], sh["window"]
    sw = sweep_mod.LayerSweep(sh["n_q_heads"], sh["n_kv_heads"], sh["head_dim"], w, torch.float32, [n], [1],
                              lam=doc["lambda"], scale=sh["scale"])
    H, R, V = [], [], []
    for layer, q, k in zip(doc["layers"], qs, ks):
        qd, kd = torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda()
        sw.score(qd, kd)
        sw.accumulate()
        rho, var = sw.pivot_metrics(qd, kd, doc["top_frac"])
        torch.cuda.synchronize()
        assert_close_floor(sw.indeg.cpu().numpy(), layer["indegree"], 1e-5, "golden in-degree")
        assert_close_floor(sw.centrality.cpu().numpy(), layer["centrality_after"], 1e-5, "golden centrality")
        assert abs(float(sw.entropy[0]) - layer["entropy"]) <= 1e-5 * layer["entropy"]
        assert abs(float(rho[0]) - layer["sparsity"]) <= 1e-5 * layer["sparsity"]
        assert abs(float(var[0]) - layer["variance"]) <= 1e-4 * layer["variance"]
        H.append(float(sw.entropy[0])); R.append(float(rho[0])); V.append(float(var[0]))
    sw.select_struct()                                   # top-1 of the earlier tokens plus the window, from C
    idx2 = torch.empty(2, dtype=torch.int32, device="cuda")
    B.structkv_select_topk(sw.centrality, sw.cu, [2], 0, idx2, sw.workspace)
    torch.cuda.synchronize()
    assert idx2.cpu().tolist() == doc["selection"]["top2"]
    assert sw.idx_struct.cpu().tolist() == doc["selection"]["top1_of_earlier_plus_window"]
    T, ls = B.structkv_transition_scores(H, R, V, doc["transition_weights"])
    assert ls == doc["transition"]["pivot_layer"]
    assert np.allclose(T, doc["transition"]["T"], rtol=0, atol=1e-3)


# ------------------------------------------------------------------ whole sweeps

def test_tiny_config_full_sweep(sweep_mod, oracle):
    wl = workloads.C1_TINY
    sw, C = sweep_against_oracle(sweep_mod, oracle, wl, range(wl.n_layers), check_dormant=True)
    sw.select_struct()
    torch.cuda.synchronize()
    got = sw.idx_struct.cpu().numpy()[:sw.rows]
    same = np.concatenate(oracle.select_topk(sw.centrality.cpu().numpy(), wl.seq_lens, wl.k_per_seq, wl.window))
    assert np.array_equal(got, same)
    assert set(workloads.hub_positions(wl)[0]) <= set(got.tolist())     # planted hubs are kept by C


@pytest.mark.parametrize("name", ["s_bf16_gqa4", "s_bf16_ragged", "s_f32_ragged"])
def test_small_sweeps(sweep_mod, oracle, name):
    wl = workloads.WORKLOADS[name]
    sweep_against_oracle(sweep_mod, oracle, wl, range(wl.n_layers), check_dormant=True)


@pytest.mark.parametrize("name", ["s_bf16_ragged", "s_f32_ragged", "s_bf16_gqa4"])
def test_fused_score_accumulate_equals_two_calls(sweep_mod, name):
    # the one-call form must give the bits of score_layer followed by accumulate_centrality
    wl = workloads.WORKLOADS[name]
    two, one = make_sweep(sweep_mod, wl), make_sweep(sweep_mod, wl)
    for l in range(3):
        x = workloads.make_layer(wl, l % wl.n_layers, "cuda")
        two.score(x.q_win, x.k)
        two.accumulate()
        one.score_accumulate(x.q_win, x.k)
        torch.cuda.synchronize()
        assert torch.equal(two.indeg, one.indeg) and torch.equal(two.centrality, one.centrality)
        assert torch.equal(two.entropy, one.entropy) and torch.equal(two.entropy_per_head, one.entropy_per_head)


def test_batch_of_64_short_sequences(sweep_mod, oracle):
    # the largest batch the ABI takes, ragged lengths from exactly one window up to a dozen key tiles
    rng = np.random.default_rng(64)
    lens = [int(x) for x in rng.integers(33, 400, 64)]
    lens[5] = 32
    lens[63] = 32
    ks = [max(0, (n - 32) // 7) for n in lens]
    wl = workloads.Workload("t_batch64", 2, 8, 2, 128, tuple(lens), 32, "bf16", tuple(ks), 0, "all")
    sweep_against_oracle(sweep_mod, oracle, wl, range(2))


def test_overlapped_sweep_equals_sequential(sweep_mod):
    # selection + gather of layer l on a side stream under the scoring of layer l+1: same bits as the plain loop
    wl = workloads.S_BF16_RAGGED
    L = 4
    layers = [workloads.make_layer(wl, l % wl.n_layers, "cuda") for l in range(L)]
    seq = make_sweep(sweep_mod, wl, n_layers_out=L)
    for l, x in enumerate(layers):
        seq.layer(x.q_win, x.k, x.v, slot=l)
    torch.cuda.synchronize()
    ovl = make_sweep(sweep_mod, wl, n_layers_out=L)
    side = torch.cuda.Stream()
    for _ in range(2):                                   # twice: buffers are reused across sweeps
        ovl.reset()
        ovl.sweep_overlapped(((x.q_win, x.k, x.v) for x in layers), side)
    torch.cuda.synchronize()
    assert torch.equal(seq.centrality, ovl.centrality)
    assert torch.equal(seq.k_cache, ovl.k_cache) and torch.equal(seq.v_cache, ovl.v_cache)
    assert torch.equal(seq.idx_kv, ovl.idx_kv)


@pytest.mark.parametrize("L,chains", [(1, 2), (4, 2), (5, 2), (7, 3), (3, 4), (9, 4)])
def test_chained_sweep_equals_sequential(sweep_mod, L, chains):
    # layer l on stream l mod chains, the recurrence kept in layer order by events: same bits
    wl = workloads.S_BF16_RAGGED
    layers = [workloads.make_layer(wl, l % wl.n_layers, "cuda") for l in range(L)]
    for l, x in enumerate(layers):
        x.k.mul_(1.0 + 0.1 * l)                          # every layer different, so a swapped order would show
    seq = make_sweep(sweep_mod, wl, n_layers_out=L)
    for l, x in enumerate(layers):
        seq.layer(x.q_win, x.k, x.v, slot=l)
    torch.cuda.synchronize()
    two = make_sweep(sweep_mod, wl, n_layers_out=L)
    sides = [torch.cuda.Stream() for _ in range(chains - 1)]
    for _ in range(2):                                   # twice: buffers are reused across sweeps
        two.reset()
        two.sweep_chains(((x.q_win, x.k, x.v) for x in layers), sides)
    torch.cuda.synchronize()
    assert torch.equal(seq.centrality, two.centrality)
    assert torch.equal(seq.k_cache, two.k_cache) and torch.equal(seq.v_cache, two.v_cache)
    assert torch.equal(seq.idx_kv, two.idx_kv) and torch.equal(seq.indeg, two.indeg)
    assert torch.equal(seq.entropy, two.entropy) and torch.equal(seq.entropy_per_head, two.entropy_per_head)


@pytest.mark.parametrize("overlap", [0, 1, 2, 4])
def test_graph_replays_equal_the_eager_sweep(sweep_mod, overlap):
    # the launch configuration bench.py times: the whole sweep captured once in a HIP graph (one stream, selection +
    # gather on a side stream, or two / four chains of layers) and replayed.  Every replay must give the eager sweep's bits; eager work
    # and synchronisations sit between the replays, and the inputs change between them.
    wl = workloads.S_BF16_W64
    L = 6 if overlap == 4 else 4
    layers = [workloads.make_layer(wl, l % wl.n_layers, "cuda") for l in range(L)]
    ref = make_sweep(sweep_mod, wl, n_layers_out=L)
    sw = make_sweep(sweep_mod, wl, n_layers_out=L)
    side = torch.cuda.Stream() if overlap else None
    sides = [side] + [torch.cuda.Stream() for _ in range(overlap - 2)] if overlap >= 2 else []

    def sweep_on(obj):
        obj.reset()
        if overlap == 1 and obj is sw:
            obj.sweep_overlapped(((x.q_win, x.k, x.v) for x in layers), side)
        elif overlap == 2 and obj is sw:
            obj.sweep_two_chains(((x.q_win, x.k, x.v) for x in layers), side)
        elif overlap > 2 and obj is sw:
            obj.sweep_chains(((x.q_win, x.k, x.v) for x in layers), sides)
        else:
            for l, x in enumerate(layers):
                obj.layer(x.q_win, x.k, x.v, slot=l)
        obj.select_struct()

    warm = torch.cuda.Stream()
    warm.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(warm):
        sweep_on(sw)                                     # every kernel once outside capture
    torch.cuda.current_stream().wait_stream(warm)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sweep_on(sw)
    for rep in range(3):
        if rep:                                          # new inputs in the same buffers, some eager work in between
            for x in layers:
                x.k.mul_(1.0 + 0.25 * rep)
                x.q_win.add_(0.125 * rep)
            sw.indeg.fill_(-1.0); sw.idx_kv.fill_(-1); sw.k_cache.zero_()
            torch.cuda.synchronize()
        sweep_on(ref)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ref.centrality, sw.centrality), rep
        assert torch.equal(ref.idx_kv, sw.idx_kv) and torch.equal(ref.idx_struct, sw.idx_struct), rep
        assert torch.equal(ref.k_cache, sw.k_cache) and torch.equal(ref.v_cache, sw.v_cache), rep
        assert torch.equal(ref.entropy, sw.entropy), rep



# ------------------------------------------------------------------ the fused layer step (Alg. 1 lines 4, 6, 16, 17)

def _both_ways(sweep_mod, wl, make_inputs, layers=2, keep_tail=None, ks=None):
    """layer() (one structkv_layer_step call) against layer_separate_calls() (the four entry points): same bits."""
    a, b = make_sweep(sweep_mod, wl), make_sweep(sweep_mod, wl)
    for sw in (a, b):
        if keep_tail is not None:
            sw.keep_tail = keep_tail
        if ks is not None:
            sw.k_per_seq = list(ks)
        sw.rows_per_seq = [k + sw.keep_tail for k in sw.k_per_seq]
        sw.rows = sum(sw.rows_per_seq)
        sw.idx_kv.fill_(-5); sw.k_cache.fill_(3.0); sw.v_cache.fill_(3.0); sw.workspace.fill_(0xCD)
    for layer in range(layers):
        q, k, v = make_inputs(layer)
        a.layer(q, k, v)
        b.layer_separate_calls(q, k, v)
        torch.cuda.synchronize()
        assert torch.equal(a.indeg, b.indeg) and torch.equal(a.centrality, b.centrality), layer
        assert torch.equal(a.entropy, b.entropy) and torch.equal(a.entropy_per_head, b.entropy_per_head), layer
        assert torch.equal(a.idx_kv, b.idx_kv), layer
        assert torch.equal(a.k_cache, b.k_cache) and torch.equal(a.v_cache, b.v_cache), layer
    return a


@pytest.mark.parametrize("name", SMALL + ["c2_llama8b_32k", "c5_ragged_batch8"])
def test_layer_step_equals_the_four_calls(sweep_mod, name):
    wl = workloads.WORKLOADS[name]

    def inputs(layer):
        x = workloads.make_layer(wl, layer, "cuda")
        return x.q_win, x.k, x.v
    _both_ways(sweep_mod, wl, inputs, layers=min(wl.n_layers, 2))
    torch.cuda.empty_cache()


def test_layer_step_degenerate_batches(sweep_mod):
    # empty sequences, zero budgets, no window, a budget that takes the whole prefix, all-equal scores (ties)
    wl = workloads.Workload("t_degenerate", 2, 8, 2, 128, (0, 200, 0, 65, 3000, 0), 32, "bf16", (0, 20, 0, 0, 2968, 0), 0)
    g = torch.Generator(device="cuda"); g.manual_seed(5)

    def inputs(layer):
        q = torch.randn(wl.batch, 8, 32, 128, generator=g, device="cuda").to(torch.bfloat16)
        k = torch.randn(2, wl.total_tokens, 128, generator=g, device="cuda").to(torch.bfloat16)
        v = torch.randn(2, wl.total_tokens, 128, generator=g, device="cuda").to(torch.bfloat16)
        if layer == 1:
            q.zero_()                     # uniform attention: every score equal, selection by index alone
        return q, k, v
    # (an empty sequence cannot keep a window: with keep_tail > 0 every sequence needs n_b >= keep_tail)
    _both_ways(sweep_mod, wl, inputs, keep_tail=0)
    _both_ways(sweep_mod, wl, inputs, keep_tail=0, ks=(0, 200, 0, 5, 1, 0))
    _both_ways(sweep_mod, wl, inputs, keep_tail=0, ks=(0, 0, 0, 0, 0, 0))
    # with the window kept: zero budgets (the window alone), the whole prefix, one token short of it
    wl2 = workloads.Workload("t_degenerate_tail", 2, 8, 2, 128, (32, 200, 65, 3000), 32, "bf16", (0, 0, 33, 2968), 0)

    def inputs2(layer):
        q = torch.randn(wl2.batch, 8, 32, 128, generator=g, device="cuda").to(torch.bfloat16)
        k = torch.randn(2, wl2.total_tokens, 128, generator=g, device="cuda").to(torch.bfloat16)
        v = torch.randn(2, wl2.total_tokens, 128, generator=g, device="cuda").to(torch.bfloat16)
        if layer == 1:
            q.zero_()
        return q, k, v
    _both_ways(sweep_mod, wl2, inputs2)
    _both_ways(sweep_mod, wl2, inputs2, ks=(0, 167, 32, 1))


def test_layer_step_odd_head_dim(sweep_mod):
    # head_dim 36 (72-byte rows: SIMT scoring, 4-byte gather units)
    wl = workloads.Workload("t_d36", 2, 4, 2, 36, (900, 70), 16, "bf16", (40, 6), 0)
    g = torch.Generator(device="cuda"); g.manual_seed(6)

    def inputs(layer):
        q = torch.randn(2, 4, 16, 36, generator=g, device="cuda").to(torch.bfloat16)
        k = torch.randn(2, 970, 36, generator=g, device="cuda").to(torch.bfloat16)
        v = torch.randn(2, 970, 36, generator=g, device="cuda").to(torch.bfloat16)
        return q, k, v
    _both_ways(sweep_mod, wl, inputs)


def test_layer_step_rejects_bad_arguments(B, sweep_mod):
    wl = workloads.S_BF16
    sw = make_sweep(sweep_mod, wl)
    x = workloads.make_layer(wl, 0, "cuda")
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.StructKVError) as e:
        B.structkv_layer_step(sw.shape, x.q_win, x.k, x.v, sw.cu, sw.k_per_seq, sw.keep_tail, sw.indeg, sw.centrality,
                              0.9, 1.0 / 32, sw.entropy, None, sw.idx_kv, sw.k_cache[0], sw.v_cache[0], small)
    assert e.value.status == B.STRUCTKV_ERR_WORKSPACE
    with pytest.raises(B.StructKVError) as e:
        B.structkv_layer_step(sw.shape, x.q_win, x.k, x.v, sw.cu, [wl.seq_lens[0]], sw.keep_tail, sw.indeg, None,
                              0.9, 1.0 / 32, sw.entropy, None, sw.idx_kv, sw.k_cache[0], sw.v_cache[0], sw.workspace)
    assert e.value.status == B.STRUCTKV_ERR_INVALID_ARG
    with pytest.raises(B.StructKVError) as e:
        B.structkv_layer_step(sw.shape, x.q_win, x.k, x.v, sw.cu, sw.k_per_seq, sw.keep_tail, sw.indeg, sw.centrality,
                              1.5, 1.0 / 32, sw.entropy, None, sw.idx_kv, sw.k_cache[0], sw.v_cache[0], sw.workspace)
    assert e.value.status == B.STRUCTKV_ERR_INVALID_ARG


# ------------------------------------------------------------------ cache-sized groups of sequences

def test_grouped_scoring_is_bit_identical(B, sweep_mod, oracle):
    # a batch whose keys (226 MB) exceed the memory-side cache can be scored group by group (pass 1, combine, pass 2
    # of a group back to back; the measurement hook's bit 16); same plan, so the same bits as one launch per kernel
    Hq, G, d, w = 32, 8, 128, 32
    lens = [40000, 300, 0, 70000, 33]
    g = torch.Generator(device="cuda"); g.manual_seed(21)
    q = torch.randn(len(lens), Hq, w, d, generator=g, device="cuda").to(torch.bfloat16)
    k = torch.randn(G, sum(lens), d, generator=g, device="cuda").to(torch.bfloat16)
    sw = sweep_mod.LayerSweep(Hq, G, d, w, torch.bfloat16, lens, [n // 20 for n in lens])
    sw.keep_tail = 0
    sw.workspace.fill_(0x5A)
    sw.score(q, k)                                             # one launch per kernel
    torch.cuda.synchronize()
    a, ea, eh = sw.indeg.clone(), sw.entropy.clone(), sw.entropy_per_head.clone()
    sw.indeg.fill_(-1.0); sw.entropy.fill_(-1.0); sw.entropy_per_head.fill_(-1.0); sw.workspace.fill_(0xA5)
    # grouped: [40000, 300, 0], [70000, 33]
    B.structkv_debug_score_steps(sw.shape, q, k, sw.cu, sw.indeg, sw.entropy, sw.entropy_per_head, sw.workspace, 15 | 16)
    torch.cuda.synchronize()
    assert torch.equal(a, sw.indeg) and torch.equal(ea, sw.entropy) and torch.equal(eh, sw.entropy_per_head)
    # kernel by kernel over the groups gives the same bits as well
    sw.indeg.fill_(-1.0); sw.workspace.fill_(0x11)
    for mask in (1, 2, 4, 8):
        B.structkv_debug_score_steps(sw.shape, q, k, sw.cu, sw.indeg, sw.entropy, sw.entropy_per_head, sw.workspace,
                                     mask | 16)
    torch.cuda.synchronize()
    assert torch.equal(a, sw.indeg) and torch.equal(ea, sw.entropy)
    # and against the oracle on the two short sequences (the long ones are covered by the full-size tests)
    for b in (1, 4):
        off = sum(lens[:b])
        D, ent, _, _ = oracle.score_layer(to_oracle_array(q[b:b + 1]), to_oracle_array(k[:, off:off + lens[b]]), Hq, G, d, w,
                                          [lens[b]])
        assert_close_floor(a[off:off + lens[b]].cpu().numpy(), D, 1e-3, "indeg seq %d" % b)
        assert_entropy(ea[b:b + 1].cpu().numpy(), ent, 1e-3)
    assert float(ea[2]) == 0.0
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ cache policy of the K tiles

@pytest.mark.parametrize("Hq,G,d,w,causal", [(2, 2, 64, 32, 0), (4, 2, 64, 32, 1), (8, 2, 64, 32, 0), (8, 2, 64, 64, 1),
                                            (2, 2, 128, 32, 1), (4, 2, 128, 32, 0), (8, 2, 128, 32, 1), (8, 2, 128, 64, 0)])
def test_streamed_k_tiles_give_the_same_bits(B, sweep_mod, Hq, G, d, w, causal):
    # every tiling of the MFMA kernels (1, 2 or 4 waves per workgroup, one or two row blocks per wave, both head
    # sizes) with the K tiles fetched non-temporally -- what the library does by itself from 256 MiB of K per layer
    # on (the full-size tests) -- against the cached fetches these sizes get: a cache policy changes no bit
    lens = [1500, 0, 4097, 333]
    g = torch.Generator(device="cuda"); g.manual_seed(1000 * Hq + d + w)
    q = torch.randn(len(lens), Hq, w, d, generator=g, device="cuda").to(torch.bfloat16)
    k = torch.randn(G, sum(lens), d, generator=g, device="cuda").to(torch.bfloat16)
    sw = sweep_mod.LayerSweep(Hq, G, d, w, torch.bfloat16, lens, [n // 10 for n in lens], causal=bool(causal))
    sw.score(q, k)
    torch.cuda.synchronize()
    a, ea, eh = sw.indeg.clone(), sw.entropy.clone(), sw.entropy_per_head.clone()
    sw.indeg.fill_(-1.0); sw.entropy.fill_(-1.0); sw.entropy_per_head.fill_(-1.0); sw.workspace.fill_(0xA5)
    B.structkv_debug_score_steps(sw.shape, q, k, sw.cu, sw.indeg, sw.entropy, sw.entropy_per_head, sw.workspace, 15 | 32)
    torch.cuda.synchronize()
    assert torch.equal(a, sw.indeg) and torch.equal(ea, sw.entropy) and torch.equal(eh, sw.entropy_per_head)
