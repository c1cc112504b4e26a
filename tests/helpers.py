"""Conversions and comparison helpers shared by the tests (no method arithmetic)."""
import numpy as np
import torch

import workloads


to_oracle_array = workloads.to_oracle_array   # torch fp32 / bf16 tensor -> the host array the oracle takes


def _tol(wl):
    return 1e-5 if wl.dtype == "f32" else 1e-3


def assert_close_floor(got, ref, rel, what):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    floor = 1e-6 * np.abs(ref).mean() if ref.size else 0.0
    err = np.abs(got - ref) / np.maximum(np.abs(ref), floor)
    worst = int(np.argmax(err)) if err.size else 0
    assert err.size == 0 or err.max() <= rel, "%s: max rel err %.3e at %d (got %r ref %r)" % (
        what, err.max(), worst, got.flat[worst], ref.flat[worst])


def assert_entropy(got, ref, rel):
    for g, r in zip(np.asarray(got, dtype=np.float64).ravel(), np.asarray(ref).ravel()):
        if abs(r) < 0.1:
            assert abs(g - r) <= 1e-4, (g, r)
        else:
            assert abs(g - r) <= rel * abs(r), (g, r)


def make_sweep(sweep_mod, wl, causal=False, n_layers_out=1):
    return sweep_mod.LayerSweep(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.torch_dtype,
                                wl.seq_lens, wl.k_per_seq, lam=wl.lam, causal=causal, n_layers_out=n_layers_out)


def oracle_layer(oracle, wl, x, causal=False):
    return oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads, wl.n_kv_heads,
                              wl.head_dim, wl.window, wl.seq_lens, causal=causal)



def sweep_against_oracle(sweep_mod, oracle, wl, layers, check_dormant=False):
    sw = make_sweep(sweep_mod, wl)
    tol = _tol(wl)
    C = np.zeros(wl.total_tokens)
    w = wl.window
    total_mass = 0.0
    for layer in layers:
        x = workloads.make_layer(wl, layer, "cuda")
        sw.layer(x.q_win, x.k, x.v)
        torch.cuda.synchronize()
        D, ent, _, _ = oracle_layer(oracle, wl, x)
        got_d = sw.indeg.cpu().numpy()
        assert_close_floor(got_d, D, tol, "indeg layer %d" % layer)
        assert_entropy(sw.entropy.cpu().numpy()[:wl.batch], ent, tol)
        total_mass += float(got_d.astype(np.float64).sum())
        oracle.accumulate(C, D, wl.lam, 1.0 / w)
        assert_close_floor(sw.centrality.cpu().numpy(), C, tol, "centrality layer %d" % layer)
        # selection: bit-identical on the GPU's own fp32 scores ...
        got_idx = sw.idx_kv.cpu().numpy()[:sw.rows]
        same_scores = np.concatenate(oracle.select_topk(got_d, wl.seq_lens, wl.k_per_seq, w))
        assert np.array_equal(got_idx, same_scores), "top-k differs on identical scores, layer %d" % layer
        # ... and end to end: only near-threshold ties may differ from the fp64 selection
        ref_idx = oracle.select_topk(D, wl.seq_lens, wl.k_per_seq, w)
        off = ro = 0
        for b, n in enumerate(wl.seq_lens):
            gi = set(got_idx[ro:ro + sw.rows_per_seq[b]].tolist())
            ri = set(ref_idx[b].tolist())
            Db = D[off:off + n]
            if wl.k_per_seq[b] > 0:
                tau = np.sort(Db[:n - w])[::-1][wl.k_per_seq[b] - 1]
                for j in gi ^ ri:
                    assert abs(Db[j] - tau) <= tol * abs(tau), (layer, b, j, Db[j], tau)
            off += n
            ro += sw.rows_per_seq[b]
        # gather: bit-exact copy of the rows the GPU selected
        idx_list, ro = [], 0
        for r in sw.rows_per_seq:
            idx_list.append(got_idx[ro:ro + r])
            ro += r
        assert np.array_equal(to_oracle_array(sw.k_cache[0][:, :sw.rows]),
                              oracle.gather_kv(to_oracle_array(x.k), idx_list, wl.seq_lens))
        assert np.array_equal(to_oracle_array(sw.v_cache[0][:, :sw.rows]),
                              oracle.gather_kv(to_oracle_array(x.v), idx_list, wl.seq_lens))
        if check_dormant:
            hubs = workloads.hub_positions(wl)
            act = workloads.hub_active(wl, layer)
            ro = 0
            n_dormant = dormant_kept = 0
            for b in range(wl.batch):
                sel = set(got_idx[ro:ro + sw.rows_per_seq[b]].tolist())
                for p, a in zip(hubs[b], act[b]):
                    if a:
                        assert p in sel, "active hub %d missed at layer %d" % (p, layer)
                    else:
                        n_dormant += 1
                        dormant_kept += p in sel
                ro += sw.rows_per_seq[b]
            # a hub that is dormant at this layer is an ordinary key here: a single-layer snapshot keeps it only
            # by chance (the budget is 3-6 % of the tokens)
            assert dormant_kept <= 0.25 * max(n_dormant, 1) + 2, (layer, dormant_kept, n_dormant)
    assert abs(total_mass - w * wl.n_q_heads * wl.batch * len(layers)) < 1e-4 * w * wl.n_q_heads * wl.batch * len(layers)
    return sw, C




def load_rational_sweep():
    """tests/golden/rational_sweep.json as floats plus the fp32 inputs that realise it:
    (doc, q [L][1,Hq,w,d] fp32, k [L][1,n,d] fp32).  Key j of a layer is (ln a_j, ln b_j, 0, 0)."""
    import json, os
    from fractions import Fraction
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "rational_sweep.json")) as f:
        doc = json.load(f)
    fr = lambda v: float(Fraction(v))
    for layer in doc["layers"]:
        layer["probs"] = np.array([[fr(x) for x in row] for row in layer["probs"]])
        for key in ("indegree", "centrality_after"):
            layer[key] = np.array([fr(x) for x in layer[key]])
        for key in ("entropy", "sparsity", "variance"):
            layer[key] = fr(layer[key]) if "/" in layer[key] else float(layer[key])
    doc["lambda"] = fr(doc["lambda"])
    doc["transition"]["T"] = [float(t) for t in doc["transition"]["T"]]
    sh = doc["shape"]
    qs, ks = [], []
    for layer in doc["layers"]:
        q = np.zeros((1, sh["n_q_heads"], sh["window"], sh["head_dim"]), np.float32)
        q[0, 0, 0, 0], q[0, 0, 1, 0], q[0, 1, 0, 1], q[0, 1, 1, 1] = 1.0, 2.0, 1.0, 2.0
        k = np.zeros((1, sh["n"], sh["head_dim"]), np.float32)
        k[0, :, 0] = np.log(np.array(layer["head0_weights"], np.float64))
        k[0, :, 1] = np.log(np.array(layer["head1_weights"], np.float64))
        qs.append(q); ks.append(k)
    return doc, qs, ks
