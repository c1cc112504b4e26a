"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Layers of each full-size configuration are generated on the GPU (the same generator bench.py uses), run
through the HIP path and compared with the CPU oracle on the same bits: in-degree, entropy and the centrality
accumulated over the sampled layers element by element (the oracle finishes a 128K-token layer in seconds on
the host cores), the top-k bit-for-bit on the GPU's own scores, the gather byte-for-byte.  Four layers of the
32K configuration, four layers of the ragged batch, an early and a late layer of the million-token sequence (each
holds active and dormant hubs), every layer of the headline 128K configuration.
"""
import numpy as np
import pytest
import torch

import workloads
from helpers import sweep_against_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sweep_mod():
    from paper_2604_06746_amd import sweep
    return sweep


@pytest.mark.parametrize("name,layers", [("c2_llama8b_32k", (0, 9, 17, 30)), ("c3_llama8b_128k", (5,)),
                                         ("c5_ragged_batch8", (3, 12, 20, 28))])
def test_full_size_layers(sweep_mod, oracle, name, layers):
    wl = workloads.WORKLOADS[name]
    sw, C = sweep_against_oracle(sweep_mod, oracle, wl, layers, check_dormant=True)
    # the structural selection on the centrality accumulated over these layers (Eq. 10), on the GPU's own scores
    sw.select_struct()
    torch.cuda.synchronize()
    got = sw.idx_struct.cpu().numpy()[:sw.rows]
    c_gpu = sw.centrality.cpu().numpy()
    assert np.array_equal(got, np.concatenate(oracle.select_topk(c_gpu, wl.seq_lens, wl.k_per_seq, wl.window)))
    torch.cuda.empty_cache()


def test_headline_config_whole_sweep(sweep_mod, oracle):
    # every layer of the configuration bench.py times: D, entropy, C, per-layer top-k and gather against the
    # oracle layer by layer, then the structural selection on the accumulated centrality
    wl = workloads.C3_128K
    sw, C = sweep_against_oracle(sweep_mod, oracle, wl, range(wl.n_layers), check_dormant=True)
    sw.select_struct()
    torch.cuda.synchronize()
    got = sw.idx_struct.cpu().numpy()[:sw.rows]
    c_gpu = sw.centrality.cpu().numpy()
    assert np.array_equal(got, np.concatenate(oracle.select_topk(c_gpu, wl.seq_lens, wl.k_per_seq, wl.window)))
    ref = oracle.select_topk(C, wl.seq_lens, wl.k_per_seq, wl.window)[0]
    n, w, k = wl.seq_lens[0], wl.window, wl.k_per_seq[0]
    tau = np.sort(C[:n - w])[::-1][k - 1]
    for j in set(got.tolist()) ^ set(ref.tolist()):
        assert abs(C[j] - tau) <= 1e-3 * abs(tau)
    hubs = workloads.hub_positions(wl)[0]
    ever = {p for i, p in enumerate(hubs) if any(workloads.hub_active(wl, l)[0][i] for l in range(wl.n_layers))}
    assert ever and ever <= set(got.tolist())
    torch.cuda.empty_cache()


@pytest.mark.parametrize("chains", [0, 2, 4])
def test_headline_graph_with_several_streams_equals_eager(sweep_mod, chains):
    # bench.py's launch configuration at full size (a few layers of it): the sweep captured in a HIP graph on
    # several streams (chains of layers, or selection + gather on a side stream), replayed twice, against
    # plain eager launches -- same bits
    from helpers import make_sweep
    wl = workloads.C3_128K
    L = 6 if chains == 4 else 4
    layers = [workloads.make_layer(wl, l, "cuda") for l in range(L)]
    ref = make_sweep(sweep_mod, wl, n_layers_out=L)
    for l, x in enumerate(layers):
        ref.layer(x.q_win, x.k, x.v, slot=l)
    ref.select_struct()
    torch.cuda.synchronize()
    sw = make_sweep(sweep_mod, wl, n_layers_out=L)
    side = torch.cuda.Stream()
    sides = [side] + [torch.cuda.Stream() for _ in range(max(chains - 2, 0))]

    def step():
        sw.reset()
        if chains:
            sw.sweep_chains(((x.q_win, x.k, x.v) for x in layers), sides)
        else:
            sw.sweep_overlapped(((x.q_win, x.k, x.v) for x in layers), side)
        sw.select_struct()

    warm = torch.cuda.Stream()
    warm.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(warm):
        step()
    torch.cuda.current_stream().wait_stream(warm)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(2):
        sw.indeg.fill_(-1.0); sw.idx_kv.fill_(-1); sw.k_cache.zero_(); sw.centrality.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ref.centrality, sw.centrality) and torch.equal(ref.idx_struct, sw.idx_struct), rep
        assert torch.equal(ref.idx_kv, sw.idx_kv), rep
        assert torch.equal(ref.k_cache, sw.k_cache) and torch.equal(ref.v_cache, sw.v_cache), rep
    del graph, layers
    torch.cuda.empty_cache()


def test_pivot_metrics_at_32k(sweep_mod, oracle):
    # Eq. 5-6 on one layer of the 32K configuration against the oracle's attention rows (268 MB of fp64)
    from paper_2604_06746_amd import binding as B
    from helpers import make_sweep, to_oracle_array
    wl = workloads.C2_32K
    sw = make_sweep(sweep_mod, wl)
    x = workloads.make_layer(wl, 7, "cuda")
    ws = torch.empty(B.structkv_pivot_workspace_bytes(sw.shape, wl.seq_lens[0]), dtype=torch.uint8, device="cuda")
    rho = torch.zeros(1, device="cuda")
    var = torch.zeros(1, device="cuda")
    B.structkv_pivot_metrics(sw.shape, x.q_win, x.k, sw.cu, 0.1, rho, var, ws)
    torch.cuda.synchronize()
    _, _, _, probs = oracle.score_layer(to_oracle_array(x.q_win), to_oracle_array(x.k), wl.n_q_heads, wl.n_kv_heads,
                                        wl.head_dim, wl.window, wl.seq_lens, want_probs=True)
    rho_ref, var_ref = oracle.pivot_metrics(probs, 0.1)
    assert abs(rho.item() - rho_ref[0]) <= 1e-3 * rho_ref[0]
    assert abs(var.item() - var_ref[0]) <= 2e-3 * var_ref[0]
    del ws
    torch.cuda.empty_cache()


def test_million_token_layers(sweep_mod, oracle):
    # an early and a late layer, both with active and with dormant hubs among the 1024 planted ones
    wl = workloads.C4_1M
    for layer in (2, 29):
        act = workloads.hub_active(wl, layer)[0]
        assert any(act) and not all(act)
    sweep_against_oracle(sweep_mod, oracle, wl, (2, 29), check_dormant=True)
    torch.cuda.empty_cache()


def test_c2_sweep_selects_planted_hubs(sweep_mod):
    # eight layers of the 32K configuration: the accumulated centrality keeps every hub that was active in
    # any of them, and the in-degree totals are w*H_q per layer
    wl = workloads.C2_32K
    from helpers import make_sweep
    sw = make_sweep(sweep_mod, wl)
    hubs = workloads.hub_positions(wl)[0]
    ever = set()
    mass = 0.0
    layers = range(8)
    for l in layers:
        x = workloads.make_layer(wl, l, "cuda")
        sw.layer(x.q_win, x.k, x.v)
        mass += float(sw.indeg.double().sum())
        ever |= {p for p, a in zip(hubs, workloads.hub_active(wl, l)[0]) if a}
    sw.select_struct()
    torch.cuda.synchronize()
    sel = set(sw.idx_struct.cpu().numpy()[:sw.rows].tolist())
    assert ever and ever <= sel
    assert abs(mass - wl.window * wl.n_q_heads * len(layers)) < 1e-4 * wl.window * wl.n_q_heads * len(layers)
