"""CPU-only checks of the C ABI: the library loads, exports what the header declares, and rejects
bad arguments before touching the GPU."""
import ctypes

import numpy as np
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    lib = os.path.join(ROOT, "paper_2604_06746_amd", "libstructkv.so")
    if not os.path.exists(lib):
        from paper_2604_06746_amd import build
        build.build(verbose=False)
    from paper_2604_06746_amd import binding
    return binding


def _declared():
    names = set()
    for header in ("structkv.h", "structkv_debug.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(structkv_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported(B):
    names = _declared()
    assert {"structkv_score_layer", "structkv_accumulate_centrality", "structkv_select_topk",
            "structkv_gather_kv"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(B.EXPORTS)
    assert B.structkv_version() >= 100


def test_workspace_query(B):
    s = B.make_shape(32, 8, 128, 64, B.STRUCTKV_DTYPE_BF16)
    a = B.structkv_workspace_bytes(s, 1, 131072)
    b = B.structkv_workspace_bytes(s, 1, 262144)
    assert 0 < a < b and a % 256 == 0
    assert 0 < B.structkv_workspace_bytes(None, 8, 500000) < a
    assert B.structkv_workspace_bytes(s, -1, 10) == 0
    assert B.structkv_workspace_bytes(s, B.STRUCTKV_MAX_BATCH + 1, 10) == 0
    bad = B.make_shape(32, 5, 128, 64, B.STRUCTKV_DTYPE_BF16)
    assert B.structkv_workspace_bytes(bad, 1, 10) == 0


def _status(B, fn, *args):
    st = fn(*args)
    return st, B.structkv_last_error()


def test_invalid_arguments_are_rejected_on_the_host(B):
    lib = B._lib
    i64 = ctypes.c_int64
    cu = (i64 * 2)(0, 100)
    fake = ctypes.c_void_p(4096)      # never dereferenced: validation fails first
    ws_bytes = 1 << 20

    def score(shape, cu_arr=cu, batch=1, ws=fake, wsb=ws_bytes, kst=128):
        return lib.structkv_score_layer(ctypes.byref(shape), fake, fake, 100 * 128, kst, batch, cu_arr, fake,
                                        fake, None, ws, wsb, None)

    ok_shape = B.make_shape(8, 2, 128, 32, B.STRUCTKV_DTYPE_BF16)
    assert score(B.make_shape(8, 3, 128, 32, 1)) == B.STRUCTKV_ERR_INVALID_ARG
    assert "divide" in B.structkv_last_error()
    assert score(B.make_shape(8, 2, 128, 0, 1)) == B.STRUCTKV_ERR_INVALID_ARG
    assert score(B.make_shape(8, 2, 1024, 32, 1)) == B.STRUCTKV_ERR_UNSUPPORTED
    assert score(B.make_shape(8, 2, 128, 32, 7)) == B.STRUCTKV_ERR_UNSUPPORTED
    assert score(B.make_shape(8, 2, 128, 32, 1, scale=-1.0)) == B.STRUCTKV_ERR_INVALID_ARG
    assert score(ok_shape, cu_arr=(i64 * 2)(1, 100)) == B.STRUCTKV_ERR_INVALID_ARG
    assert score(ok_shape, cu_arr=(i64 * 3)(0, 100, 50), batch=2) == B.STRUCTKV_ERR_INVALID_ARG
    assert score(ok_shape, batch=B.STRUCTKV_MAX_BATCH + 1) == B.STRUCTKV_ERR_UNSUPPORTED
    assert score(ok_shape, kst=64) == B.STRUCTKV_ERR_INVALID_ARG
    assert score(ok_shape, ws=None) == B.STRUCTKV_ERR_WORKSPACE
    assert score(ok_shape, ws=ctypes.c_void_p(4096 + 8)) == B.STRUCTKV_ERR_WORKSPACE
    assert score(ok_shape, wsb=16) == B.STRUCTKV_ERR_WORKSPACE
    assert "needs" in B.structkv_last_error()
    causal = B.make_shape(8, 2, 128, 32, 1, causal=True)
    assert score(causal, cu_arr=(i64 * 2)(0, 10)) == B.STRUCTKV_ERR_INVALID_ARG
    assert score(ok_shape, batch=0) == B.STRUCTKV_OK and B.structkv_last_error() == ""

    acc = lib.structkv_accumulate_centrality
    assert acc(fake, fake, 10, 0.0, 0.1, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert acc(fake, fake, 10, 1.5, 0.1, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert acc(fake, fake, 10, 0.9, 0.0, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert acc(None, fake, 10, 0.9, 0.1, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert acc(fake, fake, -1, 0.9, 0.1, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert acc(None, None, 0, 0.9, 0.1, None) == B.STRUCTKV_OK

    def fused(cen=fake, indeg=ctypes.c_void_p(8192), lam=0.9, inv_w=0.1, batch=1):
        return lib.structkv_score_layer_accumulate(ctypes.byref(ok_shape), fake, fake, 100 * 128, 128, batch, cu,
                                                   indeg, cen, lam, inv_w, fake, None, None, ws_bytes, None)
    assert fused(lam=0.0) == B.STRUCTKV_ERR_INVALID_ARG
    assert fused(inv_w=-1.0) == B.STRUCTKV_ERR_INVALID_ARG
    assert fused(cen=None) == B.STRUCTKV_ERR_INVALID_ARG
    assert fused(cen=ctypes.c_void_p(4098)) == B.STRUCTKV_ERR_INVALID_ARG
    assert fused(cen=fake, indeg=fake) == B.STRUCTKV_ERR_INVALID_ARG and "alias" in B.structkv_last_error()
    assert fused() == B.STRUCTKV_ERR_WORKSPACE            # everything else valid: stops at the NULL workspace
    assert fused(cen=None, batch=0) == B.STRUCTKV_OK

    def groups(gout=fake, batch=1, ws=None):
        return lib.structkv_score_layer_groups(ctypes.byref(ok_shape), fake, fake, 100 * 128, 128, batch, cu, fake,
                                               gout, fake, None, ws, ws_bytes, None)
    assert groups(gout=None) == B.STRUCTKV_ERR_INVALID_ARG
    assert groups(gout=ctypes.c_void_p(4097)) == B.STRUCTKV_ERR_INVALID_ARG
    assert groups() == B.STRUCTKV_ERR_WORKSPACE           # everything else valid: stops at the NULL workspace
    assert groups(gout=None, batch=0) == B.STRUCTKV_OK

    topk = lib.structkv_select_topk
    assert topk(fake, 1, cu, (i64 * 1)(101), 0, fake, fake, ws_bytes, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert topk(fake, 1, cu, (i64 * 1)(90), 32, fake, fake, ws_bytes, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert topk(fake, 1, cu, (i64 * 1)(-1), 0, fake, fake, ws_bytes, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert topk(fake, 1, cu, (i64 * 1)(10), -1, fake, fake, ws_bytes, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert topk(fake, 1, cu, (i64 * 1)(10), 200, fake, fake, ws_bytes, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert topk(fake, 1, cu, (i64 * 1)(10), 0, fake, fake, 8, None) == B.STRUCTKV_ERR_WORKSPACE
    assert topk(fake, 1, cu, (i64 * 1)(10), 0, None, fake, ws_bytes, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert topk(fake, 1, cu, (i64 * 1)(0), 0, fake, fake, ws_bytes, None) == B.STRUCTKV_OK   # nothing to do

    stat = lib.structkv_select_topk_static          # same validation; fails before it looks for its scratch
    assert stat(fake, 1, cu, (i64 * 1)(101), 0, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert stat(fake, 1, cu, (i64 * 1)(10), -1, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert stat(fake, 1, cu, None, 0, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert stat(None, 1, cu, (i64 * 1)(10), 0, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert stat(fake, 1, cu, (i64 * 1)(0), 0, fake, None) == B.STRUCTKV_OK   # nothing to do
    assert stat(None, 0, cu, None, 0, None, None) == B.STRUCTKV_OK

    def step(ks=(i64 * 1)(10), tail=32, cen=ctypes.c_void_p(8192), lam=0.9, ws=None, kdst=fake, vsrc=fake, dtok=128, batch=1):
        return lib.structkv_layer_step(ctypes.byref(ok_shape), fake, fake, vsrc, 100 * 128, 128, batch, cu, ks, tail,
                                       fake, cen, lam, 0.1, fake, None, fake, kdst, fake, 50 * 128, dtok, ws, ws_bytes,
                                       None)
    assert step(ks=(i64 * 1)(90)) == B.STRUCTKV_ERR_INVALID_ARG            # k + window > n
    assert step(ks=None) == B.STRUCTKV_ERR_INVALID_ARG
    assert step(lam=0.0) == B.STRUCTKV_ERR_INVALID_ARG
    assert step(cen=fake) == B.STRUCTKV_ERR_INVALID_ARG and "alias" in B.structkv_last_error()
    assert step(dtok=64) == B.STRUCTKV_ERR_INVALID_ARG                     # destination rows overlap
    assert step(vsrc=None) == B.STRUCTKV_ERR_INVALID_ARG                   # v_dst without v
    assert step() == B.STRUCTKV_ERR_WORKSPACE                              # everything else valid: NULL workspace
    assert step(cen=None) == B.STRUCTKV_ERR_WORKSPACE                      # the centrality is optional
    assert step(batch=0) == B.STRUCTKV_OK
    a, b_ = B.structkv_workspace_bytes(ok_shape, 1, 100), B.structkv_workspace_bytes(None, 1, 100)
    assert B.structkv_layer_step_workspace_bytes(ok_shape, 1, 100) == a + b_

    blk = lib.structkv_block_scores
    assert blk(fake, 1, cu, 0, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert blk(None, 1, cu, 16, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert blk(fake, 1, (i64 * 2)(0, -1), 16, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert blk(None, 1, (i64 * 2)(0, 0), 16, None, None) == B.STRUCTKV_OK

    tr = lib.structkv_truncate_hidden
    rows1 = (i64 * 1)(5)
    assert tr(fake, 4096, None, 4096, 4096, 2, None, None, 1, cu, rows1, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert tr(fake, 64, fake, 4096, 4096, 2, None, None, 1, cu, rows1, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert tr(None, 0, None, 0, 0, 0, fake, None, 1, cu, rows1, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert tr(None, 0, None, 0, 0, 0, None, ctypes.c_void_p(4100), 1, cu, rows1, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert tr(None, 0, None, 0, 0, 0, None, fake, 1, cu, rows1, None, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert tr(None, 0, None, 0, 0, 0, None, None, 1, cu, rows1, fake, None) == B.STRUCTKV_OK      # nothing asked for
    assert tr(None, 0, None, 0, 0, 0, None, fake, 1, cu, (i64 * 1)(0), fake, None) == B.STRUCTKV_OK

    gat = lib.structkv_gather_kv
    rows = (i64 * 1)(5)
    assert gat(fake, fake, 12800, 128, fake, fake, 640, 128, 8, 128, 3, 1, cu, rows, fake, None) == B.STRUCTKV_ERR_UNSUPPORTED
    assert gat(fake, fake, 12800, 64, fake, fake, 640, 128, 8, 128, 2, 1, cu, rows, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert gat(fake, None, 12800, 128, None, fake, 640, 128, 8, 128, 2, 1, cu, rows, fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert gat(fake, fake, 12800, 128, fake, fake, 640, 128, 8, 128, 2, 1, cu, rows, None, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert gat(fake, fake, 12800, 128, fake, fake, 640, 128, 8, 128, 2, 1, cu, (i64 * 1)(-2), fake, None) == B.STRUCTKV_ERR_INVALID_ARG
    assert gat(fake, fake, 12800, 128, fake, fake, 640, 128, 8, 128, 2, 1, cu, (i64 * 1)(0), fake, None) == B.STRUCTKV_OK


def test_binding_raises_with_message(B):
    import torch
    s = B.make_shape(8, 3, 128, 32, B.STRUCTKV_DTYPE_BF16)
    q = torch.zeros(1, 8, 32, 128, dtype=torch.bfloat16)
    k = torch.zeros(2, 100, 128, dtype=torch.bfloat16)
    out = torch.zeros(100)
    with pytest.raises(B.StructKVError) as e:
        B.structkv_score_layer(s, q, k, [0, 100], out, out, None, out, stream=0)
    assert e.value.status == B.STRUCTKV_ERR_INVALID_ARG and "divide" in str(e.value)


def test_transition_scores_hand_values(B):
    # Eq. 7-9 is host arithmetic in the library: checked against values worked out by hand (see the same cases,
    # with the working, in test_oracle_pins.py), not against the oracle's implementation of the same formulas
    T, ls = B.structkv_transition_scores([5.0, 4.9, 4.8, 2.0, 1.9], [0.2, 0.2, 0.25, 0.8, 0.8],
                                         [1.0, 1.0, 1.5, 6.0, 6.5], (0.2, 0.3, 0.5))
    assert T == pytest.approx([0.0, 0.0, 0.3 / 11 + 0.5 / 9, 1.0, 0.5 / 9]) and ls == 4
    # other weights, an entropy that also rises, a variance that mostly falls
    T, ls = B.structkv_transition_scores([4.0, 4.5, 3.5, 3.0, 3.25], [0.25, 0.125, 0.625, 0.5, 1.0],
                                         [8.0, 6.0, 7.0, 3.0, 2.0], (0.5, 0.25, 0.25))
    assert T == pytest.approx([0.0, 0.1, 1.0, 1.0 / 3, 1.0 / 12 + 0.25 + 0.15], rel=1e-14) and ls == 3
    # equal maxima: the lowest layer wins
    T, ls = B.structkv_transition_scores([2.0, 1.0, 1.0, 0.0], [0.5] * 4, [1.0] * 4, (1.0, 0.0, 0.0))
    assert T == [0.0, 1.0, 0.0, 1.0] and ls == 2
    T, ls = B.structkv_transition_scores([], [], [])
    assert T == [] and ls == 0
    T, ls = B.structkv_transition_scores([3.0, 3.0, 3.0], [0.5, 0.5, 0.5], [1.0, 1.0, 1.0])
    assert T == [0.0, 0.0, 0.0] and ls == 2
    T, ls = B.structkv_transition_scores([1.0, 0.5], [0.1, 0.4], [1.0, 1.0], (1.0, 1.0, 1.0))
    assert T == [0.0, 0.0] and ls == 2                                # a single difference: max == min
    assert B.structkv_transition_scores([1.0], [0.1], [1.0])[1] == 1


def test_pivot_metrics_arguments(B):
    lib = B._lib
    i64 = ctypes.c_int64
    cu = (i64 * 2)(0, 100)
    fake = ctypes.c_void_p(4096)
    shape = B.make_shape(8, 2, 128, 32, B.STRUCTKV_DTYPE_BF16)
    need = B.structkv_pivot_workspace_bytes(shape, 100)
    assert need > 0 and need % 256 == 0
    assert B.structkv_pivot_workspace_bytes(shape, 1 << 20) > B.structkv_pivot_workspace_bytes(shape, 1 << 10)
    assert B.structkv_pivot_workspace_bytes(B.make_shape(8, 3, 128, 32, 1), 100) == 0

    def call(frac=0.1, sp=fake, ws=fake, wsb=need, batch=1):
        return lib.structkv_pivot_metrics(ctypes.byref(shape), fake, fake, 100 * 128, 128, batch, cu, float(frac), sp, fake, ws,
                                          wsb, None)
    assert call(frac=0.0) == B.STRUCTKV_ERR_INVALID_ARG
    assert call(frac=1.5) == B.STRUCTKV_ERR_INVALID_ARG
    assert call(sp=None) == B.STRUCTKV_ERR_INVALID_ARG
    assert call(ws=None) == B.STRUCTKV_ERR_WORKSPACE
    assert call(wsb=need - 256) == B.STRUCTKV_ERR_WORKSPACE and "need" in B.structkv_last_error()
    assert call(batch=0) == B.STRUCTKV_OK

    def fused(indeg=fake, ent=fake, frac=0.1, ws=fake, batch=1):
        return lib.structkv_score_layer_pivot(ctypes.byref(shape), fake, fake, 100 * 128, 128, batch, cu, float(frac),
                                              indeg, ent, None, fake, fake, ws, need, None)
    assert fused(indeg=None) == B.STRUCTKV_ERR_INVALID_ARG and "indeg_out" in B.structkv_last_error()
    assert fused(ent=None) == B.STRUCTKV_ERR_INVALID_ARG
    assert fused(frac=-1.0) == B.STRUCTKV_ERR_INVALID_ARG
    assert fused(ws=None) == B.STRUCTKV_ERR_WORKSPACE
    assert fused(batch=0) == B.STRUCTKV_OK


def test_bench_refuses_more_than_one_gpu():
    # one GPU per box: bench.py --gpus N with N > 1 exits with a message before it touches torch or the GPU
    import subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_entry_points_exist():
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("graft_entry", os.path.join(root, "__graft_entry__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert callable(mod.build) and callable(mod.smoke)


def test_host_planning_with_stub_launchers(B):
    """Valid calls all the way through work planning and workspace carving.  Only in the host-only sanitizer
    build (tests/test_host_sanitizers.py), whose kernel launchers are stubs: no pointer is dereferenced."""
    lib = B._lib
    if not hasattr(lib, "structkv_stub_launch_count"):
        pytest.skip("the real library launches kernels; this runs against the stub build only")
    i64 = ctypes.c_int64
    fake, fake2 = ctypes.c_void_p(1 << 20), ctypes.c_void_p(1 << 21)
    rng = np.random.default_rng(3)
    before = lib.structkv_stub_launch_count()
    for (Hq, G, d, w, dtype, causal) in [(32, 8, 128, 64, 1, 0), (32, 8, 128, 32, 1, 1), (8, 8, 64, 32, 0, 0),
                                         (4, 1, 64, 8, 1, 0), (6, 2, 96, 5, 1, 0), (32, 32, 128, 64, 1, 0),
                                         (16, 2, 128, 64, 1, 0)]:
        shape = B.make_shape(Hq, G, d, w, dtype, bool(causal))
        for batch in (1, 3, B.STRUCTKV_MAX_BATCH):
            lens = [int(x) for x in rng.integers(w, 5000, size=batch)]
            if batch == 3:
                lens[1] = 0                                  # an empty sequence in the middle
            cu = (i64 * (batch + 1))(*np.concatenate([[0], np.cumsum(lens)]).tolist())
            total = int(sum(lens))
            need = B.structkv_workspace_bytes(shape, batch, total)
            assert need > 0 and need % 256 == 0
            args = (ctypes.byref(shape), fake, fake, total * d, d, batch, cu, fake, fake, None, fake2)
            assert lib.structkv_score_layer(*args, need, None) == B.STRUCTKV_OK, B.structkv_last_error()
            assert lib.structkv_score_layer(*args, need - 256, None) in (B.STRUCTKV_OK, B.STRUCTKV_ERR_WORKSPACE)
            assert lib.structkv_score_layer(*args, 256, None) == B.STRUCTKV_ERR_WORKSPACE
            ks = (i64 * batch)(*[max(n - w, 0) // 3 for n in lens])
            assert lib.structkv_select_topk(fake, batch, cu, ks, w if min(x for x in lens if x) >= w and 0 not in lens else 0,
                                            fake, fake2, need, None) == B.STRUCTKV_OK, B.structkv_last_error()
            rows = (i64 * batch)(*[int(k) for k in ks])
            assert lib.structkv_gather_kv(fake, fake, total * d, d, fake2, fake2, sum(rows) * d, d, G, d, 2, batch, cu,
                                          rows, fake, None) == B.STRUCTKV_OK, B.structkv_last_error()
            assert lib.structkv_block_scores(fake, batch, cu, 16, fake2, None) == B.STRUCTKV_OK
            tail = w if 0 not in lens else 0
            sneed = B.structkv_layer_step_workspace_bytes(shape, batch, total)
            fake3 = ctypes.c_void_p(1 << 22)
            assert lib.structkv_layer_step(ctypes.byref(shape), fake, fake, fake, total * d, d, batch, cu, ks, tail,
                                           fake3, None, 0.9, 0.1, fake, None, fake, fake2, fake2,
                                           (sum(rows) + batch * tail) * d, d, fake2, sneed, None) == B.STRUCTKV_OK, \
                B.structkv_last_error()
        pneed = B.structkv_pivot_workspace_bytes(shape, 4096)
        cu1 = (i64 * 3)(0, 4096, 4096 + 100 + w)
        assert lib.structkv_score_layer_pivot(ctypes.byref(shape), fake, fake, 5000 * d, d, 2, cu1, 0.1, fake, fake, None,
                                              fake, fake, fake2, pneed, None) == B.STRUCTKV_OK, B.structkv_last_error()
    assert lib.structkv_stub_launch_count() > before


def test_tilings_chosen_for_the_named_configurations(B):
    """The plan the host makes for the benchmark configurations: which tiling, how many keys per workgroup, which
    cache policy.  Stub build only (the stub of the MFMA scoring launcher keeps the plan it was handed, after
    checking it against what the kernels assume)."""
    lib = B._lib
    if not hasattr(lib, "structkv_stub_last_plan"):
        pytest.skip("the real library launches kernels; this runs against the stub build only")
    i64 = ctypes.c_int64
    fake, fake2 = ctypes.c_void_p(1 << 20), ctypes.c_void_p(1 << 21)

    def plan(Hq, G, d, w, lens):
        shape = B.make_shape(Hq, G, d, w, 1, False)
        cu = (i64 * (len(lens) + 1))(*np.concatenate([[0], np.cumsum(lens)]).tolist())
        total = int(sum(lens))
        need = B.structkv_workspace_bytes(shape, len(lens), total)
        assert lib.structkv_score_layer(ctypes.byref(shape), fake, fake, total * d, d, len(lens), cu, fake, fake, None,
                                        fake2, need, None) == B.STRUCTKV_OK, B.structkv_last_error()
        out = (ctypes.c_int32 * 8)()
        lib.structkv_stub_last_plan(out)
        return dict(zip(("RB", "NW", "KC", "planes", "stream_k", "RC", "grid_chunks", "path"), list(out)))

    # 128K tokens, window 64: 256 rows per KV head = four waves of 64 rows; one round of 768 workgroups; K = 256 MiB streams
    p = plan(32, 8, 128, 64, [131072])
    assert (p["RB"], p["NW"], p["RC"], p["KC"], p["stream_k"], p["path"]) == (2, 4, 4, 1376, 1, 0)
    assert p["grid_chunks"] == 96
    # 32K tokens, window 32: 128 rows = four waves of 32 rows, 512 keys each (half of the resident slots); cached fetches
    p = plan(32, 8, 128, 32, [32768])
    assert (p["RB"], p["NW"], p["RC"], p["KC"], p["stream_k"]) == (1, 4, 4, 512, 0)
    # the paper's window of 8: 32 rows, single-wave workgroups
    p = plan(32, 8, 128, 8, [32768])
    assert (p["RB"], p["NW"], p["RC"], p["KC"]) == (1, 1, 1, 256)
    # 64 rows: one wave with two row blocks; 1M tokens: several rounds, key chunks within the LDS capacity
    p = plan(16, 8, 128, 32, [4096])
    assert (p["RB"], p["NW"], p["RC"]) == (2, 1, 1)
    p = plan(32, 8, 128, 64, [1048576])
    assert (p["RB"], p["NW"], p["stream_k"]) == (2, 4, 1) and p["KC"] <= 2048 and 5 * 96 < p["grid_chunks"] <= 6 * 96
    # a ragged batch: chunks never straddle sequences
    lens = [70000, 0, 33, 16384, 100000]
    p = plan(32, 8, 128, 32, lens)
    assert p["grid_chunks"] == sum(-(-n // p["KC"]) for n in lens) and p["stream_k"] == 1     # 364 MiB of K
    p = plan(32, 8, 128, 32, [n // 2 for n in lens])
    assert p["grid_chunks"] == sum(-(-(n // 2) // p["KC"]) for n in lens) and p["stream_k"] == 0
