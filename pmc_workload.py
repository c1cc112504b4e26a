"""Small fixed workload for hardware-counter runs (rocprofv3 --pmc): a few eager layers of the sweep
plus one plain copy of known size (the gather kernel with identity indices: reads and writes
exactly copy_bytes each), which calibrates the FETCH_SIZE / WRITE_SIZE scale.

    rocprofv3 --pmc FETCH_SIZE -d out -- python3 pmc_workload.py --layers 2
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c3_llama8b_128k")
    ap.add_argument("--layers", type=int, default=2)
    ap.add_argument("--copy-mib", type=int, default=256)
    ap.add_argument("--cache-groups", action="store_true",
                    help="score each layer through the measurement hook that goes through a batch in cache-sized "
                         "groups of sequences (pass 1, combine, pass 2 of a group back to back)")
    args = ap.parse_args()
    import torch

    import workloads
    from paper_2604_06746_amd import binding as B
    from paper_2604_06746_amd import sweep as sweep_mod

    wl = workloads.WORKLOADS[args.workload]
    torch.cuda.set_device(0)
    sw = sweep_mod.LayerSweep(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.torch_dtype,
                              wl.seq_lens, wl.k_per_seq, lam=wl.lam, n_layers_out=1)
    for l in range(args.layers):
        x = workloads.make_layer(wl, l, "cuda")
        torch.cuda.synchronize()
        if args.cache_groups:
            B.structkv_debug_score_steps(sw.shape, x.q_win, x.k, sw.cu, sw.indeg, sw.entropy, sw.entropy_per_head,
                                         sw.workspace, 15 | 16)
        else:
            sw.layer(x.q_win, x.k, x.v)
        torch.cuda.synchronize()
    # calibration copy: [1, rows, 128] bf16 rows of 256 B, identity indices
    rows = args.copy_mib * 1024 * 1024 // 256
    src = torch.randn(1, rows, 128, device="cuda").to(torch.bfloat16)
    dst = torch.empty_like(src)
    idx = torch.arange(rows, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    B.structkv_gather_kv(src, None, dst, None, [0, rows], [rows], idx)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    print("pmc workload done: %s, %d layers, copy %d MiB" % (wl.name, args.layers, args.copy_mib))


if __name__ == "__main__":
    main()
