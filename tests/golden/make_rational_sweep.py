"""Writes rational_sweep.json: a worked example of the scoring sweep in exact rational arithmetic.

Nothing here touches the CPU oracle or the GPU library: every value follows from integers through the paper's
formulas (Eq. 1-10), evaluated with fractions.Fraction.  Key j of a layer is (ln a_j, ln b_j, 0, 0); head 0's two
window queries are (1,0,0,0) and (2,0,0,0), head 1's are (0,1,0,0) and (0,2,0,0); with logit scale 1 the softmax
rows are a/sum(a), a^2/sum(a^2), b/sum(b), b^2/sum(b^2).  Run: python tests/golden/make_rational_sweep.py
"""
import json
import math
import os
from fractions import Fraction as F

A = [[1, 2, 3, 4, 2], [4, 1, 1, 2, 8], [1, 1, 6, 1, 1], [1, 1, 1, 1, 1]]   # head 0 weights, one list per layer
Bw = [[2, 2, 1, 1, 4], [1, 3, 9, 1, 2], [3, 1, 1, 3, 1], [5, 1, 1, 1, 2]]  # head 1 weights
LAM, W, N, HQ = F(9, 10), 2, 5, 2           # lambda = 0.9: the paper's setting (Sec. 5.1)
WEIGHTS = [F(1, 5), F(3, 10), F(1, 2)]      # transition weights {0.2, 0.3, 0.5} (Sec. 5.1)


def main():
    layers, C = [], [F(0)] * N
    ents, rhos, variances = [], [], []
    for a, b in zip(A, Bw):
        rows = []
        for wts in (a, b):
            for r in (1, 2):
                pw = [F(x) ** r for x in wts]
                rows.append([x / sum(pw) for x in pw])                       # Eq. 1
        D = [sum(row[j] for row in rows) for j in range(N)]                  # Eq. 2 times w
        H = sum(-sum(float(p) * math.log(float(p)) for p in row) for row in rows) / len(rows)   # Eq. 4
        C = [LAM * C[j] + D[j] / W for j in range(N)]                        # Eq. 3
        pooled = [[(rows[2 * h][j] + rows[2 * h + 1][j]) / W for j in range(N)] for h in range(HQ)]
        rho = sum(max(ph) for ph in pooled) / HQ                             # Eq. 5, ceil(0.1 * 5) = 1 key
        var = sum(sum((x - F(1, N)) ** 2 for x in ph) / N for ph in pooled) / HQ   # Eq. 6
        ents.append(H); rhos.append(rho); variances.append(var)
        layers.append({"head0_weights": a, "head1_weights": b,
                       "probs": [[str(x) for x in row] for row in rows],
                       "indegree": [str(x) for x in D], "entropy": repr(H),
                       "centrality_after": [str(x) for x in C],
                       "sparsity": str(rho), "variance": str(var)})
    L = len(layers)
    top2 = sorted(sorted(range(N), key=lambda j: (-C[j], j))[:2])             # Eq. 10, ties to the lower index
    early = sorted(range(N - W), key=lambda j: (-C[j], j))[:1]
    def scaled(vals, sign):                                                   # Eq. 7-8
        d = [sign * (vals[l] - vals[l - 1]) for l in range(1, L)]
        lo, hi = min(d), max(d)
        return [float((x - lo) / (hi - lo)) if hi > lo else 0.0 for x in d]
    sH, sR, sV = scaled(ents, -1), scaled(rhos, 1), scaled(variances, 1)
    T = [0.0] + [float(WEIGHTS[0]) * x + float(WEIGHTS[1]) * y + float(WEIGHTS[2]) * z for x, y, z in zip(sH, sR, sV)]
    pivot = max(range(1, L), key=lambda l: (T[l], -l)) + 1                    # Eq. 9
    doc = {
        "_about": "Worked example in exact rational arithmetic; written by make_rational_sweep.py in this folder, "
                  "which uses neither the CPU oracle nor the GPU library.  One sequence of n = 5 keys, two query "
                  "heads sharing one KV head, head_dim 4, window w = 2, explicit logit scale 1, no causal mask. "
                  "Key j of a layer is (ln a_j, ln b_j, 0, 0); head 0's window queries are (1,0,0,0) and (2,0,0,0), "
                  "head 1's are (0,1,0,0) and (0,2,0,0).  Rows of 'probs' in the order head 0 row 0, head 0 row 1, "
                  "head 1 row 0, head 1 row 1.",
        "citations": {
            "probs": "Eq. 1: softmax over the keys of the observation-window logits",
            "indegree": "Eq. 2 without its 1/w: column sums over rows and heads; every layer's total is w*H_q = 4",
            "entropy": "Eq. 4: mean over heads and window rows of -sum_j a_j ln a_j",
            "centrality_after": "Eq. 3 / Algorithm 1: C <- lambda C + D/w with lambda = 0.9 (Sec. 5.1)",
            "sparsity": "Eq. 5, window rows pooled per head: mass of the ceil(0.1*5) = 1 largest key, mean over heads",
            "variance": "Eq. 6: population variance of the pooled per-head attention about 1/n, mean over heads",
            "selection": "Eq. 10: top-k of the final centrality, ties to the lower index; with the window kept: "
                         "top-k of the earlier tokens united with the last w tokens",
            "transition": "Eq. 7-9 with weights {0.2, 0.3, 0.5} (Sec. 5.1): min-max scaled first differences "
                          "(entropy drop, sparsity rise, variance rise), T_0 = 0, pivot layer = argmax + 1",
        },
        "shape": {"n": N, "n_q_heads": HQ, "n_kv_heads": 1, "head_dim": 4, "window": W, "scale": 1.0, "causal": 0},
        "lambda": str(LAM), "top_frac": 0.1, "transition_weights": [0.2, 0.3, 0.5],
        "layers": layers,
        "selection": {"top2": top2, "top1_of_earlier_plus_window": sorted(early + list(range(N - W, N)))},
        "transition": {"T": [repr(t) for t in T], "pivot_layer": pivot},
    }
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "rational_sweep.json"), "w") as f:
        f.write(json.dumps(doc, indent=1) + "\n")


if __name__ == "__main__":
    main()
