"""K-sort from the weights, end to end, and a report in the shape of Table I.

Alg. 1: per KV head, rank the rows of W_k by Euclidean norm, reorder the rows of W_k and of W_q alike
(Eq. (2)-(3): the scores do not change), and keep the keys in Block Floating Point.  Values are
treated the same way with their own permutation (Sec. III, last paragraph); the output then stays
in the reordered channel order and the projection after attention, W_o, gets its columns reordered
to match.  The reorder lives in the weights, so nothing is gathered at run time: both pipelines
below call quantize_append / decode_attention without a permutation, and both end in the same
model-width vector W_o . out.

Table I reports perplexity for the original and the sorted channel order at block sizes 128, 64, 32.
Perplexity needs the model's weights and a corpus; what this report measures instead, on synthetic
projections with planted large-norm rows (the paper's source of channel-consistent outliers), is the
error of the attention output against attention on the unquantized keys and values.

Every step that belongs to the method runs in libkvbfp (HIP kernels and the two host calls); torch
is used for the synthetic projections and for the unquantized reference only.

    python -m paper_2403_20137_amd.ksort_report [--tokens 4096] [--heads 8] [--group 4] [--seed 20137]
"""
import argparse
import json

import numpy as np
import torch

from . import kvbfp

D = 128


def synthetic_projections(n_kv_heads, group, d_model, n_outlier_rows, gain, seed):
    """W_q [Hq*D][d_model], W_k, W_v [Hkv*D][d_model] ~ N(0, 1/d_model); in every KV head of W_k and
    W_v a seeded set of rows is multiplied by `gain` (large-norm rows -> outlier channels)."""
    g = torch.Generator().manual_seed(seed)
    hq = n_kv_heads * group

    def mat(rows):
        return torch.randn(rows, d_model, generator=g) / d_model ** 0.5

    wq, wk, wv = mat(hq * D), mat(n_kv_heads * D), mat(n_kv_heads * D)
    for w in (wk, wv):
        for h in range(n_kv_heads):
            rows = torch.randperm(D, generator=g)[:n_outlier_rows]
            w[h * D + rows] *= gain
    return wq, wk, wv


def synthetic_output_projection(n_kv_heads, group, d_model, seed):
    """W_o [d_model][Hq*D] ~ N(0, 1/(Hq*D)): the projection that consumes the attention output."""
    g = torch.Generator().manual_seed(seed + 2)
    hq = n_kv_heads * group
    return torch.randn(d_model, hq * D, generator=g) / (hq * D) ** 0.5


def project(x, w, n_heads, dtype):
    """x [T][d_model] . w^T -> [1][T][n_heads][D] in `dtype` (one sequence)."""
    return (x @ w.t()).view(1, x.shape[0], n_heads, D).to(dtype).contiguous()


def reference_attention(q, k, v, scale):
    """fp64 softmax attention of q [1][Hq][D] over unquantized k, v [1][T][Hkv][D] (after their rounding
    to the I/O type): the quantity the BFP cache is supposed to preserve."""
    hq, hkv = q.shape[1], k.shape[2]
    grp = hq // hkv
    qd, kd, vd = q[0].double(), k[0].double(), v[0].double()
    out = torch.empty(hq, D, dtype=torch.float64, device=q.device)
    for h in range(hq):
        s = (kd[:, h // grp] @ qd[h]) * scale
        p = torch.softmax(s, dim=0)
        out[h] = p @ vd[:, h // grp]
    return out


def bfp_attention(q, k, v, block, mant_bits, scale, device):
    """quantize_append + decode_attention through the library, rows already in cache order."""
    T, hkv = k.shape[1], k.shape[2]
    layout = kvbfp.make_layout(D, block, mant_bits, hkv, 1, T)
    cache = kvbfp.alloc_cache(layout, device)
    kvbfp.quantize_append(cache, k, v)
    out = kvbfp.decode_attention(cache, q, T, scale)
    torch.cuda.synchronize()
    return out[0].double()


def rel_err(a, b):
    return float((a - b).norm() / b.norm())


def run(tokens=4096, n_kv_heads=8, group=4, d_model=1024, n_outlier_rows=4, gain=20.0, mant_bits=4,
        blocks=(128, 64, 32, 16), seed=20137, dtype=torch.bfloat16, device="cuda"):
    kvbfp.lib()
    wq, wk, wv = synthetic_projections(n_kv_heads, group, d_model, n_outlier_rows, gain, seed)
    # Alg. 1 steps 1-4 on the host, through the library
    perm_k = kvbfp.calibrate_perm_from_weights(wk, n_kv_heads, D)
    perm_v = kvbfp.calibrate_perm_from_weights(wv, n_kv_heads, D)
    wq_s = kvbfp.permute_weights(wq, n_kv_heads * group, D, perm_k, heads_per_perm=group)
    wk_s = kvbfp.permute_weights(wk, n_kv_heads, D, perm_k)
    wv_s = kvbfp.permute_weights(wv, n_kv_heads, D, perm_v)
    # Sec. III, last paragraph: the value permutation goes into the columns of the next projection
    wo = synthetic_output_projection(n_kv_heads, group, d_model, seed)
    wo_s = kvbfp.permute_weight_columns(wo, n_kv_heads * group, D, perm_v, heads_per_perm=group)
    w_out = {"original": wo.double().to(device), "sorted": wo_s.double().to(device)}

    g = torch.Generator().manual_seed(seed + 1)
    x = torch.randn(tokens, d_model, generator=g).to(device)
    xq = torch.randn(1, d_model, generator=g).to(device)
    scale = float(np.float32(D ** -0.5))
    rows = []
    pipes = {}
    for name, (q_w, k_w, v_w) in {"original": (wq, wk, wv), "sorted": (wq_s, wk_s, wv_s)}.items():
        k = project(x, k_w.to(device), n_kv_heads, dtype)
        v = project(x, v_w.to(device), n_kv_heads, dtype)
        q = project(xq, q_w.to(device), n_kv_heads * group, dtype)[:, 0].contiguous()     # [1][Hq][D]
        pipes[name] = (q, k, v, reference_attention(q, k, v, scale))
    # Eq. (2)-(3): the two pipelines compute the same attention up to the order of the output channels
    pv = torch.from_numpy(perm_v.astype(np.int64)).to(device)
    ref_o, ref_s = pipes["original"][3], pipes["sorted"][3]
    ref_s_unperm = torch.empty_like(ref_s)
    for h in range(n_kv_heads * group):
        ref_s_unperm[h, pv[h // group]] = ref_s[h]
    invariance = rel_err(ref_s_unperm, ref_o)
    # ... and after W_o (columns reordered for the sorted pipeline) the two end in the same vector
    y_ref = {name: w_out[name] @ pipes[name][3].reshape(-1) for name in pipes}
    invariance_y = rel_err(y_ref["sorted"], y_ref["original"])
    for n in blocks:
        row = {"block": n, "mant_bits": mant_bits}
        for name, (q, k, v, ref) in pipes.items():
            out = bfp_attention(q, k, v, n, mant_bits, scale, device)
            row[name] = rel_err(out, ref)
            # error of the model-width vector after the output projection, against the unquantized ORIGINAL pipeline
            row[name + "_after_w_o"] = rel_err(w_out[name] @ out.reshape(-1), y_ref["original"])
        rows.append(row)
    return {"tokens": tokens, "n_kv_heads": n_kv_heads, "group": group, "d_model": d_model,
            "outlier_rows_per_head": n_outlier_rows, "gain": gain, "dtype": str(dtype).replace("torch.", ""),
            "reorder_invariance_rel_err": invariance, "reorder_invariance_after_w_o_rel_err": invariance_y,
            "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=4096)
    ap.add_argument("--heads", type=int, default=8)
    ap.add_argument("--group", type=int, default=4)
    ap.add_argument("--mant-bits", type=int, default=4)
    ap.add_argument("--seed", type=int, default=20137)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    r = run(tokens=args.tokens, n_kv_heads=args.heads, group=args.group, mant_bits=args.mant_bits, seed=args.seed)
    if args.json:
        print(json.dumps(r))
        return
    print("attention-output error vs. unquantized keys/values (relative L2), %d tokens, %d KV heads x %d, "
          "%d planted rows x%.0f per head, %d-bit mantissas" % (r["tokens"], r["n_kv_heads"], r["group"],
                                                              r["outlier_rows_per_head"], r["gain"], args.mant_bits))
    print("reorder invariance of the unquantized attention (Eq. (2)-(3)): %.2e" % r["reorder_invariance_rel_err"])
    print("same after the output projection with reordered columns (Sec. III): %.2e"
          % r["reorder_invariance_after_w_o_rel_err"])
    print("%-12s %-12s %-12s %-20s %-20s" % ("block size", "original", "sorted", "original, after W_o", "sorted, after W_o"))
    for row in r["rows"]:
        print("%-12d %-12.4f %-12.4f %-20.4f %-20.4f" % (row["block"], row["original"], row["sorted"],
                                                     row["original_after_w_o"], row["sorted_after_w_o"]))


if __name__ == "__main__":
    main()
