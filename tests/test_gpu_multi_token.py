"""kvbfp_decode_attention_multi: the last n_q_tokens tokens of every sequence in one pass, causal among
themselves; each query token against the oracle's single-token attention over the tokens it may see."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth
from util import assert_attention_close, assert_planes_equal, dev_i32, gpu_cache, oracle_cache

pytestmark = pytest.mark.gpu
D = 128
DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@pytest.mark.parametrize("dt,p,n,G,Tq", [
    ("bf16", 4, 32, 1, 4),     # 4 virtual heads: one MFMA row group, LDS pipeline, FP4 keys
    ("bf16", 4, 16, 2, 4),     # 8 virtual heads: two row groups, LDS pipeline
    ("f16", 4, 32, 4, 2),
    ("bf16", 4, 64, 1, 8),     # register-staged pass
    ("bf16", 8, 16, 1, 8),     # 8-bit mantissas
    ("bf16", 8, 32, 2, 3),     # 6 virtual heads
    ("bf16", 4, 32, 4, 4),     # 16 virtual heads: two launches over head subsets
    ("bf16", 4, 16, 4, 8),     # 32 virtual heads: four launches
    ("bf16", 8, 32, 3, 7),     # 21 virtual heads: 8 + 8 + 5
    ("f16", 4, 32, 4, 9),      # 36 virtual heads: general pass
    ("f32", 4, 32, 2, 5),      # fp32 I/O: general pass
])
def test_each_query_token_matches_single_token_attention(dt, p, n, G, Tq):
    B, Hkv, S = 3, 2, 830
    seed = 300 + 7 * Tq + G + p
    kg = synth.outlier_gains(seed, 0, Hkv, D)
    vg = synth.outlier_gains(seed, 1, Hkv, D)
    k = synth.kv_rows(B, S, Hkv, D, dt, kg, seed, 2)
    v = synth.kv_rows(B, S, Hkv, D, dt, vg, seed, 3)
    q = torch.stack([synth.queries(B, Hkv * G, D, dt, seed + 10 * i, 4) for i in range(Tq)], dim=1)   # [B][Tq][Hq][D]
    pk = O.calibrate_perm(synth.to_f32_numpy(synth.kv_rows(1, 32, Hkv, D, dt, kg, seed, 5)[0]))
    pv = O.calibrate_perm(synth.to_f32_numpy(synth.kv_rows(1, 32, Hkv, D, dt, vg, seed, 6)[0]))
    # a full sequence ending mid-tile, one shorter than the number of query tokens, one crossing a 256-token boundary
    lens = [S, max(Tq - 2, 1), 257 + Tq // 2]
    planes = oracle_cache(k, v, n, p, S, 0, pk, pv)
    cache = gpu_cache(k.cuda(), v.cuda(), n, p, S, perm_k=pk, perm_v=pv)
    assert_planes_equal(cache, planes, "cache")
    scale = 0.09
    got = kvbfp.decode_attention_multi(cache, q.cuda(), S, scale, seq_len_dev=dev_i32(np.asarray(lens)),
                                       perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    assert got.shape == q.shape
    for i in range(Tq):
        seen = [max(l - (Tq - 1 - i), 0) for l in lens]
        want = O.decode_attention(*planes, D, n, p, synth.to_f32_numpy(q[:, i]), seen, float(np.float32(scale)), pk, pv)
        assert_attention_close(got[:, i], want, DT[dt], "query token %d of %d sees %s" % (i, Tq, seen))
        for b, l in enumerate(seen):
            if l == 0:
                assert bool((got[b, i] == 0).all())


def test_one_query_token_is_the_plain_call():
    B, Hkv, G, S = 2, 2, 4, 700
    gains = synth.outlier_gains(9, 0, Hkv, D)
    k = synth.kv_rows(B, S, Hkv, D, "bf16", gains, 9, 2, "cuda")
    v = synth.kv_rows(B, S, Hkv, D, "bf16", gains, 9, 3, "cuda")
    q = synth.queries(B, Hkv * G, D, "bf16", 9, 4, "cuda")
    cache = gpu_cache(k, v, 32, 4, S)
    a = kvbfp.decode_attention(cache, q, S, 0.1)
    b = kvbfp.decode_attention_multi(cache, q.unsqueeze(1).contiguous(), S, 0.1)
    torch.cuda.synchronize()
    assert torch.equal(a, b[:, 0])
