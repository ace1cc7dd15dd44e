"""A seeded sweep over shapes the fixed cases do not enumerate: batch, heads, group size, block size,
mantissa bits, dtype, ragged lengths, with and without permutations.  Cache bytes bit-exact, attention
within the bar, each case against the oracle."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth
from util import assert_attention_close, assert_planes_equal, dev_i32, gpu_cache, oracle_cache

pytestmark = pytest.mark.gpu
DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def _cases():
    rng = np.random.default_rng(20137)
    out = []
    for i in range(28):
        B = int(rng.integers(1, 4))
        Hkv = int(rng.integers(1, 5))
        G = int(rng.choice([1, 2, 3, 4, 6, 8, 12]))
        n = int(rng.choice([16, 32, 64, 128]))
        p = int(rng.choice([4, 8]))
        dt = str(rng.choice(["bf16", "f16", "f32"]))
        S = int(rng.integers(1, 900))
        lens = [int(rng.integers(0, S + 1)) for _ in range(B)]
        lens[int(rng.integers(0, B))] = S
        out.append((i, B, Hkv, G, n, p, dt, S, tuple(lens), bool(rng.integers(0, 2)), int(rng.choice([0, 0, 8]))))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: "c%02d_B%d_H%d_G%d_n%d_p%d_%s_S%d" % c[:8])
def test_random_configuration(case):
    i, B, Hkv, G, n, p, dt, S, lens, use_perm, qbits = case
    D = 128
    seed = 1000 + i
    kg = synth.outlier_gains(seed, 0, Hkv, D)
    vg = synth.outlier_gains(seed, 1, Hkv, D)
    k = synth.kv_rows(B, S, Hkv, D, dt, kg, seed, 2)
    v = synth.kv_rows(B, S, Hkv, D, dt, vg, seed, 3)
    q = synth.queries(B, Hkv * G, D, dt, seed, 4)
    pk = pv = None
    if use_perm:
        pk = O.calibrate_perm(synth.to_f32_numpy(synth.kv_rows(1, 32, Hkv, D, dt, kg, seed, 5)[0]))
        pv = O.calibrate_perm(synth.to_f32_numpy(synth.kv_rows(1, 32, Hkv, D, dt, vg, seed, 6)[0]))
    S_max = S + int(i % 3) * 7
    planes = oracle_cache(k, v, n, p, S_max, 0, pk, pv)
    cache = gpu_cache(k.cuda(), v.cuda(), n, p, S_max, perm_k=pk, perm_v=pv)
    assert_planes_equal(cache, planes, "cache")
    scale = float(np.float32(0.05 + 0.01 * (i % 7)))
    want = O.decode_attention(*planes, D, n, p, synth.to_f32_numpy(q), list(lens), scale, pk, pv, q_mant_bits=qbits)
    sl = dev_i32(np.asarray(lens))
    if qbits:
        got = kvbfp.decode_attention_qbfp(cache, q.cuda(), S, scale, qbits, seq_len_dev=sl, perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    else:
        got = kvbfp.decode_attention(cache, q.cuda(), S, scale, seq_len_dev=sl, perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    assert_attention_close(got, want, DT[dt], str(case))
