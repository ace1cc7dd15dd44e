"""Decode attention on seeded random combinations of everything the calls take -- element type, mantissa width,
block size, heads per kv-head, query tokens, query cast, sequence lengths next to the tile, stage and page
boundaries, one region per sequence or a pool of pages of any supported size -- each compared with the oracle
(Sec. III run-time flow; Eq. (1) for the cast).  The fixed parametrised tests cover the corners one at a time;
this one covers them in combination."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth
from test_gpu_attention import make_small
from test_gpu_paged import fill_both
from util import assert_attention_close, assert_planes_equal, dev_i32, gpu_cache, oracle_cache

pytestmark = pytest.mark.gpu

D = 128
DTYPES = [torch.bfloat16, torch.float16, torch.float32]
NAMES = {torch.bfloat16: "bf16", torch.float16: "f16", torch.float32: "f32"}


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = DTYPES[int(rng.choice(3, p=[0.5, 0.3, 0.2]))]
    p = int(rng.choice([4, 8]))
    n = int(rng.choice([16, 32, 64, 128]))
    G = int(rng.choice([1, 2, 3, 4, 5, 6, 8, 9, 12, 17]))
    Hkv = int(rng.choice([1, 2, 3]))
    B = int(rng.choice([1, 2, 3]))
    Tq = int(rng.choice([1, 1, 1, 2, 3, 5]))
    q_mant_bits = int(rng.choice([0, 0, 8]))
    page = int(rng.choice([0, 0, 16, 32, 64, 256]))          # 0: one region per sequence
    # lengths next to the boundaries the kernels have: 16-token stages, 64-token wavefront tiles, 256-token tiles
    lens = []
    for _ in range(B):
        edge = int(rng.choice([16, 64, 256, 512, 768, 1024]))
        lens.append(max(Tq, edge + int(rng.integers(-2, 3))) if rng.random() < 0.6 else int(rng.integers(Tq, 1100)))
    return dict(dtype=dtype, p=p, n=n, G=G, Hkv=Hkv, B=B, Tq=Tq, q_mant_bits=q_mant_bits, page=page, lens=lens)


@pytest.mark.parametrize("seed", range(48))
def test_random_combination_matches_oracle(seed):
    c = draw_case(seed)
    dtype, p, n, G, Hkv, B, Tq, page, lens = (c[k] for k in ("dtype", "p", "n", "G", "Hkv", "B", "Tq", "page", "lens"))
    what = "seed %d: %s p=%d n=%d G=%d Hkv=%d Tq=%d qbits=%d page=%d lens=%s" % (
        seed, NAMES[dtype], p, n, G, Hkv, Tq, c["q_mant_bits"], page, lens)
    print(what, flush=True)
    S = max(lens)
    k, v, _, pk, pv = make_small(dtype, B=B, S=S, Hkv=Hkv, G=G, seed=300 + seed)
    q = torch.stack([synth.queries(B, Hkv * G, D, NAMES[dtype], 301 + seed + 7 * i, 4) for i in range(Tq)], dim=1)
    scale = float(np.float32(128 ** -0.5))
    if page:
        pages_per_seq = -(-S // page) + 1
        pool, table, planes = fill_both(k, v, n, p, page, pages_per_seq, lens, pk, pv, seed=seed)
        got = kvbfp.decode_attention_multi_paged(pool, table, q.cuda(), S, scale, seq_len_dev=dev_i32(lens),
                                                 perm_k=dev_i32(pk), perm_v=dev_i32(pv), q_mant_bits=c["q_mant_bits"])
    else:
        S_max = S + int(seed % 3) * 5                      # the capacity need not be a multiple of anything
        planes = oracle_cache(k, v, n, p, S_max, 0, pk, pv)
        cache = gpu_cache(k.cuda(), v.cuda(), n, p, S_max, perm_k=pk, perm_v=pv)
        assert_planes_equal(cache, planes, what)
        got = kvbfp.decode_attention_multi(cache, q.cuda(), S, scale, seq_len_dev=dev_i32(lens), perm_k=dev_i32(pk),
                                           perm_v=dev_i32(pv), q_mant_bits=c["q_mant_bits"])
    torch.cuda.synchronize()
    assert got.shape == q.shape
    for i in range(Tq):
        seen = [max(l - (Tq - 1 - i), 0) for l in lens]
        want = O.decode_attention(*planes, D, n, p, synth.to_f32_numpy(q[:, i]), seen, scale, pk, pv,
                                  q_mant_bits=c["q_mant_bits"])
        assert_attention_close(got[:, i], want, dtype, what + " query token %d" % i)


@pytest.mark.parametrize("seed", range(24))
def test_random_fused_append_matches_oracle(seed):
    # kvbfp_append_decode_attention: cache bytes (the appended row among them) and output against the oracle, and
    # both against the two separate calls, on random shapes; lengths sit next to the 16 / 64 / 256-token boundaries
    from test_gpu_append_decode import _case
    rng = np.random.default_rng(5000 + seed)
    dtype = DTYPES[int(rng.choice(3, p=[0.6, 0.25, 0.15]))]
    p = int(rng.choice([4, 4, 8]))
    n = int(rng.choice([16, 32, 64, 128]))
    G = int(rng.choice([1, 2, 4, 5, 8, 12]))
    Hkv = int(rng.choice([1, 2, 4, 16]))
    B = int(rng.choice([1, 2, 4]))
    qbits = int(rng.choice([0, 0, 8]))
    lens = []
    for _ in range(B):
        edge = int(rng.choice([0, 16, 64, 256, 512, 1024]))
        lens.append(max(0, edge + int(rng.integers(-1, 3))) if rng.random() < 0.7 else int(rng.integers(1, 1200)))
    if max(lens) == 0:
        lens[0] = 1
    print("seed %d: %s p=%d n=%d G=%d Hkv=%d qbits=%d lens=%s" % (seed, NAMES[dtype], p, n, G, Hkv, qbits, lens), flush=True)
    _case(dtype, n, p, G, lens, max(lens) + int(rng.integers(0, 40)), bool(rng.integers(0, 2)), seed=400 + seed,
          qbits=qbits, Hkv=Hkv)


@pytest.mark.parametrize("seed", range(20))
def test_random_rotation_at_read_matches_oracle(seed):
    # keys cached before the rotary embedding, rotated at read (Alg. 1 step 5; Sec. II-D), on random shapes,
    # frequency bases and pairings; the 16-bit 4-bit-mantissa cases take the matrix-core pass, the rest the general one
    from test_gpu_rope_at_read import llama_theta, run_both
    rng = np.random.default_rng(7000 + seed)
    dtype = DTYPES[int(rng.choice(3, p=[0.5, 0.3, 0.2]))]
    p = int(rng.choice([4, 4, 4, 8]))
    n = int(rng.choice([16, 32, 64, 128]))
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8]))
    Hkv = int(rng.choice([1, 2, 3]))
    B = int(rng.choice([1, 2]))
    pairs = int(rng.choice([0, 1]))
    base = float(rng.choice([10000.0, 500000.0]))
    lens = []
    for _ in range(B):
        edge = int(rng.choice([16, 64, 256, 512, 1024]))
        lens.append(max(1, edge + int(rng.integers(-2, 3))) if rng.random() < 0.6 else int(rng.integers(1, 1500)))
    what = "seed %d: %s p=%d n=%d G=%d Hkv=%d pairs=%d base=%g lens=%s" % (seed, NAMES[dtype], p, n, G, Hkv, pairs, base, lens)
    print(what, flush=True)
    S = max(lens)
    k, v, q, pk, pv = make_small(dtype, B=B, S=S, Hkv=Hkv, G=G, seed=500 + seed)
    if seed % 4 == 3:
        pk = pv = None                                  # rows kept in their order: identity permutation of the parameters
    got, want = run_both(k, v, q, n, p, lens, 128 ** -0.5, pk, pv, pairs, S_max=S + seed % 7, theta=llama_theta(base))
    assert_attention_close(got, want, dtype, what)
