"""Pins for the oracle's decode attention over the packed cache (Sec. III run-time flow).  CPU only.

The attention itself is ordinary softmax attention on the decoded values, so it is pinned to
numpy's dense fp64 evaluation, to textbook softmax properties, and to the permutation
invariance of Eq. (2)-(3)."""
import numpy as np
import pytest

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import synth


def build_cache(k, v, n, p, perm_k=None, perm_v=None, S_max=None):
    B, S, H, D = k.shape
    S_max = S if S_max is None else S_max
    km, ke = O.quantize_append(k, n, p, S_max, 0, perm=perm_k)
    vm, ve = O.quantize_append(v, n, p, S_max, 0, perm=perm_v)
    return km, ke, vm, ve


def dense_attention(q, khat, vhat, scale, G):
    """numpy fp64 softmax(q K^T * scale) V; khat/vhat [B][S][Hkv][D], q [B][Hq][D]."""
    B, Hq, D = q.shape
    out = np.zeros((B, Hq, D))
    for b in range(B):
        for h in range(Hq):
            K = khat[b, :, h // G, :]
            V = vhat[b, :, h // G, :]
            s = (K @ q[b, h].astype(np.float64)) * scale
            w = np.exp(s - s.max())
            out[b, h] = (w / w.sum()) @ V
    return out


def small_inputs(seed, B=2, S=37, Hkv=2, G=2, D=128):
    rng = np.random.default_rng(seed)
    k = rng.standard_normal((B, S, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((B, S, Hkv, D)).astype(np.float32)
    k[..., [5, 64, 127]] *= 20
    v[..., [9, 33]] *= 12
    q = rng.standard_normal((B, Hkv * G, D)).astype(np.float32)
    return k, v, q


@pytest.mark.parametrize("n,p", [(16, 4), (32, 4), (128, 4), (16, 8), (64, 8)])
def test_matches_dense_numpy_attention_on_decoded_cache(n, p):
    # P9: library cross-check, including per-sequence lengths, GQA head mapping and both perms
    k, v, q = small_inputs(1)
    B, S, Hkv, D = k.shape
    G = q.shape[1] // Hkv
    rng = np.random.default_rng(2)
    pk = np.stack([rng.permutation(D) for _ in range(Hkv)]).astype(np.int32)
    pv = np.stack([rng.permutation(D) for _ in range(Hkv)]).astype(np.int32)
    km, ke, vm, ve = build_cache(k, v, n, p, pk, pv, S_max=S + 5)
    lens = [S, 11]
    scale = 1.0 / np.sqrt(D)
    out = O.decode_attention(km, ke, vm, ve, D, n, p, q, lens, scale, pk, pv)
    khat = O.dequantize(km, ke, D, n, p, 0, S, perm=pk)       # original channel order
    vhat = O.dequantize(vm, ve, D, n, p, 0, S, perm=pv)
    for b, L in enumerate(lens):
        want = dense_attention(q[b:b + 1], khat[b:b + 1, :L], vhat[b:b + 1, :L], scale, G)
        assert np.allclose(out[b], want[0], rtol=1e-12, atol=1e-13)
    # the decoded cache is close to the input it came from (ties the decode to Eq. (1))
    assert np.abs(khat - k).max() <= np.abs(k).max() / (2 ** (p - 2)) * 0.5 + 1e-12


def test_scores_are_invariant_under_a_common_permutation():
    # Eq. (2)-(3) on integer-valued data: exact equality, before and after quantization
    rng = np.random.default_rng(3)
    D, S = 128, 9
    kint = rng.integers(-7, 8, size=(1, S, 1, D)).astype(np.float32)   # representable with p = 4
    qint = rng.integers(-9, 10, size=(D,)).astype(np.float64)
    perm = rng.permutation(D).astype(np.int32).reshape(1, D)
    m0, e0 = O.quantize_append(kint, 16, 4, S, 0)
    m1, e1 = O.quantize_append(kint, 16, 4, S, 0, perm=perm)
    s_plain = O.scores(m0[0, 0], e0[0, 0], D, 16, 4, qint, 1.0)
    s_perm = O.scores(m1[0, 0], e1[0, 0], D, 16, 4, qint[perm[0]], 1.0)
    want = kint[0, :, 0, :].astype(np.float64) @ qint
    assert np.array_equal(s_plain, want) and np.array_equal(s_perm, want)


def test_full_head_block_makes_the_reorder_a_no_op():
    # Table I, n = 128 row: one block per head -> same exponent, mantissas merely permuted
    k, v, q = small_inputs(4, B=1, S=50, Hkv=2, G=1)
    D = 128
    rng = np.random.default_rng(5)
    pk = np.stack([rng.permutation(D) for _ in range(2)]).astype(np.int32)
    pv = np.stack([rng.permutation(D) for _ in range(2)]).astype(np.int32)
    c0 = build_cache(k, v, 128, 4)
    c1 = build_cache(k, v, 128, 4, pk, pv)
    assert np.array_equal(c0[1], c1[1]) and np.array_equal(c0[3], c1[3])
    o0 = O.decode_attention(*c0, D, 128, 4, q, 50, 0.09)
    o1 = O.decode_attention(*c1, D, 128, 4, q, 50, 0.09, pk, pv)
    assert np.allclose(o0, o1, rtol=1e-12, atol=1e-14)
    # with small blocks the reorder does change the result
    o2 = O.decode_attention(*build_cache(k, v, 16, 4), D, 16, 4, q, 50, 0.09)
    o3 = O.decode_attention(*build_cache(k, v, 16, 4, pk, pv), D, 16, 4, q, 50, 0.09, pk, pv)
    assert not np.allclose(o2, o3, rtol=1e-6, atol=1e-9)


def test_softmax_special_cases():
    D, n, p = 128, 16, 4
    k, v, q = small_inputs(6, B=1, S=20, Hkv=1, G=2)
    pv = np.random.default_rng(7).permutation(D).astype(np.int32).reshape(1, D)
    km, ke, vm, ve = build_cache(k, v, n, p, None, pv)
    vhat = O.dequantize(vm, ve, D, n, p, 0, 20, perm=pv)[0, :, 0, :]
    # one cached token: the output is that value row, whatever the scores
    o = O.decode_attention(km, ke, vm, ve, D, n, p, q, 1, 0.3, None, pv)
    assert np.array_equal(o[0, 0], vhat[0]) and np.array_equal(o[0, 1], vhat[0])
    # no cached token: zeros
    o = O.decode_attention(km, ke, vm, ve, D, n, p, q, 0, 0.3, None, pv)
    assert np.all(o == 0)
    # q = 0: uniform weights -> mean of the value rows
    o = O.decode_attention(km, ke, vm, ve, D, n, p, np.zeros_like(q), 20, 0.3, None, pv)
    assert np.allclose(o[0, 0], vhat.mean(axis=0), rtol=1e-13, atol=1e-15)
    # identical key rows: uniform weights again
    kk = np.repeat(k[:, :1], 20, axis=1)
    km2, ke2 = O.quantize_append(kk, n, p, 20, 0)
    o = O.decode_attention(km2, ke2, vm, ve, D, n, p, q, 20, 0.3, None, pv)
    assert np.allclose(o[0, 1], vhat.mean(axis=0), rtol=1e-12, atol=1e-14)


def test_shift_invariance_and_large_logits():
    D, n, p = 128, 16, 4
    k, v, q = small_inputs(8, B=1, S=30, Hkv=1, G=1)
    k[..., 0:16] = 0
    k[..., 3] = 4.0                     # same exactly representable value in every row
    km, ke, vm, ve = build_cache(k, v, n, p)
    q2 = q.copy()
    q2[..., 3] += 64.0                  # shifts every score by the same amount
    o1 = O.decode_attention(km, ke, vm, ve, D, n, p, q, 30, 0.25)
    o2 = O.decode_attention(km, ke, vm, ve, D, n, p, q2, 30, 0.25)
    assert np.allclose(o1, o2, rtol=1e-10, atol=1e-12)
    # scores of magnitude ~1e3: still finite and equal to the arg-max row
    o = O.decode_attention(km, ke, vm, ve, D, n, p, q * 50, 30, 1.0)
    assert np.all(np.isfinite(o))
    khat = O.dequantize(km, ke, D, n, p, 0, 30)[0, :, 0, :]
    vhat = O.dequantize(vm, ve, D, n, p, 0, 30)[0, :, 0, :]
    s = khat @ (q[0, 0].astype(np.float64) * 50)
    top = np.sort(s)[-2:]
    assert top[1] - top[0] > 40          # a clear winner, so the output is its value row
    assert np.allclose(o[0, 0], vhat[int(np.argmax(s))], rtol=1e-12, atol=1e-12)


def test_query_cast_to_bfp16_option():
    # Sec. III / Sec. IV: queries may be cast to BFP16 (8-bit mantissas) before the product.
    # With a query that is exactly representable the option changes nothing; otherwise it equals
    # running the plain path on the query quantized-and-decoded by the cast pinned elsewhere.
    D, n, p = 128, 32, 4
    k, v, q = small_inputs(9, B=1, S=25, Hkv=1, G=2)
    km, ke, vm, ve = build_cache(k, v, n, p)
    qi = np.random.default_rng(1).integers(-127, 128, size=q.shape).astype(np.float32) * 0.125
    a = O.decode_attention(km, ke, vm, ve, D, n, p, qi, 25, 0.1)
    b = O.decode_attention(km, ke, vm, ve, D, n, p, qi, 25, 0.1, q_mant_bits=8)
    assert np.array_equal(a, b)
    qm, qe = O.quantize_append(q.reshape(1, 2, 1, D), n, 8, 2, 0)
    qhat = O.dequantize(qm, qe, D, n, 8, 0, 2)[0, :, 0, :].astype(np.float32).reshape(1, 2, D)
    a = O.decode_attention(km, ke, vm, ve, D, n, p, qhat, 25, 0.1)
    b = O.decode_attention(km, ke, vm, ve, D, n, p, q, 25, 0.1, q_mant_bits=8)
    assert np.array_equal(a, b)
    c = O.decode_attention(km, ke, vm, ve, D, n, p, q, 25, 0.1)
    assert not np.array_equal(b, c) and np.allclose(b, c, rtol=0.2, atol=0.2)


def test_tiny_workload_end_to_end_is_sane():
    # the smallest benchmark configuration through the whole oracle path
    w = synth.WORKLOADS["tiny"]
    d = synth.make_workload_inputs(w)
    k, v, q = (synth.to_f32_numpy(d[x]) for x in ("k", "v", "q"))
    pk = O.calibrate_perm(synth.to_f32_numpy(d["k_calib"]))
    pv = O.calibrate_perm(synth.to_f32_numpy(d["v_calib"]))
    km, ke, vm, ve = build_cache(k, v, w.block, w.mant_bits, pk, pv)
    assert km.nbytes + ke.nbytes + vm.nbytes + ve.nbytes == 36864
    out = O.decode_attention(km, ke, vm, ve, 128, w.block, w.mant_bits, q, w.seq, 128 ** -0.5, pk, pv)
    # 4-bit keys: the scores track the unquantized ones closely (the softmax on top of them is
    # peaky for this outlier model, so the outputs themselves are only loosely comparable)
    s_exact = (k[0, :, 0, :].astype(np.float64) @ q[0, 0]) * 128 ** -0.5
    s_bfp = O.scores(km[0, 0], ke[0, 0], 128, w.block, w.mant_bits, q[0, 0][pk[0]].astype(np.float64), 128 ** -0.5)
    assert np.corrcoef(s_exact, s_bfp)[0, 1] > 0.98
    assert np.all(np.isfinite(out)) and np.abs(out).max() <= np.abs(v).max()
