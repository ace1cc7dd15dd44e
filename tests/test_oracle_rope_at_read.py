"""Pins of the oracle's rotary-embedding functions (Sec. II-D; Alg. 1 step 5; Sec. III: keys cached
before the rotation and rotated at read) against the rotation matrix of Sec. II-D written out in
full and against plain numpy attention, both in the ORIGINAL channel order."""
import numpy as np
import pytest

from oracle import kvbfp_oracle as O

D = 128


def rotation_matrix(theta, m, pair_layout):
    """The D x D matrix R_{Theta,m}: 2 x 2 blocks [[cos, -sin], [sin, cos]] on channel pairs
    (2i, 2i+1) (Sec. II-D) or (i, i + D/2) (the ordering of the footnote in Sec. III)."""
    R = np.zeros((D, D))
    for i in range(D // 2):
        a, b = (2 * i, 2 * i + 1) if pair_layout == 0 else (i, i + D // 2)
        c, s = np.cos(m * float(theta[i])), np.sin(m * float(theta[i]))
        R[a, a], R[a, b], R[b, a], R[b, b] = c, -s, s, c
    return R


def test_unpermuted_vectors_are_the_ones_the_paper_lists():
    theta = (10000.0 ** (-np.arange(D // 2) / (D // 2))).astype(np.float32)
    ident = np.arange(D, dtype=np.int32)[None, :]
    th, pa, sg = O.permute_rope(theta, ident, 0)
    assert np.array_equal(th[0], np.repeat(theta, 2))                     # [th1, th1, th2, th2, ...]
    assert pa[0, :6].tolist() == [1, 0, 3, 2, 5, 4]                      # i = [2, 1, 4, 3, ...], 0-based
    assert sg[0, :6].tolist() == [-1, 1, -1, 1, -1, 1]                   # s = [-1, 1, -1, 1, ...]
    th, pa, sg = O.permute_rope(theta, ident, 1)
    assert np.array_equal(th[0], np.concatenate([theta, theta]))          # [th1 .. th_{D/2}, th1 .. th_{D/2}]
    assert pa[0, :3].tolist() == [64, 65, 66] and pa[0, 64:67].tolist() == [0, 1, 2]
    assert np.all(sg[0, :64] == -1) and np.all(sg[0, 64:] == 1)


@pytest.mark.parametrize("pair_layout", [0, 1])
def test_permuted_parameters_rotate_the_permuted_row_like_the_matrix_rotates_the_original(pair_layout):
    rng = np.random.default_rng(3 + pair_layout)
    theta = rng.uniform(0.001, 1.0, D // 2).astype(np.float32)           # all different: a wrong index shows
    perm = np.stack([rng.permutation(D), rng.permutation(D)]).astype(np.int32)
    th, pa, sg = O.permute_rope(theta, perm, pair_layout)
    for h in range(2):
        assert sorted(pa[h].tolist()) == list(range(D))                   # partners: a permutation ...
        assert np.array_equal(pa[h][pa[h]], np.arange(D))                 # ... that is an involution
        assert np.all(sg[h] == -sg[h][pa[h]]) and np.array_equal(th[h], th[h][pa[h]])
        for m in (0, 1, 17, 4095):
            x = rng.standard_normal(D)
            want = (rotation_matrix(theta, m, pair_layout) @ x)[perm[h]]
            xp = x[perm[h]]
            ang = m * th[h].astype(np.float64)
            got = xp * np.cos(ang) + sg[h] * xp[pa[h]] * np.sin(ang)
            assert np.allclose(got, want, rtol=0, atol=1e-12)


def lossless_rows(rng, shape):
    """Integers in [-7, 7] with a +-7 in every block of 16: 4-bit BFP stores them exactly."""
    x = rng.integers(-7, 8, size=shape).astype(np.float32)
    x[..., ::16] = rng.choice([-7.0, 7.0], size=x[..., ::16].shape)
    return x


@pytest.mark.parametrize("pair_layout", [0, 1])
def test_attention_with_rotation_at_read_equals_numpy_attention_on_rotated_keys(pair_layout):
    rng = np.random.default_rng(11 + pair_layout)
    B, Hkv, G, S = 2, 2, 2, 37
    theta = (10000.0 ** (-np.arange(D // 2) / (D // 2))).astype(np.float32)
    k = lossless_rows(rng, (B, S, Hkv, D))
    v = lossless_rows(rng, (B, S, Hkv, D))
    q = rng.standard_normal((B, Hkv * G, D)).astype(np.float32)
    pk = np.stack([rng.permutation(D) for _ in range(Hkv)]).astype(np.int32)
    pv = np.stack([rng.permutation(D) for _ in range(Hkv)]).astype(np.int32)
    lens = [S, 20]
    km, ke = O.quantize_append(k, 16, 4, S, 0, perm=pk)
    vm, ve = O.quantize_append(v, 16, 4, S, 0, perm=pv)
    assert np.array_equal(O.dequantize(km, ke, D, 16, 4, 0, S, perm=pk), k)      # the cast lost nothing
    th, pa, sg = O.permute_rope(theta, pk, pair_layout)
    scale = 0.05
    got = O.decode_attention_rope(km, ke, vm, ve, D, 16, 4, q, lens, scale, th, pa, sg, perm_k=pk, perm_v=pv)
    for b in range(B):
        for h in range(Hkv * G):
            g = h // G
            kr = np.stack([rotation_matrix(theta, t, pair_layout) @ k[b, t, g].astype(np.float64)
                           for t in range(lens[b])])
            s = scale * (kr @ q[b, h].astype(np.float64))
            w = np.exp(s - s.max())
            want = (w / w.sum()) @ v[b, :lens[b], g].astype(np.float64)
            assert np.allclose(got[b, h], want, rtol=0, atol=1e-11)


def test_zero_frequencies_reduce_to_the_plain_attention():
    rng = np.random.default_rng(5)
    B, Hkv, G, S = 1, 2, 3, 50
    k = rng.standard_normal((B, S, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((B, S, Hkv, D)).astype(np.float32)
    q = rng.standard_normal((B, Hkv * G, D)).astype(np.float32)
    pk = np.stack([rng.permutation(D) for _ in range(Hkv)]).astype(np.int32)
    km, ke = O.quantize_append(k, 32, 8, S, 0, perm=pk)
    vm, ve = O.quantize_append(v, 32, 8, S, 0)
    th, pa, sg = O.permute_rope(np.zeros(D // 2, np.float32), pk, 0)
    got = O.decode_attention_rope(km, ke, vm, ve, D, 32, 8, q, [S], 0.1, th, pa, sg, perm_k=pk)
    want = O.decode_attention(km, ke, vm, ve, D, 32, 8, q, [S], 0.1, perm_k=pk)
    assert np.array_equal(got, want)


def test_scores_depend_on_the_distance_between_query_and_key_only():
    # the property rotary embeddings exist for: with q rotated at its own index, shifting every index by
    # the same amount changes nothing.  Shift = the cache starting 9 tokens later in the sequence.
    rng = np.random.default_rng(6)
    S, shift = 24, 9
    theta = (10000.0 ** (-np.arange(D // 2) / (D // 2))).astype(np.float32)
    k = lossless_rows(rng, (1, S + shift, 1, D))
    k[:, :shift] = 0                                                     # the first 9 tokens: zero keys ...
    v = lossless_rows(rng, (1, S + shift, 1, D))
    v[:, :shift] = 0
    q0 = rng.standard_normal(D)
    ident = np.arange(D, dtype=np.int32)[None, :]
    th, pa, sg = O.permute_rope(theta, ident, 0)

    def run(kk, vv, n_tok, q_index):
        qr = (rotation_matrix(theta, q_index, 0) @ q0).astype(np.float32)[None, None, :]
        km, ke = O.quantize_append(kk, 16, 4, n_tok, 0)
        vm, ve = O.quantize_append(vv, 16, 4, n_tok, 0)
        return O.decode_attention_rope(km, ke, vm, ve, D, 16, 4, qr, [n_tok], 0.07, th, pa, sg)[0, 0]

    a = run(k[:, shift:], v[:, shift:], S, S)
    b = run(k, v, S + shift, S + shift)
    # ... which add 9 tokens of score 0 and value 0 to the softmax: undo that renormalisation
    sc = lambda kk, qi: 0.07 * np.array([(rotation_matrix(theta, t, 0) @ kk[0, t, 0].astype(np.float64)) @
                                         (rotation_matrix(theta, qi, 0) @ q0).astype(np.float32).astype(np.float64)
                                         for t in range(kk.shape[1])])
    s_short, s_long = sc(k[:, shift:], S), sc(k, S + shift)
    assert np.allclose(s_long[shift:], s_short, atol=1e-5)              # q is rounded to fp32 after its rotation
    z_short = np.exp(s_short - s_short.max()).sum()
    z_long = np.exp(s_long - s_long.max()).sum()
    assert np.allclose(b * z_long * np.exp(s_long.max()), a * z_short * np.exp(s_short.max()), rtol=2e-4, atol=1e-9)
