"""Pins for the oracle's K-sort steps (Alg. 1 steps 1-4, Eq. (2)-(3)).  CPU only."""
import numpy as np
import pytest

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import synth


def test_perm_is_sorted_bijection_with_outliers_last():
    # tiny workload: 4 channels x20, 64 calibration tokens -> the four largest statistics are
    # exactly the planted channels, so they occupy the last positions (one block of 16 holds them)
    w = synth.WORKLOADS["tiny"]
    d = synth.make_workload_inputs(w)
    calib = synth.to_f32_numpy(d["k_calib"])            # [64][1][128]
    perm = O.calibrate_perm(calib, "maxabs")
    assert perm.shape == (1, 128)
    assert sorted(perm[0].tolist()) == list(range(128))
    stat = np.abs(calib[:, 0, :]).max(axis=0)
    assert np.all(np.diff(stat[perm[0]]) >= 0)
    planted = set(np.nonzero(d["k_gain"][0] > 1)[0].tolist())
    assert len(planted) == 4 and set(perm[0, -4:].tolist()) == planted
    # descending puts them first
    permd = O.calibrate_perm(calib, "maxabs", descending=True)
    assert set(permd[0, :4].tolist()) == planted
    assert np.all(np.diff(stat[permd[0]]) <= 0)


def test_ties_keep_ascending_channel_order_and_identity():
    x = np.zeros((3, 2, 8), dtype=np.float32)
    x[:, 0, :] = [[1, 5, 1, 3, 5, 0, 3, 1]] * 3         # duplicated statistics
    x[:, 1, :] = np.arange(8)                           # already sorted -> identity
    perm = O.calibrate_perm(x, "maxabs")
    assert perm[0].tolist() == [5, 0, 2, 7, 3, 6, 1, 4]
    assert perm[1].tolist() == list(range(8))
    permd = O.calibrate_perm(x, "maxabs", descending=True)
    assert permd[0].tolist() == [1, 4, 3, 6, 0, 2, 7, 5]
    assert permd[1].tolist() == list(range(7, -1, -1))


def test_l2_matches_library_argsort_of_row_norms():
    # Alg. 1: N_i = ||W_k[i, :]||, pi = argsort(N)  -- against numpy's norm + stable argsort
    rng = np.random.default_rng(1)
    H, D, F = 3, 128, 96
    w = rng.standard_normal((H * D, F)).astype(np.float32)
    big = rng.choice(H * D, size=9, replace=False)
    w[big] *= 12
    perm = O.calibrate_perm_from_weights(w, H, D)
    for h in range(H):
        norms = np.linalg.norm(w[h * D:(h + 1) * D].astype(np.float64), axis=1)
        want = np.argsort(norms, kind="stable")
        assert perm[h].tolist() == want.tolist()
    # max-abs and L2 differ in general: a row of many medium entries vs one spike
    x = np.zeros((4, 1, 2), dtype=np.float32)
    x[:, 0, 0] = 1.0          # L2 = 2, max = 1
    x[0, 0, 1] = 1.5          # L2 = 1.5, max = 1.5
    assert O.calibrate_perm(x, "maxabs")[0].tolist() == [0, 1]
    assert O.calibrate_perm(x, "l2")[0].tolist() == [1, 0]


def test_permute_weights_leaves_the_qk_product_unchanged():
    # Eq. (2)-(3): W_q^T W_k = pi(W_q)^T pi(W_k); exact on integer-valued data
    rng = np.random.default_rng(2)
    Hkv, G, D, F = 2, 3, 16, 10
    wk = rng.integers(-9, 10, size=(Hkv * D, F)).astype(np.float32)
    wq = rng.integers(-9, 10, size=(Hkv * G * D, F)).astype(np.float32)
    perm = np.stack([rng.permutation(D) for _ in range(Hkv)]).astype(np.int32)
    wk_p = O.permute_weights(wk, Hkv, D, perm, heads_per_perm=1)
    wq_p = O.permute_weights(wq, Hkv * G, D, perm, heads_per_perm=G)
    x = rng.integers(-5, 6, size=(F,)).astype(np.float64)
    for hq in range(Hkv * G):
        g = hq // G
        q, k = wq[hq * D:(hq + 1) * D] @ x, wk[g * D:(g + 1) * D] @ x
        qp, kp = wq_p[hq * D:(hq + 1) * D] @ x, wk_p[g * D:(g + 1) * D] @ x
        assert np.array_equal(qp, q[perm[g]]) and np.array_equal(kp, k[perm[g]])
        assert q @ k == qp @ kp
        a = wq[hq * D:(hq + 1) * D].T.astype(np.float64) @ wk[g * D:(g + 1) * D]
        b = wq_p[hq * D:(hq + 1) * D].T.astype(np.float64) @ wk_p[g * D:(g + 1) * D]
        assert np.array_equal(a, b)


def test_sorting_by_weight_norm_orders_key_magnitudes():
    # Sec. II-C: large-norm rows of W_k are what makes a key channel an outlier channel
    rng = np.random.default_rng(3)
    D, F = 128, 256
    wk = rng.standard_normal((D, F)).astype(np.float32)
    planted = [7, 40, 99]
    wk[planted] *= 15
    perm = O.calibrate_perm_from_weights(wk, 1, D)
    assert set(perm[0, -3:].tolist()) == set(planted)
    xs = rng.standard_normal((64, F))
    keys = (xs @ wk.T.astype(np.float64)).astype(np.float32).reshape(64, 1, D)
    assert set(O.calibrate_perm(keys, "maxabs")[0, -3:].tolist()) == set(planted)


@pytest.mark.parametrize("n", [32, 64, 128])       # the block sizes of Table I
def test_reorder_lowers_quantization_error_except_at_full_head_blocks(n):
    # Table I direction: the reorder helps for blocks smaller than the head, and a block that
    # spans the whole head (n = 128) cannot benefit -- the error is then identical.
    w = synth.WORKLOADS["llama2_7b_4k"]
    d = synth.make_workload_inputs(w, seq=192)
    k = synth.to_f32_numpy(d["k"])[:, :, :4]                    # [1][192][4][128]
    calib = synth.to_f32_numpy(d["k_calib"])[:, :4]
    perm = O.calibrate_perm(calib, "maxabs")
    S = k.shape[1]
    m0, e0 = O.quantize_append(k, n, 4, S, 0)
    m1, e1 = O.quantize_append(k, n, 4, S, 0, perm=perm)
    err0 = ((O.dequantize(m0, e0, 128, n, 4, 0, S) - k) ** 2).mean()
    err1 = ((O.dequantize(m1, e1, 128, n, 4, 0, S, perm=perm) - k) ** 2).mean()
    if n == 128:
        assert err1 == pytest.approx(err0, rel=1e-12)
    else:
        assert err1 < 0.9 * err0


def test_permute_weight_columns_carries_the_value_permutation_into_the_next_projection():
    # Sec. III, last paragraph: with W_v's rows and W_o's columns reordered alike, W_o' (P W_v' x) =
    # W_o (P W_v x) for any mixing P over tokens; exact on integer-valued data.  Several query heads
    # share a KV head's permutation.
    rng = np.random.default_rng(5)
    Hkv, G, D, F, T = 2, 3, 8, 6, 5
    wv = rng.integers(-9, 10, size=(Hkv * D, F)).astype(np.float32)
    wo = rng.integers(-9, 10, size=(F, Hkv * G * D)).astype(np.float32)
    perm = np.stack([rng.permutation(D) for _ in range(Hkv)]).astype(np.int32)
    wv_p = O.permute_weights(wv, Hkv, D, perm)
    wo_p = O.permute_weight_columns(wo, Hkv * G, D, perm, heads_per_perm=G)
    # written out: column (h, j) of the result is column (h, perm[h // G][j]) of the input
    for h in range(Hkv * G):
        for j in range(D):
            assert np.array_equal(wo_p[:, h * D + j], wo[:, h * D + perm[h // G][j]])
    x = rng.integers(-5, 6, size=(T, F)).astype(np.float64)
    mix = rng.integers(0, 4, size=(Hkv * G, T)).astype(np.float64)          # one row of "probabilities" per query head
    v = (x @ wv.T.astype(np.float64)).reshape(T, Hkv, D)
    v_p = (x @ wv_p.T.astype(np.float64)).reshape(T, Hkv, D)
    o = np.stack([mix[h] @ v[:, h // G] for h in range(Hkv * G)]).reshape(-1)
    o_p = np.stack([mix[h] @ v_p[:, h // G] for h in range(Hkv * G)]).reshape(-1)
    assert not np.array_equal(o, o_p)
    assert np.array_equal(wo.astype(np.float64) @ o, wo_p.astype(np.float64) @ o_p)
    # a transposed reading (scatter instead of gather) would break the product
    wo_wrong = np.empty_like(wo)
    for h in range(Hkv * G):
        wo_wrong[:, h * D + perm[h // G]] = wo[:, h * D:(h + 1) * D]
    assert not np.array_equal(wo_wrong.astype(np.float64) @ o_p, wo.astype(np.float64) @ o)
