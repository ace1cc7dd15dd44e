"""Rotary embeddings and the reorder (Sec. II-D, Alg. 1 step 5).

The build applies the permutation to RoPE's output when a row is appended instead of folding it into
W_k and rotating cached keys at read.  These CPU checks pin the two facts that choice rests on:
the scores are unchanged, and channel-consistent outliers survive the rotation as consistent
outlier *pairs* that the max-|x| statistic still gathers into few blocks."""
import numpy as np

from oracle import kvbfp_oracle as O

D = 128


def rope(x, pos, theta):
    """Eq. (RoFreq): consecutive pairs (2i, 2i+1) rotated by pos * theta_i.  x: [T][D], pos: [T]."""
    ang = pos[:, None] * theta[None, :]
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[:, 0::2] = x[:, 0::2] * c - x[:, 1::2] * s
    out[:, 1::2] = x[:, 1::2] * c + x[:, 0::2] * s
    return out


def test_scores_do_not_depend_on_where_the_permutation_is_applied():
    rng = np.random.default_rng(0)
    theta = 10000.0 ** (-np.arange(D // 2) / (D // 2))
    T = 50
    k = rng.standard_normal((T, D))
    q = rng.standard_normal((1, D))
    pos = np.arange(T, dtype=np.float64)
    perm = rng.permutation(D)
    want = rope(k, pos, theta) @ rope(q, np.array([float(T)]), theta)[0]
    # permutation applied to the rotated vectors (this build)
    got_after = rope(k, pos, theta)[:, perm] @ rope(q, np.array([float(T)]), theta)[0][perm]
    assert np.allclose(got_after, want, rtol=1e-13, atol=1e-12)
    # Alg. 1 step 5: rows permuted first, then RoPE with permuted frequencies, partners and signs
    theta_full = np.repeat(theta, 2)                         # [th1, th1, th2, th2, ...]
    partner = np.arange(D) ^ 1                               # i = [2,1,4,3,...] (0-based: j xor 1)
    sign = np.where(np.arange(D) % 2 == 0, -1.0, 1.0)        # s = [-1, 1, -1, 1, ...]
    inv = np.argsort(perm)

    def rope_permuted(xp, p):                                # xp = x[:, perm]
        th, sg, pa = theta_full[perm], sign[perm], inv[partner[perm]]
        ang = p[:, None] * th[None, :]
        return xp * np.cos(ang) + sg[None, :] * xp[:, pa] * np.sin(ang)

    got_alg1 = rope_permuted(k[:, perm], pos) @ rope_permuted(q[:, perm], np.array([float(T)]))[0]
    assert np.allclose(got_alg1, want, rtol=1e-13, atol=1e-12)


def test_outliers_survive_rope_as_pairs_and_sorting_still_helps():
    rng = np.random.default_rng(1)
    theta = 10000.0 ** (-np.arange(D // 2) / (D // 2))
    T = 512
    k = rng.standard_normal((T, D)).astype(np.float32)
    outliers = [5, 40, 77, 102]
    k[:, outliers] *= 20.0
    kr = rope(k.astype(np.float64), np.arange(T, dtype=np.float64), theta).astype(np.float32)
    calib = rope((rng.standard_normal((256, D)) * np.where(np.isin(np.arange(D), outliers), 20.0, 1.0)),
                 np.arange(256, dtype=np.float64), theta).astype(np.float32)
    perm = O.calibrate_perm(calib.reshape(256, 1, D))[0]
    # the eight channels of the four rotation pairs rank last (slow pairs keep the outlier mostly in one
    # channel, but its partner still sees it at some positions)
    pairs = sorted({c for o in outliers for c in (o, o ^ 1) if theta[o // 2] * 256 > 1.0} | set(outliers))
    assert set(outliers) <= set(perm[-8:].tolist())
    assert set(perm[-len(pairs):].tolist()) <= {c for o in outliers for c in (o, o ^ 1)}

    def mse(p):
        x = kr.reshape(1, T, 1, D)
        m, e = O.quantize_append(x, 32, 4, T, 0, perm=None if p is None else p.reshape(1, D))
        back = O.dequantize(m, e, D, 32, 4, 0, T, perm=None if p is None else p.reshape(1, D))
        return float(np.mean((back[0, :, 0, :] - kr) ** 2))

    assert mse(perm) < 0.8 * mse(None)
