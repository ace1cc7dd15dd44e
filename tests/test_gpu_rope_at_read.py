"""GPU parity of decode attention over keys cached before the rotary embedding and rotated at read
with the reordered parameters (Sec. III; Alg. 1 step 5), against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth
from test_gpu_attention import make_small
from util import assert_attention_close, assert_planes_equal, dev_i32, gpu_cache, oracle_cache

pytestmark = pytest.mark.gpu

D = 128


def llama_theta(base=10000.0):
    return (base ** (-np.arange(D // 2, dtype=np.float64) / (D // 2))).astype(np.float32)


def run_both(k, v, q, n, p, lens, scale, pk, pv, pairs, S_max=None, theta=None, profile=False):
    B, S, Hkv, _ = k.shape
    S_max = S if S_max is None else S_max
    theta = llama_theta() if theta is None else theta
    ident = np.tile(np.arange(D, dtype=np.int32), (Hkv, 1))
    planes = oracle_cache(k, v, n, p, S_max, 0, pk, pv)
    cache = gpu_cache(k.cuda(), v.cuda(), n, p, S_max, perm_k=pk, perm_v=pv)
    assert_planes_equal(cache, planes, "cache before attention")
    th_o, pa_o, sg_o = O.permute_rope(theta, ident if pk is None else pk, pairs)
    want = O.decode_attention_rope(*planes, D, n, p, synth.to_f32_numpy(q), lens, float(np.float32(scale)),
                                   th_o, pa_o, sg_o, perm_k=pk, perm_v=pv)
    th, pa, sg = kvbfp.permute_rope(theta, ident if pk is None else pk, pairs)      # the library's own host call
    sl = dev_i32(np.broadcast_to(np.asarray(lens), (B,)))
    got = kvbfp.decode_attention_rope(cache, q.cuda(), int(np.max(lens)), float(np.float32(scale)),
                                      torch.from_numpy(th).cuda(), torch.from_numpy(pa).cuda(),
                                      torch.from_numpy(sg).cuda(), seq_len_dev=sl, perm_k=dev_i32(pk),
                                      perm_v=dev_i32(pv), profile=profile)
    torch.cuda.synchronize()
    return got, want


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
@pytest.mark.parametrize("p,n", [(4, 16), (4, 32), (4, 128), (8, 16), (8, 64)])
@pytest.mark.parametrize("G,pairs", [(1, 0), (4, 1), (6, 0)])
def test_rotation_at_read_matches_oracle(dtype, p, n, G, pairs):
    # 700 tokens: two full 256-token tiles and a ragged third; the second sequence stops mid-tile
    k, v, q, pk, pv = make_small(dtype, B=2, S=700, Hkv=2, G=G, seed=120 + G)
    got, want = run_both(k, v, q, n, p, [700, 259], 128 ** -0.5, pk, pv, pairs, S_max=720)
    assert_attention_close(got, want, dtype, "p=%d n=%d G=%d pairs=%d" % (p, n, G, pairs))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rotation_is_not_a_no_op_and_rows_need_not_be_reordered(dtype):
    k, v, q, _, _ = make_small(dtype, B=1, S=300, Hkv=2, G=2, seed=130)
    got, want = run_both(k, v, q, 32, 4, [300], 0.1, None, None, 1)
    assert_attention_close(got, want, dtype)
    plain = kvbfp.decode_attention(gpu_cache(k.cuda(), v.cuda(), 32, 4, 300), q.cuda(), 300, float(np.float32(0.1)))
    torch.cuda.synchronize()
    assert (plain.double().cpu() - got.double().cpu()).norm() > 1e-2 * got.double().cpu().norm()


def test_token_indices_beyond_100k_keep_fp32_accuracy():
    # angles up to 1.3e5 radians at the highest frequency (theta = 1): the sequence is long enough for
    # many splits, the kernel's tile phasors are stepped across all of them, and fp32 I/O holds the 1e-5 bar
    S = 131072 + 300
    k, v, q, pk, pv = make_small(torch.float32, B=1, S=S, Hkv=1, G=2, seed=140)
    got, want = run_both(k, v, q, 32, 4, [S], 128 ** -0.5, pk, pv, 1)
    assert_attention_close(got, want, torch.float32)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_token_indices_beyond_100k_with_16_bit_io(dtype):
    # the matrix-core pass: per-tile phasors stepped in fp32 from a double-precision start over 45 tiles
    # per wavefront (12 splits), angles up to 1.3e5 radians
    S = 131072 + 300
    k, v, q, pk, pv = make_small(dtype, B=1, S=S, Hkv=1, G=4, seed=141)
    got, want = run_both(k, v, q, 32, 4, [S], 128 ** -0.5, pk, pv, 1)
    assert_attention_close(got, want, dtype)


@pytest.mark.parametrize("n", [16, 32, 128])
@pytest.mark.parametrize("k_shift,q_shift", [(-100, 0), (100, 0), (0, 90), (0, -90), (-60, -50)])
def test_rotation_at_read_at_the_ends_of_the_range(n, k_shift, q_shift):
    # block exponents are applied after the matrix product and the query is normalised per 32 channels:
    # keys and queries anywhere in the fp32 range, with the softmax scale that brings the logits back
    dtype = torch.bfloat16
    B, S, Hkv, G = 2, 600, 2, 4
    g = synth.outlier_gains(6, 0, Hkv, D)
    mk = lambda t, sh: (t * 2.0 ** sh).to(dtype)
    k = mk(synth.kv_rows(B, S, Hkv, D, "f32", g, 6, 2), k_shift)
    v = synth.kv_rows(B, S, Hkv, D, "bf16", g, 6, 3)
    q = mk(synth.queries(B, Hkv * G, D, "f32", 6, 4), q_shift)
    pk = O.calibrate_perm(synth.to_f32_numpy(k[0, :64]))
    scale = float(np.float32(D ** -0.5) * np.float32(2.0 ** (-(k_shift + q_shift))))
    got, want = run_both(k, v, q, n, 4, [S, 259], scale, pk, None, 0)
    assert bool(torch.isfinite(got).all())
    assert_attention_close(got, want, dtype, "n=%d shifts k %d q %d" % (n, k_shift, q_shift))


def test_blocks_of_16_with_very_different_exponents_inside_one_chunk():
    # every second block of 16 channels 2^30 below its neighbour: the smaller block is scaled down inside
    # the conversion, and what falls below 2^-24 of the larger block's unit is dropped
    dtype = torch.bfloat16
    k, v, q, pk, pv = make_small(dtype, B=1, S=400, Hkv=2, G=4, seed=151)
    damp = torch.ones(D)
    damp[torch.arange(D) % 32 >= 16] = 2.0 ** -30
    k = (k.float() * damp).to(dtype)
    got, want = run_both(k, v, q, 16, 4, [400], 0.3, None, pv, 1)
    assert_attention_close(got, want, dtype)


def test_profile_variant_returns_the_same_result_and_two_durations():
    k, v, q, pk, pv = make_small(torch.bfloat16, B=2, S=600, Hkv=2, G=4, seed=150)
    (got, split_ms, combine_ms), want = run_both(k, v, q, 16, 4, [600, 1], 0.09, pk, pv, 0, profile=True)
    assert_attention_close(got, want, torch.bfloat16)
    assert split_ms > 0 and combine_ms > 0
