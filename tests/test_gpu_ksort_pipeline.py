"""Alg. 1 end to end on the GPU path: permutation from the weights, reordered projections, BFP cache,
decode attention; and the qualitative content of Table I on the synthetic outlier model."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import ksort_report as R
from paper_2403_20137_amd import kvbfp, synth
from util import assert_attention_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def report():
    return R.run(tokens=1536, n_kv_heads=2, group=2, d_model=256, blocks=(128, 64, 32, 16), seed=7)


def test_reorder_leaves_unquantized_attention_alone(report):
    # Eq. (2)-(3): same scores, same outputs up to the channel order (inputs are rounded to bf16 once)
    assert report["reorder_invariance_rel_err"] < 5e-3


def test_reordered_output_projection_ends_in_the_same_vector(report):
    # Sec. III, last paragraph: W_o with reordered columns consumes the output in cache order
    assert report["reorder_invariance_after_w_o_rel_err"] < 5e-3
    rows = {r["block"]: r for r in report["rows"]}
    for n in (64, 32, 16):
        assert rows[n]["sorted_after_w_o"] < 0.9 * rows[n]["original_after_w_o"], (n, rows[n])


def test_sorting_lowers_the_error_below_the_full_row_block(report):
    rows = {r["block"]: r for r in report["rows"]}
    # Table I, n = 128: one block per row, the order inside it cannot matter
    assert abs(rows[128]["sorted"] - rows[128]["original"]) < 0.03 * rows[128]["original"]
    # Table I, n = 64 and 32: with the outlier channels gathered into few blocks the error drops
    for n in (64, 32, 16):
        assert rows[n]["sorted"] < 0.9 * rows[n]["original"], (n, rows[n])
    # and sorted + smaller blocks is the best of all
    assert rows[32]["sorted"] < rows[128]["sorted"]


def test_sorted_pipeline_matches_oracle():
    torch.manual_seed(3)
    hkv, grp, dm, T = 2, 2, 256, 700
    wq, wk, wv = R.synthetic_projections(hkv, grp, dm, 4, 20.0, seed=11)
    perm_k = kvbfp.calibrate_perm_from_weights(wk, hkv, R.D)
    perm_v = kvbfp.calibrate_perm_from_weights(wv, hkv, R.D)
    assert np.array_equal(perm_k, O.calibrate_perm_from_weights(wk.numpy(), hkv, R.D))
    assert np.array_equal(perm_v, O.calibrate_perm_from_weights(wv.numpy(), hkv, R.D))
    wq_s = kvbfp.permute_weights(wq, hkv * grp, R.D, perm_k, heads_per_perm=grp)
    wk_s = kvbfp.permute_weights(wk, hkv, R.D, perm_k)
    wv_s = kvbfp.permute_weights(wv, hkv, R.D, perm_v)
    assert np.array_equal(wk_s.numpy(), O.permute_weights(wk.numpy(), hkv, R.D, perm_k))
    assert np.array_equal(wq_s.numpy(), O.permute_weights(wq.numpy(), hkv * grp, R.D, perm_k, grp))
    wo = R.synthetic_output_projection(hkv, grp, dm, seed=11)
    wo_s = kvbfp.permute_weight_columns(wo, hkv * grp, R.D, perm_v, heads_per_perm=grp)
    assert np.array_equal(wo_s.numpy(), O.permute_weight_columns(wo.numpy(), hkv * grp, R.D, perm_v, grp))
    x = torch.randn(T, dm)
    xq = torch.randn(1, dm)
    k = R.project(x, wk_s, hkv, torch.bfloat16)
    v = R.project(x, wv_s, hkv, torch.bfloat16)
    q = R.project(xq, wq_s, hkv * grp, torch.bfloat16)[:, 0].contiguous()
    scale = float(np.float32(R.D ** -0.5))
    got = R.bfp_attention(q.cuda(), k.cuda(), v.cuda(), 32, 4, scale, "cuda")
    km, ke = O.quantize_append(synth.to_f32_numpy(k), 32, 4, T, 0)
    vm, ve = O.quantize_append(synth.to_f32_numpy(v), 32, 4, T, 0)
    want = O.decode_attention(km, ke, vm, ve, R.D, 32, 4, synth.to_f32_numpy(q), [T], scale)
    assert_attention_close(got.to(torch.bfloat16).unsqueeze(0), want, torch.bfloat16, "sorted pipeline")
