"""GPU parity of decode attention over the packed cache against the oracle (fp64), through the C ABI.
Tolerance: max over (batch, head) of the relative L2 error, 2e-3 for fp16/bf16 I/O, 1e-5 for fp32."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth
from util import DT_NAME, assert_attention_close, assert_planes_equal, dev_i32, gpu_cache, oracle_cache

pytestmark = pytest.mark.gpu


def run_both(k, v, q, n, p, lens, scale, pk=None, pv=None, S_max=None, use_seq_len=True, q_mant_bits=0):
    """k, v: CPU tensors [B][S][Hkv][D]; q: CPU [B][Hq][D].  Returns (gpu_out, oracle_out)."""
    B, S, Hkv, D = k.shape
    S_max = S if S_max is None else S_max
    planes = oracle_cache(k, v, n, p, S_max, 0, pk, pv)
    cache = gpu_cache(k.cuda(), v.cuda(), n, p, S_max, perm_k=pk, perm_v=pv)
    assert_planes_equal(cache, planes, "cache before attention")
    want = O.decode_attention(*planes, D, n, p, synth.to_f32_numpy(q), lens, float(np.float32(scale)), pk, pv,
                              q_mant_bits=q_mant_bits)
    max_len = int(np.max(lens))
    sl = dev_i32(np.broadcast_to(np.asarray(lens), (B,))) if use_seq_len else None
    if q_mant_bits:
        got = kvbfp.decode_attention_qbfp(cache, q.cuda(), max_len, float(np.float32(scale)), q_mant_bits,
                                          seq_len_dev=sl, perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    else:
        got = kvbfp.decode_attention(cache, q.cuda(), max_len, float(np.float32(scale)), seq_len_dev=sl,
                                     perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    return got, want


def make_small(dtype, B, S, Hkv, G, seed):
    D = 128
    kg = synth.outlier_gains(seed, 0, Hkv, D)
    vg = synth.outlier_gains(seed, 1, Hkv, D)
    k = synth.kv_rows(B, S, Hkv, D, DT_NAME[dtype], kg, seed, 2)
    v = synth.kv_rows(B, S, Hkv, D, DT_NAME[dtype], vg, seed, 3)
    q = synth.queries(B, Hkv * G, D, DT_NAME[dtype], seed, 4)
    calib_k = synth.kv_rows(1, 64, Hkv, D, DT_NAME[dtype], kg, seed, 5)[0]
    calib_v = synth.kv_rows(1, 64, Hkv, D, DT_NAME[dtype], vg, seed, 6)[0]
    pk = O.calibrate_perm(synth.to_f32_numpy(calib_k))
    pv = O.calibrate_perm(synth.to_f32_numpy(calib_v))
    return k, v, q, pk, pv


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
@pytest.mark.parametrize("p,n", [(4, 16), (4, 32), (4, 64), (4, 128), (8, 16), (8, 32), (8, 64), (8, 128)])
@pytest.mark.parametrize("G", [1, 4])
def test_decode_attention_matches_oracle(dtype, p, n, G):
    # 700 tokens: two full 256-token tiles and a ragged third; the second sequence stops mid-tile
    k, v, q, pk, pv = make_small(dtype, B=2, S=700, Hkv=2, G=G, seed=20 + G)
    got, want = run_both(k, v, q, n, p, [700, 259], 128 ** -0.5, pk, pv, S_max=720)
    assert_attention_close(got, want, dtype, "p=%d n=%d G=%d" % (p, n, G))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("p,n", [(4, 16), (4, 32), (4, 64), (8, 16), (8, 128)])
@pytest.mark.parametrize("G,qbits", [(1, 8), (4, 8), (4, 4), (6, 8)])
def test_query_cast_to_bfp_matches_oracle(dtype, p, n, G, qbits):
    # Sec. III / Sec. IV: the query enters the score product as BFP (8-bit mantissas in the paper's
    # experiments); the cast is decided on exact fp32 values on both sides, so the tolerance is the
    # one of the plain path.
    k, v, q, pk, pv = make_small(dtype, B=2, S=600, Hkv=2, G=G, seed=70 + G)
    got, want = run_both(k, v, q, n, p, [600, 77], 128 ** -0.5, pk, pv, q_mant_bits=qbits)
    assert_attention_close(got, want, dtype, "qbits=%d p=%d n=%d G=%d" % (qbits, p, n, G))
    # and the option is not a no-op: 4-bit queries move the result far beyond the tolerance
    if qbits == 4:
        plain = kvbfp.decode_attention(gpu_cache(k.cuda(), v.cuda(), n, p, 600, perm_k=pk, perm_v=pv), q.cuda(), 600,
                                       float(np.float32(128 ** -0.5)), perm_k=dev_i32(pk), perm_v=dev_i32(pv))
        torch.cuda.synchronize()
        assert (plain.double().cpu() - got.double().cpu()).norm() > 1e-2 * got.double().cpu().norm()


@pytest.mark.parametrize("p,n", [(4, 16), (4, 32), (4, 128), (8, 16), (8, 64)])
@pytest.mark.parametrize("G", [7, 8, 12])
def test_fp32_io_with_wide_groups(p, n, G):
    # fp32 I/O on the matrix cores: three bf16 limbs for the query and for the probabilities, two head
    # groups per workgroup (G > 4) and a second launch over the heads beyond the eighth (G = 12); long
    # enough for several splits, with the second sequence ending inside the first tile
    k, v, q, pk, pv = make_small(torch.float32, B=2, S=1500, Hkv=2, G=G, seed=90 + G)
    got, want = run_both(k, v, q, n, p, [1500, 131], 128 ** -0.5, pk, pv)
    assert_attention_close(got, want, torch.float32, "p=%d n=%d G=%d" % (p, n, G))


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("n", [16, 32])
@pytest.mark.parametrize("G", [10, 16, 20])
def test_sixteen_heads_per_workgroup(dtype, n, G):
    # more than 8 heads per kv-head in the LDS pipeline: one launch serves up to 16 (G = 20: 16 + 4);
    # several splits, the second sequence ends inside a tile, the third holds a single token
    k, v, q, pk, pv = make_small(dtype, B=3, S=2100, Hkv=2, G=G, seed=200 + G)
    got, want = run_both(k, v, q, n, 4, [2100, 777, 1], 128 ** -0.5, pk, pv)
    assert_attention_close(got, want, dtype, "n=%d G=%d" % (n, G))


@pytest.mark.parametrize("p", [4, 8])
@pytest.mark.parametrize("G", [2, 3, 5, 8, 9, 16, 24, 32, 40])
def test_group_sizes_and_no_permutation(G, p):
    k, v, q, _, _ = make_small(torch.bfloat16, B=1, S=300, Hkv=3, G=G, seed=40 + G)
    got, want = run_both(k, v, q, 32, p, [300], 0.11, None, None, use_seq_len=False)
    assert_attention_close(got, want, torch.bfloat16)


def test_sequence_length_edge_cases():
    # lengths 0 (zeros out), 1 (the value row itself), tile boundary, one past it, full
    k, v, q, pk, pv = make_small(torch.float16, B=5, S=513, Hkv=2, G=2, seed=50)
    lens = [0, 1, 256, 257, 513]
    got, want = run_both(k, v, q, 16, 4, lens, 128 ** -0.5, pk, pv, S_max=600)
    g = got.cpu().float().numpy()
    assert np.all(g[0] == 0)
    assert_attention_close(got[1:], want[1:], torch.float16)
    # length 1: exactly the decoded value row, un-permuted, rounded once to fp16
    planes = oracle_cache(k, v, 16, 4, 600, 0, pk, pv)
    v0 = O.dequantize(planes[2], planes[3], 128, 16, 4, 0, 1, perm=pv)[1, 0]       # [Hkv][D]
    want_row = torch.from_numpy(v0).to(torch.float16)
    for h in range(4):
        assert torch.equal(got[1, h].cpu(), want_row[h // 2])


def test_split_count_does_not_change_the_result_beyond_rounding():
    # the same cache attended through different max_seq / max_len (hence different split plans)
    k, v, q, pk, pv = make_small(torch.float32, B=1, S=3000, Hkv=1, G=2, seed=60)
    got_a, want = run_both(k, v, q, 32, 4, [3000], 128 ** -0.5, pk, pv, S_max=3000)
    got_b, _ = run_both(k, v, q, 32, 4, [3000], 128 ** -0.5, pk, pv, S_max=4096)
    assert_attention_close(got_a, want, torch.float32)
    assert_attention_close(got_b, want, torch.float32)
    # attending to a prefix only
    planes = oracle_cache(k, v, 32, 4, 3000, 0, pk, pv)
    cache = gpu_cache(k.cuda(), v.cuda(), 32, 4, 3000, perm_k=pk, perm_v=pv)
    want = O.decode_attention(*planes, 128, 32, 4, synth.to_f32_numpy(q), [1000], float(np.float32(128 ** -0.5)), pk, pv)
    got = kvbfp.decode_attention(cache, q.cuda(), 1000, 128 ** -0.5, perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    assert_attention_close(got, want, torch.float32)


def test_large_logits_stay_finite_and_accurate():
    k, v, q, pk, pv = make_small(torch.float32, B=1, S=400, Hkv=1, G=1, seed=70)
    got, want = run_both(k, v, q * 40, 16, 4, [400], 1.0, pk, pv)
    assert bool(torch.isfinite(got).all())
    assert_attention_close(got, want, torch.float32)


def test_tiny_workload_full_parity():
    # smallest benchmark configuration end to end: perm from the library, cache bytes, attention
    w = synth.WORKLOADS["tiny"]
    d = synth.make_workload_inputs(w)
    pk = kvbfp.calibrate_perm(d["k_calib"])
    pv = kvbfp.calibrate_perm(d["v_calib"])
    assert np.array_equal(pk, O.calibrate_perm(synth.to_f32_numpy(d["k_calib"])))
    assert np.array_equal(pv, O.calibrate_perm(synth.to_f32_numpy(d["v_calib"])))
    got, want = run_both(d["k"], d["v"], d["q"], w.block, w.mant_bits, [w.seq], w.head_dim ** -0.5, pk, pv)
    assert_attention_close(got, want, torch.float32)


def test_llama2_7b_4k_full_parity():
    w = synth.WORKLOADS["llama2_7b_4k"]
    d = synth.make_workload_inputs(w)
    pk = kvbfp.calibrate_perm(d["k_calib"])
    pv = kvbfp.calibrate_perm(d["v_calib"])
    got, want = run_both(d["k"], d["v"], d["q"], w.block, w.mant_bits, [w.seq], w.head_dim ** -0.5, pk, pv)
    assert_attention_close(got, want, torch.float16)


@pytest.mark.parametrize("offset", [1, 4])
@pytest.mark.parametrize("p,n,dtype", [(4, 32, torch.bfloat16), (8, 16, torch.float32)])
def test_exponent_planes_at_odd_addresses(offset, p, n, dtype):
    # exponent planes that are not 16-byte aligned take the general pass, which reads them byte by byte
    # (the mantissa planes must be aligned: see test_library_host.py); same bar against the oracle
    k, v, q, pk, pv = make_small(dtype, B=2, S=600, Hkv=2, G=4, seed=300 + offset)
    planes = oracle_cache(k, v, n, p, 600, 0, pk, pv)
    cache = gpu_cache(k.cuda(), v.cuda(), n, p, 600, perm_k=pk, perm_v=pv)
    moved = []
    for t in (cache.k_exp, cache.v_exp):
        buf = torch.zeros((t.numel() + 64,), dtype=torch.uint8, device="cuda")
        view = buf[offset:offset + t.numel()].view(t.shape)
        view.copy_(t)
        assert view.data_ptr() % 16 == offset
        moved.append(view)
    odd = kvbfp.Cache(cache.layout, cache.k_mant, moved[0], cache.v_mant, moved[1])
    scale = float(np.float32(128 ** -0.5))
    want = O.decode_attention(*planes, 128, n, p, synth.to_f32_numpy(q), [600, 333], scale, pk, pv)
    got = kvbfp.decode_attention(odd, q.cuda(), 600, scale, seq_len_dev=dev_i32(np.asarray([600, 333])),
                                 perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    assert_attention_close(got, want, dtype, "exponent planes at +%d" % offset)
    # appending through the odd planes writes the same bytes
    kvbfp.quantize_append(odd, k.cuda(), v.cuda(), perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    assert_planes_equal(odd, planes, "append into exponent planes at +%d" % offset)


@pytest.mark.parametrize("n,G", [(32, 4), (16, 8), (64, 4)])
def test_split_partials_before_the_output_rounding(n, G):
    # The arithmetic of the 16-bit passes, separately from the one rounding of the output: the workspace
    # holds the fp32 partial results of the splits, [B][Hq][n_splits][128] unnormalised outputs followed by
    # [B][Hq][n_splits][2] (running maximum in base-2 units, normaliser).  Merged here in fp64, they must
    # agree with the oracle far below a bf16 step.
    B, S, Hkv, D = 2, 2100, 2, 128
    k, v, q, pk, _ = make_small(torch.bfloat16, B=B, S=S, Hkv=Hkv, G=G, seed=400 + n)
    planes = oracle_cache(k, v, n, 4, S, 0, pk, None)
    cache = gpu_cache(k.cuda(), v.cuda(), n, 4, S, perm_k=pk)
    scale = float(np.float32(D ** -0.5))
    Hq = Hkv * G
    need = kvbfp.decode_workspace_bytes(cache.layout, Hq, S)
    n_splits = need // (B * Hq * (D + 2) * 4)
    assert n_splits * B * Hq * (D + 2) * 4 == need and n_splits > 1
    ws = torch.zeros((need,), dtype=torch.uint8, device="cuda")
    lens = [S, 1111]
    kvbfp.decode_attention(cache, q.cuda(), S, scale, seq_len_dev=dev_i32(np.asarray(lens)), perm_k=dev_i32(pk),
                           workspace=ws)
    torch.cuda.synchronize()
    f = ws.view(torch.float32).cpu().double().numpy()
    po = f[:B * Hq * n_splits * D].reshape(B, Hq, n_splits, D)
    ml = f[B * Hq * n_splits * D:].reshape(B, Hq, n_splits, 2)
    m, l = ml[..., 0], ml[..., 1]
    M = m.max(axis=-1, keepdims=True)
    wgt = np.where(np.isfinite(m), np.exp2(m - M), 0.0)
    merged = (wgt[..., None] * po).sum(axis=2) / (wgt * l).sum(axis=-1)[..., None]
    want = O.decode_attention(*planes, D, n, 4, synth.to_f32_numpy(q), lens, scale, pk, None)
    err = np.linalg.norm(merged - want, axis=-1) / np.linalg.norm(want, axis=-1)
    print("block %d, %d heads per kv-head: worst rel-L2 of the fp32 partials %.2e" % (n, G, err.max()))
    assert err.max() <= 1e-4, err


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("n", [32, 64, 128])
@pytest.mark.parametrize("G", [1, 4, 6])
def test_integer_score_product_of_8_bit_codes(dtype, n, G):
    # 8-bit keys and an 8-bit BFP query, blocks of 32 and wider: the scores are integer matrix products of the
    # codes with the two block exponents added afterwards (Sec. II-B), in the LDS pipeline
    k, v, q, pk, pv = make_small(dtype, B=2, S=700, Hkv=2, G=G, seed=40 + G + n)
    got, want = run_both(k, v, q, n, 8, [700, 259], 128 ** -0.5, pk, pv, S_max=720, q_mant_bits=8)
    assert_attention_close(got, want, dtype, "integer scores n=%d G=%d" % (n, G))


def test_integer_score_product_at_the_ends_of_the_range():
    # queries and keys far from 1: the exponent sum of a group is formed in integers and applied once
    dtype = torch.bfloat16
    for k_shift, q_shift in ((-100, 60), (90, -100), (-60, -50)):
        k, v, q, pk, pv = make_small(dtype, B=1, S=400, Hkv=2, G=4, seed=47)
        k = (k.float() * 2.0 ** k_shift).to(dtype)
        q = (q.float() * 2.0 ** q_shift).to(dtype)
        scale = float(np.float32(128 ** -0.5) * np.float32(2.0 ** (-(k_shift + q_shift))))
        got, want = run_both(k, v, q, 32, 8, [400], scale, pk, pv, q_mant_bits=8)
        assert_attention_close(got, want, dtype, "integer scores, shifts %d %d" % (k_shift, q_shift))
