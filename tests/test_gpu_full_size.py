"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times: the whole
cache is written and attended on the GPU, and sampled (batch, kv-head) units are recomputed by the
oracle from the same inputs (copied back from the device) and compared: packed bytes bit-exact,
attention within tolerance."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth
from util import assert_attention_close, dev_i32

pytestmark = pytest.mark.gpu

SAMPLES = {  # workload -> sampled (batch, kv-head) units
    "batched_8k_p4": [(0, 0), (7, 13), (15, 31)],
    "batched_8k_p8": [(3, 5), (15, 30)],
    "llama3_8b_gqa_32k": [(0, 0), (5, 3), (7, 7)],
    "long_128k": [(0, 2), (0, 7)],
    "gqa_32k_n64": [(1, 2), (7, 6)],         # the headline shapes at Table I's other block sizes and at 8 bits
    "gqa_32k_n128": [(2, 1), (6, 7)],
    "gqa_32k_p8n16": [(0, 4), (5, 0)],
    "gqa_32k_p8n32": [(3, 3), (4, 6)],       # with the query cast to 8-bit BFP: the integer score product
}
Q_MANT_BITS = {"gqa_32k_p8n32": 8}


@pytest.mark.parametrize("name", list(SAMPLES))
def test_full_size_sampled_units(name):
    w = synth.WORKLOADS[name]
    tdt = synth.TORCH_DTYPES[w.dtype]
    d = synth.make_workload_inputs(w, device="cuda")
    pk = kvbfp.calibrate_perm(d["k_calib"].cpu())
    pv = kvbfp.calibrate_perm(d["v_calib"].cpu())
    S_max = w.seq + 1
    L = kvbfp.make_layout(w.head_dim, w.block, w.mant_bits, w.n_kv_heads, w.batch, S_max)
    cache = kvbfp.alloc_cache(L, "cuda", fill=0)
    pkd, pvd = dev_i32(pk), dev_i32(pv)
    kvbfp.quantize_append(cache, d["k"], d["v"], pos0=0, perm_k=pkd, perm_v=pvd)          # bulk prefill
    k1 = synth.kv_rows(w.batch, 1, w.n_kv_heads, w.head_dim, w.dtype, d["k_gain"], synth.BASE_SEED, synth.TID_K_NEW, "cuda")
    v1 = synth.kv_rows(w.batch, 1, w.n_kv_heads, w.head_dim, w.dtype, d["v_gain"], synth.BASE_SEED, synth.TID_V_NEW, "cuda")
    pos = torch.full((w.batch,), w.seq, dtype=torch.int32, device="cuda")
    kvbfp.quantize_append(cache, k1, v1, pos_dev=pos, perm_k=pkd, perm_v=pvd)             # one decode-step append
    scale = float(np.float32(w.head_dim ** -0.5))
    qbits = Q_MANT_BITS.get(name, 0)
    if qbits:
        out = kvbfp.decode_attention_qbfp(cache, d["q"], w.seq + 1, scale, qbits, perm_k=pkd, perm_v=pvd)
    else:
        out = kvbfp.decode_attention(cache, d["q"], w.seq + 1, scale, perm_k=pkd, perm_v=pvd)
    torch.cuda.synchronize()
    G = w.group
    worst = 0.0
    for (b, h) in SAMPLES[name]:
        kk = torch.cat([d["k"][b:b + 1, :, h:h + 1], k1[b:b + 1, :, h:h + 1]], dim=1).cpu()
        vv = torch.cat([d["v"][b:b + 1, :, h:h + 1], v1[b:b + 1, :, h:h + 1]], dim=1).cpu()
        km, ke = O.quantize_append(synth.to_f32_numpy(kk), w.block, w.mant_bits, S_max, 0, perm=pk[h:h + 1])
        vm, ve = O.quantize_append(synth.to_f32_numpy(vv), w.block, w.mant_bits, S_max, 0, perm=pv[h:h + 1])
        for got, ref, nm in ((cache.k_mant, km, "k_mant"), (cache.k_exp, ke, "k_exp"),
                             (cache.v_mant, vm, "v_mant"), (cache.v_exp, ve, "v_exp")):
            assert np.array_equal(got[b, h].cpu().numpy(), ref[0, 0]), (name, b, h, nm)
        qq = synth.to_f32_numpy(d["q"][b:b + 1, h * G:(h + 1) * G])
        want = O.decode_attention(km, ke, vm, ve, w.head_dim, w.block, w.mant_bits, qq, [w.seq + 1], scale,
                                  pk[h:h + 1], pv[h:h + 1], q_mant_bits=qbits)
        per_head, _ = assert_attention_close(out[b:b + 1, h * G:(h + 1) * G], want, tdt, "%s unit (%d,%d)" % (name, b, h))
        worst = max(worst, per_head)
    print("%s: worst rel-L2 over sampled units %.3e" % (name, worst))


def test_bulk_prefill_bytes_sampled():
    # 32 layers x 8 KV heads x 4096 tokens quantized in one call (the layer index plays the batch role)
    w = synth.WORKLOADS["prefill_bulk"]
    d = synth.make_workload_inputs(w, device="cuda", with_calibration=False)
    L = kvbfp.make_layout(w.head_dim, w.block, w.mant_bits, w.n_kv_heads, w.batch, w.seq)
    cache = kvbfp.alloc_cache(L, "cuda", fill=0)
    kvbfp.quantize_append(cache, d["k"], d["v"], pos0=0)
    torch.cuda.synchronize()
    for (b, h) in [(0, 0), (17, 4), (31, 7)]:
        for src, mant, exp in ((d["k"], cache.k_mant, cache.k_exp), (d["v"], cache.v_mant, cache.v_exp)):
            x = synth.to_f32_numpy(src[b:b + 1, :, h:h + 1])
            m, e = O.quantize_append(x, w.block, w.mant_bits, w.seq, 0)
            assert np.array_equal(mant[b, h].cpu().numpy(), m[0, 0])
            assert np.array_equal(exp[b, h].cpu().numpy(), e[0, 0])


def test_full_size_paged_and_rotation_at_read():
    """The headline workload once more (a) as a pool of 256-token pages scattered by a seeded shuffle:
    attention must return the contiguous call's bits, and sampled pages must hold the contiguous cache's
    bytes; (b) read with rotation at read (keys taken as cached before the rotary embedding): sampled units
    against the oracle."""
    name = "llama3_8b_gqa_32k"
    w = synth.WORKLOADS[name]
    tdt = synth.TORCH_DTYPES[w.dtype]
    d = synth.make_workload_inputs(w, device="cuda")
    pk = kvbfp.calibrate_perm(d["k_calib"].cpu())
    pv = kvbfp.calibrate_perm(d["v_calib"].cpu())
    pkd, pvd = dev_i32(pk), dev_i32(pv)
    S = w.seq
    L = kvbfp.make_layout(w.head_dim, w.block, w.mant_bits, w.n_kv_heads, w.batch, S)
    cache = kvbfp.alloc_cache(L, "cuda", fill=0)
    kvbfp.quantize_append(cache, d["k"], d["v"], pos0=0, perm_k=pkd, perm_v=pvd)
    scale = float(np.float32(w.head_dim ** -0.5))
    flat = kvbfp.decode_attention(cache, d["q"], S, scale, perm_k=pkd, perm_v=pvd)
    # (a) pages
    page = 256
    per_seq = S // page
    rng = np.random.default_rng(synth.BASE_SEED)
    table = rng.permutation(w.batch * per_seq).reshape(w.batch, per_seq).astype(np.int32)
    pool = kvbfp.alloc_cache(kvbfp.make_layout(w.head_dim, w.block, w.mant_bits, w.n_kv_heads, w.batch * per_seq, page),
                             "cuda", fill=0)
    kvbfp.quantize_append_paged(pool, dev_i32(table), d["k"], d["v"], pos0=0, perm_k=pkd, perm_v=pvd)
    paged = kvbfp.decode_attention_paged(pool, dev_i32(table), d["q"], S, scale, perm_k=pkd, perm_v=pvd)
    torch.cuda.synchronize()
    assert torch.equal(flat, paged)
    for (b, i) in [(0, 0), (3, 77), (7, per_seq - 1)]:
        for src, dst in zip(cache.planes(), pool.planes()):
            assert torch.equal(src[b, :, i * page:(i + 1) * page], dst[int(table[b, i])]), (b, i)
    # (b) rotation at read
    theta = (10000.0 ** (-np.arange(w.head_dim // 2, dtype=np.float64) / (w.head_dim // 2))).astype(np.float32)
    th, pa, sg = kvbfp.permute_rope(theta, pk, kvbfp.ROPE_PAIRS_HALF_SPLIT)
    out = kvbfp.decode_attention_rope(cache, d["q"], S, scale, torch.from_numpy(th).cuda(), torch.from_numpy(pa).cuda(),
                                      torch.from_numpy(sg).cuda(), perm_k=pkd, perm_v=pvd)
    torch.cuda.synchronize()
    G = w.group
    tho, pao, sgo = O.permute_rope(theta, pk, 1)
    for (b, h) in [(0, 0), (6, 5)]:
        planes = [t[b:b + 1, h:h + 1].cpu().numpy() for t in cache.planes()]
        qq = synth.to_f32_numpy(d["q"][b:b + 1, h * G:(h + 1) * G])
        want = O.decode_attention_rope(*planes, w.head_dim, w.block, w.mant_bits, qq, [S], scale, tho[h:h + 1],
                                       pao[h:h + 1], sgo[h:h + 1], perm_k=pk[h:h + 1], perm_v=pv[h:h + 1])
        assert_attention_close(out[b:b + 1, h * G:(h + 1) * G], want, tdt, "rotation at read, unit (%d,%d)" % (b, h))
