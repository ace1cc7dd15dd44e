"""GPU parity of the cache write / read-back kernels against the oracle: packed bytes bit-exact.
Everything goes through the C ABI (paper_2403_20137_amd.kvbfp -> libkvbfp.so)."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth
from util import DT_NAME, assert_planes_equal, dev_i32, gpu_cache, oracle_cache

pytestmark = pytest.mark.gpu


def plant_special_values(x, p):
    """Overwrite a few rows of x ([B][T][H][D], any float dtype, CPU) with the cases a cast can get
    wrong: zeros and negative zeros, subnormals, exact rounding ties, the exponent-bump boundary,
    the largest finite value, an all-zero row."""
    qmax = 2 ** (p - 1) - 1
    fi = torch.finfo(x.dtype)
    B, T, H, D = x.shape
    x[0, 0, 0, :] = 0
    x[0, 0, 0, 5] = -0.0
    x[0, 1, 0, :16] = torch.tensor([0.0, -0.0, fi.tiny, -fi.tiny, fi.tiny / 2, fi.tiny / 4, 0, 0,
                                    fi.smallest_normal * 3, 0, 0, 0, 0, 0, 0, 0], dtype=x.dtype)
    x[0, 1, 0, 16:32] = 0                                       # whole block zero
    x[0, 2, 0, :] = fi.smallest_normal / 8                      # whole row subnormal
    x[0, 2, 0, 3] = -fi.smallest_normal / 2
    ties = torch.arange(0, 2 * qmax + 2, dtype=torch.float32) * 0.5
    x[0, 3, 0, :len(ties[:D])] = ties[:D].to(x.dtype)           # k + 1/2 ties at scale 1
    x[0, 4, 0, :] = 1.0
    x[0, 4, 0, 0] = (qmax + 0.5) * 4                            # exactly on the bump boundary
    x[0, 4, 0, 40] = -(qmax + 0.5) * 4
    x[0, 5, 0, :] = 0.25
    x[0, 5, 0, 17] = fi.max
    x[0, 5, 0, 99] = -fi.max
    x[0, 6, 0, :] = float(torch.nextafter(torch.tensor((qmax + 0.5) * 2, dtype=x.dtype), torch.tensor(0, dtype=x.dtype)))
    x[0, 7, 0, :] = -1e-3
    x[0, 7, 0, 64:] = 3e4
    return x


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
@pytest.mark.parametrize("p", [4, 8])
@pytest.mark.parametrize("n", [16, 32, 64, 128])
@pytest.mark.parametrize("with_perm", [False, True])
def test_quantize_append_bytes_bit_exact(dtype, p, n, with_perm):
    B, T, H, D, S_max, pos0 = 2, 37, 3, 128, 50, 5          # 222 rows: 13 full groups of 16 + a ragged one
    kg = synth.outlier_gains(3, 0, H, D)
    vg = synth.outlier_gains(3, 1, H, D)
    k = synth.kv_rows(B, T, H, D, DT_NAME[dtype], kg, 3, 10)
    v = synth.kv_rows(B, T, H, D, DT_NAME[dtype], vg, 3, 11)
    # spread magnitudes over many binades, per row
    lo, hi = (-10, 5) if dtype == torch.float16 else (-20, 12)          # stay finite in fp16
    sc = (2.0 ** torch.randint(lo, hi, (B, T, H, 1), generator=torch.Generator().manual_seed(1))).to(dtype)
    k, v = plant_special_values(k * sc, p), plant_special_values(v * sc.flip(1), p)
    assert bool(torch.isfinite(k).all()) and bool(torch.isfinite(v).all())
    pk = pv = None
    if with_perm:
        rng = np.random.default_rng(5)
        pk = np.stack([rng.permutation(D) for _ in range(H)]).astype(np.int32)
        pv = np.stack([rng.permutation(D) for _ in range(H)]).astype(np.int32)
    want = oracle_cache(k, v, n, p, S_max, pos0, pk, pv, fill=0xA5)
    cache = gpu_cache(k.cuda(), v.cuda(), n, p, S_max, pos0=pos0, perm_k=pk, perm_v=pv, fill=0xA5)
    assert_planes_equal(cache, want, "dtype=%s p=%d n=%d perm=%s" % (dtype, p, n, with_perm))


def test_per_sequence_positions_strided_and_unaligned_inputs():
    B, T, H, D, S_max, n, p = 3, 4, 2, 128, 40, 32, 4
    kbig = synth.gaussian((B, T, H, 2 * D + 8), 7, 0).to(torch.bfloat16).cuda()
    vbig = synth.gaussian((B, T, H, 2 * D + 8), 7, 1).to(torch.bfloat16).cuda()
    pos = np.array([0, 36, 17], dtype=np.int32)
    for lo in (0, D, 3):                       # aligned, aligned at an offset, unaligned start
        kview, vview = kbig[..., lo:lo + D], vbig[..., lo:lo + D]
        assert kview.stride(3) == 1 and kview.stride(2) == 2 * D + 8
        want = oracle_cache(kview.cpu(), vview.cpu(), n, p, S_max, pos, fill=0x11)
        L = kvbfp.make_layout(D, n, p, H, B, S_max)
        cache = kvbfp.alloc_cache(L, "cuda", fill=0x11)
        kvbfp.quantize_append(cache, kview, vview, pos_dev=dev_i32(pos))
        torch.cuda.synchronize()
        assert_planes_equal(cache, want, "strided view starting at channel %d" % lo)


def test_rows_outside_the_cache_are_dropped_and_single_tensor_calls():
    B, T, H, D, S_max, n, p = 2, 6, 2, 128, 8, 16, 4
    k = synth.gaussian((B, T, H, D), 8, 0).to(torch.float16)
    v = synth.gaussian((B, T, H, D), 8, 1).to(torch.float16)
    pos = np.array([5, -2], dtype=np.int32)        # sequence 0 overflows by 3 rows, sequence 1 starts before 0
    L = kvbfp.make_layout(D, n, p, H, B, S_max)
    cache = kvbfp.alloc_cache(L, "cuda", fill=0x77)
    kvbfp.quantize_append(cache, k.cuda(), v.cuda(), pos_dev=dev_i32(pos))
    torch.cuda.synchronize()
    want = [np.full(t.shape, 0x77, np.uint8) for t in cache.planes()]
    kf, vf = synth.to_f32_numpy(k), synth.to_f32_numpy(v)
    for b in range(B):
        for t in range(T):
            ps = int(pos[b]) + t
            if 0 <= ps < S_max:
                for x, mi in ((kf, 0), (vf, 2)):
                    m, e = O.quantize_append(x[b:b + 1, t:t + 1], n, p, 1, 0)
                    want[mi][b, :, ps] = m[0, :, 0]
                    want[mi + 1][b, :, ps] = e[0, :, 0]
    assert_planes_equal(cache, want, "dropped rows")
    # keys only / values only leave the other planes untouched
    cache2 = kvbfp.alloc_cache(L, "cuda", fill=0x33)
    kvbfp.quantize_append(cache2, k.cuda(), None, pos0=0)
    torch.cuda.synchronize()
    assert bool((cache2.v_mant == 0x33).all()) and bool((cache2.v_exp == 0x33).all())
    km, ke = O.quantize_append(kf, n, p, S_max, 0, mant=np.full(want[0].shape, 0x33, np.uint8),
                               exp=np.full(want[1].shape, 0x33, np.uint8))
    assert np.array_equal(cache2.k_mant.cpu().numpy(), km) and np.array_equal(cache2.k_exp.cpu().numpy(), ke)
    kvbfp.quantize_append(cache2, None, v.cuda(), pos0=2)
    torch.cuda.synchronize()
    vm, ve = O.quantize_append(vf, n, p, S_max, 2, mant=np.full(want[0].shape, 0x33, np.uint8),
                               exp=np.full(want[1].shape, 0x33, np.uint8))
    assert np.array_equal(cache2.v_mant.cpu().numpy(), vm) and np.array_equal(cache2.v_exp.cpu().numpy(), ve)
    assert np.array_equal(cache2.k_mant.cpu().numpy(), km)


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
@pytest.mark.parametrize("p,n", [(4, 16), (4, 32), (8, 16), (4, 128), (8, 64)])
@pytest.mark.parametrize("with_perm", [False, True])
def test_dequantize_matches_oracle(dtype, p, n, with_perm):
    B, T, H, D = 2, 21, 3, 128
    rng = np.random.default_rng(9)
    # arbitrary bytes: every code and a wide range of exponents, including E = 0 and 255
    ms, es = O.plane_shapes(B, H, D, n, p, T + 3)
    mant = rng.integers(0, 256, size=ms, dtype=np.uint8)
    exp = rng.integers(90, 160, size=es).astype(np.uint8)
    exp[0, 0, 0, :], exp[0, 0, 1, :], exp[0, 0, 2, :], exp[0, 0, 3, :] = 0, 1, 255, 254
    exp[1, 1, 2] = 255
    exp[1, 2, 3] = 1
    perm = np.stack([rng.permutation(D) for _ in range(H)]).astype(np.int32) if with_perm else None
    L = kvbfp.make_layout(D, n, p, H, B, T + 3)
    planes = [torch.from_numpy(a).cuda() for a in (mant, exp)]
    for which in (0, 1):
        cache = kvbfp.Cache(L, planes[0], planes[1], None, None) if which == 0 else \
            kvbfp.Cache(L, None, None, planes[0], planes[1])
        got = kvbfp.dequantize(cache, which, 2, T, dtype=dtype, perm=dev_i32(perm))
        torch.cuda.synchronize()
        want = torch.from_numpy(O.dequantize(mant, exp, D, n, p, 2, T, perm=perm)).to(dtype)
        g = got.cpu()
        if dtype == torch.float32:
            assert torch.equal(g.view(torch.int32), want.view(torch.int32))
        else:
            assert torch.equal(g.view(torch.int16), want.view(torch.int16))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_dequantize_many_rows_ragged_tail_and_unaligned_permutation(dtype):
    # 3 x 5 x 211 rows: many 64-row workgroups and a ragged last one; the permutation once 16-byte aligned and
    # once at an address that is only 4-byte aligned (its entries are then loaded one by one): same bits
    B, T, H, D, n, p = 3, 211, 5, 128, 32, 4
    rng = np.random.default_rng(19)
    ms, es = O.plane_shapes(B, H, D, n, p, T + 5)
    mant = rng.integers(0, 256, size=ms, dtype=np.uint8)
    exp = rng.integers(100, 150, size=es).astype(np.uint8)
    perm = np.stack([rng.permutation(D) for _ in range(H)]).astype(np.int32)
    L = kvbfp.make_layout(D, n, p, H, B, T + 5)
    cache = kvbfp.Cache(L, torch.from_numpy(mant).cuda(), torch.from_numpy(exp).cuda(), None, None)
    want = torch.from_numpy(O.dequantize(mant, exp, D, n, p, 3, T, perm=perm)).to(dtype)
    aligned = dev_i32(perm)
    holder = torch.zeros(H * D + 1, dtype=torch.int32, device="cuda")
    holder[1:] = aligned.reshape(-1)
    shifted = holder[1:].view(H, D)
    assert aligned.data_ptr() % 16 == 0 and shifted.data_ptr() % 16 == 4
    for pr in (aligned, shifted):
        got = kvbfp.dequantize(cache, 0, 3, T, dtype=dtype, perm=pr)
        torch.cuda.synchronize()
        assert torch.equal(got.cpu().view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                           want.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))


def test_round_trip_through_both_kernels():
    # cast then decode on the GPU: within half a mantissa step of the input (Sec. II-B)
    w = synth.WORKLOADS["llama2_7b_4k"]
    d = synth.make_workload_inputs(w, seq=300, device="cuda", with_calibration=False)
    cache = gpu_cache(d["k"], d["v"], w.block, w.mant_bits, 300)
    back = kvbfp.dequantize(cache, 0, 0, 300, dtype=torch.float32)
    e = cache.k_exp.to(torch.int32).permute(0, 2, 1, 3)                     # [B][S][H][NB]
    step = torch.ldexp(torch.ones((), device="cuda"), e - 127 - (w.mant_bits - 2))
    step = step.repeat_interleave(w.block, dim=-1)
    assert bool(((back - d["k"].float()).abs() <= 0.5 * step).all())
