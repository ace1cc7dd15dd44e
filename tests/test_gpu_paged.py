"""Paged caches: the same bytes and the same attention as the contiguous cache, with every sequence's
tokens scattered over a pool of pages through a block table.  Paging is addressing only, so the
oracle is the contiguous one: pages are gathered back through the table before the comparison."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth
from test_gpu_attention import make_small
from util import assert_attention_close, dev_i32, oracle_cache

pytestmark = pytest.mark.gpu

D = 128
SENTINEL = 0xA5


def make_pool(B, Hkv, n, p, page, pages_per_seq, lens, seed, spare=3):
    """A pool with a few spare pages and a block table that scatters the pages each sequence needs;
    entries a sequence never reaches hold an invalid page number."""
    rng = np.random.default_rng(seed)
    need = [(l + page - 1) // page for l in lens]
    n_pages = sum(need) + spare
    order = rng.permutation(n_pages)
    table = np.full((B, pages_per_seq), -7, dtype=np.int32)
    at = 0
    for b in range(B):
        table[b, :need[b]] = order[at:at + need[b]]
        at += need[b]
    L = kvbfp.make_layout(D, n, p, Hkv, n_pages, page)
    pool = kvbfp.alloc_cache(L, "cuda", fill=SENTINEL)
    return pool, table, need


def gather_pages(pool, table, need, B, S_max, page):
    """The pool's rows in sequence order, [B][Hkv][S_max][..] per plane (numpy); rows of pages a sequence
    does not own are filled with the sentinel."""
    out = []
    for t in pool.planes():
        src = t.cpu().numpy()
        dst = np.full((B,) + src.shape[1:2] + (S_max,) + src.shape[3:], SENTINEL, dtype=np.uint8)
        for b in range(B):
            for i in range(need[b]):
                hi = min((i + 1) * page, S_max)
                dst[b, :, i * page:hi] = src[table[b, i], :, :hi - i * page]
        out.append(dst)
    return out


def fill_both(k, v, n, p, page, pages_per_seq, lens, pk, pv, seed, chunks=(None,)):
    """k, v: CPU [B][S][Hkv][D].  Writes lens[b] tokens of every sequence into a paged pool (GPU) and into
    contiguous planes (oracle); returns (pool, table_dev, planes)."""
    B, S, Hkv, _ = k.shape
    pool, table, need = make_pool(B, Hkv, n, p, page, pages_per_seq, lens, seed)
    table_dev = dev_i32(table)
    S_max = pages_per_seq * page
    # oracle: every sequence holds its first lens[b] tokens, the rest keeps the sentinel
    planes = None
    for b in range(B):
        one = oracle_cache(k[b:b + 1, :lens[b]], v[b:b + 1, :lens[b]], n, p, S_max, 0,
                           None if pk is None else pk, None if pv is None else pv, fill=SENTINEL)
        planes = [x.copy() for x in one] if planes is None else [np.concatenate([a, c]) for a, c in zip(planes, one)]
    # GPU: the longest prefix all sequences share in bulk, then token by token with per-sequence positions
    common = min(lens)
    kd, vd = k.cuda(), v.cuda()
    kvbfp.quantize_append_paged(pool, table_dev, kd[:, :common], vd[:, :common], pos0=0, perm_k=dev_i32(pk),
                                perm_v=dev_i32(pv))
    for b in range(B):
        if lens[b] > common:      # the tail of sequence b alone: a table of one row
            kvbfp.quantize_append_paged(pool, table_dev[b:b + 1].contiguous(), kd[b:b + 1, common:lens[b]],
                                        vd[b:b + 1, common:lens[b]], pos_dev=dev_i32([common]),
                                        perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    got = gather_pages(pool, table, need, B, S_max, page)
    for name, g, w in zip(("k_mant", "k_exp", "v_mant", "v_exp"), got, planes):
        for b in range(B):
            assert np.array_equal(g[b, :, :lens[b]], w[b, :, :lens[b]]), (name, b)
            own = need[b] * page
            assert np.all(g[b, :, lens[b]:own] == SENTINEL), (name, b, "rows after the last token were written")
    return pool, table_dev, planes


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
@pytest.mark.parametrize("p,n", [(4, 16), (4, 32), (4, 64), (8, 16), (8, 128)])
@pytest.mark.parametrize("G,page", [(1, 256), (4, 256), (8, 512), (4, 64), (2, 128), (4, 16), (8, 32), (1, 16)])
def test_paged_cache_matches_oracle(dtype, p, n, G, page):
    # 1300 and 700 tokens: six and three 256-token pages (or three and two of 512), last page ragged
    lens = [1300, 700]
    k, v, q, pk, pv = make_small(dtype, B=2, S=1300, Hkv=2, G=G, seed=160 + G)
    pool, table, planes = fill_both(k, v, n, p, page, -(-1300 // page) + 2, lens, pk, pv, seed=G + page)
    want = O.decode_attention(*planes, D, n, p, synth.to_f32_numpy(q), lens, float(np.float32(128 ** -0.5)), pk, pv)
    got = kvbfp.decode_attention_paged(pool, table, q.cuda(), 1300, float(np.float32(128 ** -0.5)),
                                       seq_len_dev=dev_i32(lens), perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    assert_attention_close(got, want, dtype, "p=%d n=%d G=%d page=%d" % (p, n, G, page))


def test_paged_equals_contiguous_bit_for_bit_and_wide_groups():
    # same kernels, same order of operations: the paged result is the contiguous one exactly; G = 40 takes
    # the general pass, G = 12 two launches of the matrix-core pass
    for G, page in ((12, 256), (40, 256), (40, 64), (12, 16), (40, 32)):
        lens = [900, 900]
        k, v, q, pk, pv = make_small(torch.bfloat16, B=2, S=900, Hkv=1, G=G, seed=170 + G)
        pool, table, planes = fill_both(k, v, 32, 4, page, 1024 // page, lens, pk, pv, seed=G)
        L = kvbfp.make_layout(D, 32, 4, 1, 2, 1024)
        flat = kvbfp.alloc_cache(L, "cuda", fill=0)
        kvbfp.quantize_append(flat, k.cuda(), v.cuda(), perm_k=dev_i32(pk), perm_v=dev_i32(pv))
        a = kvbfp.decode_attention(flat, q.cuda(), 900, 0.1, perm_k=dev_i32(pk), perm_v=dev_i32(pv))
        b = kvbfp.decode_attention_paged(pool, table, q.cuda(), 900, 0.1, perm_k=dev_i32(pk), perm_v=dev_i32(pv))
        torch.cuda.synchronize()
        assert torch.equal(a, b)
        want = O.decode_attention(*planes, D, 32, 4, synth.to_f32_numpy(q), lens, float(np.float32(0.1)), pk, pv)
        assert_attention_close(b, want, torch.bfloat16)


def test_query_cast_and_profile_variant_on_pages():
    lens = [600, 300, 10]
    k, v, q, pk, pv = make_small(torch.bfloat16, B=3, S=600, Hkv=2, G=4, seed=180)
    pool, table, planes = fill_both(k, v, 16, 4, 256, 3, lens, pk, pv, seed=9)
    want = O.decode_attention(*planes, D, 16, 4, synth.to_f32_numpy(q), lens, float(np.float32(0.09)), pk, pv,
                              q_mant_bits=8)
    got, split_ms, combine_ms = kvbfp.decode_attention_paged(pool, table, q.cuda(), 600, float(np.float32(0.09)),
                                                            q_mant_bits=8, seq_len_dev=dev_i32(lens),
                                                            perm_k=dev_i32(pk), perm_v=dev_i32(pv), profile=True)
    assert_attention_close(got, want, torch.bfloat16)
    assert split_ms > 0 and combine_ms > 0


@pytest.mark.parametrize("page", [128, 16])
def test_integer_score_product_on_pages(page):
    # 8-bit keys in blocks of 32, query cast to 8-bit BFP: the int8 matrix product of the LDS pipeline over a pool
    lens = [700, 300]
    k, v, q, pk, pv = make_small(torch.bfloat16, B=2, S=700, Hkv=2, G=6, seed=185)
    pool, table, planes = fill_both(k, v, 32, 8, page, 768 // page, lens, pk, pv, seed=11)
    want = O.decode_attention(*planes, D, 32, 8, synth.to_f32_numpy(q), lens, float(np.float32(0.09)), pk, pv,
                              q_mant_bits=8)
    got = kvbfp.decode_attention_paged(pool, table, q.cuda(), 700, float(np.float32(0.09)), q_mant_bits=8,
                                       seq_len_dev=dev_i32(lens), perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    assert_attention_close(got, want, torch.bfloat16)


def test_dequantize_from_pages_equals_the_oracle():
    lens = [500, 321]
    k, v, q, pk, pv = make_small(torch.bfloat16, B=2, S=500, Hkv=2, G=1, seed=190)
    pool, table, planes = fill_both(k, v, 32, 8, 128, 4, lens, pk, pv, seed=3)
    for which, (m, e), perm in ((0, planes[0:2], pk), (1, planes[2:4], pv)):
        want = O.dequantize(m, e, D, 32, 8, 100, 221, perm=perm)           # tokens 100..320 exist in both sequences
        got = kvbfp.dequantize_paged(pool, table, which, 100, 221, dtype=torch.float32, perm=dev_i32(perm))
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy().astype(np.float64), want)


def test_paged_argument_errors():
    L = kvbfp.make_layout(D, 32, 4, 2, 4, 384)          # 384 tokens per page: not a power of two
    pool = kvbfp.alloc_cache(L, "cuda", fill=0)
    table = dev_i32(np.zeros((1, 2)))
    q = torch.zeros(1, 2, D, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(kvbfp.KvbfpError) as ei:
        kvbfp.decode_attention_paged(pool, table, q, 100, 0.1)
    assert "page" in str(ei.value)
    L = kvbfp.make_layout(D, 32, 4, 2, 4, 256)
    pool = kvbfp.alloc_cache(L, "cuda", fill=0)
    with pytest.raises(kvbfp.KvbfpError):               # 2 pages of 256 hold 512 tokens
        kvbfp.decode_attention_paged(pool, table, q, 513, 0.1)
    x = torch.zeros(1, 2, 2, D, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(kvbfp.KvbfpError):
        kvbfp.quantize_append_paged(pool, table, x, x, pos0=511)


@pytest.mark.parametrize("dtype,p,n,G,page,Hkv", [
    (torch.bfloat16, 4, 32, 4, 256, 64),    # 64 kv-heads: several splits, the cast runs inside the split pass
    (torch.bfloat16, 4, 16, 2, 64, 64),
    (torch.float16, 4, 64, 1, 128, 64),
    (torch.bfloat16, 4, 128, 8, 512, 2),
    (torch.bfloat16, 8, 16, 2, 256, 2),     # 8-bit mantissas and fp32 I/O: the cache-write kernel goes first
    (torch.float32, 4, 32, 2, 128, 2),
    (torch.bfloat16, 4, 32, 4, 16, 64),     # pages of 16 and 32 tokens: a page per stage of a tile
    (torch.bfloat16, 8, 32, 2, 32, 2),
    (torch.float32, 4, 16, 1, 16, 2),
])
def test_current_token_appended_and_attended_on_pages(dtype, p, n, G, page, Hkv):
    # the current tokens: the first row of a fresh page (1025 = 4 x 256 + 1 = 16 x 64 + 1), mid-page, the very
    # first token of a sequence, and an empty sequence that must stay untouched
    lens = [1025, 700, 1, 0]
    B, S = 4, 1025
    k, v, q, pk, pv = make_small(dtype, B=B, S=S, Hkv=Hkv, G=G, seed=210 + n + G)
    pages_per_seq = -(-S // page) + 1
    before = [max(l - 1, 0) for l in lens]
    # before the call: every sequence holds all but its current token (an empty one gets a page anyway)
    pool, table, need = make_pool(B, Hkv, n, p, page, pages_per_seq, [max(l, 1) for l in lens], seed=n + page)
    table_dev = dev_i32(table)
    kd, vd = k.cuda(), v.cuda()
    for b in range(B):
        if before[b]:
            kvbfp.quantize_append_paged(pool, table_dev[b:b + 1].contiguous(), kd[b:b + 1, :before[b]],
                                        vd[b:b + 1, :before[b]], pos0=0, perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    idx = torch.tensor([max(l - 1, 0) for l in lens])
    k_new = torch.stack([k[b, idx[b]] for b in range(B)]).cuda()           # [B][Hkv][D]
    v_new = torch.stack([v[b, idx[b]] for b in range(B)]).cuda()
    scale = float(np.float32(0.09))
    got = kvbfp.append_decode_attention_paged(pool, table_dev, k_new, v_new, q.cuda(), S, scale,
                                              seq_len_dev=dev_i32(lens), perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    S_max = pages_per_seq * page
    planes = None
    for b in range(B):
        take = max(lens[b], 1)           # an empty sequence: cast one token, then wipe it again
        one = oracle_cache(k[b:b + 1, :take], v[b:b + 1, :take], n, p, S_max, 0, pk, pv, fill=SENTINEL)
        if lens[b] == 0:
            for x in one:
                x[:] = SENTINEL
        planes = [x.copy() for x in one] if planes is None else [np.concatenate([a, c]) for a, c in zip(planes, one)]
    have = gather_pages(pool, table, need, B, S_max, page)
    for name, g, w in zip(("k_mant", "k_exp", "v_mant", "v_exp"), have, planes):
        for b in range(B):
            assert np.array_equal(g[b, :, :lens[b]], w[b, :, :lens[b]]), (name, b)
            assert np.all(g[b, :, lens[b]:need[b] * page] == SENTINEL), (name, b, "rows after the current token")
    units = None if Hkv <= 2 else [(0, 0), (0, Hkv - 1), (1, 17), (2, 40), (3, 5)]
    if units is None:
        want = O.decode_attention(*planes, D, n, p, synth.to_f32_numpy(q), lens, scale, pk, pv)
        assert_attention_close(got, want, dtype, "p=%d n=%d G=%d page=%d" % (p, n, G, page))
    else:           # the oracle on a few (sequence, kv-head) units
        qf = synth.to_f32_numpy(q).reshape(B, Hkv, G, D)
        for b, h in units:
            sub = [x[b:b + 1, h:h + 1] for x in planes]
            want = O.decode_attention(*sub, D, n, p, qf[b:b + 1, h], [lens[b]], scale,
                                      None if pk is None else pk[h:h + 1], None if pv is None else pv[h:h + 1])
            assert_attention_close(got.reshape(B, Hkv, G, D)[b:b + 1, h], want, dtype, "unit %s" % ((b, h),))
    assert bool((got[3] == 0).all())


@pytest.mark.parametrize("dtype,p,n,G,Tq,page", [
    (torch.bfloat16, 4, 32, 2, 4, 256),
    (torch.float16, 4, 16, 1, 8, 64),
    (torch.bfloat16, 8, 32, 3, 7, 128),     # 21 virtual heads: three launches over head subsets
    (torch.bfloat16, 4, 64, 4, 9, 256),     # 36 virtual heads: general pass
    (torch.bfloat16, 4, 32, 4, 4, 16),
    (torch.bfloat16, 8, 16, 2, 3, 32),
    (torch.float16, 4, 128, 5, 8, 16),      # 40 virtual heads: general pass over pages of 16
])
def test_several_query_tokens_on_pages(dtype, p, n, G, Tq, page):
    lens = [830, max(Tq - 2, 1), 257 + Tq // 2]
    k, v, q0, pk, pv = make_small(dtype, B=3, S=830, Hkv=2, G=G, seed=230 + Tq)
    pool, table, planes = fill_both(k, v, n, p, page, -(-830 // page) + 1, lens, pk, pv, seed=Tq + page)
    name = {torch.bfloat16: "bf16", torch.float16: "f16", torch.float32: "f32"}[dtype]
    q = torch.stack([synth.queries(3, 2 * G, D, name, 231 + 10 * i, 4) for i in range(Tq)], dim=1)
    scale = float(np.float32(0.09))
    got = kvbfp.decode_attention_multi_paged(pool, table, q.cuda(), 830, scale, seq_len_dev=dev_i32(lens),
                                             perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    assert got.shape == q.shape
    for i in range(Tq):
        seen = [max(l - (Tq - 1 - i), 0) for l in lens]
        want = O.decode_attention(*planes, D, n, p, synth.to_f32_numpy(q[:, i]), seen, scale, pk, pv)
        assert_attention_close(got[:, i], want, dtype, "query token %d of %d sees %s" % (i, Tq, seen))


@pytest.mark.parametrize("page", [16, 256])
def test_many_tiles_per_wavefront_on_pages(page):
    # 768 (sequence, kv-head) units leave one split per unit, so every wavefront walks 67 tiles: more than the 64 whose
    # page numbers it fetches at kernel start -- the last ones are looked up when they are due.  Sampled units
    # against the oracle (bytes through the table bit for bit, attention within the bar).
    B, Hkv, G, S, n, p = 96, 8, 2, 66 * 256 + 37, 32, 4
    gains = synth.outlier_gains(77, 0, Hkv, D)
    k = synth.kv_rows(B, S, Hkv, D, "bf16", gains, 77, 2, "cuda")
    v = synth.kv_rows(B, S, Hkv, D, "bf16", gains, 77, 3, "cuda")
    q = synth.queries(B, Hkv * G, D, "bf16", 77, 4, "cuda")
    rng = np.random.default_rng(page)
    pk = np.stack([rng.permutation(D) for _ in range(Hkv)]).astype(np.int32)
    pv = np.stack([rng.permutation(D) for _ in range(Hkv)]).astype(np.int32)
    per_seq = -(-S // page)
    table = rng.permutation(B * per_seq).reshape(B, per_seq).astype(np.int32)
    table_dev = dev_i32(table)
    L = kvbfp.make_layout(D, n, p, Hkv, B * per_seq, page)
    pool = kvbfp.alloc_cache(L, "cuda", fill=SENTINEL)
    kvbfp.quantize_append_paged(pool, table_dev, k, v, pos0=0, perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    scale = float(np.float32(128 ** -0.5))
    got = kvbfp.decode_attention_paged(pool, table_dev, q, S, scale, perm_k=dev_i32(pk), perm_v=dev_i32(pv))
    torch.cuda.synchronize()
    for (b, h) in [(0, 0), (41, 5), (95, 7)]:
        km, ke = O.quantize_append(synth.to_f32_numpy(k[b:b + 1, :, h:h + 1].cpu()), n, p, per_seq * page, 0, perm=pk[h:h + 1])
        vm, ve = O.quantize_append(synth.to_f32_numpy(v[b:b + 1, :, h:h + 1].cpu()), n, p, per_seq * page, 0, perm=pv[h:h + 1])
        pages = torch.as_tensor(table[b], device="cuda", dtype=torch.long)
        for plane, ref, nm in ((pool.k_mant, km, "k_mant"), (pool.k_exp, ke, "k_exp"), (pool.v_mant, vm, "v_mant"),
                               (pool.v_exp, ve, "v_exp")):
            rows = plane[pages, h].reshape(per_seq * page, -1)[:S].cpu().numpy()
            assert np.array_equal(rows, ref[0, 0, :S]), (nm, b, h)
        want = O.decode_attention(km, ke, vm, ve, D, n, p, synth.to_f32_numpy(q[b:b + 1, h * G:(h + 1) * G].cpu()), [S], scale,
                                  pk[h:h + 1], pv[h:h + 1])
        assert_attention_close(got[b:b + 1, h * G:(h + 1) * G], want, torch.bfloat16, "page %d unit (%d,%d)" % (page, b, h))
