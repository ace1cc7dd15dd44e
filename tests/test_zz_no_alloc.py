"""kvbfp_decode_attention_noalloc (split partials in the library's fixed device array, no workspace argument,
no allocation) returns what kvbfp_decode_attention_qbfp returns with a caller's workspace: same launches,
so the outputs are compared bit for bit; the oracle bar is checked on top.  Two calls in a row, the second
on a smaller input, share the array."""
import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth
from util import assert_attention_close, dev_i32, gpu_cache, oracle_cache

pytestmark = pytest.mark.gpu
D = 128
DT = {torch.float32: "f32", torch.float16: "f16", torch.bfloat16: "bf16"}


def _inputs(dtype, B, S, Hkv, G, seed):
    gains = synth.outlier_gains(seed, 0, Hkv, D)
    k = synth.kv_rows(B, S, Hkv, D, DT[dtype], gains, seed, 2, "cuda")
    v = synth.kv_rows(B, S, Hkv, D, DT[dtype], gains, seed, 3, "cuda")
    q = synth.queries(B, Hkv * G, D, DT[dtype], seed, 4, "cuda")
    return k, v, q


def _both(dtype, n, p, B, S, Hkv, G, lens, seed, qbits=0):
    k, v, q = _inputs(dtype, B, S, Hkv, G, seed)
    cache = gpu_cache(k, v, n, p, S)
    lens_t = dev_i32(np.asarray(lens))
    scale = float(np.float32(D ** -0.5))
    want = kvbfp.decode_attention_qbfp(cache, q, S, scale, qbits, seq_len_dev=lens_t)
    got = torch.full_like(q, float("nan"))
    kvbfp.decode_attention_noalloc(cache, q, S, scale, got, q_mant_bits=qbits, seq_len_dev=lens_t)
    torch.cuda.synchronize()
    assert torch.equal(got, want), "noalloc call differs from the call with a workspace"
    planes = oracle_cache(k.cpu(), v.cpu(), n, p, S, 0)
    ref = O.decode_attention(*planes, D, n, p, synth.to_f32_numpy(q.cpu()), list(lens), scale,
                             q_mant_bits=qbits)
    assert_attention_close(got, ref, dtype, "noalloc")


def test_two_calls_in_a_row_the_second_smaller():
    # first: 3 sequences x 2 kv-heads x 4 heads, several splits with ragged tails and an empty sequence;
    # second: a smaller geometry (other block size, fewer heads, shorter) through the same array
    _both(torch.bfloat16, 32, 4, 3, 2100, 2, 4, [2100, 1333, 0], seed=11)
    _both(torch.bfloat16, 16, 4, 1, 300, 1, 2, [257], seed=12)
    # and once more large after small, 8-bit mantissas and an fp32 query cast to BFP
    _both(torch.float32, 64, 8, 2, 1500, 2, 2, [1500, 77], seed=13, qbits=8)


def test_a_geometry_beyond_the_array_is_refused_before_any_launch():
    # 64 sequences x 32 heads x 6 splits x 130 floats = 6.4 MB of partials > 4 MiB
    L = kvbfp.make_layout(D, 32, 4, 2, 64, 4096)
    assert kvbfp.decode_workspace_bytes(L, 32, 4096) > kvbfp.NOALLOC_SCRATCH_BYTES
    cache = kvbfp.alloc_cache(L, "cuda", fill=0)
    q = torch.zeros((64, 32, D), dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, 3.0)
    with pytest.raises(kvbfp.KvbfpError) as e:
        kvbfp.decode_attention_noalloc(cache, q, 4096, 0.1, out)
    assert e.value.status == kvbfp.ERR_WORKSPACE and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 3.0).all()), "nothing may have been launched"
