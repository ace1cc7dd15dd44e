"""CPU-side tests of libkvbfp: the library loads, exports the whole C ABI, its host functions agree
with the oracle, and argument errors are reported before anything is launched.  No GPU needed."""
import ctypes as C
import os
import re

import numpy as np
import pytest
import torch

from oracle import kvbfp_oracle as O
from paper_2403_20137_amd import kvbfp, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "kvbfp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvbfp_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(kvbfp.EXPORTS)
    lib = kvbfp.lib()
    for n in names:
        assert getattr(lib, n) is not None
    assert "gfx950" in kvbfp.version()


def test_cache_bytes_matches_format_definition():
    L = kvbfp.make_layout(128, 32, 4, 8, 8, 32768)
    m, e = kvbfp.cache_bytes(L)
    assert m == 8 * 8 * 32768 * 64 and e == 8 * 8 * 32768 * 4
    assert 2 * (m + e) == synth.WORKLOADS["llama3_8b_gqa_32k"].cache_bytes()
    bad = kvbfp.make_layout(128, 48, 4, 8, 8, 16)
    with pytest.raises(kvbfp.KvbfpError):
        kvbfp.cache_bytes(bad)


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
@pytest.mark.parametrize("descending", [False, True])
def test_calibrate_perm_equals_oracle(dtype, descending):
    g = synth.outlier_gains(1, 0, 4, 128)
    x = synth.kv_rows(1, 96, 4, 128, {torch.float32: "f32", torch.float16: "f16", torch.bfloat16: "bf16"}[dtype],
                      g, 1, 5)[0]
    x[:, 1, 7] = x[:, 1, 3]                     # force a tie
    x[:, 2, :] = 0                              # a head of all-equal statistics
    got = kvbfp.calibrate_perm(x, kvbfp.STAT_MAXABS, descending)
    want = O.calibrate_perm(synth.to_f32_numpy(x), "maxabs", descending)
    assert np.array_equal(got, want)
    got = kvbfp.calibrate_perm(x, kvbfp.STAT_L2, descending)
    want = O.calibrate_perm(synth.to_f32_numpy(x), "l2", descending)
    assert np.array_equal(got, want)


def test_calibrate_from_weights_and_permute_weights_equal_oracle():
    rng = np.random.default_rng(4)
    H, G, D, F = 2, 3, 128, 40
    wk = rng.standard_normal((H * D, F)).astype(np.float32)
    wk[rng.choice(H * D, 7, replace=False)] *= 9
    wq = rng.standard_normal((H * G * D, F)).astype(np.float32)
    perm = kvbfp.calibrate_perm_from_weights(wk, H, D)
    assert np.array_equal(perm, O.calibrate_perm_from_weights(wk, H, D))
    assert np.array_equal(kvbfp.permute_weights(wk, H, D, perm), O.permute_weights(wk, H, D, perm))
    assert np.array_equal(kvbfp.permute_weights(wq, H * G, D, perm, G), O.permute_weights(wq, H * G, D, perm, G))
    # 16-bit rows move as whole bit patterns
    wq16 = torch.from_numpy(wq).to(torch.bfloat16)
    out = kvbfp.permute_weights(wq16, H * G, D, perm, G)
    want = O.permute_weights(synth.to_f32_numpy(wq16), H * G, D, perm, G)
    assert np.array_equal(synth.to_f32_numpy(out), want)


@pytest.mark.parametrize("pairs", [0, 1])
def test_permute_rope_equals_oracle(pairs):
    # Alg. 1 step 5 on the host: frequencies, partner positions and sine signs in the reordered order
    rng = np.random.default_rng(8 + pairs)
    theta = rng.uniform(1e-4, 1.0, 64).astype(np.float32)
    perm = np.stack([rng.permutation(128) for _ in range(5)]).astype(np.int32)
    got = kvbfp.permute_rope(theta, perm, pairs)
    want = O.permute_rope(theta, perm, pairs)
    for g, w in zip(got, want):
        assert g.dtype == w.dtype and np.array_equal(g, w)
    bad = perm.copy()
    bad[2, 0] = bad[2, 1]
    with pytest.raises(kvbfp.KvbfpError) as ei:
        kvbfp.permute_rope(theta, bad, pairs)
    assert ei.value.status == kvbfp.ERR_INVALID_ARG and "permutation" in str(ei.value)
    with pytest.raises(kvbfp.KvbfpError):
        kvbfp.permute_rope(theta, perm, 2)


def test_host_argument_errors():
    w = np.zeros((256, 4), dtype=np.float32)
    perm = np.tile(np.arange(128, dtype=np.int32), (2, 1))
    bad = perm.copy()
    bad[1, 5] = 6                                # duplicate entry
    with pytest.raises(kvbfp.KvbfpError) as ei:
        kvbfp.permute_weights(w, 2, 128, bad)
    assert ei.value.status == kvbfp.ERR_INVALID_ARG and "permutation" in str(ei.value)
    with pytest.raises(kvbfp.KvbfpError):
        kvbfp.permute_weights(w, 2, 128, perm, heads_per_perm=3)
    lib = kvbfp.lib()
    # overlapping in/out
    rc = lib.kvbfp_permute_weights(w.ctypes.data, w.ctypes.data + 16, kvbfp.F32, 2, 128, 4, 1, perm.ctypes.data)
    assert rc == kvbfp.ERR_INVALID_ARG and "overlap" in kvbfp.last_error()
    rc = lib.kvbfp_calibrate_perm(None, kvbfp.F32, 1, 1, 128, 128, 128, 1, 0, 0, perm.ctypes.data)
    assert rc == kvbfp.ERR_INVALID_ARG
    rc = lib.kvbfp_calibrate_perm(w.ctypes.data, 7, 1, 1, 128, 128, 128, 1, 0, 0, perm.ctypes.data)
    assert rc == kvbfp.ERR_INVALID_ARG


def test_device_calls_reject_bad_arguments_before_launching():
    # every case below fails validation on the host, so no HIP call is made (runs without a GPU)
    lib = kvbfp.lib()
    good = kvbfp.make_layout(128, 32, 4, 2, 1, 64)
    ptrs = kvbfp.CachePtrs(0x1000, 0x1000, 0x1000, 0x1000)
    fake = C.c_void_p(0x1000)

    def qa(layout, n_new=1, pos0=0, dtype=kvbfp.BF16, cache=ptrs):
        return lib.kvbfp_quantize_append(C.byref(layout), C.byref(cache), fake, fake, dtype, n_new,
                                         256, 256, 128, pos0, None, None, None, None)

    assert qa(kvbfp.make_layout(64, 32, 4, 2, 1, 64)) == kvbfp.ERR_UNSUPPORTED
    assert qa(kvbfp.make_layout(128, 24, 4, 2, 1, 64)) == kvbfp.ERR_UNSUPPORTED
    assert qa(kvbfp.make_layout(128, 32, 5, 2, 1, 64)) == kvbfp.ERR_UNSUPPORTED
    assert qa(kvbfp.make_layout(128, 32, 4, 0, 1, 64)) == kvbfp.ERR_INVALID_ARG
    wrong_size = kvbfp.make_layout(128, 32, 4, 2, 1, 64)
    wrong_size.struct_bytes = 8
    assert qa(wrong_size) == kvbfp.ERR_INVALID_ARG
    assert qa(good, n_new=-1) == kvbfp.ERR_INVALID_ARG
    assert qa(good, n_new=2, pos0=63) == kvbfp.ERR_INVALID_ARG and "max_seq" in kvbfp.last_error()
    assert qa(good, dtype=9) == kvbfp.ERR_INVALID_ARG
    assert qa(good, cache=kvbfp.CachePtrs(0, 0, 0x1000, 0x1000)) == kvbfp.ERR_INVALID_ARG
    assert qa(good, n_new=0) == kvbfp.OK            # nothing to do is not an error, nothing launched

    def dq(which=0, t0=0, n_tok=1, out=fake):
        return lib.kvbfp_dequantize(C.byref(good), C.byref(ptrs), which, t0, n_tok, None, out, kvbfp.F32, None)

    assert dq(which=2) == kvbfp.ERR_INVALID_ARG
    assert dq(t0=60, n_tok=5) == kvbfp.ERR_INVALID_ARG
    assert dq(out=None) == kvbfp.ERR_INVALID_ARG
    assert dq(n_tok=0) == kvbfp.OK

    def da(n_q=4, max_len=64, ws=fake, ws_bytes=1 << 30, scale=0.1, q=fake):
        return lib.kvbfp_decode_attention(C.byref(good), C.byref(ptrs), n_q, q, kvbfp.BF16, None, max_len,
                                          scale, None, None, fake, ws, ws_bytes, None)

    assert da(n_q=3) == kvbfp.ERR_INVALID_ARG
    assert da(max_len=65) == kvbfp.ERR_INVALID_ARG
    assert da(max_len=0) == kvbfp.ERR_INVALID_ARG
    assert da(q=None) == kvbfp.ERR_INVALID_ARG
    assert da(scale=float("nan")) == kvbfp.ERR_INVALID_ARG

    def daq(qbits, n_q=4):
        return lib.kvbfp_decode_attention_qbfp(C.byref(good), C.byref(ptrs), n_q, fake, kvbfp.BF16, None, 64,
                                               0.1, None, None, qbits, fake, fake, 1 << 30, None)

    assert daq(5) == kvbfp.ERR_INVALID_ARG and "q_mant_bits" in kvbfp.last_error()
    assert daq(-8) == kvbfp.ERR_INVALID_ARG
    assert daq(8, n_q=3) == kvbfp.ERR_INVALID_ARG      # the other checks are those of the plain call
    def dar(theta=fake, partner=fake, sign=fake):
        return lib.kvbfp_decode_attention_rope(C.byref(good), C.byref(ptrs), 4, fake, kvbfp.BF16, None, 64, 0.1,
                                               None, None, theta, partner, sign, fake, None, 0, None, None)

    assert dar(theta=None) == kvbfp.ERR_INVALID_ARG and "rope" in kvbfp.last_error()
    assert dar(partner=None) == kvbfp.ERR_INVALID_ARG
    assert dar(sign=None) == kvbfp.ERR_INVALID_ARG
    assert dar() == kvbfp.ERR_WORKSPACE                # complete arguments reach the workspace check
    def dap(pool, stride=2, batch=1, max_len=300, table=fake):
        return lib.kvbfp_decode_attention_paged(C.byref(pool), C.byref(ptrs), table, stride, batch, 4, fake, kvbfp.BF16,
                                                None, max_len, 0.1, None, None, 0, fake, None, 0, None, None)

    pages = kvbfp.make_layout(128, 32, 4, 2, 6, 256)
    assert dap(kvbfp.make_layout(128, 32, 4, 2, 6, 384)) == kvbfp.ERR_UNSUPPORTED and "page" in kvbfp.last_error()
    assert dap(kvbfp.make_layout(128, 32, 4, 2, 6, 8)) == kvbfp.ERR_UNSUPPORTED           # below 16 tokens per page
    assert dap(kvbfp.make_layout(128, 32, 4, 2, 40, 16), stride=20) == kvbfp.ERR_WORKSPACE  # pages of 16 tokens are taken
    assert dap(pages, table=None) == kvbfp.ERR_INVALID_ARG
    assert dap(pages, batch=0) == kvbfp.ERR_INVALID_ARG
    assert dap(pages, max_len=513) == kvbfp.ERR_INVALID_ARG          # two pages of 256 tokens
    assert dap(pages) == kvbfp.ERR_WORKSPACE                          # complete arguments reach the workspace check
    assert kvbfp.decode_workspace_bytes_paged(pages, 2, 3, 4, 512) == kvbfp.decode_workspace_bytes(
        kvbfp.make_layout(128, 32, 4, 2, 3, 512), 4, 512)
    assert lib.kvbfp_quantize_append_paged(C.byref(pages), C.byref(ptrs), fake, 2, 1, fake, fake, kvbfp.BF16, 2, 256,
                                           256, 128, 511, None, None, None, None) == kvbfp.ERR_INVALID_ARG
    assert da(ws=None) == kvbfp.ERR_WORKSPACE
    assert da(ws_bytes=16) == kvbfp.ERR_WORKSPACE and "workspace" in kvbfp.last_error()
    assert da(ws=C.c_void_p(0x1010)) == kvbfp.ERR_WORKSPACE
    need = kvbfp.decode_workspace_bytes(good, 4, 64)
    assert need > 0 and need % 4 == 0
    assert kvbfp.decode_workspace_bytes(good, 3, 64) == 0


def test_workspace_grows_with_splits_and_heads():
    L = kvbfp.make_layout(128, 16, 4, 8, 1, 131072)
    a = kvbfp.decode_workspace_bytes(L, 32, 131072)
    b = kvbfp.decode_workspace_bytes(L, 32, 256)
    assert a > b > 0
    assert b == 1 * 32 * 1 * 130 * 4


def test_misaligned_mantissa_planes_are_refused_before_any_launch():
    # device calls move mantissa rows with 8- and 16-byte accesses; a plane at an odd address is an
    # argument error (checked on the host: the pointers below are never dereferenced)
    L = kvbfp.make_layout(128, 32, 4, 2, 1, 64)
    lib = kvbfp.lib()
    for bad in (0, 2):
        planes = [0x10000, 0x20000, 0x30000, 0x40000]
        planes[bad] += 8
        ptrs = kvbfp.CachePtrs(*planes)
        rc = lib.kvbfp_decode_attention(C.byref(L), C.byref(ptrs), 2, C.c_void_p(0x50000), kvbfp.BF16, None, 64,
                                        C.c_float(0.1), None, None, C.c_void_p(0x60000), C.c_void_p(0x70000),
                                        C.c_size_t(1 << 20), None)
        assert rc == kvbfp.ERR_INVALID_ARG and "16-byte aligned" in kvbfp.last_error()
        rc = lib.kvbfp_quantize_append(C.byref(L), C.byref(ptrs), C.c_void_p(0x50000), C.c_void_p(0x58000), kvbfp.BF16,
                                       1, 256, 256, 128, 0, None, None, None, None)
        assert rc == kvbfp.ERR_INVALID_ARG and "16-byte aligned" in kvbfp.last_error()


def test_noalloc_entry_rejects_what_does_not_fit_without_touching_the_gpu():
    L = kvbfp.make_layout(128, 32, 4, 2, 64, 4096)
    assert kvbfp.decode_workspace_bytes(L, 32, 4096) > kvbfp.NOALLOC_SCRATCH_BYTES
    ptrs = kvbfp.CachePtrs(0x10000, 0x20000, 0x30000, 0x40000)
    rc = kvbfp.lib().kvbfp_decode_attention_noalloc(C.byref(L), C.byref(ptrs), 32, C.c_void_p(0x50000), kvbfp.BF16, None,
                                                    4096, C.c_float(0.1), None, None, 0, C.c_void_p(0x60000), None)
    assert rc == kvbfp.ERR_WORKSPACE and "scratch" in kvbfp.last_error()


def test_permute_weight_columns_equals_oracle_and_rejects_bad_input():
    rng = np.random.default_rng(21)
    H, G, D, R = 2, 4, 128, 37
    wo = rng.standard_normal((R, H * G * D)).astype(np.float32)
    perm = np.stack([rng.permutation(D) for _ in range(H)]).astype(np.int32)
    assert np.array_equal(kvbfp.permute_weight_columns(wo, H * G, D, perm, G),
                          O.permute_weight_columns(wo, H * G, D, perm, G))
    wo16 = torch.from_numpy(wo).to(torch.bfloat16)
    out = kvbfp.permute_weight_columns(wo16, H * G, D, perm, G)
    assert out.dtype == torch.bfloat16
    assert np.array_equal(synth.to_f32_numpy(out), O.permute_weight_columns(synth.to_f32_numpy(wo16), H * G, D, perm, G))
    bad = perm.copy()
    bad[1, 5] = bad[1, 6]
    with pytest.raises(kvbfp.KvbfpError):
        kvbfp.permute_weight_columns(wo, H * G, D, bad, G)
    with pytest.raises(kvbfp.KvbfpError):
        kvbfp.permute_weight_columns(wo, H * G, D, perm, 3)
    rc = kvbfp.lib().kvbfp_permute_weight_columns(wo.ctypes.data, wo.ctypes.data + 64, kvbfp.F32, R, H * G, D, G,
                                                  perm.ctypes.data)
    assert rc == kvbfp.ERR_INVALID_ARG and "overlap" in kvbfp.last_error()
