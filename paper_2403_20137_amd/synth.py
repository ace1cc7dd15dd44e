"""Seeded synthetic inputs shaped like the paper's workload (Sec. IV: Llama-2-7B keys with
channel-consistent outliers, Sec. II-C).  Used by the tests and the benchmark for BOTH the
oracle and the HIP path; holds none of the method's arithmetic (no quantization, no sorting,
no attention) -- only random draws, the outlier gains and dtype rounding.

Data model: every K or V tensor is N(0,1) per element; per KV head a seeded set of outlier
channels is multiplied by a gain for ALL tokens (calibration and cached alike), which is the
"outliers sit in fixed channels" structure the method exploits.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

BASE_SEED = 20137

TORCH_DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq: int
    dtype: str            # "f32" | "f16" | "bf16"
    block: int
    mant_bits: int
    outlier_count: tuple  # inclusive (lo, hi) outlier channels per KV head
    outlier_gain: tuple   # (lo, hi): log-uniform gain range; lo == hi -> fixed gain
    n_calib: int = 256
    extra: dict = field(default_factory=dict)

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    def row_pair_bytes(self):
        d, n, p = self.head_dim, self.block, self.mant_bits
        return 2 * (d * p // 8 + d // n)

    def cache_bytes(self, seq=None):
        s = self.seq if seq is None else seq
        return self.batch * self.n_kv_heads * s * self.row_pair_bytes()


# The five configurations the benchmark contract names, as concrete shapes.
WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 1, 128, 256, "f32", 16, 4, (4, 4), (20.0, 20.0), n_calib=64),
    "llama2_7b_4k": Workload("llama2_7b_4k", 1, 32, 32, 128, 4096, "f16", 32, 4, (2, 6), (10.0, 50.0)),
    "batched_8k_p4": Workload("batched_8k_p4", 16, 32, 32, 128, 8192, "bf16", 16, 4, (2, 6), (10.0, 50.0)),
    "batched_8k_p8": Workload("batched_8k_p8", 16, 32, 32, 128, 8192, "bf16", 16, 8, (2, 6), (10.0, 50.0)),
    "llama3_8b_gqa_32k": Workload("llama3_8b_gqa_32k", 8, 32, 8, 128, 32768, "bf16", 32, 4, (2, 6), (20.0, 20.0)),
    "long_128k": Workload("long_128k", 1, 32, 8, 128, 131072, "bf16", 16, 4, (2, 6), (20.0, 20.0)),
    # not one of the contract's configurations: 8 query heads per kv-head (two MFMA row groups per pass)
    "gqa8_32k": Workload("gqa8_32k", 8, 64, 8, 128, 32768, "bf16", 32, 4, (2, 6), (20.0, 20.0)),
    # the headline shapes with the paper's other block sizes (Table I) and with 8-bit mantissas
    "gqa_32k_n64": Workload("gqa_32k_n64", 8, 32, 8, 128, 32768, "bf16", 64, 4, (2, 6), (20.0, 20.0)),
    "gqa_32k_n128": Workload("gqa_32k_n128", 8, 32, 8, 128, 32768, "bf16", 128, 4, (2, 6), (20.0, 20.0)),
    "gqa_32k_p8n16": Workload("gqa_32k_p8n16", 8, 32, 8, 128, 32768, "bf16", 16, 8, (2, 6), (20.0, 20.0)),
    "gqa_32k_p8n32": Workload("gqa_32k_p8n32", 8, 32, 8, 128, 32768, "bf16", 32, 8, (2, 6), (20.0, 20.0)),
    # the headline shapes with 96 sequences: 768 (sequence, kv-head) units, one split each, 3.4 GB per call
    "gqa_32k_b96": Workload("gqa_32k_b96", 96, 32, 8, 128, 32768, "bf16", 32, 4, (2, 6), (20.0, 20.0)),
    "prefill_bulk": Workload("prefill_bulk", 32, 8, 8, 128, 4096, "bf16", 16, 4, (2, 6), (10.0, 50.0),
                             extra={"note": "32 layers x 8 KV heads x 4096 tokens, layer index plays the batch role"}),
}


def _tensor_seed(seed: int, tensor_id: int) -> int:
    return (int(seed) * 1000003 + int(tensor_id) * 7919 + 12345) % (2 ** 62)


def outlier_gains(seed: int, tensor_id: int, n_heads: int, head_dim: int,
                  count=(2, 6), gain=(10.0, 50.0)) -> np.ndarray:
    """float32 [n_heads][head_dim]: 1.0 except on the seeded outlier channels of each head."""
    rng = np.random.Generator(np.random.Philox(key=_tensor_seed(seed, tensor_id)))
    g = np.ones((n_heads, head_dim), dtype=np.float32)
    for h in range(n_heads):
        c = int(rng.integers(count[0], count[1] + 1))
        ch = rng.permutation(head_dim)[:c]
        if gain[0] == gain[1]:
            vals = np.full(c, gain[0])
        else:
            vals = np.exp(rng.uniform(math.log(gain[0]), math.log(gain[1]), size=c))
        g[h, ch] = vals.astype(np.float32)
    return g


def gaussian(shape, seed: int, tensor_id: int, device="cpu") -> torch.Tensor:
    """float32 N(0,1) tensor from a generator seeded by (seed, tensor_id) on `device`.
    The stream depends on the device type, so both sides of a comparison must be fed from
    the same call (generate once, copy)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(_tensor_seed(seed, tensor_id))
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def kv_rows(batch, n_tok, n_heads, head_dim, dtype, gains, seed, tensor_id, device="cpu",
            chunk_tokens=8192) -> torch.Tensor:
    """[batch][n_tok][n_heads][head_dim] tensor of `dtype`: N(0,1) times the per-(head, channel)
    gains, rounded once to `dtype`."""
    tdt = TORCH_DTYPES[dtype]
    out = torch.empty((batch, n_tok, n_heads, head_dim), dtype=tdt, device=device)
    g = torch.as_tensor(gains, dtype=torch.float32, device=device).view(1, 1, n_heads, head_dim)
    gen = torch.Generator(device=device)
    gen.manual_seed(_tensor_seed(seed, tensor_id))
    for b in range(batch):
        for t0 in range(0, n_tok, chunk_tokens):
            t1 = min(n_tok, t0 + chunk_tokens)
            x = torch.randn((1, t1 - t0, n_heads, head_dim), generator=gen, device=device,
                            dtype=torch.float32)
            out[b:b + 1, t0:t1] = (x * g).to(tdt)
    return out


def queries(batch, n_q_heads, head_dim, dtype, seed, tensor_id, device="cpu") -> torch.Tensor:
    return gaussian((batch, n_q_heads, head_dim), seed, tensor_id, device).to(TORCH_DTYPES[dtype])


# tensor ids (one stream per logical tensor)
TID_K_GAIN, TID_V_GAIN, TID_K_CALIB, TID_V_CALIB, TID_K, TID_V, TID_Q, TID_K_NEW, TID_V_NEW = range(9)


def make_workload_inputs(w: Workload, seed: int = BASE_SEED, device="cpu", seq=None, batch=None,
                         with_calibration=True):
    """All inputs of one workload as a dict of torch tensors on `device` (gains as numpy)."""
    seq = w.seq if seq is None else seq
    batch = w.batch if batch is None else batch
    kg = outlier_gains(seed, TID_K_GAIN, w.n_kv_heads, w.head_dim, w.outlier_count, w.outlier_gain)
    vg = outlier_gains(seed, TID_V_GAIN, w.n_kv_heads, w.head_dim, w.outlier_count, w.outlier_gain)
    d = {"k_gain": kg, "v_gain": vg}
    if with_calibration:
        d["k_calib"] = kv_rows(1, w.n_calib, w.n_kv_heads, w.head_dim, w.dtype, kg, seed, TID_K_CALIB, device)[0]
        d["v_calib"] = kv_rows(1, w.n_calib, w.n_kv_heads, w.head_dim, w.dtype, vg, seed, TID_V_CALIB, device)[0]
    d["k"] = kv_rows(batch, seq, w.n_kv_heads, w.head_dim, w.dtype, kg, seed, TID_K, device)
    d["v"] = kv_rows(batch, seq, w.n_kv_heads, w.head_dim, w.dtype, vg, seed, TID_V, device)
    d["q"] = queries(batch, w.n_q_heads, w.head_dim, w.dtype, seed, TID_Q, device)
    return d


def to_f32_numpy(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a tensor to float32 numpy (host)."""
    return t.detach().to("cpu").to(torch.float32).contiguous().numpy()
