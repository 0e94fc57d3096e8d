"""Seeded synthetic inputs: model weights, filter weights and prompts.

This module only draws numbers.  It contains none of the decoding method's
arithmetic (no transformer op, no softmax, no filter evaluation, no decode
rule), so both the CPU checker and the HIP path may be fed from it without
sharing any computation.

Every value is a pure function of (seed, tensor name, element index): a
counter-based integer hash (two rounds of a 32-bit xorshift-multiply mixer,
exact integer arithmetic, identical on CPU and GPU) selects one of 65536
equiprobable quantiles of the standard normal from a table that is computed
once, on the CPU, in float64.  The same call therefore yields bit-identical
tensors on ``cpu`` and on ``cuda`` devices, which is what lets a 16 GB model
be generated directly in HBM while a CPU checker regenerates exactly the
same weights, one tensor at a time, on the host.

The model family (the paper treats the dLLM as a black box M(X); shapes are
those of its LLaDA-8B workload): pre-norm transformer, RMSNorm, rotary
embeddings, SwiGLU FFN, untied LM head, no biases.  All weight matrices are
stored row-major ``[out_features, in_features]``.
"""
from __future__ import annotations

import dataclasses
import os
import zlib
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Iterator, Tuple

import numpy as np
import torch

_M32 = 0xFFFFFFFF
_MULT = 0x45D9F3B  # < 2**27, so products of 32-bit values stay below 2**59
_CHUNK = 1 << 24


@dataclasses.dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    mask_id: int
    eos_id: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "bf16"  # "fp32" or "bf16"


@dataclasses.dataclass(frozen=True)
class Workload:
    """One decoding workload: model shape plus the decode arguments of Alg. 2 / Alg. 3."""
    name: str
    model: ModelShape
    batch: int
    prompt_len: int
    gen_len: int
    block_len: int
    filter_hidden: int
    threshold: float
    eotp: bool = False
    eotp_step: bool = False  # step-granular EoTP (Sec. 3.3) instead of the block-granular Alg. 3
    prefix_cache: bool = False
    dual_cache: bool = False
    bias_from: int = -1      # generation position from which the EOS logit bias applies (-1: none)
    bias_value: float = 0.0
    prompt_hi: int = 0       # prompt ids are uniform in [0, prompt_hi)


_TINY = ModelShape(2, 128, 4, 32, 512, 1024, 1023, 1022, dtype="fp32")
_MID = ModelShape(8, 1024, 16, 64, 2816, 32000, 31999, 31998, dtype="bf16")
_8B = ModelShape(32, 4096, 32, 128, 12288, 126464, 126336, 126081, dtype="bf16")

WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", _TINY, 1, 32, 64, 32, 64, 0.5, prompt_hi=1022),
    "mid": Workload("mid", _MID, 8, 128, 256, 32, 128, 0.7, prompt_hi=31998),
    "8b_g256": Workload("8b_g256", _8B, 1, 256, 256, 32, 128, 0.9, prompt_hi=126081),
    "8b_b8_g256": Workload("8b_b8_g256", _8B, 8, 256, 256, 32, 128, 0.9, prompt_hi=126081),
    "8b_g1024_eotp": Workload("8b_g1024_eotp", _8B, 1, 256, 1024, 32, 128, 0.9, eotp=True,
                              bias_from=300, bias_value=20.0, prompt_hi=126081),
    "8b_g1024_eotp_step": Workload("8b_g1024_eotp_step", _8B, 1, 256, 1024, 32, 128, 0.9, eotp=True, eotp_step=True,
                                   bias_from=300, bias_value=20.0, prompt_hi=126081),
    "8b_g1024_dual": Workload("8b_g1024_dual", _8B, 1, 256, 1024, 32, 128, 0.9, eotp=True, dual_cache=True,
                              bias_from=300, bias_value=20.0, prompt_hi=126081),
    "8b_b8_g1024_dual": Workload("8b_b8_g1024_dual", _8B, 8, 256, 1024, 32, 128, 0.9, eotp=True, dual_cache=True,
                                 bias_from=300, bias_value=20.0, prompt_hi=126081),
    "8b_b32_prefix": Workload("8b_b32_prefix", _8B, 32, 512, 512, 64, 128, 0.9, eotp=True,
                              prefix_cache=True, bias_from=400, bias_value=20.0, prompt_hi=126081),
}


def with_layers(w: Workload, n_layers: int) -> Workload:
    """Same widths / vocabulary / decode arguments at a reduced depth."""
    return dataclasses.replace(w, model=dataclasses.replace(w.model, n_layers=n_layers),
                               name=f"{w.name}_L{n_layers}")


# --------------------------------------------------------------------------- hashing
def _mix(x: torch.Tensor) -> torch.Tensor:
    x = (((x >> 16) ^ x) * _MULT) & _M32
    x = (((x >> 16) ^ x) * _MULT) & _M32
    return (x >> 16) ^ x


def _mix_int(x: int) -> int:
    x &= _M32
    x = (((x >> 16) ^ x) * _MULT) & _M32
    x = (((x >> 16) ^ x) * _MULT) & _M32
    return (x >> 16) ^ x


def _key(seed: int, name: str) -> int:
    return _mix_int(_mix_int(seed) ^ (zlib.crc32(name.encode()) & _M32))


def _bits(seed: int, name: str, start: int, count: int, device) -> torch.Tensor:
    """32 hashed bits (as int64 in [0, 2**32)) for elements start..start+count of tensor `name`."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix(_mix(idx) ^ _key(seed, name))


_Z_TABLE = None


def _z_table() -> torch.Tensor:
    """65536 standard-normal quantiles at the bin midpoints, float64, CPU."""
    global _Z_TABLE
    if _Z_TABLE is None:
        k = torch.arange(65536, dtype=torch.float64)
        _Z_TABLE = torch.erfinv(2.0 * (k + 0.5) / 65536.0 - 1.0) * (2.0 ** 0.5)
    return _Z_TABLE


def _mix_np(x: np.ndarray) -> np.ndarray:
    """Same mixer on uint32 arrays (unsigned multiplication wraps, so no masking is needed)."""
    m, sh = np.uint32(_MULT), np.uint32(16)
    x ^= x >> sh
    x *= m
    x ^= x >> sh
    x *= m
    x ^= x >> sh
    return x


def _normal_cpu(seed: int, name: str, n: int, table: torch.Tensor) -> torch.Tensor:
    """Host fast path of `normal`: identical values, numpy uint32 arithmetic on a thread pool."""
    key = np.uint32(_key(seed, name))
    out = torch.empty(n, dtype=table.dtype)
    two_byte = table.element_size() == 2
    tab = (table.view(torch.int16) if two_byte else table).numpy()
    dst = (out.view(torch.int16) if two_byte else out).numpy()
    chunk = 1 << 18

    def work(s0):
        c = min(chunk, n - s0)
        x = _mix_np(np.arange(s0, s0 + c, dtype=np.uint32))
        x ^= key
        dst[s0:s0 + c] = tab[_mix_np(x) >> np.uint32(16)]

    with ThreadPoolExecutor(max(1, min(16, os.cpu_count() or 1))) as ex:
        list(ex.map(work, range(0, n, chunk)))
    return out


def normal(seed: int, name: str, shape: Tuple[int, ...], std: float, dtype: torch.dtype,
           device="cpu", force_torch: bool = False) -> torch.Tensor:
    """Tensor of N(0, std^2) draws (truncated at about 4.2 sigma, 65536 levels)."""
    n = 1
    for s in shape:
        n *= int(s)
    assert n < (1 << 32)
    table = (_z_table() * std).to(torch.float32).to(dtype)
    if torch.device(device).type == "cpu" and not force_torch:
        return _normal_cpu(seed, name, n, table).view(*shape)
    table = table.to(device)
    out = torch.empty(n, dtype=dtype, device=device)
    for s0 in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s0)
        out[s0:s0 + c] = table[_bits(seed, name, s0, c, device) >> 16]
    return out.view(*shape)


def uniform_ints(seed: int, name: str, shape: Tuple[int, ...], hi: int, device="cpu") -> torch.Tensor:
    """int32 tensor of draws uniform on [0, hi)."""
    n = 1
    for s in shape:
        n *= int(s)
    out = (_bits(seed, name, 0, n, device) * hi) >> 32
    return out.to(torch.int32).view(*shape)


# --------------------------------------------------------------------------- model / filter / prompt
def weight_specs(m: ModelShape) -> Iterator[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) of every model tensor in a fixed order; kind is 'w' (matrix) or 'g' (norm gain)."""
    d, f, v = m.d_model, m.d_ffn, m.vocab
    yield "tok_emb", (v, d), "w"
    for l in range(m.n_layers):
        p = f"layers.{l}."
        yield p + "attn_norm_g", (d,), "g"
        yield p + "wq", (d, d), "w"
        yield p + "wk", (d, d), "w"
        yield p + "wv", (d, d), "w"
        yield p + "wo", (d, d), "w"
        yield p + "ffn_norm_g", (d,), "g"
        yield p + "w_gate", (f, d), "w"
        yield p + "w_up", (f, d), "w"
        yield p + "w_down", (d, f), "w"
    yield "final_norm_g", (d,), "g"
    yield "lm_head", (v, d), "w"


def torch_dtype(m: ModelShape) -> torch.dtype:
    return torch.float32 if m.dtype == "fp32" else torch.bfloat16


def make_tensor(m: ModelShape, seed: int, name: str, shape, kind: str, device="cpu",
                init_std: float = 0.02) -> torch.Tensor:
    dt = torch_dtype(m)
    if kind == "g":
        return torch.ones(shape, dtype=dt, device=device)
    return normal(seed, name, shape, init_std, dt, device)


def make_weights(m: ModelShape, seed: int, device="cpu", init_std: float = 0.02,
                 lm_head_scale: float = 1.0) -> Dict[str, torch.Tensor]:
    """All model tensors: matrices N(0, init_std^2), RMSNorm gains 1.

    lm_head_scale > 1 gives the "peaked" test variant: logits spread out, so confidences cover
    (0, 1) instead of sitting near 1/vocab as they do for a plain random-init model.
    """
    return {name: make_tensor(m, seed, name, shape, kind, device,
                              init_std * (lm_head_scale if name == "lm_head" else 1.0))
            for name, shape, kind in weight_specs(m)}


def make_filter(seed: int, block_len: int, hidden: int, device="cpu", n_layers: int = 2) -> Dict[str, torch.Tensor]:
    """MLP filter parameters {w1, b1, ..., wN, bN}, fp32: W ~ N(0, 1/fan_in), b ~ N(0, 1).  Two layers
    is the paper's filter; one and four are the depth variants of Table 3 (hidden widths all `hidden`).

    Biases of order one spread the filter outputs over (0, 1); with a random-init
    language model every confidence is about 1e-3, so a small-weight filter would
    put every decision on top of the threshold.
    """
    f32 = torch.float32
    dims = [block_len] + [hidden] * (n_layers - 1) + [block_len]
    out = {}
    for k in range(1, n_layers + 1):
        fan_in, fan_out = dims[k - 1], dims[k]
        out[f"w{k}"] = normal(seed, f"filter.w{k}", (fan_out, fan_in), fan_in ** -0.5, f32, device)
        out[f"b{k}"] = normal(seed, f"filter.b{k}", (fan_out,), 1.0, f32, device)
    return out


def threshold_filter(block_len: int, theta: float, sharpness: float = 200.0, device="cpu") -> Dict[str, torch.Tensor]:
    """The filter that turns the decoder into fixed-threshold confidence decoding (the baseline of
    Sec. 2 / Table 1): W1 = I, W2 = sharpness * I, b2 = -sharpness * theta, so that the filter output
    exceeds 0.5 exactly when the position's confidence exceeds theta (committed positions enter as 1.0)."""
    f32 = torch.float32
    eye = torch.eye(block_len, dtype=f32, device=device)
    return {"w1": eye.clone(), "b1": torch.zeros(block_len, dtype=f32, device=device),
            "w2": eye * sharpness, "b2": torch.full((block_len,), -sharpness * theta, dtype=f32, device=device)}


def make_prompt(seed: int, batch: int, prompt_len: int, hi: int, device="cpu") -> torch.Tensor:
    """int32 [batch, prompt_len], ids uniform on [0, hi) (hi excludes the EOS and mask ids)."""
    return uniform_ints(seed, "prompt", (batch, prompt_len), hi, device)


def to_numpy(t: torch.Tensor):
    """CPU numpy view; bf16 tensors come back as their uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
