"""Seeded, synthetic stand-ins for the policy weights and the query batches of the PPO rollout.

The paper trains on TL;DR prompts with Pythia checkpoints (Dataset Details; Setup -> Tech stack);
neither is available, so every tensor here is drawn from a counter-based generator keyed by
(seed, tensor name).  Any tensor can therefore be regenerated alone, on either side of the
oracle / HIP comparison, and both sides see bit-identical inputs.

Shapes follow the paper: queries are left-padded to a fixed length (Dataset Details, item
"SFT dataset for PPO training"), responses have a fixed sampled length (PPO Details, "EOS
trick"), the end-of-sequence id is 0 (Figure "reward logits" caption).
"""
from __future__ import annotations

import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np
from numpy.random import Generator, Philox

VOCAB = 50304
ID_HI = 50277  # query ids are drawn from [1, ID_HI); ID_HI itself serves as the pad id


@dataclass(frozen=True)
class ModelConfig:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    rotary_dims: int
    d_ff: int
    vocab: int = VOCAB
    dtype: str = "bf16"  # "fp32" or "bf16": storage type of the weights
    eos_id: int = 0
    pad_id: int = ID_HI
    ln_eps: float = 1e-5
    rope_base: float = 10000.0

    def with_(self, **kw) -> "ModelConfig":
        return replace(self, **kw)


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelConfig
    batch: int
    query_len: int
    new_tokens: int
    min_len: int  # true query lengths are uniform in [min_len, max_len]
    max_len: int
    temperature: float = 0.7
    weight_seed: int = 0
    data_seed: int = 0
    sample_seed: int = 0


def _wl(i, name, model, batch, lq, n, lo, hi):
    return Workload(name, model, batch, lq, n, lo, hi, 0.7, 1000 + i, 2000 + i, 3000 + i)


WORKLOADS = {
    1: _wl(1, "pythia-70m-shape/fp32/B2", ModelConfig(6, 512, 8, 64, 16, 2048, dtype="fp32"), 2, 64, 16, 48, 64),
    2: _wl(2, "pythia-160m-shape/bf16/B64", ModelConfig(12, 768, 12, 64, 16, 3072), 64, 512, 53, 128, 512),
    3: _wl(3, "pythia-1b-shape/bf16/B256", ModelConfig(16, 2048, 8, 256, 64, 8192), 256, 512, 53, 128, 512),
    4: _wl(4, "pythia-2.8b-shape/bf16/B256", ModelConfig(32, 2560, 32, 80, 20, 10240), 256, 512, 53, 128, 512),
    5: _wl(5, "pythia-6.9b-shape/bf16/B512", ModelConfig(32, 4096, 32, 128, 32, 16384), 512, 512, 53, 128, 512),
}


# ----------------------------------------------------------------------------------------------
# bf16 rounding of host data (input preparation: the weights of a bf16 model are bf16 numbers)
# ----------------------------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array holding the bf16-rounded values of x."""
    return (bf16_bits(x).astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(np.shape(x))


# ----------------------------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------------------------
_LAYER_TENSORS = (
    "ln1_g", "ln1_b", "ln2_g", "ln2_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "w_fc1", "b_fc1", "w_fc2", "b_fc2",
)


def weight_names(cfg: ModelConfig):
    names = ["embed_in"]
    for l in range(cfg.n_layers):
        names += [f"layers.{l}.{t}" for t in _LAYER_TENSORS]
    names += ["lnf_g", "lnf_b", "embed_out", "value_w"]
    return names


def weight_shape(cfg: ModelConfig, name: str):
    d, f, v = cfg.d_model, cfg.d_ff, cfg.vocab
    base = name.split(".")[-1]
    return {
        "embed_in": (v, d), "embed_out": (v, d), "value_w": (d,),
        "lnf_g": (d,), "lnf_b": (d,),
        "ln1_g": (d,), "ln1_b": (d,), "ln2_g": (d,), "ln2_b": (d,),
        "w_qkv": (3 * d, d), "b_qkv": (3 * d,),  # rows: all q heads | all k heads | all v heads
        "w_o": (d, d), "b_o": (d,),
        "w_fc1": (f, d), "b_fc1": (f,),
        "w_fc2": (d, f), "b_fc2": (d,),
    }[base]


def _rng(seed: int, name: str) -> Generator:
    return Generator(Philox(key=[np.uint64(seed), np.uint64(zlib.crc32(name.encode()))]))


def make_tensor(cfg: ModelConfig, seed: int, name: str, variant: str = "bench") -> np.ndarray:
    """One weight tensor as float32 (already rounded to bf16 values when cfg.dtype == 'bf16').

    variant 'bench': matrices and linear biases ~ N(0, 0.02), LayerNorm gain 1 / bias 0.
    variant 'test' : LayerNorm gain ~ N(1, 0.1), bias ~ N(0, 0.1), so those paths are exercised.
    The value head follows the reward-head initialisation N(0, 1/sqrt(d_model+1)) (Reward Model
    Details, "Reward head initialization").
    """
    shape = weight_shape(cfg, name)
    base = name.split(".")[-1]
    g = _rng(seed, name)
    if base in ("ln1_g", "ln2_g", "lnf_g"):
        if variant == "bench":
            x = np.ones(shape, np.float32)
        else:
            x = (1.0 + 0.1 * g.standard_normal(shape, dtype=np.float32)).astype(np.float32)
    elif base in ("ln1_b", "ln2_b", "lnf_b"):
        if variant == "bench":
            x = np.zeros(shape, np.float32)
        else:
            x = (0.1 * g.standard_normal(shape, dtype=np.float32)).astype(np.float32)
    elif base == "value_w":
        std = np.float32(1.0 / np.sqrt(cfg.d_model + 1.0))
        x = g.standard_normal(shape, dtype=np.float32) * std
    else:
        x = g.standard_normal(shape, dtype=np.float32)
        x *= np.float32(0.02)
    if cfg.dtype == "bf16":
        x = round_to_bf16(x)
    return x


def make_weights(cfg: ModelConfig, seed: int, variant: str = "bench", threads: int = 8) -> dict:
    """All weight tensors of the model, name -> float32 array, plus the scalar 'value_b'."""
    names = weight_names(cfg)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        arrs = list(ex.map(lambda n: make_tensor(cfg, seed, n, variant), names))
    w = dict(zip(names, arrs))
    w["value_b"] = np.float32(0.0 if variant == "bench" else 0.3)
    return w


def boost_eos(cfg: ModelConfig, w: dict, alpha: float) -> dict:
    """Test helper: make the EOS logit roughly `alpha` at every position.

    Needs a non-zero final-LayerNorm bias ('test' variant): the EOS row of the output embedding is
    set parallel to that bias, so logits[eos] = alpha + (a zero-mean term).  With random-init
    weights EOS is otherwise sampled with probability ~2e-5 per step and the stop mask is never
    exercised.
    """
    b = w["lnf_b"].astype(np.float64)
    row = (alpha * b / float(b @ b)).astype(np.float32)
    out = dict(w)
    eo = w["embed_out"].copy()
    eo[cfg.eos_id] = round_to_bf16(row) if cfg.dtype == "bf16" else row
    out["embed_out"] = eo
    return out


def boost_eos_bias(cfg: ModelConfig, w: dict, alpha: float) -> dict:
    """Test helper: raise the EOS logit by `alpha` at every position while every weight stays at its
    initialisation scale.

    The final LayerNorm's bias gets a component along the EOS row e of the output embedding,
    lnf_b += alpha * e / (e . e): the EOS logit rises by alpha, any other logit v by
    alpha * (e_v . e) / (e . e), which is small for random rows.  No row of the output embedding is
    touched (unlike boost_eos, whose EOS row is tens of times larger than N(0, 0.02) weights), so
    rounding errors of the hidden state are weighted as in the real model.  In bf16 mode the new bias
    is rounded to bf16 (the storage type), which moves the boost by a fraction of a percent."""
    e = w["embed_out"][cfg.eos_id].astype(np.float64)
    b = w["lnf_b"].astype(np.float64) + alpha * e / float(e @ e)
    out = dict(w)
    out["lnf_b"] = round_to_bf16(b.astype(np.float32)) if cfg.dtype == "bf16" else b.astype(np.float32)
    return out


# ----------------------------------------------------------------------------------------------
# queries
# ----------------------------------------------------------------------------------------------
def make_queries(wl: Workload, seed: int | None = None, batch: int | None = None):
    """Left-padded query ids int32 [B, Lq] and mask uint8 [B, Lq] (1 = real token)."""
    seed = wl.data_seed if seed is None else seed
    B = wl.batch if batch is None else batch
    Lq = wl.query_len
    g = _rng(seed, "queries")
    lens = g.integers(wl.min_len, wl.max_len + 1, size=B)
    ids = g.integers(1, ID_HI, size=(B, Lq)).astype(np.int32)
    col = np.arange(Lq)[None, :]
    mask = (col >= (Lq - lens)[:, None]).astype(np.uint8)
    queries = np.where(mask == 1, ids, np.int32(wl.model.pad_id)).astype(np.int32)
    return queries, mask


def make_random_responses(wl: Workload, queries: np.ndarray, pad_mask: np.ndarray, seed: int):
    """A (B, Lq+N) token batch and mask with random response ids of random lengths in [1, N]:
    a scoring input that does not depend on the sampler."""
    B, Lq = queries.shape
    N = wl.new_tokens
    g = _rng(seed, "responses")
    rl = g.integers(1, N + 1, size=B)
    resp = g.integers(1, ID_HI, size=(B, N)).astype(np.int32)
    col = np.arange(N)[None, :]
    rmask = (col < rl[:, None]).astype(np.uint8)
    resp = np.where(rmask == 1, resp, np.int32(wl.model.pad_id)).astype(np.int32)
    tokens = np.concatenate([queries, resp], axis=1)
    mask = np.concatenate([pad_mask, rmask], axis=1)
    return tokens, mask
