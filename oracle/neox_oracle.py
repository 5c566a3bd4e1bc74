"""CPU oracle for the PPO rollout + rescoring path.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.

What it computes (paper passages in brackets):
  * the policy forward pass: the GPT-NeoX / Pythia decoder the paper takes from the
    `transformers` library [General Details, "Setup -> Tech stack"], with dropout off
    ["Model -> Disable dropout"];
  * rollout: left-padded queries [Dataset Details, "left pad the queries"], a fixed number of
    tokens sampled at temperature 0.7 [PPO hyperparameter table, "Sampling Temperature"], then
    truncation at the first EOS with padding after it [PPO Details, "EOS trick", steps 1-2];
  * rescoring: a teacher-forced forward over the (B, query+response) batch with the attention mask
    adjusted for the left padding [Reward Model Details, "Minor numerical differences ..."],
    giving the per-token log-probabilities of the KL term [Preliminaries, Eq. (RL)] and PPO ratio,
    and per-token values from a scalar linear head [Preliminaries, Step 2; PPO Details, "Value
    model initializes from the reward model"].

Everything is float64 numpy on the float32 weight values it is handed; `@` (matmul),
scipy.special.erf and numpy's exp/log are the only library steps.  The one place where floating
point decides an integer -- the sampled token -- is taken in float32, the precision of the GPU
sampler: float32(logit)/float32(T) + float32(gumbel), ties to the lowest id.

The paper does not describe the architecture, the noise generator or the index conventions; the
readings taken here are listed where each function implements them.

Pins (tests/test_oracle_*.py): HF transformers GPT-NeoX forward on a tiny random model, brute
force no-cache decoding, closed forms (zero output embedding, zero-layer model, single token),
left-padding invariance, causality, Gumbel-max frequency test against softmax, rope identities.
Unpinned against paper-printed numbers: the paper prints none for this path.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64
_U64 = np.uint64


# ----------------------------------------------------------------------------------------------
# weights access: float32 storage -> float64 on use
# ----------------------------------------------------------------------------------------------
class OracleModel:
    """Holds the name -> float32 array dict and hands out float64 views of single tensors."""

    def __init__(self, weights: dict, cfg, cache_f64: bool = True):
        self.w = weights
        self.cfg = cfg
        self._cache = {} if cache_f64 else None

    def get(self, name: str) -> np.ndarray:
        if self._cache is not None and name in self._cache:
            return self._cache[name]
        a = np.asarray(self.w[name], dtype=F64)
        if self._cache is not None:
            self._cache[name] = a
        return a

    def layer(self, l: int, name: str) -> np.ndarray:
        return self.get(f"layers.{l}.{name}")


# ----------------------------------------------------------------------------------------------
# building blocks of the decoder (GPT-NeoX as used through `transformers`, Tech stack)
# ----------------------------------------------------------------------------------------------
def layer_norm(x, g, b, eps):
    """Per-row (x - mean) / sqrt(biased variance + eps) * g + b."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    return xc / np.sqrt(var + eps) * g + b


def gelu_erf(x):
    """Exact GELU: x * Phi(x)."""
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def rope(u, pos, rotary_dims, base):
    """Partial rotary embedding.  u: [n, H, hd]; pos: [n] integer positions.

    Only dims [0, r) of each head rotate; dim i < r/2 pairs with dim i + r/2 and the pair turns by
    the angle pos * base^(-2i/r)."""
    r = rotary_dims
    half = r // 2
    inv_freq = base ** (-(np.arange(half, dtype=F64) * 2.0) / r)
    ang = np.asarray(pos, dtype=F64)[:, None] * inv_freq[None, :]  # [n, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    out = u.copy()
    a = u[..., :half]
    b = u[..., half:r]
    out[..., :half] = a * c - b * s
    out[..., half:r] = b * c + a * s
    return out


def attention(q, q_pos, K, V, k_pos, head_dim):
    """softmax(q k^T / sqrt(hd)) v over the keys whose position is <= the query's.

    q: [n, H, hd] at positions q_pos [n]; K, V: [m, H, hd] at positions k_pos [m]
    (all of one sequence; padding never enters K/V, so no pad term exists)."""
    n, H, hd = q.shape
    allowed = np.asarray(k_pos)[None, :] <= np.asarray(q_pos)[:, None]  # [n, m]
    out = np.empty_like(q)
    scale = 1.0 / math.sqrt(head_dim)
    for h in range(H):
        s = (q[:, h, :] @ K[:, h, :].T) * scale
        s = np.where(allowed, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ V[:, h, :]
    return out


def decoder_layer(m: OracleModel, l: int, x, pos, past=None):
    """x <- x + Attn(LN1(x)) + MLP(LN2(x))  (parallel residual).

    x: [n, d] rows of ONE sequence at positions pos.  past = (K, V, k_pos) of earlier positions of
    the same sequence or None.  Returns new x and the extended (K, V, k_pos)."""
    cfg = m.cfg
    H, hd, d = cfg.n_heads, cfg.head_dim, cfg.d_model
    a = layer_norm(x, m.layer(l, "ln1_g"), m.layer(l, "ln1_b"), cfg.ln_eps)
    mm = layer_norm(x, m.layer(l, "ln2_g"), m.layer(l, "ln2_b"), cfg.ln_eps)
    qkv = a @ m.layer(l, "w_qkv").T + m.layer(l, "b_qkv")  # rows of w_qkv: q heads | k heads | v heads
    n = x.shape[0]
    q = qkv[:, 0 * d:1 * d].reshape(n, H, hd)
    k = qkv[:, 1 * d:2 * d].reshape(n, H, hd)
    v = qkv[:, 2 * d:3 * d].reshape(n, H, hd)
    q = rope(q, pos, cfg.rotary_dims, cfg.rope_base)
    k = rope(k, pos, cfg.rotary_dims, cfg.rope_base)
    if past is not None:
        K = np.concatenate([past[0], k], axis=0)
        V = np.concatenate([past[1], v], axis=0)
        k_pos = np.concatenate([past[2], np.asarray(pos)])
    else:
        K, V, k_pos = k, v, np.asarray(pos)
    o = attention(q, pos, K, V, k_pos, hd).reshape(n, d)
    attn = o @ m.layer(l, "w_o").T + m.layer(l, "b_o")
    hid = gelu_erf(mm @ m.layer(l, "w_fc1").T + m.layer(l, "b_fc1"))
    mlp = hid @ m.layer(l, "w_fc2").T + m.layer(l, "b_fc2")
    return x + attn + mlp, (K, V, k_pos)


def forward_sequence(m: OracleModel, token_ids, pos, cache=None):
    """Run all layers over the rows of one sequence.

    token_ids, pos: [n].  cache: list (per layer) of (K, V, k_pos) from earlier positions, or None.
    Returns (x [n, d] before the final LayerNorm, new cache)."""
    x = m.get("embed_in")[np.asarray(token_ids)]
    new_cache = []
    for l in range(m.cfg.n_layers):
        x, kv = decoder_layer(m, l, x, pos, None if cache is None else cache[l])
        new_cache.append(kv)
    return x, new_cache


def heads(m: OracleModel, x):
    """Final LayerNorm, then the LM head (no bias, untied) and the scalar value head."""
    cfg = m.cfg
    h = layer_norm(x, m.get("lnf_g"), m.get("lnf_b"), cfg.ln_eps)
    logits = h @ m.get("embed_out").T
    values = h @ m.get("value_w") + float(m.w["value_b"])
    return logits, values


def log_softmax_at(logits, temperature, target):
    """log softmax(logits / T)[target] for one row (float64)."""
    z = logits / float(np.float32(temperature))
    mx = z.max()
    return z[target] - (mx + math.log(np.exp(z - mx).sum()))


# ----------------------------------------------------------------------------------------------
# sampling noise: a counter-based hash keyed by (seed, sequence, step, token id)
# ----------------------------------------------------------------------------------------------
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)


def _fmix(x):
    """64-bit xor-shift-multiply finaliser (two multiply rounds) on a uint64 array."""
    with np.errstate(over="ignore"):
        x = x ^ (x >> _U64(30))
        x = x * _M1
        x = x ^ (x >> _U64(27))
        x = x * _M2
        x = x ^ (x >> _U64(31))
    return x


def noise_bits(seed: int, seq: int, step: int, vocab: int) -> np.ndarray:
    """Top 32 bits of the hash for every token id of one (sequence, step): uint32 [vocab].

    key_row = fmix(seed + G*(seq+1)); key_step = fmix(key_row + G*(step+1));
    h(v) = fmix(key_step + G*(v+1)), all arithmetic modulo 2^64."""
    with np.errstate(over="ignore"):
        kr = _fmix(np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=_U64) + _GOLDEN * _U64(seq + 1))
        ks = _fmix(kr + _GOLDEN * _U64(step + 1))
        v = np.arange(1, vocab + 1, dtype=_U64)
        h = _fmix(ks + _GOLDEN * v)
    return (h >> _U64(32)).astype(np.uint32)


def gumbel_from_bits(k: np.ndarray) -> np.ndarray:
    """Standard Gumbel variates from 32-bit integers: u = (k + 1/2) / 2^32 lies strictly inside
    (0, 1); g = -ln(-ln u).  Computed in float64, returned as float32 (the sampler's precision)."""
    u = (k.astype(F64) + 0.5) * 2.0 ** -32
    return (-np.log(-np.log(u))).astype(np.float32)


def sample_token(logits, temperature, g32):
    """Gumbel-max draw from softmax(logits / T): argmax_v (z_v + g_v), ties to the lowest id.

    The decision is taken in float32.  Returns (token, log-prob of it under softmax(logits/T),
    perturbed float32 scores)."""
    t32 = np.float32(temperature)
    z32 = logits.astype(np.float32) / t32
    score = z32 + g32
    tok = int(np.argmax(score))  # numpy returns the first maximum
    return tok, log_softmax_at(logits, temperature, tok), score


# ----------------------------------------------------------------------------------------------
# the two entry points
# ----------------------------------------------------------------------------------------------
def _row_span(mask_row):
    """Real tokens of a row form one contiguous run [start, end); returns (start, end)."""
    idx = np.flatnonzero(mask_row)
    if idx.size == 0:
        return 0, 0
    start, end = int(idx[0]), int(idx[-1]) + 1
    if end - start != idx.size:
        raise ValueError("mask row is not one contiguous run of real tokens")
    return start, end


def rollout_generate(m: OracleModel, queries, pad_mask, seed, temperature, max_new_tokens, seq_id_base=0):
    """Sample `max_new_tokens` tokens per row after a left-padded query.

    Positions count real tokens only (a row's first real token is position 0), and padding never
    enters the attention.  Step t of row b draws noise keyed (seed, seq_id_base+b, t, v).  After
    the first EOS a row emits pad_id with log-prob 0; lengths[b] counts the tokens up to and
    including EOS (max_new_tokens if none).  One prefill pass plus max_new_tokens-1 single-token
    passes: the last sampled token is never fed back.

    Returns tokens int32 [B, Lq+N] (query copied), logprobs float64 [B, N], lengths int32 [B]."""
    cfg = m.cfg
    queries = np.asarray(queries)
    pad_mask = np.asarray(pad_mask)
    B, Lq = queries.shape
    N = int(max_new_tokens)
    tokens = np.full((B, Lq + N), cfg.pad_id, dtype=np.int32)
    tokens[:, :Lq] = queries
    logprobs = np.zeros((B, N), dtype=F64)
    lengths = np.full((B,), N, dtype=np.int32)
    for b in range(B):
        start, end = _row_span(pad_mask[b])
        if end != Lq and end != 0:
            raise ValueError("queries must be left-padded")
        n = end - start
        if n == 0:  # an all-pad row has nothing to condition on: emitted as all pad, length 0
            lengths[b] = 0
            continue
        x, cache = forward_sequence(m, queries[b, start:end], np.arange(n))
        logits, _ = heads(m, x[-1:])
        finished = False
        for t in range(N):
            g = gumbel_from_bits(noise_bits(seed, seq_id_base + b, t, cfg.vocab))
            tok, lp, _ = sample_token(logits[0], temperature, g)
            if not finished:
                tokens[b, Lq + t] = tok
                logprobs[b, t] = lp
                if tok == cfg.eos_id:
                    finished = True
                    lengths[b] = t + 1
            if t < N - 1:
                # the paper keeps sampling past EOS and truncates afterwards; what is fed back after
                # EOS cannot change any kept output, so the sampled token is fed either way
                x, cache = forward_sequence(m, np.array([tok]), np.array([n + t]), cache)
                logits, _ = heads(m, x)
    return tokens, logprobs, lengths


def score_sequences(m: OracleModel, tokens, mask, temperature):
    """Teacher-forced pass over a (B, L) batch.

    logprobs[b, t] = log softmax(logits[b, t-1] / T)[tokens[b, t]] for every real t whose
    predecessor is real, 0 elsewhere.  values[b, t] = value head at t (unshifted) for real t,
    0 elsewhere.  Returns two float64 [B, L] arrays."""
    tokens = np.asarray(tokens)
    mask = np.asarray(mask)
    B, L = tokens.shape
    logprobs = np.zeros((B, L), dtype=F64)
    values = np.zeros((B, L), dtype=F64)
    for b in range(B):
        start, end = _row_span(mask[b])
        n = end - start
        if n == 0:
            continue
        x, _ = forward_sequence(m, tokens[b, start:end], np.arange(n))
        logits, val = heads(m, x)
        values[b, start:end] = val
        for i in range(1, n):
            logprobs[b, start + i] = log_softmax_at(logits[i - 1], temperature, int(tokens[b, start + i]))
    return logprobs, values


def logits_rows(m: OracleModel, tokens, mask, rows_bt):
    """Raw (pre-temperature) logits at the listed (row, column) pairs: float64 [n, vocab]."""
    tokens = np.asarray(tokens)
    mask = np.asarray(mask)
    out = np.zeros((len(rows_bt), m.cfg.vocab), dtype=F64)
    by_row = {}
    for i, (b, t) in enumerate(rows_bt):
        by_row.setdefault(int(b), []).append((i, int(t)))
    for b, items in by_row.items():
        start, end = _row_span(mask[b])
        x, _ = forward_sequence(m, tokens[b, start:end], np.arange(end - start))
        logits, _ = heads(m, x)
        for i, t in items:
            if not (start <= t < end):
                raise ValueError("requested a padded position")
            out[i] = logits[t - start]
    return out


def verify_rollout(m: OracleModel, tokens, pad_mask, seed, temperature, max_new_tokens, rows=None,
                   seq_id_base=0):
    """Replay a rollout teacher-forced on ITS OWN tokens and grade each sampled token.

    For every checked row b and step t (up to and including the first EOS) the oracle's perturbed
    float32 scores are computed on the prefix the rollout actually produced.  Returns a list of
    dicts with: row, step, token, argmax (the oracle's choice), deficit (= max score -
    score[token], 0 when they agree), margin (oracle's top-1 minus top-2 score) and logprob (the
    oracle's log-prob of the rollout's token).  A step is acceptable when deficit <= the near-tie
    threshold, which is how "identical tokens except where the oracle's top-2 margin is tiny" is
    checked without one legal divergence cascading."""
    cfg = m.cfg
    tokens = np.asarray(tokens)
    pad_mask = np.asarray(pad_mask)
    B, Lq = pad_mask.shape
    N = int(max_new_tokens)
    rows = range(B) if rows is None else rows
    report = []
    for b in rows:
        start, end = _row_span(pad_mask[b])
        n = end - start
        if n == 0:
            continue
        resp = tokens[b, Lq:Lq + N]
        eos = np.flatnonzero(resp == cfg.eos_id)
        length = int(eos[0]) + 1 if eos.size else N
        seq = np.concatenate([tokens[b, start:Lq], resp[:length]])
        x, _ = forward_sequence(m, seq, np.arange(seq.size))
        logits, _ = heads(m, x[n - 1:n - 1 + length])
        for t in range(length):
            g = gumbel_from_bits(noise_bits(seed, seq_id_base + b, t, cfg.vocab))
            arg, _, score = sample_token(logits[t], temperature, g)
            tok = int(resp[t])
            top2 = np.partition(score, -2)[-2:]
            report.append(dict(row=int(b), step=t, token=tok, argmax=arg,
                               deficit=float(score[arg] - score[tok]),
                               margin=float(top2[1] - top2[0]),
                               logprob=log_softmax_at(logits[t], temperature, tok)))
    return report
