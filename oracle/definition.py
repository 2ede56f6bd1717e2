"""Definition-level transformer in numpy fp64.  TEST INFRASTRUCTURE ONLY.

No KV cache and no early exit: the whole token sequence is pushed through every layer at once
with an explicit T x T causal mask, which is the textbook definition of what a decoder-only
model computes (Sec. III: hidden states h_t^(l), l = 1..L, final head g_L, Eq. 1).  The C oracle's
incremental decoding is pinned to this file; this file's own pieces are pinned to library routines
in tests/test_oracle_primitives.py.

Conventions (the paper treats the backbone as a black box; these follow the stated workload
shapes): pre-norm residual blocks, RMSNorm with gain, rotary embedding on pairs (i, i + hd/2) with
angle pos * base^(-2i/hd), grouped-query attention where consecutive query heads share a KV head,
scores scaled by 1/sqrt(hd), SwiGLU MLP, no biases.
"""
from __future__ import annotations

import numpy as np


def widen(w: np.ndarray) -> np.ndarray:
    """matrix -> float64 (uint16 arrays hold bf16 bit patterns)"""
    if w.dtype == np.uint16:
        return (w.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return w.astype(np.float64)


def rmsnorm(x: np.ndarray, gamma: np.ndarray, eps: float) -> np.ndarray:
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * gamma.astype(np.float64)


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """x: [T, heads, hd]; pos: [T]"""
    hd = x.shape[-1]
    half = hd // 2
    theta = base ** (-2.0 * np.arange(half) / hd)
    ang = pos[:, None].astype(np.float64) * theta[None, :]          # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """q: [T, nq, hd]; k, v: [T, nkv, hd] -> [T, nq, hd]; query head h reads kv head h // (nq/nkv)"""
    T, nq, hd = q.shape
    group = nq // k.shape[1]
    out = np.empty_like(q)
    mask = np.tril(np.ones((T, T), dtype=bool))
    for h in range(nq):
        kh, vh = k[:, h // group, :], v[:, h // group, :]
        s = (q[:, h, :] @ kh.T) / np.sqrt(hd)
        s = np.where(mask, s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=-1, keepdims=True)
        out[:, h, :] = p @ vh
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def bf16_storage(x: np.ndarray) -> np.ndarray:
    """values as they read back from a bf16 store (library cast: fp32 -> bf16, nearest even)"""
    import torch
    return torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


def hidden_states(shape, weights: dict, tokens: np.ndarray, kv_bf16: bool = False) -> np.ndarray:
    """h[l, t, :] for l = 0..L (l = 0 is the embedding, l >= 1 is the residual stream after
    block l) of every position of `tokens`, all computed in one full-sequence pass.
    kv_bf16: keys (after the rotary embedding) and values pass through a bf16 store, as they do
    in a bf16 KV cache."""
    T = len(tokens)
    L, d, hd = shape.n_layers, shape.d_model, shape.head_dim
    nq, nkv = shape.n_q_heads, shape.n_kv_heads
    pos = np.arange(T)
    h = widen(weights["embed"])[np.asarray(tokens)]
    hs = np.empty((L + 1, T, d))
    hs[0] = h
    for l in range(L):
        n = rmsnorm(h, weights["attn_norm"][l], shape.rms_eps)
        q = (n @ widen(weights["wq"][l]).T).reshape(T, nq, hd)
        k = (n @ widen(weights["wk"][l]).T).reshape(T, nkv, hd)
        v = (n @ widen(weights["wv"][l]).T).reshape(T, nkv, hd)
        q, k = rope(q, pos, shape.rope_base), rope(k, pos, shape.rope_base)
        if kv_bf16:
            k, v = bf16_storage(k), bf16_storage(v)
        a = causal_attention(q, k, v).reshape(T, nq * hd)
        h = h + a @ widen(weights["wo"][l]).T
        n = rmsnorm(h, weights["mlp_norm"][l], shape.rms_eps)
        act = silu(n @ widen(weights["wg"][l]).T) * (n @ widen(weights["wu"][l]).T)
        h = h + act @ widen(weights["wd"][l]).T
        hs[l + 1] = h
    return hs


def final_logits(shape, weights: dict, h_last: np.ndarray) -> np.ndarray:
    """g_L of Eq. 1 on hidden states [.., d] of the last layer"""
    n = rmsnorm(h_last, weights["final_norm"], shape.rms_eps)
    return n @ widen(weights["lm_head"]).T


def lens_logits(shape, weights: dict, h_e: np.ndarray) -> np.ndarray:
    """g_e of Eq. 2: unembedding of the normed, affinely translated intermediate state"""
    u = h_e + h_e @ widen(weights["lens_a"]).T + weights["lens_b"].astype(np.float64)
    n = rmsnorm(u, weights["lens_norm"], shape.rms_eps)
    return n @ widen(weights["lens_head"]).T


def greedy_standard(shape, weights: dict, prompt: np.ndarray, n_new: int):
    """Standard greedy decoding by full recomputation at every step: the input of the first step
    is the last prompt token.  Returns (tokens[n_new], logits[n_new, V])."""
    seq = list(int(t) for t in prompt)
    toks, logs = [], []
    for _ in range(n_new):
        hs = hidden_states(shape, weights, np.array(seq))
        lg = final_logits(shape, weights, hs[-1, -1])
        y = int(np.argmax(lg))
        toks.append(y)
        logs.append(lg)
        seq.append(y)
    return np.array(toks), np.array(logs)
