"""Decoder-only transformer forward in numpy fp64 (test infrastructure).

The base model M of Section 4.1 (input embedding V, output embedding U, next
token distribution p_M) is, for this repository's configurations, a pre-norm
Llama-style decoder: RMSNorm, multi-head attention with rotary position
embedding (rotate-half pairing), SwiGLU feed-forward, no biases, a final
RMSNorm and an untied output embedding.  A model call on an input block of
shape (k, w+1) whose context is KV-cached (Section 3) is `forward_block`.

Weights are read as stored (fp32 values, bf16-representable for bf16 models)
and widened to fp64; no activation is rounded to a lower precision.  The
widening is exact, so when it happens changes no result: by default every
matrix is widened once in the constructor; `widen_at_use=True` keeps the layer
matrices as stored and widens one layer at a time inside the forward pass,
which bounds memory for deep, wide models.
"""
from __future__ import annotations

import numpy as np


class KVCache:
    """Keys and values of the cached context, one pair of arrays per layer,
    shapes [P, n_kv_heads, head_dim].  Section 3: every context token but the
    final one is cached."""

    def __init__(self, n_layers, n_kv_heads, head_dim):
        self.k = [np.zeros((0, n_kv_heads, head_dim)) for _ in range(n_layers)]
        self.v = [np.zeros((0, n_kv_heads, head_dim)) for _ in range(n_layers)]

    def __len__(self):
        return self.k[0].shape[0]

    def append(self, layer, k_new, v_new):
        self.k[layer] = np.concatenate([self.k[layer], k_new], axis=0)
        self.v[layer] = np.concatenate([self.v[layer], v_new], axis=0)

    def truncated(self, n):
        c = KVCache(len(self.k), self.k[0].shape[1], self.k[0].shape[2])
        c.k = [a[:n].copy() for a in self.k]
        c.v = [a[:n].copy() for a in self.v]
        return c


class Model:
    def __init__(self, desc: dict, weights: dict, widen_at_use: bool = False):
        self.desc = dict(desc)
        f64 = lambda a: np.asarray(a, dtype=np.float64)
        self.tok_emb = f64(weights["tok_emb"])        # V  (input embedding), [vocab][d]
        self.unemb = f64(weights["unemb"])            # U^T (output embedding), [vocab][d]
        self.final_norm = f64(weights["final_norm"])
        self.widen_at_use = bool(widen_at_use)
        if self.widen_at_use:
            self.layers = [dict(lw) for lw in weights["layers"]]          # as stored; widened per layer in the forward pass
        else:
            self.layers = [{k: f64(v) for k, v in lw.items()} for lw in weights["layers"]]
        self.L = desc["n_layers"]
        self.H = desc["n_heads"]
        self.Hkv = desc["n_kv_heads"]
        self.hd = desc["head_dim"]
        self.eps = float(desc["rms_eps"])
        self.theta = float(desc["rope_theta"])

    # -- layer pieces -------------------------------------------------------
    def rmsnorm(self, x, g):
        """x * rsqrt(mean(x^2) + eps) * g over the last axis."""
        ms = np.mean(x * x, axis=-1, keepdims=True)
        return x / np.sqrt(ms + self.eps) * g

    def rope(self, x, pos):
        """Rotary embedding, rotate-half pairing: element i pairs with i + hd/2,
        angle pos * theta^(-2i/hd).  x: [..., T, heads, hd], pos: [T]."""
        half = self.hd // 2
        inv = self.theta ** (-np.arange(half, dtype=np.float64) * 2.0 / self.hd)
        ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]      # [T, half]
        c = np.cos(ang)[:, None, :]
        s = np.sin(ang)[:, None, :]
        x1, x2 = x[..., :half], x[..., half:]
        return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)

    @staticmethod
    def silu(x):
        with np.errstate(over="ignore"):            # exp(-x) -> inf for very negative x gives x / inf = -0
            return x / (1.0 + np.exp(-x))

    def _expand_kv(self, a):
        """[..., Hkv, hd] -> [..., H, hd] (query head h reads kv head h // (H/Hkv))."""
        if self.Hkv == self.H:
            return a
        return np.repeat(a, self.H // self.Hkv, axis=-2)

    # -- the model call of Section 3 -----------------------------------------
    def forward_block(self, tokens, cache: KVCache | None = None, want_logits=True):
        """Model call on a block of shape (k, c): row r holds c tokens at positions
        P .. P+c-1, where P = len(cache) context tokens are KV-cached and shared
        by every row ("repeat the context to form k identical rows", Section 4.1).
        Token (r, j) attends to the cached context and to (r, 0..j).

        Returns (logits [k, c, vocab] or None, block_kv) where block_kv[layer] is
        (K [k, c, Hkv, hd], V [k, c, Hkv, hd]) for the block's own positions.
        """
        tokens = np.asarray(tokens)
        k, c = tokens.shape
        P = 0 if cache is None else len(cache)
        pos = np.arange(P, P + c)
        h = self.tok_emb[tokens]                                  # [k, c, d]
        scale = 1.0 / np.sqrt(self.hd)
        causal = np.tril(np.ones((c, c), dtype=bool))             # [query j, key s]: s <= j
        block_kv = []
        for li, lw in enumerate(self.layers):
            if self.widen_at_use:
                lw = {name: np.asarray(a, dtype=np.float64) for name, a in lw.items()}
            x = self.rmsnorm(h, lw["attn_norm"])
            q = (x @ lw["wq"].T).reshape(k, c, self.H, self.hd)
            kk = (x @ lw["wk"].T).reshape(k, c, self.Hkv, self.hd)
            vv = (x @ lw["wv"].T).reshape(k, c, self.Hkv, self.hd)
            q = self.rope(q, pos)
            kk = self.rope(kk, pos)
            block_kv.append((kk, vv))
            kb, vb = self._expand_kv(kk), self._expand_kv(vv)
            # scores and weighted sums as stacked matrix products, heads moved in front of the token axis:
            # q_h [k, H, c, hd]; keys and values of the block [k, H, c, hd], of the cached context [H, P, hd]
            q_h = q.transpose(0, 2, 1, 3)
            kb_h, vb_h = kb.transpose(0, 2, 1, 3), vb.transpose(0, 2, 1, 3)
            s_blk = (q_h @ kb_h.transpose(0, 1, 3, 2)) * scale      # [k, H, c (query j), c (key s)]
            s_blk = np.where(causal[None, None], s_blk, -np.inf)
            if P > 0:
                kp_h = self._expand_kv(cache.k[li]).transpose(1, 0, 2)       # [H, P, hd]
                vp_h = self._expand_kv(cache.v[li]).transpose(1, 0, 2)
                s_pre = (q_h @ kp_h.transpose(0, 2, 1)[None]) * scale       # [k, H, c, P]
                s = np.concatenate([s_pre, s_blk], axis=-1)
            else:
                s = s_blk
            s = s - s.max(axis=-1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=-1, keepdims=True)
            a = p[..., P:] @ vb_h                                    # [k, H, c, hd]
            if P > 0:
                a = a + p[..., :P] @ vp_h[None]
            a = a.transpose(0, 2, 1, 3)                              # [k, c, H, hd]
            h = h + a.reshape(k, c, self.H * self.hd) @ lw["wo"].T
            x = self.rmsnorm(h, lw["mlp_norm"])
            h = h + (self.silu(x @ lw["w_gate"].T) * (x @ lw["w_up"].T)) @ lw["w_down"].T
        logits = None
        if want_logits:
            logits = self.rmsnorm(h, self.final_norm) @ self.unemb.T
        return logits, block_kv

    def forward_full(self, tokens):
        """Logits [n, vocab] of the whole sequence with no cache at all."""
        logits, _ = self.forward_block(np.asarray(tokens)[None, :], None)
        return logits[0]


def greedy_argmax(logits):
    """Greedy next-token choice; equal logits go to the lowest token id."""
    return np.argmax(logits, axis=-1).astype(np.int32)       # numpy returns the first maximum
