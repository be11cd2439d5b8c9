"""Seeded synthetic inputs: model shapes, weights and prompt token streams.

This module only *generates data*.  It holds none of the method's arithmetic
(no transformer maths, no drafting, no acceptance rule): the CPU oracle and the
HIP library both consume the buffers produced here and share nothing else.

The shapes follow the benchmark configurations of this repository (tiny fp32
decoder, small bf16 decoder, 7B-shaped bf16 decoder, long-context stress,
large-vocabulary sweep).  The token streams stand in for the paper's
benchmark prompts (Section 5, "Datasets and models"), the random-normal
weights for its trained checkpoints; neither is available offline.
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# model shapes
# --------------------------------------------------------------------------

def _model(n_layers, d_model, n_heads, d_ffn, vocab, dtype, head_dim=None):
    return dict(
        n_layers=n_layers, d_model=d_model, n_heads=n_heads, n_kv_heads=n_heads,
        head_dim=head_dim if head_dim is not None else d_model // n_heads,
        d_ffn=d_ffn, vocab=vocab, dtype=dtype, rms_eps=1e-5, rope_theta=10000.0,
    )


MODELS = {
    "tiny":   _model(2, 128, 4, 512, 512, "f32"),
    "small":  _model(12, 768, 12, 3072, 32000, "bf16"),
    "7b":     _model(32, 4096, 32, 14336, 32000, "bf16"),
    "3b":     _model(28, 3072, 24, 8192, 128256, "bf16"),
}

# run recipes: which model, prompt recipe and draft configuration each benchmark
# configuration uses.  q = N-1 query tokens for a "context N-gram".
RUNS = {
    "cfg1": dict(model="tiny", prompt_len=128, prompt="motif", k=4, w=3,
                 k_ctx_max=2, q_min=2, q_max=2, n_gen=64),
    "cfg2": dict(model="small", prompt_len=1024, prompt="spans", copied=0.30, k=8, w=4,
                 k_ctx_max=8, q_min=2, q_max=2, n_gen=256),
    "cfg3": dict(model="7b", prompt_len=2048, prompt="spans", copied=0.30, k=10, w=5,
                 k_ctx_max=5, q_min=3, q_max=3, n_gen=512),
    "cfg4": dict(model="7b", prompt_len=16384, prompt="spans", copied=0.50, k=16, w=6,
                 k_ctx_max=16, q_min=1, q_max=3, n_gen=64),
    "cfg5": dict(model="3b", prompt_len=4096, prompt="spans", copied=0.30, k=10, w=5,
                 k_ctx_max=10, q_min=2, q_max=2, n_gen=64),
}


def reduced_layers(model: dict, n_layers: int) -> dict:
    """Same widths, fewer layers (a twin the CPU oracle can run end to end)."""
    m = dict(model)
    m["n_layers"] = n_layers
    return m


# --------------------------------------------------------------------------
# bf16 storage helpers (round-to-nearest-even from fp32)
# --------------------------------------------------------------------------

def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 values (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16-representable fp32 value."""
    return bf16_to_f32(bf16_bits(a))


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------

LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")


def layer_shapes(m: dict) -> dict:
    d, f = m["d_model"], m["d_ffn"]
    dq = m["n_heads"] * m["head_dim"]
    dkv = m["n_kv_heads"] * m["head_dim"]
    return dict(attn_norm=(d,), wq=(dq, d), wk=(dkv, d), wv=(dkv, d), wo=(d, dq),
                mlp_norm=(d,), w_gate=(f, d), w_up=(f, d), w_down=(d, f))


def make_weights(m: dict, seed: int = 0, std: float = 0.02, random_gains: bool = False) -> dict:
    """Random-normal(0, std^2) matrices, row-major [out][in], as fp32 arrays.

    For a bf16 model every value is rounded to bf16 first, so the returned fp32
    arrays hold exactly the stored values.  Norm gains are 1 unless
    ``random_gains`` (then 1 + 0.1 N(0,1), to exercise the gain path).
    Returns {"tok_emb", "unemb", "final_norm", "layers": [ {name: array} ]}.
    """
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x77]))
    rnd = bf16_round if m["dtype"] == "bf16" else (lambda a: a)

    def mat(shape):
        return rnd((rng.standard_normal(shape, dtype=np.float32) * np.float32(std)))

    def gain(shape):
        if random_gains:
            return rnd((1.0 + 0.1 * rng.standard_normal(shape)).astype(np.float32))
        return np.ones(shape, dtype=np.float32)

    V, d = m["vocab"], m["d_model"]
    w = dict(tok_emb=mat((V, d)), unemb=mat((V, d)), final_norm=gain((d,)), layers=[])
    shapes = layer_shapes(m)
    for _ in range(m["n_layers"]):
        lw = {}
        for name in LAYER_TENSORS:
            lw[name] = gain(shapes[name]) if name.endswith("norm") else mat(shapes[name])
        w["layers"].append(lw)
    return w


# --------------------------------------------------------------------------
# prompts
# --------------------------------------------------------------------------

def zipf_cdf(vocab: int, s: float = 1.1) -> np.ndarray:
    p = 1.0 / np.arange(1, vocab + 1, dtype=np.float64) ** s
    c = np.cumsum(p)
    return c / c[-1]


def _zipf_draw(rng, cdf, n):
    u = rng.random(n)
    return np.minimum(np.searchsorted(cdf, u, side="left"), len(cdf) - 1).astype(np.int32)


def prompt_motif(vocab: int, n: int = 128, seed: int = 1, motif_len: int = 8, period: int = 32) -> np.ndarray:
    """Zipf(1.1) stream with one motif written at offsets 0, period, 2*period, ..."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x51]))
    cdf = zipf_cdf(vocab)
    x = _zipf_draw(rng, cdf, n)
    motif = _zipf_draw(rng, cdf, motif_len)
    for o in range(0, n - motif_len + 1, period):
        x[o:o + motif_len] = motif
    return x


def prompt_spans(vocab: int, n: int, copied: float = 0.30, seed: int = 1) -> np.ndarray:
    """Zipf(1.1) stream in which about a fraction ``copied`` of the positions
    belongs to spans of 4..16 tokens copied from a uniformly chosen earlier start."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x52]))
    cdf = zipf_cdf(vocab)
    p_start = copied / (copied + 10.0 * (1.0 - copied))   # mean span length is 10
    x = np.empty(n, dtype=np.int32)
    fresh = _zipf_draw(rng, cdf, n)
    i = 0
    while i < n:
        if i >= 16 and rng.random() < p_start:
            ln = int(rng.integers(4, 17))
            src = int(rng.integers(0, i))
            for t in range(ln):                      # src + t < i always holds: a forward, possibly overlapping copy
                if i >= n:
                    break
                x[i] = x[src + t]
                i += 1
        else:
            x[i] = fresh[i]
            i += 1
    return x


def make_prompt(run: dict, vocab: int, seed: int = 1) -> np.ndarray:
    if run["prompt"] == "motif":
        return prompt_motif(vocab, run["prompt_len"], seed)
    return prompt_spans(vocab, run["prompt_len"], run["copied"], seed)


def make_weights_device(m: dict, seed: int = 0, std: float = 0.02, device: str = "cuda") -> dict:
    """Same structure as make_weights, generated on the device with torch's seeded generator
    (for shapes too large to draw on the host in reasonable time).  The stream differs from
    make_weights'; tensors are of the model's storage type."""
    import torch
    dt = torch.bfloat16 if m["dtype"] == "bf16" else torch.float32
    gen = torch.Generator(device=device)
    gen.manual_seed(1000003 * seed + 0x77)

    def mat(shape):
        return (torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * std).to(dt)

    def gain(shape):
        return torch.ones(shape, device=device, dtype=dt)

    V, d = m["vocab"], m["d_model"]
    w = dict(tok_emb=mat((V, d)), unemb=mat((V, d)), final_norm=gain((d,)), layers=[])
    shapes = layer_shapes(m)
    for _ in range(m["n_layers"]):
        w["layers"].append({name: (gain(shapes[name]) if name.endswith("norm") else mat(shapes[name]))
                            for name in LAYER_TENSORS})
    return w
