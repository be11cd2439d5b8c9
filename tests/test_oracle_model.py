"""Pins for the oracle's transformer forward: closed forms, invariants and
special cases that reduce to textbook or library routines.  CPU only."""
import copy

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import Model, KVCache, prefill


def tiny(seed=0, **over):
    desc = dict(si.MODELS["tiny"])
    desc.update(over)
    return desc, si.make_weights(desc, seed=seed, random_gains=True)


# ---------------------------------------------------------------------------
# RMSNorm, SiLU, RoPE: closed forms
# ---------------------------------------------------------------------------

def test_rmsnorm_constant_vector_closed_form():
    desc, w = tiny()
    m = Model(desc, w)
    for c in (1e-4, 0.5, 3.0):
        x = np.full((1, 8), c)
        out = m.rmsnorm(x, np.ones(8))
        # mean(x^2) = c^2, so every element is c / sqrt(c^2 + eps): eps sits inside the root
        assert np.allclose(out, c / np.sqrt(c * c + desc["rms_eps"]), rtol=1e-14)
    assert np.all(m.rmsnorm(np.zeros((2, 8)), np.ones(8)) == 0.0)


def test_rmsnorm_unit_rms_and_gain():
    desc, w = tiny(rms_eps=0.0)
    m = Model(desc, w)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64))
    g = rng.standard_normal(64)
    y = m.rmsnorm(x, np.ones(64))
    assert np.allclose(np.mean(y * y, axis=-1), 1.0, rtol=1e-13)
    assert np.allclose(m.rmsnorm(7.3 * x, np.ones(64)), y, rtol=1e-13)     # scale invariant at eps = 0
    assert np.allclose(m.rmsnorm(x, g), y * g, rtol=1e-13)


def test_silu_limits():
    assert Model.silu(np.array([0.0]))[0] == 0.0
    assert np.isclose(Model.silu(np.array([40.0]))[0], 40.0, rtol=1e-15)
    assert abs(Model.silu(np.array([-40.0]))[0]) < 1e-15
    # silu(x) - silu(-x) = x  (x*sigmoid(x) + x*sigmoid(-x) = x)
    x = np.linspace(-5, 5, 11)
    assert np.allclose(Model.silu(x) - Model.silu(-x), x, atol=1e-14)


def test_rope_is_complex_rotation_on_half_pairs():
    desc, w = tiny()
    m = Model(desc, w)
    hd = m.hd
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, 3, hd))           # [T, heads, hd]
    pos = np.array([0, 1, 2, 17, 100, 4095])
    y = m.rope(x, pos)
    # textbook form: z_i = x_i + 1j * x_{i+hd/2} is multiplied by exp(1j * pos * theta^(-2i/hd))
    z = x[..., : hd // 2] + 1j * x[..., hd // 2:]
    freq = desc["rope_theta"] ** (-2.0 * np.arange(hd // 2) / hd)
    zr = z * np.exp(1j * pos[:, None, None] * freq[None, None, :])
    assert np.allclose(y[..., : hd // 2], zr.real, atol=1e-12)
    assert np.allclose(y[..., hd // 2:], zr.imag, atol=1e-12)
    assert np.array_equal(y[0], x[0])             # position 0 is the identity


def test_rope_scores_depend_on_relative_position_only():
    desc, w = tiny()
    m = Model(desc, w)
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 1, m.hd))
    k = rng.standard_normal((1, 1, m.hd))
    base = np.sum(m.rope(q, [9]) * m.rope(k, [4]))
    for shift in (1, 50, 1000):
        assert np.isclose(np.sum(m.rope(q, [9 + shift]) * m.rope(k, [4 + shift])), base, atol=1e-10)
    assert not np.isclose(np.sum(m.rope(q, [9]) * m.rope(k, [5])), base, atol=1e-6)


# ---------------------------------------------------------------------------
# attention structure
# ---------------------------------------------------------------------------

def test_single_token_logits_ignore_wq_wk():
    """With one key the softmax weight is 1, so the attention output is v: the
    logits of a 1-token sequence cannot depend on W_q or W_k."""
    desc, w = tiny()
    ref = Model(desc, w).forward_full([7])
    w2 = copy.deepcopy(w)
    rng = np.random.default_rng(3)
    for lw in w2["layers"]:
        lw["wq"] = rng.standard_normal(lw["wq"].shape).astype(np.float32)
        lw["wk"] = rng.standard_normal(lw["wk"].shape).astype(np.float32)
    assert np.allclose(Model(desc, w2).forward_full([7]), ref, atol=1e-13)


def _uniform_attention_model(d=16, H=2, vocab=16):
    """One layer, W_q = 0 (uniform softmax), W_v = W_o = identity, MLP switched off
    (W_gate = 0), unit-RMS embeddings, eps = 0, identity unembedding."""
    hd = d // H
    desc = dict(n_layers=1, d_model=d, n_heads=H, n_kv_heads=H, head_dim=hd, d_ffn=8, vocab=vocab,
                dtype="f32", rms_eps=0.0, rope_theta=10000.0)
    rng = np.random.default_rng(4)
    E = rng.standard_normal((vocab, d))
    E /= np.sqrt(np.mean(E * E, axis=1, keepdims=True))
    eye = np.eye(d)
    layer = dict(attn_norm=np.ones(d), wq=np.zeros((d, d)), wk=rng.standard_normal((d, d)), wv=eye, wo=eye,
                 mlp_norm=np.ones(d), w_gate=np.zeros((8, d)), w_up=rng.standard_normal((8, d)),
                 w_down=rng.standard_normal((d, 8)))
    w = dict(tok_emb=E, unemb=np.eye(d), final_norm=np.ones(d), layers=[layer])
    return desc, w, E


def test_uniform_attention_closed_form_pins_visible_set():
    """W_q = 0 makes every visible key equally likely, so the attention output of
    block token (r, j) is the plain mean of the embeddings of the cached context
    and of row r's tokens 0..j -- and of nothing else."""
    desc, w, E = _uniform_attention_model()
    m = Model(desc, w)
    prompt = [3, 1, 4, 1, 5]
    st = prefill(m, prompt)                     # caches the 5 prompt tokens
    block = np.array([[9, 2, 6], [9, 5, 3], [9, 8, 7]])
    logits, _ = m.forward_block(block, st.cache)
    for r in range(3):
        for j in range(3):
            vis = prompt + [int(t) for t in block[r, : j + 1]]
            h = E[block[r, j]] + E[vis].mean(axis=0)
            expect = h / np.sqrt(np.mean(h * h))              # final norm (eps = 0, gain 1), identity unembedding
            assert np.allclose(logits[r, j], expect, atol=1e-12), (r, j)


def test_causality_future_tokens_do_not_matter():
    desc, w = tiny()
    m = Model(desc, w)
    a = m.forward_full([5, 9, 2, 77, 31, 8])
    b = m.forward_full([5, 9, 2, 400, 12, 13])
    assert np.allclose(a[:3], b[:3], atol=1e-13)
    assert not np.allclose(a[3], b[3], atol=1e-6)


def test_block_with_cache_equals_uncached_forward_per_row():
    """A (k, c) block on a cached context gives, for every row r and column j, the
    logits of the plain uncached forward of context ++ row r's tokens 0..j."""
    desc, w = tiny()
    m = Model(desc, w)
    prompt = list(si.prompt_motif(desc["vocab"], 24, seed=3))
    st = prefill(m, prompt)
    rng = np.random.default_rng(5)
    block = rng.integers(0, desc["vocab"], size=(3, 4))
    logits, _ = m.forward_block(block, st.cache)
    for r in range(3):
        full = m.forward_full(prompt + [int(t) for t in block[r]])
        assert np.allclose(logits[r], full[len(prompt):], atol=1e-12)


def test_gqa_equals_mha_with_repeated_kv_heads():
    desc, w = tiny()
    desc_g = dict(desc, n_kv_heads=2)
    wg = si.make_weights(desc_g, seed=1)
    # the same model written as MHA: each kv head's rows are repeated for its group
    wm = copy.deepcopy(wg)
    hd, grp = desc["head_dim"], desc["n_heads"] // 2
    for lw in wm["layers"]:
        for name in ("wk", "wv"):
            a = lw[name].reshape(2, hd, -1)
            lw[name] = np.repeat(a, grp, axis=0).reshape(desc["n_heads"] * hd, -1)
    toks = [1, 2, 3, 4, 5, 6, 7]
    assert np.allclose(Model(desc_g, wg).forward_full(toks), Model(desc, wm).forward_full(toks), atol=1e-13)


# ---------------------------------------------------------------------------
# feed-forward roles
# ---------------------------------------------------------------------------

def test_zero_gate_switches_mlp_off_and_large_gate_is_relu():
    desc, w = tiny()
    w0 = copy.deepcopy(w)
    for lw in w0["layers"]:
        lw["w_down"] = np.zeros_like(lw["w_down"])
    no_mlp = Model(desc, w0).forward_full([4, 8, 15])
    wz = copy.deepcopy(w)
    for lw in wz["layers"]:
        lw["w_gate"] = np.zeros_like(lw["w_gate"])       # silu(0) = 0 kills the product whatever W_up is
    assert np.allclose(Model(desc, wz).forward_full([4, 8, 15]), no_mlp, atol=1e-13)

    # one layer, huge gate: silu(s*g) -> s*relu(g); the MLP becomes W_down (s*relu(W_gate x) * (W_up x))
    desc1 = dict(desc, n_layers=1)
    w1 = si.make_weights(desc1, seed=2)
    s = 1e6
    wl = copy.deepcopy(w1)
    wl["layers"][0]["w_gate"] = w1["layers"][0]["w_gate"] * s
    wl["layers"][0]["w_down"] = w1["layers"][0]["w_down"] / s
    m = Model(desc1, wl)
    toks = [4, 8, 15]
    got = m.forward_full(toks)
    # rebuild the same logits from a library-routine attention residual plus the relu closed form
    ma = Model(desc1, w1)
    lw = {k: np.asarray(v, dtype=np.float64) for k, v in w1["layers"][0].items()}
    h_attn = _attention_residual_bruteforce(ma, toks)
    x = ma.rmsnorm(h_attn, lw["mlp_norm"])
    mlp = (np.maximum(x @ lw["w_gate"].T, 0.0) * (x @ lw["w_up"].T)) @ lw["w_down"].T
    expect = ma.rmsnorm(h_attn + mlp, ma.final_norm) @ ma.unemb.T
    # silu(s*g) differs from s*relu(g) only where |s*g| is O(1): an O(1/s) effect after W_down / s
    assert np.allclose(got, expect, atol=1e-6)
    assert not np.allclose(got, Model(desc1, w1).forward_full(toks), atol=1e-3)


def _attention_residual_bruteforce(m, toks):
    """Textbook single-layer causal attention with library routines (torch)."""
    lw = m.layers[0]
    e = torch.tensor(m.tok_emb[np.asarray(toks)])
    x = F.rms_norm(e, (e.shape[-1],), torch.tensor(lw["attn_norm"]), eps=m.eps)
    T = len(toks)
    q = (x @ torch.tensor(lw["wq"]).T).view(T, m.H, m.hd)
    k = (x @ torch.tensor(lw["wk"]).T).view(T, m.Hkv, m.hd)
    v = (x @ torch.tensor(lw["wv"]).T).view(T, m.Hkv, m.hd)
    q, k = _torch_rope(q, m), _torch_rope(k, m)
    a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
    a = a.transpose(0, 1).reshape(T, m.H * m.hd)
    return (e + a @ torch.tensor(lw["wo"]).T).numpy()


def _torch_rope(x, m, pos0=0):
    T, _, hd = x.shape
    freq = m.theta ** (-2.0 * torch.arange(hd // 2, dtype=torch.float64) / hd)
    ang = (torch.arange(T, dtype=torch.float64) + pos0)[:, None] * freq[None, :]
    z = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


# ---------------------------------------------------------------------------
# whole forward against library building blocks
# ---------------------------------------------------------------------------

def _torch_forward(m: Model, toks):
    """The same decoder assembled from torch library routines (rms_norm,
    scaled_dot_product_attention with its default 1/sqrt(head_dim) scale, silu)."""
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    h = t(m.tok_emb)[torch.tensor(toks)]
    T, d = h.shape
    for lw in m.layers:
        x = F.rms_norm(h, (d,), t(lw["attn_norm"]), eps=m.eps)
        q = F.linear(x, t(lw["wq"])).view(T, m.H, m.hd)
        k = F.linear(x, t(lw["wk"])).view(T, m.Hkv, m.hd)
        v = F.linear(x, t(lw["wv"])).view(T, m.Hkv, m.hd)
        q, k = _torch_rope(q, m), _torch_rope(k, m)
        rep = m.H // m.Hkv
        k, v = k.repeat_interleave(rep, dim=1), v.repeat_interleave(rep, dim=1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
        h = h + F.linear(a.transpose(0, 1).reshape(T, m.H * m.hd), t(lw["wo"]))
        x = F.rms_norm(h, (d,), t(lw["mlp_norm"]), eps=m.eps)
        h = h + F.linear(F.silu(F.linear(x, t(lw["w_gate"]))) * F.linear(x, t(lw["w_up"])), t(lw["w_down"]))
    return F.linear(F.rms_norm(h, (d,), t(m.final_norm), eps=m.eps), t(m.unemb)).numpy()


@pytest.mark.parametrize("kv_heads", [4, 2])
def test_forward_matches_torch_library_assembly(kv_heads):
    desc, _ = tiny()
    desc = dict(desc, n_kv_heads=kv_heads)
    w = si.make_weights(desc, seed=6, std=0.2, random_gains=True)     # std 0.2: attention far from uniform
    m = Model(desc, w)
    toks = [int(t) for t in si.prompt_motif(desc["vocab"], 40, seed=9)]
    assert np.allclose(m.forward_full(toks), _torch_forward(m, toks), atol=1e-10)


def test_zero_output_projections_reduce_logits_to_embedding_path():
    """W_o = W_down = 0 leaves the residual stream equal to the embedding, so the
    logits are U . RMSNorm(E[x]) at every position."""
    desc, w = tiny()
    for lw in w["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["w_down"] = np.zeros_like(lw["w_down"])
    m = Model(desc, w)
    toks = [11, 300, 42]
    got = m.forward_full(toks)
    for j, t in enumerate(toks):
        e = m.tok_emb[t]
        expect = m.unemb @ (e / np.sqrt(np.mean(e * e) + desc["rms_eps"]) * m.final_norm)
        assert np.allclose(got[j], expect, atol=1e-13)
