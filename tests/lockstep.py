"""Lock-step comparison of the HIP path with the CPU oracle (test helper).

After every step the harness compares drafts, greedy grid, accepted lengths,
winner, new tokens and logits.  Integer results must agree exactly, except
where floating point decides them and the oracle's own margin between the two
candidates is below the logit tolerance (then the disagreement is counted as
tolerated and the oracle's history is forced to the GPU's committed tokens so
one near-tie cannot desynchronise the rest of the run).
"""
from __future__ import annotations

import numpy as np

import oracle


TOL = {"f32": 1e-4, "bf16": 2e-2}     # max abs logit error relative to the position's logit scale


class Report:
    def __init__(self):
        self.steps = 0
        self.tolerated_argmax = 0
        self.tolerated_draft = 0
        self.max_rel_logit_err = 0.0
        self.new_hist = {}
        self.ctx_rows = 0

    def __repr__(self):
        return (f"steps={self.steps} tolerated_argmax={self.tolerated_argmax} tolerated_draft={self.tolerated_draft} "
                f"max_rel_logit_err={self.max_rel_logit_err:.3e} new_hist={self.new_hist} ctx_rows={self.ctx_rows}")


def _check_argmax(gpu_tok, logits, tol, rep, what):
    """gpu_tok must be the oracle's argmax, or lie within the tolerated margin of it."""
    o_tok = int(np.argmax(logits))
    if int(gpu_tok) == o_tok:
        return
    scale = float(np.max(np.abs(logits)))
    margin = float(logits[o_tok] - logits[int(gpu_tok)])
    assert margin < tol * scale, f"{what}: GPU token {gpu_tok} vs oracle {o_tok}, margin {margin:.3e} >= {tol * scale:.3e}"
    rep.tolerated_argmax += 1


def check_drafts(g_drafts, g_src, g_nctx, st, bigram, cfg, tol, rep):
    """Context rows are integer work: exact.  Bigram rows may differ only between
    ids whose oracle scores are closer than tol * max|z|."""
    o_drafts, o_src, o_nctx = oracle.build_drafts(st.tokens, bigram, cfg["k"], cfg["w"], cfg["k_ctx_max"],
                                                  cfg["q_min"], cfg["q_max"])
    assert g_nctx == o_nctx, f"context rows found: GPU {g_nctx} vs oracle {o_nctx}"
    assert np.array_equal(g_src, o_src)
    assert np.array_equal(g_drafts[:o_nctx], o_drafts[:o_nctx]), "context rows differ"
    if np.array_equal(g_drafts, o_drafts):
        return
    for r in range(o_nctx, cfg["k"]):
        prev = st.tokens[-1]
        for j in range(cfg["w"]):
            g, o = int(g_drafts[r, j]), int(o_drafts[r, j])
            if g != o:
                z = bigram.scores(prev)
                # rank r-o_nctx for column 0, rank 0 afterwards: either way the two ids must be a near tie
                assert abs(z[g] - z[o]) < tol * np.max(np.abs(z)), f"bigram row {r} col {j}: GPU {g} vs oracle {o}"
                rep.tolerated_draft += 1
                break                       # the rest of the chain follows the GPU's token
            prev = g


def run(ctx, model, prompt, n_gen, cfg, tol, check_logits=True, injected=None, max_steps=None, bigram=None,
        oracle_chunk=None, on_step=None):
    """Lock-step decode.  `injected(step, st) -> drafts or None` replaces the built
    drafts for some steps (coverage of every accepted length).  `oracle_chunk`: the oracle
    takes the prompt in pieces of that many tokens (bounded memory at long contexts).
    `on_step(step)` is called after every verify call of the GPU.  Returns a Report."""
    rep = Report()
    bigram = bigram or oracle.Bigram(model.tok_emb, model.unemb)
    ctx.prefill(prompt)
    st = oracle.prefill(model, prompt, chunk=oracle_chunk)
    g_first = int(ctx.get_tokens()[-1])
    _check_argmax(g_first, st.first_logits, tol, rep, "first token")
    st.tokens[-1] = g_first
    n0 = len(prompt)
    while len(st.tokens) - n0 < n_gen and (max_steps is None or rep.steps < max_steps):
        left = n_gen - (len(st.tokens) - n0)
        drafts = injected(rep.steps, st) if injected else None
        if drafts is None:
            g_drafts, g_src, g_nctx = ctx.build_drafts(cfg)
            check_drafts(g_drafts, g_src, g_nctx, st, bigram, cfg, tol, rep)
            rep.ctx_rows += g_nctx
            res_g = ctx.verify_step(None, cfg["k"], cfg["w"], want_logits=check_logits)
            drafts = g_drafts
        else:
            drafts = np.asarray(drafts, dtype=np.int32)
            res_g = ctx.verify_step(drafts, want_logits=check_logits)
        if on_step:
            on_step(rep.steps)
        res_o = oracle.verify_step(model, st, drafts)
        k, w = drafts.shape
        if check_logits:
            scale = np.max(np.abs(res_o["logits"]), axis=-1)
            err = np.max(np.abs(res_g["logits"] - res_o["logits"]), axis=-1) / scale
            rep.max_rel_logit_err = max(rep.max_rel_logit_err, float(err.max()))
            assert err.max() <= tol, f"step {rep.steps}: logit error {err.max():.3e} of scale exceeds {tol}"
        for r in range(k):
            for j in range(w + 1):
                _check_argmax(res_g["greedy"][r, j], res_o["logits"][r, j], tol, rep, f"step {rep.steps} greedy[{r}][{j}]")
        # integer work on the GPU's own greedy grid must be exact
        a = oracle.accept_lengths(drafts, res_g["greedy"])
        assert np.array_equal(res_g["accept_len"], a), f"step {rep.steps}: accept_len {res_g['accept_len']} vs {a}"
        win, n_acc = oracle.select_winner(a)
        assert (res_g["winner"], res_g["n_accept"], res_g["n_new"]) == (win, n_acc, n_acc + 1)
        new = [int(t) for t in drafts[win, :n_acc]] + [int(res_g["greedy"][win, n_acc])]
        assert list(res_g["new_tokens"]) == new
        n_new = ctx.commit(left)
        assert n_new == min(len(new), left)
        forced = dict(res_o, winner=win)
        oracle.commit(st, forced, max_new=left, tokens_override=new)
        assert list(ctx.get_tokens()) == st.tokens, f"step {rep.steps}: committed histories differ"
        rep.new_hist[n_new] = rep.new_hist.get(n_new, 0) + 1
        rep.steps += 1
    return rep
