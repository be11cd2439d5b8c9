"""Pins for the oracle's guess-and-verify step and decode loops: the method's
defining invariant (speculative greedy == plain greedy), injected drafts with a
known accepted length, closed-form accept-all, cache consistency.  CPU only."""
import copy

import numpy as np
import pytest

import synth_inputs as si
from oracle import (Model, Bigram, ModelBigram, rank_ids, prefill, verify_step, commit, accept_lengths, select_winner,
                    greedy_plain, greedy_plain_cached, greedy_speculative, build_drafts)


@pytest.fixture(scope="module")
def tiny():
    desc = si.MODELS["tiny"]
    w = si.make_weights(desc, seed=0)
    run = si.RUNS["cfg1"]
    prompt = si.make_prompt(run, desc["vocab"], seed=1)
    m = Model(desc, w)
    plain = greedy_plain(m, prompt, 24)             # the definition: no cache, whole sequence re-run per token
    return desc, w, run, prompt, m, plain


def test_accept_lengths_and_winner_by_hand():
    drafts = np.array([[5, 6, 7], [5, 6, 9], [1, 6, 7], [5, 6, 7]])
    greedy = np.array([[5, 6, 9, 0], [5, 6, 9, 4], [5, 6, 7, 1], [5, 6, 7, 2]])
    a = accept_lengths(drafts, greedy)
    assert list(a) == [2, 3, 0, 3]
    assert select_winner(a) == (1, 3)               # rows 1 and 3 tie at 3: the lower row wins
    assert select_winner(np.array([0, 0, 0])) == (0, 0)
    assert list(accept_lengths(np.zeros((2, 0), dtype=np.int32), np.array([[3], [3]]))) == [0, 0]


def test_cached_plain_equals_uncached_plain(tiny):
    desc, w, run, prompt, m, plain = tiny
    assert greedy_plain_cached(m, prompt, 24) == plain


def test_speculative_equals_plain_greedy_cfg1(tiny):
    """The defining invariant: whatever the drafts, the committed tokens are the
    plain greedy tokens."""
    desc, w, run, prompt, m, plain = tiny
    gen, stats = greedy_speculative(m, prompt, 24, run["k"], run["w"], run["k_ctx_max"], run["q_min"], run["q_max"])
    assert gen == plain
    assert sum(stats["new_hist"]) == stats["calls"]


@pytest.mark.parametrize("k,w,kc,qmin,qmax", [(1, 0, 0, 1, 1), (1, 5, 1, 1, 1), (6, 2, 0, 1, 1), (5, 4, 5, 1, 3)])
def test_speculative_equals_plain_greedy_other_shapes(tiny, k, w, kc, qmin, qmax):
    desc, w_, run, prompt, m, plain = tiny
    gen, _ = greedy_speculative(m, prompt, 24, k, w, kc, qmin, qmax)
    assert gen == plain


def test_injected_drafts_accept_exactly_up_to_the_corruption(tiny):
    desc, w_, run, prompt, m, plain = tiny
    st = prefill(m, prompt)
    assert st.tokens[-1] == plain[0]
    w = 5
    truth = plain[1:1 + w]
    V = desc["vocab"]
    rows = []
    for c in range(w + 1):                      # row c: correct for c tokens, then wrong
        row = list(truth)
        if c < w:
            row[c] = (truth[c] + 1 + c) % V
        rows.append(row)
    res = verify_step(m, st, np.array(rows))
    assert list(res["accept_len"]) == list(range(w + 1))
    assert res["winner"] == w and res["n_accept"] == w
    assert res["new_tokens"] == plain[1:w + 2]
    # every row that accepted at least a tokens saw the same inputs up to column a: same greedy token there
    for a in range(w + 1):
        col = {int(res["greedy"][r, a]) for r in range(a, w + 1)}
        assert col == {plain[1 + a]}
    # rows in another order, with a duplicate: same tokens, winner = first of the best rows
    perm = [3, 5, 0, 5, 1]
    res2 = verify_step(m, st, np.array([rows[i] for i in perm]))
    assert list(res2["accept_len"]) == perm and res2["winner"] == 1
    assert res2["new_tokens"] == res["new_tokens"]
    assert np.array_equal(res2["greedy"][1], res2["greedy"][3])


def test_all_wrong_drafts_reduce_to_a_plain_decode_step(tiny):
    desc, w_, run, prompt, m, plain = tiny
    st = prefill(m, prompt)
    wrong = np.array([[(plain[1] + 1 + r) % desc["vocab"], 0, 0] for r in range(3)])
    res = verify_step(m, st, wrong)
    assert res["n_accept"] == 0 and res["winner"] == 0 and res["new_tokens"] == [plain[1]]
    res1 = verify_step(m, st, np.zeros((1, 0), dtype=np.int32))          # (k, w) = (1, 0)
    assert res1["new_tokens"] == [plain[1]]
    assert np.allclose(res["logits"][:, 0], res1["logits"][0, 0], atol=1e-12)    # column 0 is the same in every row


def test_commit_keeps_the_cache_consistent_with_a_fresh_prefill(tiny):
    desc, w_, run, prompt, m, plain = tiny
    st = prefill(m, prompt)
    truth = plain[1:4]
    drafts = np.array([[truth[0], truth[1], (truth[2] + 1) % desc["vocab"]], [truth[0], 0, 0]])
    res = verify_step(m, st, drafts)
    assert res["n_accept"] == 2
    n_new = commit(st, res)
    assert n_new == 3 and st.tokens == [int(t) for t in prompt] + plain[:4]
    fresh = prefill(m, st.tokens[:-1])
    assert fresh.tokens[-1] == st.tokens[-1]
    for li in range(desc["n_layers"]):
        assert np.allclose(st.cache.k[li], fresh.cache.k[li], atol=1e-12)
        assert np.allclose(st.cache.v[li], fresh.cache.v[li], atol=1e-12)
    nxt = verify_step(m, st, np.zeros((1, 0), dtype=np.int32))
    assert nxt["new_tokens"] == [plain[4]]
    # budget truncation
    st2 = prefill(m, prompt)
    assert commit(st2, verify_step(m, st2, drafts), max_new=2) == 2
    assert st2.tokens == [int(t) for t in prompt] + plain[:3] and len(st2.cache) == len(st2.tokens) - 1


def test_zero_output_projections_accept_the_whole_bigram_chain():
    """W_o = W_down = 0: the model's logits are U . RMSNorm(E[x]), whose argmax is
    the bigram's top-1 (a positive per-vector scale cannot change ranks, gains
    are 1).  So bigram row 0 -- the chain of top-1s -- is accepted in full."""
    desc = si.MODELS["tiny"]
    w = si.make_weights(desc, seed=3)
    for lw in w["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["w_down"] = np.zeros_like(lw["w_down"])
    m = Model(desc, w)
    b = Bigram(m.tok_emb, m.unemb)
    st = prefill(m, [10, 20, 30])
    drafts, src, n_ctx = build_drafts(st.tokens, b, k=4, w=6, k_ctx_max=0, q_min=1, q_max=1)
    res = verify_step(m, st, drafts)
    assert res["winner"] == 0 and res["n_accept"] == 6
    assert list(res["accept_len"][1:]) == [0, 0, 0]               # ranks 2..4 start with a different token
    gen, stats = greedy_speculative(m, [10, 20, 30], 29, 4, 6, 0, 1, 1)
    assert stats["new_hist"][7] == stats["calls"] == 4            # 1 from prefill + 4 calls x 7 tokens


def test_full_model_bigram_closed_form_and_ranks():
    """Section 4.1's bigram is the whole model on a one-token context.  (1) With W_o = W_down = 0
    and a random final gain g its scores have the closed form U . (g * E[x] / rms(E[x])): one key
    means attention returns v, which the zero output projection discards.  (2) With gains of 1 the
    scores are a positive multiple of the direct path's U . E[x], so both bigrams rank alike."""
    desc = si.MODELS["tiny"]
    w = si.make_weights(desc, seed=5, random_gains=True)
    for lw in w["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["w_down"] = np.zeros_like(lw["w_down"])
    m = Model(desc, w)
    mb = ModelBigram(lambda x: m.forward_full([x])[-1])
    for x in (0, 7, 511):
        e = np.asarray(w["tok_emb"][x], dtype=np.float64)
        closed = np.asarray(w["unemb"], np.float64) @ (np.asarray(w["final_norm"], np.float64) * e /
                                                       np.sqrt(np.mean(e * e) + desc["rms_eps"]))
        assert np.allclose(mb.scores(x), closed, rtol=1e-12, atol=1e-12)
        assert list(mb.topk(x, 5)) == list(rank_ids(closed, 5)) and mb.next1(x) == int(rank_ids(closed, 1)[0])
    w1 = si.make_weights(desc, seed=5)
    for lw in w1["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["w_down"] = np.zeros_like(lw["w_down"])
    m1 = Model(desc, w1)
    mb1, direct = ModelBigram(lambda x: m1.forward_full([x])[-1]), Bigram(m1.tok_emb, m1.unemb)
    for x in (3, 100):
        assert list(mb1.topk(x, 16)) == list(direct.topk(x, 16))
        assert mb1.rows(x, 3, 4) == direct.rows(x, 3, 4)


def test_full_model_bigram_differs_from_direct_path_but_keeps_the_invariant(tiny):
    """On a model with live layers the two bigrams draft differently; the committed tokens are
    plain greedy either way (the method's invariant does not depend on the drafts)."""
    desc, w, run, prompt, m, plain = tiny
    mb = ModelBigram(lambda x: m.forward_full([x])[-1])
    direct = Bigram(m.tok_emb, m.unemb)
    assert any(list(mb.topk(x, 4)) != list(direct.topk(x, 4)) for x in range(0, 512, 37))
    gen, stats = greedy_speculative(m, prompt, 24, run["k"], run["w"], run["k_ctx_max"], run["q_min"], run["q_max"], bigram=mb)
    assert list(gen) == list(plain)


def test_attention_cost_model_counts():
    """Section 3: each of the k rows multiplies w+1 queries by l+w keys."""
    for (l, k, w) in [(25, 1, 0), (100, 10, 5), (500, 32, 15)]:
        pairs = sum(1 for r in range(k) for j in range(w + 1) for s in range((l - 1) + j + 1))
        assert pairs == k * ((w + 1) * (l - 1) + (w + 1) * (w + 2) // 2)
        assert pairs <= k * (w + 1) * (l + w)


# ---------------------------------------------------------------------------
# the greedy tie rule, the per-strategy bookkeeping, and the memory-bounded forms
# ---------------------------------------------------------------------------

def test_greedy_argmax_takes_the_lowest_id_among_equal_logits():
    """Exact ties, hand-made: the FIRST maximum wins, in every position of a batch (a "last maximum" or a
    "strictly greater from the right" scan fails each of these)."""
    from oracle.model import greedy_argmax
    assert int(greedy_argmax(np.array([1.0, 3.0, 3.0, 2.0]))) == 1
    assert int(greedy_argmax(np.array([0.0, 5.0, 5.0]))) == 1            # the tie reaches the last entry
    assert int(greedy_argmax(np.array([7.0, 7.0, 7.0, 7.0]))) == 0          # all equal
    assert int(greedy_argmax(np.array([-2.0, -1.0, -3.0, -1.0]))) == 1      # negative logits
    assert int(greedy_argmax(np.array([0.0, -0.0, 0.0]))) == 0              # +0 and -0 compare equal
    grid = np.array([[[1.0, 1.0, 0.0], [0.0, 2.0, 2.0]], [[3.0, 0.0, 3.0], [0.0, 0.0, 0.0]]])
    out = greedy_argmax(grid)
    assert out.dtype == np.int32 and out.tolist() == [[0, 1], [0, 0]]


class _ScriptedModel:
    """A 'model' whose greedy prediction after token t is S[t], whatever came before: one-hot logits,
    one layer of empty keys/values.  Offers what prefill / verify_step / commit use."""
    L, Hkv, hd = 1, 1, 1

    def __init__(self, succ):
        self.succ = np.asarray(succ)

    def forward_block(self, tokens, cache=None, want_logits=True):
        tokens = np.asarray(tokens)
        k, c = tokens.shape
        logits = np.zeros((k, c, len(self.succ)))
        for r in range(k):
            for j in range(c):
                logits[r, j, self.succ[tokens[r, j]]] = 1.0
        kv = [(np.zeros((k, c, 1, 1)), np.zeros((k, c, 1, 1)))]
        return logits, kv


class _ScriptedBigram:
    """Ranked first tokens from a table, chain through `nxt`."""

    def __init__(self, top, nxt):
        self.top, self.nxt = top, nxt

    def rows(self, x, k_big, w):
        out = []
        for t in self.top[x][:k_big]:
            row = [t]
            while len(row) < w:
                row.append(self.nxt[row[-1]])
            out.append(tuple(row[:w]))
        return out


def test_strategy_bookkeeping_on_a_hand_worked_four_call_run():
    """accept_hist / rank_hist / alloc_hist / new_hist / winner_src / ctx_rows of greedy_speculative, worked by
    hand (Section 5.2's ablation quantities).  Model: next token S[t], S = two 4-cycles.  k=3, w=2, at most 2
    context rows, q=2, 8 tokens.  Prompt 0 1 7 7 0 1 7 7 0 1; the prefill appends S[1] = 2.
      call 1: query (1,2) never occurred: 0 context rows; bigram rows (4,5) (3,5) (5,6); the model says 3 then 0:
              row 1 keeps 1 token -> bigram win, rank 1, 1 accepted, appends 3 0.
      call 2: query (3,0) never occurred; bigram rows (2,3) (3,5) (4,5), the model says 1: nothing accepted, row 0
              (a bigram row) 'wins' with 0 accepted -> no rank entry, appends 1.
      call 3: query (0,1) occurred at 0, 4 (then 7 7) and 8 (then 2 3): context rows (7,7) [count 2], (2,3); one bigram
              row (3,5); the model says 2 then 3: row 1 keeps 2 -> context win, rank 1, appends 2 3 0.
      call 4: query (3,0) occurred at 11 (then 1 2): context row (1,2), bigram rows (2,3) (3,5); row 0 keeps 2 ->
              context win, rank 0, 2 accepted, but only 1 token of budget is left: appends 1."""
    S = [1, 2, 3, 0, 5, 6, 7, 4]
    nxt = list(S)
    nxt[3] = 5                                           # the chain is wrong after token 3
    top = {2: [4, 3, 5], 0: [2, 3, 4], 1: [3, 2, 6]}
    prompt = [0, 1, 7, 7, 0, 1, 7, 7, 0, 1]
    gen, st = greedy_speculative(_ScriptedModel(S), prompt, 8, 3, 2, 2, 2, 2, bigram=_ScriptedBigram(top, nxt))
    assert gen == [2, 3, 0, 1, 2, 3, 0, 1]
    assert st["calls"] == 4
    assert st["new_hist"] == [0, 2, 1, 1]
    assert st["winner_src"] == [2, 2]
    assert st["ctx_rows"] == [0, 0, 2, 1]
    assert st["accept_hist"] == [[0, 0, 2], [1, 1, 0]]
    assert st["rank_hist"] == [[1, 1, 0], [0, 1, 0]]
    assert st["alloc_hist"] == [2, 1, 1, 0]
    assert st["tokens_per_call"] == 7 / 4


def test_chunked_prefill_and_widening_at_use_change_nothing(tiny):
    """The memory-bounded forms used for long contexts and deep models: a prompt fed in pieces through the
    cached block call gives the cache and first token of the one-piece prefill (up to fp64 summation order),
    and widening the layer matrices at use instead of up front gives bit-identical logits."""
    desc, w, run, prompt, m, plain = tiny
    whole = prefill(m, prompt)
    for chunk in (1, 7, 50, 127, 128, 500):
        st = prefill(m, prompt, chunk=chunk)
        assert st.tokens == whole.tokens and len(st.cache) == len(prompt)
        for li in range(m.L):
            assert np.allclose(st.cache.k[li], whole.cache.k[li], rtol=0, atol=1e-12)
            assert np.allclose(st.cache.v[li], whole.cache.v[li], rtol=0, atol=1e-12)
        assert np.allclose(st.first_logits, whole.first_logits, rtol=0, atol=1e-12)
    lazy = Model(desc, w, widen_at_use=True)
    assert lazy.layers[0]["wq"].dtype == np.float32                     # kept as stored
    assert np.array_equal(lazy.forward_full(prompt[:40]), m.forward_full(prompt[:40]))
    bdesc = si.reduced_layers(si.MODELS["small"], 1)
    bdesc = dict(bdesc, vocab=256, d_model=64, n_heads=2, n_kv_heads=2, head_dim=32, d_ffn=128)
    bw = si.make_weights(bdesc, seed=3)
    assert np.array_equal(Model(bdesc, bw, widen_at_use=True).forward_full([1, 2, 3, 4, 5]),
                          Model(bdesc, bw).forward_full([1, 2, 3, 4, 5]))


def test_adaptive_context_cap_by_hand_and_the_invariant(tiny):
    from oracle import adaptive_context_cap
    wins = [5, 3, 1, 1, 0, 0]                                  # 10 context wins: 5 by the first row, 3 by the second, ...
    assert adaptive_context_cap(wins, 6, 90, 8) == 3           # 5 + 3 + 1 = 9 of 10 reach 90 %
    assert adaptive_context_cap(wins, 6, 80, 8) == 2           # 8 of 10
    assert adaptive_context_cap(wins, 6, 81, 8) == 3
    assert adaptive_context_cap(wins, 6, 100, 8) == 4          # every win
    assert adaptive_context_cap(wins, 2, 100, 8) == 2          # never above the configured cap
    assert adaptive_context_cap(wins, 6, 90, 11) == 6          # not warmed up: the configured cap
    assert adaptive_context_cap([7, 0, 0], 3, 90, 1) == 1      # all wins in the first row
    assert adaptive_context_cap([0, 0, 0], 3, 90, 1) == 3      # no wins yet
    assert adaptive_context_cap([0, 0, 4], 3, 1, 1) == 3       # the first rows never won: the cap still reaches the row that did
    desc, w, run, prompt, m, plain = tiny
    gen, st = greedy_speculative(m, prompt, 24, 5, 4, 5, 1, 3, allocation=dict(coverage_percent=50, warmup_wins=1))
    assert gen == plain                                        # whatever the allocation, the tokens are the greedy tokens
