"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import copy

import numpy as np
import pytest

import synth_inputs as si
import oracle
import paper_2411_03786_amd as ngg
from lockstep import run as lockstep_run, TOL

pytestmark = pytest.mark.gpu


def _setup(desc, run, seed=0, max_k=None, max_w=None, extra_seq=0, **wkw):
    w = si.make_weights(desc, seed=seed, **wkw)
    prompt = si.make_prompt(run, desc["vocab"], seed=1)
    model = oracle.Model(desc, w)
    ctx = ngg.Context(desc, w, max_seq=run["prompt_len"] + run["n_gen"] + 8 + extra_seq,
                      max_k=max_k or run["k"], max_w=max_w if max_w is not None else run["w"])
    return w, prompt, model, ctx


# ---------------------------------------------------------------------------------------------
# config 1: tiny fp32 decoder, whole run in lock-step
# ---------------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def tiny():
    desc, run = si.MODELS["tiny"], si.RUNS["cfg1"]
    w, prompt, model, ctx = _setup(desc, run, max_k=32, max_w=8, extra_seq=64)
    yield desc, run, w, prompt, model, ctx
    ctx.close()


def test_cfg1_lockstep_fp32(tiny):
    desc, run, w, prompt, model, ctx = tiny
    rep = lockstep_run(ctx, model, prompt, run["n_gen"], run, TOL["f32"])
    print("cfg1:", rep)
    assert rep.tolerated_argmax == 0 and rep.tolerated_draft == 0
    assert rep.max_rel_logit_err <= 1e-4
    assert max(rep.new_hist) > 1              # multi-token commits were exercised


def test_cfg1_matches_oracle_plain_greedy_and_gpu_plain_equals_speculative(tiny):
    desc, run, w, prompt, model, ctx = tiny
    want = oracle.greedy_plain_cached(model, prompt, 40)
    got_spec, stats = ctx.greedy_decode(prompt, 40, run)
    got_plain, stats_p = ctx.greedy_decode(prompt, 40, None)
    assert list(got_spec) == want and list(got_plain) == want
    assert stats_p["calls"] == 39 and stats_p["new_hist"][1] == 39
    assert stats["calls"] < 39 and sum(i * c for i, c in enumerate(stats["new_hist"])) == 39
    # the ablation quantities of Section 5.2 (accepted length and rank by strategy, rows per strategy)
    _, o_stats = oracle.greedy_speculative(model, prompt, 40, run["k"], run["w"], run["k_ctx_max"], run["q_min"], run["q_max"])
    assert stats["calls"] == o_stats["calls"] and stats["winner_src"] == o_stats["winner_src"]
    for s_ in (0, 1):
        assert stats["accept_hist"][s_][:run["w"] + 1] == o_stats["accept_hist"][s_]
        assert stats["rank_hist"][s_][:run["k"]] == o_stats["rank_hist"][s_]
    assert stats["alloc_hist"][:run["k"] + 1] == o_stats["alloc_hist"]
    assert sum(stats["alloc_hist"]) == stats["calls"] == sum(map(sum, stats["accept_hist"]))


def test_decode_more_in_pieces_equals_greedy_decode_and_the_oracle(tiny):
    """The library-side loop resumed from the committed state: pieces of at most 3 verify calls, the token
    budget shrinking as in one greedy_decode call, give its tokens and its statistics, and the oracle's."""
    desc, run, w, prompt, model, ctx = tiny
    want = oracle.greedy_plain_cached(model, prompt, 40)
    _, whole = ctx.greedy_decode(prompt, 40, run)
    ctx.prefill(prompt)                                   # appends the first token
    toks, left, total = [int(ctx.get_tokens()[-1])], 39, None
    while left > 0:
        out, st = ctx.decode_more(left, 3, run)
        assert 1 <= st["calls"] <= 3 and st["tokens"] == len(out) >= st["calls"]
        toks += [int(t) for t in out]
        left -= len(out)
        if total is None:
            total = st
        else:
            for key in ("calls", "ctx_rows"):
                total[key] += st[key]
            for key in ("new_hist", "winner_src", "alloc_hist"):
                total[key] = [a + b for a, b in zip(total[key], st[key])]
            for key in ("accept_hist", "rank_hist"):
                total[key] = [[a + b for a, b in zip(ra, rb)] for ra, rb in zip(total[key], st[key])]
    assert toks == want and list(ctx.get_tokens()) == list(prompt) + want
    for key in ("calls", "ctx_rows", "new_hist", "winner_src", "alloc_hist", "accept_hist", "rank_hist"):
        assert total[key] == whole[key], key
    with pytest.raises(ngg.NggError) as e:
        ctx.decode_more(0, 1, run)
    assert e.value.status == ngg.NGG_EINVAL
    with pytest.raises(ngg.NggError) as e:
        ctx.decode_more(10 ** 6, 1, run)
    assert e.value.status == ngg.NGG_ECAPACITY


def test_graph_replay_equals_stream_launches(tiny):
    """ngg_decode_more can replay captured steps (mode 1: whenever a step qualifies; mode 2, the default: where it
    measures faster).  The same generation with the replay switched off (every step launched on the stream) must
    give the same tokens and the same statistics in both modes, for two block shapes and the single-token loop; the replaying run is cut into calls of three steps with launches on the stream in between
    (a verify call that is not committed), crosses several changes of the attention slice count (a new capture
    each) and ends on steps that the remaining budget clamps (launched on the stream)."""
    desc, run, w, prompt, model, ctx = tiny
    n_gen = 70
    want = oracle.greedy_plain_cached(model, prompt, n_gen)
    plain = dict(k=1, w=0, k_ctx_max=0, q_min=1, q_max=1)
    keys = ("calls", "tokens", "new_hist", "accept_hist", "rank_hist", "winner_src", "ctx_rows", "alloc_hist")
    try:
        for cfg in (run, dict(run, k=8, w=5, k_ctx_max=4), None):
            ctx.step_graphs(0)
            ctx.prefill(prompt)
            ref, st_ref = ctx.decode_more(n_gen - 1, 10 ** 6, cfg)
            ctx.step_graphs(2)
            ctx.prefill(prompt)
            auto, st_auto = ctx.decode_more(n_gen - 1, 10 ** 6, cfg)
            assert list(auto) == list(ref)
            ctx.step_graphs(1)
            ctx.prefill(prompt)
            before = ctx.debug_peek("step_graphs", np.int32)[0]
            whole, st_whole = ctx.decode_more(n_gen - 1, 10 ** 6, cfg)
            after = ctx.debug_peek("step_graphs", np.int32)[0]
            assert after[0] == 1 and after[1] == 0 and after[3] - before[3] >= st_whole["calls"] // 2, (before, after)
            assert list(whole) == list(ref) == want[1:]
            for key in keys:
                assert np.array_equal(np.asarray(st_whole[key]), np.asarray(st_ref[key])), key
                assert np.array_equal(np.asarray(st_auto[key]), np.asarray(st_ref[key])), key
            ctx.prefill(prompt)
            out = []
            c = cfg or plain
            while len(out) < n_gen - 1:
                toks, _ = ctx.decode_more(n_gen - 1 - len(out), 3, cfg)
                out += list(toks)
                ctx.build_drafts(c)                                   # stream launches between the replays
                ctx.verify_step(None, c["k"], c["w"])
            assert out == want[1:]
    finally:
        ctx.step_graphs(2)


def test_injected_drafts_every_accept_length(tiny):
    desc, run, w, prompt, model, ctx = tiny
    V = desc["vocab"]
    truth = oracle.greedy_plain_cached(model, prompt, 40)
    wd = 5

    def inject(step, st):
        done = len(st.tokens) - len(prompt)              # generated so far; truth[done:] comes next
        nxt = truth[done:done + wd]
        if len(nxt) < wd:
            return None
        cmax = step % (wd + 1)                             # longest correct prefix present in this step
        rows = []
        for c in range(cmax + 1):                          # row c: correct for c tokens, then wrong
            row = list(nxt)
            if c < wd:
                row[c] = (row[c] + 1 + c) % V
            rows.append(row)
        rot = step % len(rows)                             # move the best row around the batch
        return np.array(rows[rot:] + rows[:rot], dtype=np.int32)

    cfg = dict(run, k=6, w=wd)
    rep = lockstep_run(ctx, model, prompt, 36, cfg, TOL["f32"], injected=inject)
    print("injected:", rep)
    assert set(rep.new_hist) >= {1, 2, 3, 4, 5, 6}
    assert rep.tolerated_argmax == 0


def test_bigram_scores_and_next1_table(tiny):
    desc, run, w, prompt, model, ctx = tiny
    ctx.prefill(prompt)
    ctx.build_drafts(run)
    z, _ = ctx.debug_peek("z", np.float32)
    x_last = int(ctx.get_tokens()[-1])
    zo = oracle.bigram_scores(model.tok_emb, model.unemb, x_last)
    assert np.max(np.abs(z - zo)) <= 1e-5 * np.max(np.abs(zo))
    next1, _ = ctx.debug_peek("next1", np.int32)
    b = oracle.Bigram(model.tok_emb, model.unemb)
    for x in range(desc["vocab"]):
        if next1[x] != b.next1(x):
            s = b.scores(x)
            assert s[b.next1(x)] - s[next1[x]] < 1e-5 * np.max(np.abs(s))


# 1, 9, 112, 288, 6, 40, 65 and 96 block rows: GEMM row tiles of 1, 7, 8 (several passes), 3, 5 and 6 column blocks
@pytest.mark.parametrize("k,w", [(1, 0), (8, 0), (32, 0), (1, 8), (16, 6), (32, 8), (3, 1), (8, 4), (13, 4), (12, 7)])
def test_block_shapes_including_more_than_64_rows(tiny, k, w):
    desc, run, _, prompt, model, ctx = tiny
    cfg = dict(k=k, w=w, k_ctx_max=k, q_min=1, q_max=3)
    rep = lockstep_run(ctx, model, prompt, 12, cfg, TOL["f32"], max_steps=4)
    assert rep.tolerated_argmax == 0 and rep.max_rel_logit_err <= 1e-4


@pytest.mark.parametrize("n_prompt", [1, 2, 63, 64, 65, 127, 128, 129, 250])
def test_prefill_chunk_boundaries(tiny, n_prompt):
    desc, run, _, _, model, ctx = tiny
    prompt = si.prompt_spans(desc["vocab"], n_prompt, 0.5, seed=7)
    rep = lockstep_run(ctx, model, prompt, 6, run, TOL["f32"])
    assert rep.tolerated_argmax == 0


def test_same_step_twice_is_bit_identical(tiny):
    desc, run, _, prompt, model, ctx = tiny
    ctx.prefill(prompt)
    d, _, _ = ctx.build_drafts(run)
    a = ctx.verify_step(d, want_logits=True)
    b = ctx.verify_step(d, want_logits=True)
    assert np.array_equal(a["logits"], b["logits"]) and np.array_equal(a["greedy"], b["greedy"])


def _successor_model(period=None, seed=4):
    """A tiny decoder whose greedy next token is a known function of the last one, so
    that generated tokens recur in the context and the matcher has work to do:
    W_o = W_down = 0 leaves the residual stream equal to the embedding, and the output
    embedding of token succ(x) is the input embedding of x, so the model predicts
    succ(x) = (x + 1) mod period (tokens >= period map to themselves)."""
    desc = dict(si.MODELS["tiny"])
    w = si.make_weights(desc, seed=seed)
    for lw in w["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["w_down"] = np.zeros_like(lw["w_down"])
    V = desc["vocab"]
    period = period or V
    succ = np.arange(V)
    succ[:period] = (np.arange(period) + 1) % period
    unemb = np.empty_like(w["tok_emb"])
    unemb[succ[:period]] = w["tok_emb"][:period]
    unemb[period:] = w["tok_emb"][period:]
    w["unemb"] = unemb
    return desc, w, succ


def test_matcher_on_many_context_cuts():
    """Context rows are integer work: exact agreement at many context lengths, with
    back-off over q = 3, 2, 1 and real multi-group, tied-count hits.  The prompt
    follows the successor rule most of the time, so the generated token recurs."""
    desc, w, succ = _successor_model()
    model = oracle.Model(desc, w)
    ctx = ngg.Context(desc, w, max_seq=400, max_k=8, max_w=8)
    b = oracle.Bigram(model.tok_emb, model.unemb)
    rng = np.random.default_rng(11)
    x = [3]
    for _ in range(330):
        x.append(int(succ[x[-1]]) if rng.random() < 0.75 else int(rng.integers(0, 12)))
    x = np.array(x, dtype=np.int32)
    hits, multi = 0, 0
    for cut in list(range(3, 60)) + list(range(60, 330, 7)):
        ctx.prefill(x[:cut])
        toks = [int(t) for t in ctx.get_tokens()]
        assert toks[-1] == succ[toks[-2]]
        for cfg in (dict(k=8, w=3, k_ctx_max=8, q_min=1, q_max=3), dict(k=4, w=2, k_ctx_max=2, q_min=2, q_max=2),
                    dict(k=5, w=8, k_ctx_max=5, q_min=1, q_max=1), dict(k=8, w=1, k_ctx_max=5, q_min=2, q_max=3)):
            g_d, g_src, g_n = ctx.build_drafts(cfg)
            o_d, o_src, o_n = oracle.build_drafts(toks, b, cfg["k"], cfg["w"], cfg["k_ctx_max"], cfg["q_min"], cfg["q_max"])
            assert g_n == o_n and np.array_equal(g_src, o_src) and np.array_equal(g_d[:o_n], o_d[:o_n]), (cut, cfg)
            assert np.array_equal(g_d, o_d), (cut, cfg)
            hits += g_n
            multi += g_n > 1
    ctx.close()
    assert hits > 300 and multi > 50


def test_degenerate_contexts_for_the_matcher():
    for period, start, n in ((1, 0, 200), (3, 0, 180), (7, 2, 150)):
        desc, w, succ = _successor_model(period)
        model = oracle.Model(desc, w)
        ctx = ngg.Context(desc, w, max_seq=256, max_k=6, max_w=4)
        b = oracle.Bigram(model.tok_emb, model.unemb)
        x = [start]
        while len(x) < n:
            x.append(int(succ[x[-1]]))
        ctx.prefill(np.array(x, dtype=np.int32))
        toks = [int(t) for t in ctx.get_tokens()]
        assert toks[-1] == succ[toks[-2]]
        g_d, g_src, g_n = ctx.build_drafts(dict(k=6, w=4, k_ctx_max=6, q_min=1, q_max=3))
        o_d, o_src, o_n = oracle.build_drafts(toks, b, 6, 4, 6, 1, 3)
        assert g_n == o_n == 1 and np.array_equal(g_d, o_d)
        # a whole speculative run on the periodic stream: every call accepts all w drafted tokens
        out, stats = ctx.greedy_decode(np.array(x, dtype=np.int32), 41, dict(k=6, w=4, k_ctx_max=6, q_min=1, q_max=3))
        assert list(out) == oracle.greedy_plain_cached(model, x, 41)
        assert stats["new_hist"][5] == stats["calls"] == 8
        ctx.close()


def test_matcher_on_long_contexts_with_thousands_of_matches():
    """Contexts of several thousand tokens whose last token is frequent: hundreds to thousands of matching
    windows, grouped through the hash table and ranked by repeated selection; exact against the oracle.
    The model predicts succ(x) = x + 1, and every cut ends on a token whose successor is frequent in the
    stream, so the generated last token has many earlier occurrences."""
    desc, w, succ = _successor_model()
    ctx = ngg.Context(desc, w, max_seq=5200, max_k=32, max_w=8)
    rng = np.random.default_rng(21)
    streams = ((si.prompt_spans(desc["vocab"], 5000, copied=0.5, seed=6), 0), (rng.integers(0, 4, 2500).astype(np.int32), 1),
               (np.tile(np.array([3, 1, 4, 1, 5], dtype=np.int32), 600), 3), (np.zeros(3000, dtype=np.int32) + 2, 1))
    rows_found = 0
    for x, last in streams:
        for cut in (len(x), len(x) - 1, len(x) // 2 + 3):
            piece = x[:cut].copy()
            piece[-1] = last
            ctx.prefill(piece)
            toks = [int(t) for t in ctx.get_tokens()]
            assert toks[-1] == last + 1
            for cfg in (dict(k=16, w=6, k_ctx_max=16, q_min=1, q_max=3), dict(k=32, w=2, k_ctx_max=32, q_min=1, q_max=1),
                        dict(k=5, w=8, k_ctx_max=3, q_min=2, q_max=2)):
                g_d, g_src, g_n = ctx.build_drafts(cfg)
                want = oracle.context_rows(toks, cfg["w"], cfg["k_ctx_max"], cfg["q_min"], cfg["q_max"])
                assert g_n == len(want) and [tuple(int(t) for t in r) for r in g_d[:g_n]] == [tuple(r) for r in want], (len(x), cut, cfg)
                rows_found += g_n
    ctx.close()
    assert rows_found > 100


def test_adaptive_allocation_follows_the_oracle():
    """The adaptive row allocation (fewer context rows once their wins are seen to sit in the first ranks)
    inside the library's decode loop: same tokens, same per-call allocation and statistics as the oracle
    under the same rule, and a different allocation than the fixed cap on a stream where the context wins."""
    desc, w, succ = _successor_model(period=9)
    model = oracle.Model(desc, w)
    rng = np.random.default_rng(5)
    x = [2]
    for _ in range(150):
        x.append(int(succ[x[-1]]) if rng.random() < 0.8 else int(rng.integers(0, 9)))
    cfg = dict(k=8, w=3, k_ctx_max=8, q_min=1, q_max=2)
    ctx = ngg.Context(desc, w, max_seq=400, max_k=8, max_w=4)
    fixed_tok, fixed = ctx.greedy_decode(x, 60, cfg)
    with pytest.raises(ngg.NggError) as e:
        ctx.allocation(1, 0, 3)
    assert e.value.status == ngg.NGG_EINVAL
    ctx.allocation(1, 90, 3)
    got, st = ctx.greedy_decode(x, 60, cfg)
    ctx.allocation(0)
    again, st_fixed = ctx.greedy_decode(x, 60, cfg)
    ctx.close()
    want, o_st = oracle.greedy_speculative(model, x, 60, cfg["k"], cfg["w"], cfg["k_ctx_max"], cfg["q_min"], cfg["q_max"],
                                           allocation=dict(coverage_percent=90, warmup_wins=3))
    assert list(got) == want == list(fixed_tok) == list(again)
    assert st["calls"] == o_st["calls"] and st["alloc_hist"][:9] == o_st["alloc_hist"] and st["ctx_rows"] == sum(o_st["ctx_rows"])
    assert st["winner_src"] == o_st["winner_src"] and st["rank_hist"][0][:8] == o_st["rank_hist"][0]
    assert st_fixed["alloc_hist"] == fixed["alloc_hist"]                      # back to the fixed rule
    assert st["alloc_hist"] != fixed["alloc_hist"] and st["ctx_rows"] < fixed["ctx_rows"]
    print("adaptive allocation:", st["alloc_hist"][:9], "fixed:", fixed["alloc_hist"][:9])


def test_seeded_sweep_of_block_shapes_prompt_lengths_and_query_lengths(tiny):
    """Forty seeded combinations of k, w, context-row cap, query back-off range and prompt length on the tiny fp32
    model, two steps each, everything compared with the oracle (no tolerated disagreement in fp32)."""
    desc, run, w, prompt0, model, ctx = tiny
    rng = np.random.default_rng(2024)
    for case in range(40):
        k, wd = int(rng.integers(1, 33)), int(rng.integers(0, 9))
        q_min = int(rng.integers(1, 4))
        cfg = dict(k=k, w=wd, k_ctx_max=int(rng.integers(0, k + 1)), q_min=q_min, q_max=int(rng.integers(q_min, 5)))
        n_prompt = int(rng.integers(1, 200))
        prompt = si.prompt_spans(desc["vocab"], n_prompt, float(rng.uniform(0.1, 0.7)), seed=100 + case)
        print("case", case, cfg, n_prompt, flush=True)
        rep = lockstep_run(ctx, model, prompt, 2 * (wd + 1), cfg, TOL["f32"], max_steps=2)
        assert rep.tolerated_argmax == 0 and rep.tolerated_draft == 0 and rep.max_rel_logit_err <= 1e-4, (case, cfg, n_prompt)


def test_seeded_sweep_of_the_matcher_without_a_model():
    """Two hundred seeded token streams (alphabet 2 .. 5000 symbols, 1 .. 4000 tokens, with and without copied
    spans) x random (w, k_ctx_max, q_min, q_max): the context rows of the allocation-free entry point, which runs
    the same matcher kernel on a caller's token buffer, against the oracle, exactly."""
    import torch
    rng = np.random.default_rng(77)
    rows_total = 0
    for case in range(200):
        n = int(rng.integers(1, 4001))
        vocab = int(rng.choice([2, 3, 7, 50, 512, 5000]))
        x = (si.prompt_spans(vocab, n, float(rng.uniform(0.0, 0.8)), seed=500 + case) if rng.random() < 0.7
             else rng.integers(0, vocab, n).astype(np.int32))
        wd, kc = int(rng.integers(1, 33)), int(rng.integers(1, 33))
        q0 = int(rng.integers(1, 5)); q1 = int(rng.integers(q0, 8))
        t = torch.tensor(x, device="cuda")
        rows = torch.full((kc, wd), -1, dtype=torch.int32, device="cuda")
        n_rows = torch.zeros(1, dtype=torch.int32, device="cuda")
        ngg.context_drafts_static(t, wd, kc, q0, q1, rows, n_rows)
        torch.cuda.synchronize()
        want = oracle.context_rows(x, wd, kc, q0, q1)
        got = rows.cpu().numpy()[:int(n_rows.item())]
        assert [tuple(int(v) for v in r) for r in got] == [tuple(r) for r in want], (case, n, vocab, wd, kc, q0, q1)
        rows_total += len(want)
    assert rows_total > 500


def test_row_permutation_and_duplicate_rows(tiny):
    """Rows are independent given the shared prefix: a duplicate row gets the same logits as its original,
    permuting the rows permutes the results, and the committed tokens do not change (the winner is the
    first of the best rows in either order)."""
    desc, run, w, prompt, model, ctx = tiny
    truth = oracle.greedy_plain_cached(model, prompt, 8)
    ctx.prefill(prompt)
    assert int(ctx.get_tokens()[-1]) == truth[0]
    rng = np.random.default_rng(11)
    d = rng.integers(0, desc["vocab"], size=(4, 3)).astype(np.int32)
    d[1] = truth[1:4]                                     # the true continuation: accepted whole
    d[2, :2] = truth[1:3]                                 # right for two tokens, then wrong
    d[2, 2] = (truth[3] + 1) % desc["vocab"]
    d[3] = d[1]                                           # duplicate of the best row
    a = ctx.verify_step(d, want_logits=True)
    assert list(a["accept_len"])[1:] == [3, 2, 3] and a["winner"] == 1 and list(a["new_tokens"]) == truth[1:5]
    scale = np.max(np.abs(a["logits"]))
    assert np.max(np.abs(a["logits"][3] - a["logits"][1])) <= 1e-5 * scale
    assert np.array_equal(a["greedy"][3], a["greedy"][1])
    # rows 1 and 2 share two draft tokens: the same inputs up to column 2
    assert np.max(np.abs(a["logits"][2, :3] - a["logits"][1, :3])) <= 1e-5 * scale
    perm = [3, 2, 0, 1]
    b = ctx.verify_step(d[perm], want_logits=True)
    assert np.max(np.abs(b["logits"] - a["logits"][perm])) <= 1e-5 * scale
    assert np.array_equal(b["greedy"], a["greedy"][perm]) and list(b["accept_len"]) == list(a["accept_len"][perm])
    assert b["winner"] == 0 and list(b["new_tokens"]) == list(a["new_tokens"])


def test_profile_classes_count_launches_and_sampling(tiny):
    """HIP-event brackets per kernel class: one span per launch (n_layers per layer kernel and model call),
    one in every N with ngg_profile_sample, none when switched off; results are not affected."""
    desc, run, w, prompt, model, ctx = tiny
    L = desc["n_layers"]
    ctx.prefill(prompt)
    ref = ctx.verify_step(None, 1, 0)["new_tokens"]
    ctx.profile_reset()
    ctx.profile_enable(-1)
    for _ in range(3):
        assert list(ctx.verify_step(None, 1, 0)["new_tokens"]) == list(ref)
    prof = ctx.profile_read()
    for cls in ("gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down", "attention"):
        ms, cnt = prof[cls]
        assert cnt == 3 * L and ms > 0.0, cls
    assert prof["gemm_unembed"][1] == 3 and prof["norm"][1] == 3 * (2 * L + 1)
    ctx.profile_reset()
    ctx.profile_sample(L + 1)                            # one gate/up launch in every L + 1
    ctx.profile_enable(1 << ngg.PROF_CLASSES.index("gemm_gateup"))
    for _ in range(L + 1):
        ctx.verify_step(None, 1, 0)
    prof = ctx.profile_read()
    assert prof["gemm_gateup"][1] == L and prof["gemm_qkv"][1] == 0
    ctx.profile_enable(0)
    ctx.profile_sample(1)
    ctx.profile_reset()
    ctx.verify_step(None, 1, 0)
    assert all(cnt == 0 for _, cnt in ctx.profile_read().values())
    assert ctx.profile_bracket_overhead() > 0.0
    with pytest.raises(ngg.NggError):
        ctx.profile_sample(0)


def test_state_and_capacity_errors(tiny):
    desc, run, w, prompt, model, _ = tiny
    ctx = ngg.Context(desc, w, max_seq=140, max_k=4, max_w=3)
    with pytest.raises(ngg.NggError) as e:
        ctx.verify_step(np.zeros((2, 2), dtype=np.int32))
    assert e.value.status == ngg.NGG_ESTATE
    with pytest.raises(ngg.NggError) as e:
        ctx.commit()
    assert e.value.status == ngg.NGG_ESTATE
    with pytest.raises(ngg.NggError) as e:
        ctx.decode_more(4, 2, run)                        # nothing to continue from
    assert e.value.status == ngg.NGG_ESTATE
    ctx.prefill(prompt)                                   # n = 129
    with pytest.raises(ngg.NggError) as e:
        ctx.verify_step(np.zeros((5, 2), dtype=np.int32))
    assert e.value.status == ngg.NGG_ECAPACITY
    with pytest.raises(ngg.NggError) as e:
        ctx.verify_step(np.full((2, 2), desc["vocab"], dtype=np.int32))
    assert e.value.status == ngg.NGG_EINVAL
    with pytest.raises(ngg.NggError) as e:
        ctx.verify_step(None, 2, 2)                       # no drafts on the device
    assert e.value.status == ngg.NGG_ESTATE
    with pytest.raises(ngg.NggError) as e:
        ctx.prefill(np.zeros(200, dtype=np.int32))
    assert e.value.status == ngg.NGG_ECAPACITY
    ctx.prefill(prompt)
    ctx.verify_step(np.zeros((2, 2), dtype=np.int32))
    with pytest.raises(ngg.NggError) as e:
        ctx.commit(0)
    assert e.value.status == ngg.NGG_EINVAL
    assert ctx.commit(1) == 1
    with pytest.raises(ngg.NggError):
        ctx.commit()                                      # already committed
    # decode right up to max_seq
    out, _ = ctx.greedy_decode(prompt, 12, run)
    assert list(out) == oracle.greedy_plain_cached(model, prompt, 12)
    with pytest.raises(ngg.NggError) as e:
        ctx.greedy_decode(prompt, 13, run)
    assert e.value.status == ngg.NGG_ECAPACITY
    ctx.close()


def test_grouped_query_attention_and_random_gains():
    desc = dict(si.MODELS["tiny"], n_kv_heads=2)
    run = si.RUNS["cfg1"]
    w, prompt, model, ctx = _setup(desc, run, seed=5, random_gains=True)
    rep = lockstep_run(ctx, model, prompt, 24, run, TOL["f32"])
    ctx.close()
    assert rep.tolerated_argmax == 0 and rep.max_rel_logit_err <= 1e-4


@pytest.mark.parametrize("hd,heads,kv", [(64, 12, 4), (128, 8, 2), (32, 8, 1)])
def test_grouped_query_attention_16_bit(hd, heads, kv):
    """Grouped-query attention in the 16-bit configuration, every head_dim the library takes, random gains: 3, 4 and
    8 query heads per key/value head; verify blocks (shared kernel), single-token steps (stream kernel), prefill."""
    desc = dict(si.reduced_layers(si.MODELS["small"], 2), n_heads=heads, n_kv_heads=kv, head_dim=hd, d_model=heads * hd,
                vocab=4096)
    run = dict(si.RUNS["cfg2"], prompt_len=300, n_gen=12)
    w, prompt, model, ctx = _setup(desc, run, seed=6, random_gains=True)
    rep = lockstep_run(ctx, model, prompt, 12, run, TOL["bf16"], max_steps=3)
    rep1 = lockstep_run(ctx, model, prompt[:77], 5, dict(k=1, w=0, k_ctx_max=0, q_min=1, q_max=1), TOL["bf16"])
    ctx.close()
    print("16-bit GQA:", hd, heads, kv, rep, rep1)
    assert rep.max_rel_logit_err <= 2e-2 and rep1.max_rel_logit_err <= 2e-2


def test_weight_rescaling_keeps_small_rows_exact_16_bit():
    """The library multiplies bf16 weights as fp16 operands after an exact power-of-two rescale per matrix.  Output
    embedding rows spread over 18 binary orders of magnitude (the smallest far below fp16's normal range before the
    rescale) must all give bigram scores as accurate as fp32 accumulation allows, relative to each row's own size."""
    desc = dict(si.reduced_layers(si.MODELS["small"], 1), vocab=2048)
    run = dict(si.RUNS["cfg2"], prompt_len=64, n_gen=4)
    w = si.make_weights(desc, seed=8)
    exps = np.random.default_rng(8).integers(-12, 7, desc["vocab"])
    w["unemb"] = (w["unemb"] * (2.0 ** exps)[:, None]).astype(np.float32)          # exact: powers of two on bf16 values
    ctx = ngg.Context(desc, w, max_seq=128, max_k=8, max_w=4)
    prompt = si.make_prompt(run, desc["vocab"], seed=1)
    ctx.prefill(prompt)
    x_last = int(ctx.get_tokens()[-1])
    ctx.build_drafts(run)
    z, _ = ctx.debug_peek("z", np.float32)
    ctx.close()
    zo = oracle.bigram_scores(w["tok_emb"], w["unemb"], x_last)
    row_size = np.linalg.norm(w["unemb"].astype(np.float64), axis=1) * np.linalg.norm(w["tok_emb"][x_last].astype(np.float64))
    rel = np.abs(z - zo) / row_size
    print("rescaled rows: max error relative to |u_v||e| =", rel.max(), "at exponent", exps[int(np.argmax(rel))])
    assert rel.max() <= 1e-5


def test_damped_residual_variant_accepts_bigram_rows():
    """W_o and W_down scaled by 1e-2: the embedding path dominates, so bigram rows
    are accepted (a labelled variant for coverage, not a headline configuration)."""
    desc, run = si.MODELS["tiny"], si.RUNS["cfg1"]
    w = si.make_weights(desc, seed=2)
    for lw in w["layers"]:
        lw["wo"] = lw["wo"] * np.float32(1e-2)
        lw["w_down"] = lw["w_down"] * np.float32(1e-2)
    prompt = si.make_prompt(run, desc["vocab"], seed=3)
    model = oracle.Model(desc, w)
    ctx = ngg.Context(desc, w, max_seq=256, max_k=4, max_w=3)
    cfg = dict(run, k_ctx_max=0)
    rep = lockstep_run(ctx, model, prompt, 40, cfg, TOL["f32"])
    ctx.close()
    print("damped:", rep)
    assert max(rep.new_hist) > 1


# ---------------------------------------------------------------------------------------------
# the paper's own bigram: the whole model on one-token contexts, as a precomputed table
# ---------------------------------------------------------------------------------------------

def _check_table_rows(table, mb, xs, tol):
    """Rows of the GPU table against the oracle's ranking; ids may differ only at near-ties."""
    K = table.shape[1]
    swaps = 0
    for x in xs:
        z = mb.scores(int(x))
        order = oracle.rank_ids(z, K)
        for i in range(K):
            g, o = int(table[x, i]), int(order[i])
            if g != o:
                assert abs(z[g] - z[o]) < tol * np.max(np.abs(z)), f"table[{x}][{i}]: GPU {g} vs oracle {o}"
                swaps += 1
    return swaps


def test_full_model_bigram_table_fp32(tiny):
    desc, run, _, prompt, model, ctx = tiny
    with pytest.raises(ngg.NggError) as e:
        ctx.bigram_source(1)                                   # no table yet
    assert e.value.status == ngg.NGG_ESTATE
    with pytest.raises(ngg.NggError) as e:
        ctx.bigram_table_build(4)                              # fewer ranks than max_k rows
    assert e.value.status == ngg.NGG_EINVAL
    ctx.bigram_table_build(32)
    table = ctx.debug_peek("bg_table", np.int32)[0].reshape(desc["vocab"], 32)
    mb = oracle.ModelBigram(lambda x: model.forward_full([x])[-1])
    assert _check_table_rows(table, mb, range(desc["vocab"]), TOL["f32"]) == 0     # every one-token context
    ctx.bigram_source(1)
    try:
        rep = lockstep_run(ctx, model, prompt, 40, run, TOL["f32"], bigram=mb)
        cfg = dict(k=16, w=6, k_ctx_max=4, q_min=1, q_max=3)
        rep2 = lockstep_run(ctx, model, prompt, 20, cfg, TOL["f32"], bigram=mb, max_steps=4)
    finally:
        ctx.bigram_source(0)
    print("table mode:", rep, rep2)
    assert rep.tolerated_argmax == 0 and rep.tolerated_draft == 0 and rep2.tolerated_draft == 0
    rep3 = lockstep_run(ctx, model, prompt, 12, run, TOL["f32"])                    # back on the direct path
    assert rep3.tolerated_draft == 0


def test_full_model_bigram_table_bf16():
    """Small bf16 widths, 3 layers, vocabulary 32000: the table of all 32000 one-token contexts,
    sampled rows against the oracle, then a few steps in table mode."""
    desc = si.reduced_layers(si.MODELS["small"], 3)
    run = dict(si.RUNS["cfg2"], prompt_len=200, n_gen=24)
    w, prompt, model, ctx = _setup(desc, run)
    ctx.bigram_table_build(run["k"])
    table = ctx.debug_peek("bg_table", np.int32)[0].reshape(desc["vocab"], run["k"])
    mb = oracle.ModelBigram(lambda x: model.forward_full([x])[-1])
    xs = [0, 1, 31999] + [int(t) for t in np.random.default_rng(3).integers(0, desc["vocab"], 13)]
    swaps = _check_table_rows(table, mb, xs, TOL["bf16"])
    ctx.bigram_source(1)
    rep = lockstep_run(ctx, model, prompt, 24, run, TOL["bf16"], bigram=mb, max_steps=4)
    ctx.close()
    print("bf16 table:", swaps, "near-tie swaps in", len(xs), "rows;", rep)
    assert rep.max_rel_logit_err <= 2e-2


# ---------------------------------------------------------------------------------------------
# the model unigram (q = 0 drafts)
# ---------------------------------------------------------------------------------------------

def _check_unigram(top, d, tol):
    """GPU ranking of the nearest tokens against the oracle's distances; swaps only between near-ties."""
    order = oracle.rank_ids(-d, len(top))
    swaps = 0
    for g, o in zip(top, order):
        if int(g) != int(o):
            assert abs(d[int(g)] - d[int(o)]) < tol * np.max(d), f"unigram: GPU {g} vs oracle {o}"
            swaps += 1
    return swaps


def test_unigram_drafts_fp32(tiny):
    desc, run, w, prompt, model, ctx = tiny
    with pytest.raises(ngg.NggError) as e:
        ctx.bigram_source(2)                                   # not built yet
    assert e.value.status == ngg.NGG_ESTATE
    ctx.unigram_build(32)
    top = ctx.debug_peek("uni_top", np.int32)[0]
    ug = oracle.UnigramDrafts(w["tok_emb"], w["unemb"], oracle.Bigram(model.tok_emb, model.unemb))
    assert _check_unigram(top, ug.d, TOL["f32"]) == 0
    ctx.bigram_source(2)
    try:
        rep = lockstep_run(ctx, model, prompt, 30, run, TOL["f32"], bigram=ug)
        rep2 = lockstep_run(ctx, model, prompt, 12, dict(k=16, w=6, k_ctx_max=3, q_min=1, q_max=3), TOL["f32"], bigram=ug, max_steps=3)
    finally:
        ctx.bigram_source(0)
    print("unigram mode:", rep, rep2)
    assert rep.tolerated_draft == 0 and rep2.tolerated_draft == 0 and rep.tolerated_argmax == 0


def test_unigram_bf16_vocabulary_32000():
    desc = si.reduced_layers(si.MODELS["small"], 2)
    run = dict(si.RUNS["cfg2"], prompt_len=150, n_gen=16)
    w, prompt, model, ctx = _setup(desc, run)
    ctx.unigram_build(16)
    top = ctx.debug_peek("uni_top", np.int32)[0]
    ug = oracle.UnigramDrafts(w["tok_emb"], w["unemb"], oracle.Bigram(model.tok_emb, model.unemb))
    swaps = _check_unigram(top, ug.d, TOL["bf16"])
    ctx.bigram_source(2)
    g_drafts, g_src, g_nctx = None, None, None
    ctx.prefill(prompt)
    g_drafts, g_src, g_nctx = ctx.build_drafts(run)
    ctx.close()
    print("bf16 unigram:", swaps, "near-tie swaps in 16;", list(top[:6]), "first draft tokens", list(g_drafts[g_nctx:, 0]))
    assert list(g_drafts[g_nctx:, 0]) == [int(t) for t in top[:run["k"] - g_nctx]]      # rows start with the kept tokens, in order


# ---------------------------------------------------------------------------------------------
# bf16 configurations
# ---------------------------------------------------------------------------------------------

def test_cfg2_small_bf16_lockstep():
    desc, run = si.MODELS["small"], si.RUNS["cfg2"]
    w, prompt, model, ctx = _setup(desc, run)
    rep = lockstep_run(ctx, model, prompt, run["n_gen"], run, TOL["bf16"])       # all 256 tokens, logits at every step
    print("cfg2:", rep)
    assert rep.max_rel_logit_err <= 2e-2
    # The GPU's own plain decoding of the same prompt: in bf16 the two GPU runs round differently (other
    # key spans, other block shapes), so they may part at a near-tie; each is checked against the oracle
    # with the margin rule instead of against the other.
    rep_plain = lockstep_run(ctx, model, prompt, 40, dict(k=1, w=0, k_ctx_max=0, q_min=1, q_max=1), TOL["bf16"])
    ctx.close()
    print("cfg2 plain:", rep_plain)
    positions = rep.steps * run["k"] * (run["w"] + 1)
    assert rep.tolerated_argmax <= 0.1 * positions


@pytest.mark.parametrize("k,w", [(16, 0), (16, 6), (32, 8), (13, 4), (12, 7), (13, 9), (20, 7), (32, 7), (20, 14), (32, 32)])
def test_bf16_blocks_of_more_than_64_rows(k, w):
    """Blocks of 112, 288, 65 and 96 rows on the small 16-bit widths (3 layers): GEMM row tiles of 7, 8, 5
    and 6 column blocks and the attention workgroups with two query groups per wave; then the wide GEMM
    kernel (more than 128 rows in one pass over the weights): 130, 160, 256 and 288 rows (tiles of 10, 10, 16
    and 18 row blocks), 300 rows (two row tiles of 160 in one launch) and 1056 rows (four row tiles of 272)."""
    desc = si.reduced_layers(si.MODELS["small"], 3)
    run = dict(si.RUNS["cfg2"], prompt_len=333, k=k, w=w, k_ctx_max=k, q_min=1, q_max=3, n_gen=30)
    w_, prompt, model, ctx = _setup(desc, run)
    rep = lockstep_run(ctx, model, prompt, 30, run, TOL["bf16"], max_steps=4)
    ctx.close()
    print("wide block:", k, w, rep)
    assert rep.max_rel_logit_err <= 2e-2


def test_prefill_piece_boundaries_16_bit():
    """Prompt lengths around the row tiles of the prefill (16-bit models take pieces of up to 2048 tokens; the wide
    GEMM kernel cuts a piece into tiles of up to 288 rows, the skinny kernel takes up to 128 rows) and around the
    piece boundary itself, on the small 16-bit widths (2 layers).  A context created with a short max_seq has
    shorter pieces (max_seq rounded up to 256): the second loop runs the same prompts through 768-token pieces."""
    desc = si.reduced_layers(si.MODELS["small"], 2)
    run = dict(si.RUNS["cfg2"], prompt_len=2400, n_gen=8)
    w_, _, model, ctx = _setup(desc, run)
    for n_prompt in (129, 200, 256, 257, 288, 289, 300, 513, 577, 1000, 2047, 2048, 2049, 2305):
        prompt = si.prompt_spans(desc["vocab"], n_prompt, 0.3, seed=7)
        rep = lockstep_run(ctx, model, prompt, 4, run, TOL["bf16"], max_steps=1)
        assert rep.max_rel_logit_err <= 2e-2, n_prompt
    ctx.close()
    run = dict(si.RUNS["cfg2"], prompt_len=700, n_gen=8)                  # max_seq 716: pieces of 768 tokens
    w_, _, model, ctx = _setup(desc, run)
    for n_prompt in (255, 384, 640, 700):
        prompt = si.prompt_spans(desc["vocab"], n_prompt, 0.3, seed=7)
        rep = lockstep_run(ctx, model, prompt, 4, run, TOL["bf16"], max_steps=1)
        assert rep.max_rel_logit_err <= 2e-2, n_prompt
    ctx.close()


def test_row_tiles_of_256_with_an_odd_number_of_contraction_slices_16_bit():
    """The 32x32x16 GEMM kernel takes tiles of 192 and 256 rows; its main loop handles two 64-element slices of the
    contraction per trip and one more after it when their number is odd.  Widths of 192 (3 slices) and 448 (7 slices),
    2 layers: a 512-token prompt is prefilled as two 256-row tiles (all four GEMMs on that kernel), then verify blocks
    of 241 and 177 rows (one tile of 256 and of 192 rows: q/k/v and gate/up on it) and a step of the default shape."""
    desc = dict(si.reduced_layers(si.MODELS["small"], 2), n_heads=3, n_kv_heads=3, head_dim=64, d_model=192, d_ffn=448,
                vocab=4096)
    run = dict(si.RUNS["cfg2"], prompt_len=512, n_gen=64)
    w_, prompt, model, ctx = _setup(desc, run, max_k=16, max_w=15)
    rep = lockstep_run(ctx, model, prompt, 8, run, TOL["bf16"], max_steps=1)
    assert rep.max_rel_logit_err <= 2e-2, rep
    for k, wd in ((16, 15), (16, 11)):
        cfg = dict(run, k=k, w=wd, k_ctx_max=4)
        rep = lockstep_run(ctx, model, prompt, 2 * (wd + 1), cfg, TOL["bf16"], max_steps=1)
        print("odd slices:", k, wd, rep)
        assert rep.max_rel_logit_err <= 2e-2, (k, wd, rep)
    ctx.close()


def test_7b_width_two_layer_twin_bf16_lockstep():
    """7B widths (d 4096, 32 heads of 128, FFN 14336, vocab 32000) with 2 layers so
    the oracle can run it: prompt 2048, k=10, w=5 -- the launch shapes of config 3."""
    desc = si.reduced_layers(si.MODELS["7b"], 2)
    run = dict(si.RUNS["cfg3"], n_gen=20)
    w, prompt, model, ctx = _setup(desc, run)
    rep = lockstep_run(ctx, model, prompt, 20, run, TOL["bf16"], max_steps=6)
    ctx.close()
    print("7b twin:", rep)
    assert rep.max_rel_logit_err <= 2e-2


def test_7b_width_one_layer_twin_long_context_shape():
    """The long-context configuration's draft shape (k=16, w=6: 112 block rows, query back-off q=3..1)
    at 7B widths, one layer, prompt 1536: the 128-row GEMM tiles at K = 4096 / 14336 and the
    two-query-group attention workgroups at head_dim 128."""
    desc = si.reduced_layers(si.MODELS["7b"], 1)
    run = dict(si.RUNS["cfg4"], prompt_len=1536, n_gen=20)
    w, prompt, model, ctx = _setup(desc, run)
    rep = lockstep_run(ctx, model, prompt, 20, run, TOL["bf16"], max_steps=3)
    ctx.close()
    print("7b one-layer twin, k=16 w=6:", rep)
    assert rep.max_rel_logit_err <= 2e-2


def test_7b_width_one_layer_twin_at_the_long_context_configurations_own_length():
    """Config 4 at its own context: prompt 16384 (50 % copied spans), k=16, w=6 (112 block rows), query
    back-off q = 3..1, 7B widths, one layer.  The oracle takes the prompt in 512-token pieces through its
    cached block call.  Covers what the shorter twins do not reach: rotary angles, cache tiles and the key
    list at positions up to 16.4K, and the attention launch this shape takes (its slice count and workgroup
    count are asserted, so a change of the layout shows up here)."""
    desc = si.reduced_layers(si.MODELS["7b"], 1)
    run = dict(si.RUNS["cfg4"], n_gen=16)
    assert run["prompt_len"] == 16384 and (run["k"], run["w"]) == (16, 6)
    w = si.make_weights(desc, seed=0)
    prompt = si.make_prompt(run, desc["vocab"], seed=1)
    model = oracle.Model(desc, w, widen_at_use=True)
    ctx = ngg.Context(desc, w, max_seq=run["prompt_len"] + 64, max_k=run["k"], max_w=run["w"])
    layouts = []
    rep = lockstep_run(ctx, model, prompt, 16, run, TOL["bf16"], max_steps=2, oracle_chunk=512,
                       on_step=lambda step: layouts.append(ctx.debug_peek("attn_layout", np.int32)[0].tolist()))
    ctx.close()
    print("7b one-layer twin at 16384 tokens, k=16 w=6:", rep, layouts)
    assert rep.steps == 2 and rep.max_rel_logit_err <= 2e-2
    for n_splits, wgs, M, P in layouts:
        assert M == 1 + 16 * 6 and P >= 16384             # 97 distinct block tokens: the shared first column is computed once
        assert n_splits >= 8 and wgs >= 256               # the key list of every head is cut into slices that fill the chip
    assert layouts[0][:2] == list(EXPECTED_LONG_CONTEXT_LAYOUT), layouts[0]


EXPECTED_LONG_CONTEXT_LAYOUT = (16, 512)      # slices per head, workgroups (two per CU) at M = 112, P = 16384, 32 heads


@pytest.mark.parametrize("k,w", [(10, 5), (32, 8)])
def test_3b_width_one_layer_twin_at_the_large_vocabulary_configurations_own_length(k, w):
    """Config 5 at its own context: prompt 4096, 3B widths (24 heads of 128, vocabulary 128256), one layer;
    k=10, w=5 and the largest block of its grid, k=32, w=8 (288 rows)."""
    desc = si.reduced_layers(si.MODELS["3b"], 1)
    run = dict(si.RUNS["cfg5"], k=k, w=w, k_ctx_max=k, n_gen=20)
    assert run["prompt_len"] == 4096
    w_ = si.make_weights(desc, seed=0)
    prompt = si.make_prompt(run, desc["vocab"], seed=1)
    model = oracle.Model(desc, w_, widen_at_use=True)
    ctx = ngg.Context(desc, w_, max_seq=run["prompt_len"] + 64, max_k=k, max_w=w)
    layouts = []
    rep = lockstep_run(ctx, model, prompt, 20, run, TOL["bf16"], max_steps=2, oracle_chunk=1024,
                       on_step=lambda step: layouts.append(ctx.debug_peek("attn_layout", np.int32)[0].tolist()))
    ctx.close()
    print("3b one-layer twin at 4096 tokens:", k, w, rep, layouts)
    assert rep.steps == 2 and rep.max_rel_logit_err <= 2e-2
    assert layouts[0][2] == 1 + k * w and layouts[0][3] >= 4096 and layouts[0][1] >= 240


@pytest.mark.parametrize("k,w", [(10, 5), (32, 8)])
def test_3b_width_one_layer_twin_large_vocabulary(k, w):
    """The large-vocabulary configuration's widths (d 3072, 24 heads of 128, FFN 8192, vocab 128256),
    one layer, prompt 512: bigram sweep, next1 table and argmax over 128256 rows; k=32, w=8 is the
    largest block of its sweep (288 rows: three passes of 128-row tiles)."""
    desc = si.reduced_layers(si.MODELS["3b"], 1)
    run = dict(si.RUNS["cfg5"], prompt_len=512, k=k, w=w, k_ctx_max=k, n_gen=20)
    w_, prompt, model, ctx = _setup(desc, run)
    rep = lockstep_run(ctx, model, prompt, 20, run, TOL["bf16"], max_steps=2)
    ctx.close()
    print("3b one-layer twin:", k, w, rep)
    assert rep.max_rel_logit_err <= 2e-2
