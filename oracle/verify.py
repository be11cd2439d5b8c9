"""Guess-and-verify step and decode loops, CPU oracle (test infrastructure).

Section 3 fixes the verify call (input block (k, w+1): the one uncached context
token followed by w drafted tokens per row).  The introduction fixes the
acceptance rule (a drafted token is kept when the base model would have
predicted it).  Appendix D fixes the commit (every row's cache becomes that of
the longest accepted speculation).  Because only tokens the model itself would
have produced are kept, the committed sequence equals plain greedy decoding;
`greedy_plain` is that definition, written out with no cache at all.
"""
from __future__ import annotations

import numpy as np

from .model import Model, KVCache, greedy_argmax
from .drafts import Bigram, build_drafts


def accept_lengths(drafts, greedy):
    """a[r] = number of leading drafted tokens of row r that equal the model's
    greedy prediction at the preceding block position: drafts[r][i] == greedy[r][i]
    for all i < a[r].  drafts [k, w], greedy [k, w+1]."""
    drafts = np.asarray(drafts)
    greedy = np.asarray(greedy)
    k, w = drafts.shape
    a = np.zeros(k, dtype=np.int32)
    for r in range(k):
        n = 0
        while n < w and drafts[r, n] == greedy[r, n]:
            n += 1
        a[r] = n
    return a


def select_winner(a):
    """Row with the longest accepted prefix; equal lengths go to the lowest row."""
    a = np.asarray(a)
    r = int(np.argmax(a))
    return r, int(a[r])


class State:
    """tokens: the whole context (prompt + generated), the last one uncached;
    cache: keys/values of tokens[:-1]."""

    def __init__(self, tokens, cache: KVCache):
        self.tokens = [int(t) for t in tokens]
        self.cache = cache


def prefill(model: Model, prompt, chunk: int | None = None, progress=None) -> State:
    """Run the prompt, cache all of it, append the first greedy token.  With
    `chunk`, the prompt goes through the model in pieces of that many tokens, each
    a (1, chunk) block on the cache of the pieces before it: the same causal
    forward pass (Section 3's block call with k = 1), with bounded memory.
    `progress(tokens_done)` is called after every piece."""
    prompt = [int(t) for t in prompt]
    cache = KVCache(model.L, model.Hkv, model.hd)
    step = len(prompt) if not chunk else int(chunk)
    for p0 in range(0, len(prompt), step):
        piece = np.asarray(prompt[p0:p0 + step])[None, :]
        last = p0 + step >= len(prompt)
        logits, kv = model.forward_block(piece, cache if p0 else None, want_logits=last)
        for li, (kk, vv) in enumerate(kv):
            cache.append(li, kk[0], vv[0])
        if progress:
            progress(min(p0 + step, len(prompt)))
    first = int(greedy_argmax(logits[0, -1]))
    st = State(prompt + [first], cache)
    st.first_logits = logits[0, -1]              # logits that chose the first generated token
    return st


def verify_step(model: Model, state: State, drafts):
    """One model call on the block [x_last, drafts[r]] for every row r, then the
    per-position greedy tokens, accepted lengths and the winner.  Does not change
    the state.  New tokens = the winner's accepted drafts plus the model's own
    prediction after them (1 .. w+1 tokens)."""
    drafts = np.asarray(drafts, dtype=np.int32)
    k, w = drafts.shape
    block = np.concatenate([np.full((k, 1), state.tokens[-1], dtype=np.int32), drafts], axis=1)
    logits, kv = model.forward_block(block, state.cache)
    greedy = greedy_argmax(logits)
    a = accept_lengths(drafts, greedy)
    r, n_acc = select_winner(a)
    new_tokens = [int(t) for t in drafts[r, :n_acc]] + [int(greedy[r, n_acc])]
    return dict(block=block, logits=logits, greedy=greedy, accept_len=a, winner=r,
                n_accept=n_acc, new_tokens=new_tokens, block_kv=kv)


def commit(state: State, res: dict, max_new: int | None = None, tokens_override=None) -> int:
    """Append the new tokens (at most max_new) and the winner row's keys/values
    for the block columns they came from.  `tokens_override` lets a lock-step
    comparison force a different (tolerated) final token."""
    new = list(res["new_tokens"] if tokens_override is None else tokens_override)
    if max_new is not None:
        new = new[:max_new]
    n_new = len(new)
    r = res["winner"]
    for li, (kk, vv) in enumerate(res["block_kv"]):
        state.cache.append(li, kk[r, :n_new], vv[r, :n_new])
    state.tokens.extend(int(t) for t in new)
    return n_new


def greedy_plain(model: Model, prompt, n_gen: int):
    """Plain greedy decoding with no cache: the whole sequence is re-run for
    every new token.  This is the definition the speculative loop must equal."""
    toks = [int(t) for t in prompt]
    for _ in range(n_gen):
        logits = model.forward_full(toks)
        toks.append(int(greedy_argmax(logits[-1])))
    return toks[len(prompt):]


def greedy_plain_cached(model: Model, prompt, n_gen: int):
    """Plain greedy decoding, one (1, 1) model call per token on the KV cache:
    the (k, w) = (1, 0) case of the verify step."""
    st = prefill(model, prompt)
    out = [st.tokens[-1]]
    while len(out) < n_gen:
        res = verify_step(model, st, np.zeros((1, 0), dtype=np.int32))
        commit(st, res)
        out.append(st.tokens[-1])
    return out[:n_gen]


def adaptive_context_cap(ctx_rank_wins, k_ctx_max: int, coverage_percent: int, warmup_wins: int) -> int:
    """Context rows allowed in the next call under the adaptive allocation: the ablation of Section 5.2 finds
    the context strategy's wins in its first few rows while it often fills the whole batch.  Once
    `warmup_wins` calls were won by a context row (with an accepted token), allow the smallest number of
    leading context rows that held `coverage_percent` of those wins; at least 1, at most k_ctx_max."""
    total = sum(ctx_rank_wins)
    if total < warmup_wins:
        return k_ctx_max
    seen = 0
    for r, n in enumerate(ctx_rank_wins):
        seen += n
        if 100 * seen >= coverage_percent * total:
            return min(k_ctx_max, max(1, r + 1))
    return k_ctx_max


def greedy_speculative(model: Model, prompt, n_gen: int, k: int, w: int, k_ctx_max: int,
                       q_min: int, q_max: int, bigram: Bigram | None = None, allocation: dict | None = None):
    """Greedy decoding with batched learning-free drafts.  Returns
    (generated tokens [n_gen], stats) with stats = calls, tokens per call,
    histogram of new tokens per call, winner source counts, context rows found.
    `allocation` = dict(coverage_percent, warmup_wins) switches the row allocation
    from the fixed cap k_ctx_max (Section 4.3) to adaptive_context_cap."""
    bigram = bigram or Bigram(model.tok_emb, model.unemb)
    st = prefill(model, prompt)
    n0 = len(prompt)
    # accept_hist / rank_hist / alloc_hist: the quantities of the ablation on strategies (Section 5.2)
    stats = dict(calls=0, new_hist=[0] * (w + 2), winner_src=[0, 0], ctx_rows=[],
                 accept_hist=[[0] * (w + 1), [0] * (w + 1)], rank_hist=[[0] * k, [0] * k], alloc_hist=[0] * (k + 1))
    while len(st.tokens) - n0 < n_gen:
        cap = k_ctx_max
        if allocation:
            cap = adaptive_context_cap(stats["rank_hist"][0], k_ctx_max, allocation["coverage_percent"], allocation["warmup_wins"])
        drafts, src, n_ctx = build_drafts(st.tokens, bigram, k, w, cap, q_min, q_max)
        res = verify_step(model, st, drafts)
        n_new = commit(st, res, max_new=n_gen - (len(st.tokens) - n0))
        stats["calls"] += 1
        stats["new_hist"][n_new] += 1
        ws = int(src[res["winner"]])
        stats["winner_src"][ws] += 1
        stats["ctx_rows"].append(n_ctx)
        stats["accept_hist"][ws][res["n_accept"]] += 1
        if res["n_accept"] > 0:
            stats["rank_hist"][ws][res["winner"] - n_ctx if ws else res["winner"]] += 1
        stats["alloc_hist"][n_ctx] += 1
    gen = st.tokens[n0:n0 + n_gen]
    stats["tokens_per_call"] = (len(gen) - 1) / max(1, stats["calls"])
    return gen, stats
