"""Pins for the oracle's draft construction (Sections 4.1-4.3): hand-worked
cases, closed forms and brute force on tiny inputs.  CPU only."""
import os

import numpy as np
import pytest

import synth_inputs as si
from oracle import (context_ngram_groups, context_rows, bigram_scores, rank_ids, Bigram, build_drafts,
                    unigram_distances, UnigramDrafts)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "context_ngram_cases.txt")


def _golden_cases():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, ctx, exp = [p.strip() for p in line.split("|")]
        q, w = [int(t) for t in head.split()]
        rows = []
        if exp != "-":
            for item in exp.split():
                toks, cnt, last = item.split(":")
                rows.append((tuple(int(t) for t in toks.split(",")), int(cnt), int(last)))
        cases.append((q, w, [int(t) for t in ctx.split()], rows))
    return cases


@pytest.mark.parametrize("q,w,ctx,rows", _golden_cases())
def test_matcher_hand_worked_cases(q, w, ctx, rows):
    assert context_ngram_groups(ctx, q, w) == rows


def _brute_force_groups(x, q, w):
    """Quadratic enumeration: every matching window is compared with every other."""
    n = len(x)
    starts = [i for i in range(n) if i + q + w <= n and all(x[i + t] == x[n - q + t] for t in range(q))]
    out = []
    for i in starts:
        same = [j for j in starts if all(x[j + q + t] == x[i + q + t] for t in range(w))]
        if i == max(same):                                   # one representative per continuation: its last match
            out.append((tuple(x[i + q:i + q + w]), len(same), i))
    # rank: repeatedly pull the best remaining (count, then later start)
    ranked = []
    while out:
        best = out[0]
        for g in out[1:]:
            if g[1] > best[1] or (g[1] == best[1] and g[2] > best[2]):
                best = g
        ranked.append(best)
        out.remove(best)
    return ranked


@pytest.mark.parametrize("seed", range(8))
def test_matcher_equals_brute_force_on_small_alphabets(seed):
    rng = np.random.default_rng(seed)
    for _ in range(40):
        n = int(rng.integers(1, 60))
        x = [int(t) for t in rng.integers(0, int(rng.integers(1, 4)) + 1, size=n)]   # alphabet of 1..4 symbols
        q, w = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        assert context_ngram_groups(x, q, w) == _brute_force_groups(x, q, w)


def test_matcher_closed_forms():
    # constant stream: one continuation, n-q-w+1 occurrences, last start n-q-w
    for n, q, w in [(10, 1, 1), (33, 3, 5), (7, 2, 5)]:
        assert context_ngram_groups([4] * n, q, w) == [((4,) * w, n - q - w + 1, n - q - w)]
    # period-p stream of distinct symbols, whole periods: the query matches once per period and every match
    # has the same continuation
    p, reps, q, w = 5, 6, 2, 3
    x = list(range(p)) * reps
    n = len(x)
    (cont, cnt, last), = context_ngram_groups(x, q, w)
    assert cont == tuple((n + t) % p for t in range(w))      # what the period dictates comes next
    assert cnt == reps - 1 and last == n - p - q
    # tokens that never occurred before: nothing
    assert context_ngram_groups(list(range(20)), 1, 1) == []


def test_matcher_on_synthetic_prompts_matches_brute_force():
    x = [int(t) for t in si.prompt_spans(32000, 600, 0.5, seed=4)]
    hits = 0
    for cut in range(50, 600, 7):
        for q in (1, 2, 3):
            g = context_ngram_groups(x[:cut], q, 4)
            assert g == _brute_force_groups(x[:cut], q, 4)
            hits += bool(g)
    assert hits > 20                                         # the copied spans do produce matches


def _library_groups(x, q, w):
    """The matcher through torch's library routines: sliding windows (unfold), rows equal to the query,
    distinct continuations with their counts (unique over rows).  The order of equal counts is not
    defined this way (Appendix B of the paper ranks with a top-k over the counts), so the caller
    compares only where the counts are distinct."""
    import torch
    t = torch.tensor(x, dtype=torch.int64)
    if len(x) < q + w:
        return []
    win = t.unfold(0, q + w, 1)                              # [n - q - w + 1][q + w]
    hit = (win[:, :q] == t[len(x) - q:]).all(dim=1)
    cont = win[hit][:, q:]
    if cont.shape[0] == 0:
        return []
    uniq, counts = torch.unique(cont, dim=0, return_counts=True)
    order = torch.argsort(counts, descending=True, stable=True)
    return [(tuple(int(v) for v in uniq[i]), int(counts[i])) for i in order]


@pytest.mark.parametrize("seed", range(6))
def test_matcher_agrees_with_unfold_unique_counts_where_counts_are_distinct(seed):
    """Streams built from a few motifs repeated a different number of times each, so that no two
    continuations of the final query share a count: there the library's ranking is unambiguous."""
    rng = np.random.default_rng(100 + seed)
    q, w = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    query = [int(v) for v in rng.integers(0, 5, size=q)]
    conts, x = set(), []
    n_motifs = int(rng.integers(2, 5))
    while len(conts) < n_motifs:
        conts.add(tuple(int(v) for v in rng.integers(5, 12, size=w)))     # continuation tokens never look like a query token
    pieces = []
    for reps, c in enumerate(sorted(conts), start=1):       # motif number i occurs i times: distinct counts
        pieces += [query + list(c)] * reps
    for i in rng.permutation(len(pieces)):
        x += pieces[i] + [int(v) for v in rng.integers(12, 20, size=int(rng.integers(0, 3)))]   # filler that matches nothing
    x += query
    got = context_ngram_groups(x, q, w)
    lib = _library_groups(x, q, w)
    assert len({c for _, c in lib}) == len(lib) == n_motifs  # the construction worked: distinct counts
    assert [(g[0], g[1]) for g in got] == lib
    # the oracle's third field is the last start of each continuation
    for cont, cnt, last in got:
        starts = [i for i in range(len(x) - q - w + 1) if x[i:i + q] == query and tuple(x[i + q:i + q + w]) == cont]
        assert len(starts) == cnt and last == max(starts)


def test_context_rows_backoff_cap_and_dedup():
    x = [1, 2, 3, 9, 9, 2, 3, 8, 8, 7, 3, 6, 6, 1, 2, 3]
    # q=3 ("1 2 3") -> 9 9 ; q=2 ("2 3") -> 8 8 (later), 9 9 (dup) ; q=1 ("3") -> 6 6, 8 8 (dup), 9 9 (dup)
    assert context_rows(x, 2, 8, 1, 3) == [(9, 9), (8, 8), (6, 6)]
    assert context_rows(x, 2, 2, 1, 3) == [(9, 9), (8, 8)]
    assert context_rows(x, 2, 8, 3, 3) == [(9, 9)]
    assert context_rows(x, 2, 8, 1, 1) == [(6, 6), (8, 8), (9, 9)]
    assert context_rows(x, 2, 0, 1, 3) == []


# -- bigram ---------------------------------------------------------------------

def test_bigram_scores_are_plain_dot_products():
    rng = np.random.default_rng(0)
    E, U = rng.standard_normal((7, 5)), rng.standard_normal((7, 5))
    z = bigram_scores(E, U, 3)
    for v in range(7):
        assert np.isclose(z[v], sum(U[v, i] * E[3, i] for i in range(5)), rtol=1e-14)


def _select_by_loop(z, k):
    left = list(range(len(z)))
    out = []
    for _ in range(k):
        best = left[0]
        for v in left[1:]:
            if z[v] > z[best]:                  # strict: an equal later id never displaces an earlier one
                best = v
        out.append(best)
        left.remove(best)
    return out


def test_rank_ids_against_selection_loop_with_ties():
    rng = np.random.default_rng(1)
    for _ in range(50):
        V = int(rng.integers(1, 40))
        z = rng.integers(0, 6, size=V).astype(np.float64)        # many exact ties
        k = int(rng.integers(1, V + 1))
        assert list(rank_ids(z, k)) == _select_by_loop(z, k)
    z = rng.standard_normal(100)
    assert sorted(rank_ids(z, 100)) == list(range(100))           # k = V is a permutation
    assert list(rank_ids(np.arange(10.0), 3)) == [9, 8, 7]


def test_duplicate_unembedding_rows_rank_by_id():
    rng = np.random.default_rng(2)
    E, U = rng.standard_normal((6, 4)), rng.standard_normal((6, 4))
    U[4] = U[1]                                                    # exact tie between ids 1 and 4
    b = Bigram(E, U)
    for x in range(6):
        order = list(b.topk(x, 6))
        assert order.index(1) + 1 == order.index(4)


def test_chain_rows_follow_the_top1_bigram():
    m = si.MODELS["tiny"]
    w = si.make_weights(m, seed=0)
    b = Bigram(w["tok_emb"], w["unemb"])
    rows = b.rows(17, 5, 4)
    top = list(b.topk(17, 5))
    assert [r[0] for r in rows] == top
    assert b.next1(17) == top[0]
    for r in rows:
        for j in range(3):
            assert r[j + 1] == b.next1(r[j]) == int(np.argmax(b.scores(r[j])))


# -- mixed strategy ---------------------------------------------------------------

def test_mixed_strategy_rows_and_sources():
    m = si.MODELS["tiny"]
    wts = si.make_weights(m, seed=0)
    b = Bigram(wts["tok_emb"], wts["unemb"])
    x = [1, 2, 3, 9, 9, 2, 3, 8, 8, 7, 3, 6, 6, 1, 2, 3]
    d, src, n_ctx = build_drafts(x, b, k=5, w=2, k_ctx_max=5, q_min=1, q_max=3)
    assert n_ctx == 3 and list(src) == [0, 0, 0, 1, 1]
    assert [tuple(r) for r in d[:3]] == [(9, 9), (8, 8), (6, 6)]
    assert [tuple(r) for r in d[3:]] == b.rows(3, 2, 2)
    # cap on context rows: the bigram takes what is left
    d, src, n_ctx = build_drafts(x, b, k=5, w=2, k_ctx_max=1, q_min=1, q_max=3)
    assert n_ctx == 1 and list(src) == [0, 1, 1, 1, 1]
    assert [tuple(r) for r in d[1:]] == b.rows(3, 4, 2)
    # nothing in the context: all bigram
    d, src, n_ctx = build_drafts(list(range(30, 40)), b, k=3, w=2, k_ctx_max=3, q_min=1, q_max=1)
    assert n_ctx == 0 and list(src) == [1, 1, 1] and [tuple(r) for r in d] == b.rows(39, 3, 2)
    # more context rows than k: the first k by rank
    d, src, n_ctx = build_drafts(x, b, k=2, w=2, k_ctx_max=8, q_min=1, q_max=3)
    assert n_ctx == 2 and [tuple(r) for r in d] == [(9, 9), (8, 8)]
    # w = 0: plain decoding, an empty batch
    d, src, n_ctx = build_drafts(x, b, k=1, w=0, k_ctx_max=1, q_min=1, q_max=1)
    assert d.shape == (1, 0) and n_ctx == 0


def test_unigram_distance_brute_force_gram_form_and_special_cases():
    """Section 4.1, "Unigram": d(x) = ||u_x - u_mean||_V.  Pins: the double loop over the definition's
    sum, the Gram-matrix form (a^T (E^T E) a), invariance to a common shift of all output embeddings,
    and orthonormal input embeddings (E^T E = I), where the distance is the plain Euclidean one."""
    rng = np.random.default_rng(11)
    V, d = 23, 6
    e, u = rng.normal(size=(V, d)), rng.normal(size=(V, d))
    got = unigram_distances(e, u)
    mean = [sum(u[x][i] for x in range(V)) / V for i in range(d)]
    for x in (0, 5, 22):
        a = [u[x][i] - mean[i] for i in range(d)]
        total = 0.0
        for y in range(V):
            dot = sum(a[i] * e[y][i] for i in range(d))
            total += dot * dot
        assert abs(got[x] - total ** 0.5) < 1e-12
    c = u - u.mean(axis=0)
    assert np.allclose(got ** 2, np.einsum("xi,ij,xj->x", c, e.T @ e, c), rtol=1e-12)
    assert np.allclose(unigram_distances(e, u + rng.normal(size=(1, d))), got, rtol=1e-10)
    q, _ = np.linalg.qr(rng.normal(size=(V, d)))             # V x d with orthonormal columns: E^T E = I
    assert np.allclose(unigram_distances(q, u), np.linalg.norm(c, axis=1), rtol=1e-12)
    # a token whose output embedding is the mean has distance 0 and ranks first
    u2 = u.copy()
    u2[7] = (u2.sum(axis=0) - u2[7]) / (V - 1)               # makes row 7 equal to the mean of all rows
    assert abs(unigram_distances(e, u2)[7]) < 1e-12


def test_unigram_rows_ignore_the_context_and_chain_like_bigram_rows():
    desc = si.MODELS["tiny"]
    w = si.make_weights(desc, seed=2)
    b = Bigram(w["tok_emb"], w["unemb"])
    ug = UnigramDrafts(w["tok_emb"], w["unemb"], b)
    d = unigram_distances(w["tok_emb"], w["unemb"])
    assert list(ug.order[:5]) == sorted(range(desc["vocab"]), key=lambda x: (d[x], x))[:5]
    rows = ug.rows(123, 3, 4)
    assert rows == ug.rows(7, 3, 4)                          # q = 0: no context token enters
    for i, row in enumerate(rows):
        assert row[0] == ug.order[i] and all(row[j + 1] == b.next1(row[j]) for j in range(3))
    drafts, src, n_ctx = build_drafts([1, 2, 3, 1, 2, 3, 1, 2], ug, k=4, w=2, k_ctx_max=2, q_min=2, q_max=2)
    assert n_ctx == 1 and tuple(drafts[0]) == (3, 1) and [tuple(r) for r in drafts[1:]] == ug.rows(2, 3, 2)
