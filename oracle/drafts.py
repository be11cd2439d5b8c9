"""Learning-free draft construction, CPU oracle (test infrastructure).

Section 4.1: model-derived bigram, its top-k as a k x 1 batch of drafts, and the
extension to w > 1 tokens by re-applying the bigram.  Section 4.2: context
N-grams (earlier occurrences of the last q tokens, the w tokens that follow,
ranked by count, ties to the later match).  Section 4.3: mixed strategy
(context rows first, the extended bigram fills the rest).

Readings taken where the paper leaves a choice (all listed in the design notes):
the bigram used on the step is the direct path z = U^T-row . E[x] (no
transformer layers, no normalisation); equal scores rank by ascending token
id; the extension chains the bigram's top-1; only windows whose w-token
continuation lies fully inside the context count as matches.
"""
from __future__ import annotations

import numpy as np


# -- context N-grams (Section 4.2) -------------------------------------------

def context_ngram_groups(tokens, q: int, w: int):
    """All earlier occurrences of the last q context tokens, grouped by the w
    tokens that follow.  Returns a list of (continuation tuple, count, last_start)
    ordered by (count descending, last_start descending): more frequent first,
    ties to the match that occurs later in the context.

    A window starts at i, 0 <= i <= n-q-w, so its continuation x[i+q .. i+q+w)
    is complete; the query's own position (i = n-q) has no continuation and is
    never a match."""
    x = [int(t) for t in tokens]
    n = len(x)
    if q < 1 or w < 1 or n < q + w:
        return []
    query = x[n - q:]
    groups = {}
    for i in range(0, n - q - w + 1):
        if x[i:i + q] == query:
            cont = tuple(x[i + q:i + q + w])
            cnt, _ = groups.get(cont, (0, -1))
            groups[cont] = (cnt + 1, i)          # i increases, so this is the last start
    ranked = sorted(groups.items(), key=lambda kv: (-kv[1][0], -kv[1][1]))
    return [(cont, cnt, last) for cont, (cnt, last) in ranked]


def context_rows(tokens, w: int, k_ctx_max: int, q_min: int, q_max: int):
    """Up to k_ctx_max distinct continuations.  Query lengths are tried from
    q_max down to q_min (a back-off; with q_min == q_max this is exactly the
    matcher of Section 4.2); a continuation already taken is skipped."""
    rows = []
    for q in range(q_max, q_min - 1, -1):
        for cont, _, _ in context_ngram_groups(tokens, q, w):
            if len(rows) >= k_ctx_max:
                return rows
            if cont not in rows:
                rows.append(cont)
    return rows[:k_ctx_max]


# -- model bigram (Section 4.1) ------------------------------------------------

def bigram_scores(tok_emb, unemb, x: int):
    """z[v] = <unemb[v], tok_emb[x]> for every vocabulary entry v, in fp64."""
    return np.asarray(unemb, dtype=np.float64) @ np.asarray(tok_emb[x], dtype=np.float64)


def rank_ids(z, k: int):
    """The k token ids with the largest score, by (score descending, id ascending)."""
    z = np.asarray(z)
    order = np.lexsort((np.arange(len(z)), -z))       # last key is primary
    return order[:k].astype(np.int32)


class Bigram:
    """Top-k next tokens under the model bigram and its chained extension."""

    def __init__(self, tok_emb, unemb):
        self.tok_emb = np.asarray(tok_emb, dtype=np.float64)
        self.unemb = np.asarray(unemb, dtype=np.float64)
        self._next1 = {}

    def scores(self, x: int):
        return bigram_scores(self.tok_emb, self.unemb, x)

    def topk(self, x: int, k: int):
        return rank_ids(self.scores(x), k)

    def next1(self, x: int) -> int:
        """The bigram's single best next token (the O(1) lookup of Section 4.1,
        filled lazily)."""
        x = int(x)
        if x not in self._next1:
            self._next1[x] = int(rank_ids(self.scores(x), 1)[0])
        return self._next1[x]

    def rows(self, x: int, k_big: int, w: int):
        """k_big drafts of w tokens: row i starts with the bigram's i-th ranked
        token and continues by repeatedly applying the top-1 bigram."""
        out = []
        for t in self.topk(x, k_big):
            row = [int(t)]
            while len(row) < w:
                row.append(self.next1(row[-1]))
            out.append(tuple(row[:w]))
        return out


class ModelBigram(Bigram):
    """The paper's own bigram (Section 4.1, "Model bigram"): p_M(. | x) is the
    next-token distribution of the WHOLE model on the one-token context x, so
    scores(x) are the model's logits after running it on [x].  `logits_of(x)`
    is that model call (e.g. lambda x: model.forward_full([x])[-1]); ranking,
    chaining and the lazily filled top-1 lookup are those of Bigram."""

    def __init__(self, logits_of):
        self.logits_of = logits_of
        self._scores = {}
        self._next1 = {}

    def scores(self, x: int):
        x = int(x)
        if x not in self._scores:
            self._scores[x] = np.asarray(self.logits_of(x), dtype=np.float64)
        return self._scores[x]


# -- model unigram (Section 4.1, "Unigram") -------------------------------------

def unigram_distances(tok_emb, unemb):
    """d(x) = || u_x - u_mean ||_V for every token x, where u_x is the output
    embedding of x, u_mean the mean output embedding, and the norm comes from the
    inner product <a, b>_V = sum over tokens y of (a . v_y)(b . v_y) with v_y the
    input embeddings.  So d(x) is the Euclidean length of the vector
    ((u_x - u_mean) . v_y)_y.  The paper's listing computes a different quantity
    and returns nothing; the text's definition is the one followed here."""
    e = np.asarray(tok_emb, dtype=np.float64)
    u = np.asarray(unemb, dtype=np.float64)
    centred = u - u.mean(axis=0, keepdims=True)
    return np.sqrt(np.sum((centred @ e.T) ** 2, axis=1))


class UnigramDrafts:
    """Draft rows from the unigram p(x) ~ exp(-d(x)): row i starts with the token of
    i-th smallest distance (ties to the lower id), whatever the context, and is
    extended like a bigram row, by the chain of the bigram's top-1.  Offers the
    interface build_drafts uses (rows) on top of an existing Bigram."""

    def __init__(self, tok_emb, unemb, bigram):
        self.d = unigram_distances(tok_emb, unemb)
        self.order = rank_ids(-self.d, len(self.d))
        self.bigram = bigram

    def scores(self, x: int):
        return self.bigram.scores(x)

    def next1(self, x: int) -> int:
        return self.bigram.next1(x)

    def rows(self, x: int, k_big: int, w: int):
        out = []
        for t in self.order[:k_big]:
            row = [int(t)]
            while len(row) < w:
                row.append(self.bigram.next1(row[-1]))
            out.append(tuple(row[:w]))
        return out


# -- mixed strategy (Section 4.3) -----------------------------------------------

def build_drafts(tokens, bigram: Bigram, k: int, w: int, k_ctx_max: int, q_min: int, q_max: int):
    """The k x w draft batch: as many context rows as were found (at most
    k_ctx_max), in rank order, then extended-bigram rows in rank order.
    Returns (drafts int32 [k, w], row_src int8 [k] with 0 = context, 1 = bigram,
    n_ctx).  w == 0 gives an empty batch (plain decoding)."""
    drafts = np.zeros((k, w), dtype=np.int32)
    src = np.ones(k, dtype=np.int8)
    if w == 0:
        return drafts, src, 0
    ctx = context_rows(tokens, w, min(k_ctx_max, k), q_min, q_max)
    n_ctx = len(ctx)
    rows = list(ctx) + bigram.rows(int(tokens[-1]), k - n_ctx, w)
    for r, row in enumerate(rows):
        drafts[r] = row
    src[:n_ctx] = 0
    return drafts, src, n_ctx
