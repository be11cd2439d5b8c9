"""The allocation-free entry point ngg_context_drafts_static against ngg_build_drafts (and the oracle),
through the C ABI: two calls in a row on one GPU, the second on a smaller input (the static scratch
keeps the first call's contents).  Needs an MI355X."""
import numpy as np
import pytest

import synth_inputs as si
import oracle
import paper_2411_03786_amd as ngg

pytestmark = pytest.mark.gpu


def _static_rows(tokens, w, k_ctx_max, q_min, q_max):
    import torch
    t = torch.tensor(np.asarray(tokens, dtype=np.int32), device="cuda")
    rows = torch.full((k_ctx_max, w), -7, dtype=torch.int32, device="cuda")
    n_rows = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    ngg.context_drafts_static(t, w, k_ctx_max, q_min, q_max, rows, n_rows)
    torch.cuda.synchronize()
    n = int(n_rows.item())
    out = rows.cpu().numpy()
    assert (out[n:] == -7).all()                               # rows beyond the count are left untouched
    return out[:n], n


def test_static_entry_equals_build_drafts_twice_second_call_smaller():
    desc = si.MODELS["tiny"]
    w = si.make_weights(desc, seed=0)
    ctx = ngg.Context(desc, w, max_seq=6200, max_k=16, max_w=6)
    stream = si.prompt_spans(desc["vocab"], 6000, copied=0.5, seed=5)
    cfgs = (dict(k=16, w=6, k_ctx_max=16, q_min=1, q_max=3), dict(k=8, w=3, k_ctx_max=8, q_min=1, q_max=1))
    found = 0
    for n_prompt in (6000, 700):                              # the second call's input is smaller
        ctx.prefill(stream[:n_prompt])
        toks = ctx.get_tokens()
        for cfg in cfgs:
            g_d, g_src, g_n = ctx.build_drafts(cfg)
            rows, n = _static_rows(toks, cfg["w"], cfg["k_ctx_max"], cfg["q_min"], cfg["q_max"])
            assert n == g_n and np.array_equal(rows, g_d[:g_n]), (n_prompt, cfg)
            want = oracle.context_rows(toks, cfg["w"], cfg["k_ctx_max"], cfg["q_min"], cfg["q_max"])
            assert [tuple(int(t) for t in r) for r in rows] == [tuple(r) for r in want], (n_prompt, cfg)
            found += n
    ctx.close()
    assert found >= 10


def test_static_entry_at_its_limit_and_on_degenerate_streams_against_the_oracle():
    """No context object at all: token streams up to NGG_STATIC_MAX_TOKENS, then much shorter ones."""
    V = 32000
    rng = np.random.default_rng(3)
    n_max = ngg.NGG_STATIC_MAX_TOKENS
    streams = [si.prompt_spans(V, n_max, copied=0.5, seed=9),                       # Zipf + copied spans, at the limit
               np.zeros(20000, dtype=np.int32) + 5,                                   # constant: every window matches, one group
               np.tile(np.arange(7, dtype=np.int32), 3000)[:16385],                   # period 7
               si.prompt_spans(512, 9000, copied=0.3, seed=2),                        # small vocabulary: thousands of matches at q = 1
               rng.integers(0, 3, 3000).astype(np.int32),                             # three symbols: many groups with large counts
               si.prompt_spans(V, 300, copied=0.5, seed=9),
               np.array([1, 2], dtype=np.int32), np.array([4], dtype=np.int32)]
    for x in streams:
        for (w, kc, q0, q1) in ((6, 16, 1, 3), (3, 32, 1, 1), (1, 5, 2, 4), (32, 4, 1, 2)):
            rows, n = _static_rows(x, w, kc, q0, q1)
            want = oracle.context_rows(x, w, kc, q0, q1)
            assert n == len(want) and [tuple(int(t) for t in r) for r in rows] == [tuple(r) for r in want], (len(x), w, kc, q0, q1)


def test_matcher_time_is_linear_in_the_matches():
    """A constant 16K-token context makes every window a match of one group (the quadratic grouping this
    replaces took ~1e9 token compares there); a Zipf stream with a frequent last token has thousands of
    matches in thousands of groups.  Both must stay far below a verify step (milliseconds)."""
    import torch
    for x in (np.zeros(16384, dtype=np.int32) + 9, si.prompt_spans(64, 16384, copied=0.3, seed=4)):
        t = torch.tensor(x, device="cuda")
        rows = torch.zeros((16, 6), dtype=torch.int32, device="cuda")
        n_rows = torch.zeros(1, dtype=torch.int32, device="cuda")
        ngg.context_drafts_static(t, 6, 16, 1, 3, rows, n_rows)           # warm-up (module load, symbol lookup)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            ngg.context_drafts_static(t, 6, 16, 1, 3, rows, n_rows)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        print(f"matcher on 16384 tokens ({'constant' if x[0] == x[1] == 9 else 'Zipf over 64 symbols'}): {ms * 1e3:.0f} us per call")
        assert ms < 5.0


def test_static_entry_rejects_what_it_cannot_hold():
    import torch
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    rows = torch.zeros((4, 4), dtype=torch.int32, device="cuda")
    n_rows = torch.zeros(1, dtype=torch.int32, device="cuda")
    for kw, status in ((dict(n=ngg.NGG_STATIC_MAX_TOKENS + 1), ngg.NGG_ECAPACITY), (dict(n=0), ngg.NGG_ECAPACITY)):
        with pytest.raises(ngg.NggError) as e:
            ngg.context_drafts_static(t, 4, 4, 1, 2, rows, n_rows, **kw)
        assert e.value.status == status
    for args in ((0, 4, 1, 2), (33, 1, 1, 1), (4, 0, 1, 2), (4, 4, 0, 2), (4, 4, 3, 2), (4, 4, 1, 65)):
        with pytest.raises(ngg.NggError) as e:
            ngg.context_drafts_static(t, args[0], args[1], args[2], args[3], torch.zeros(33 * 33, dtype=torch.int32, device="cuda"), n_rows)
        assert e.value.status == ngg.NGG_EINVAL
    torch.cuda.synchronize()
