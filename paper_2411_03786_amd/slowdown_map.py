"""Slowdown of a (k, w+1) verify call against the single-token call, over context length, k and w
(the experiment of Section 3, Figure 1, on this library and an MI355X).

  python -m paper_2411_03786_amd.slowdown_map [--model 7b] [--ctx 25,100,500,2048]
         [--k 1,2,4,8,10,16,25,32] [--w 0,1,2,3,5,8,10,15] [--reps 10] [--out FILE.md]

For every context length the model call on a (k, w+1) block is timed (ngg_verify_step on drafts left
on the device; no commit, so every call sees the same state) and divided by the (1, 1) call at the
same context.  Prints one markdown table per context length and the largest k*w whose slowdown stays
under 1.15, 1.25 and 1.5 (the paper reads its optimal (k, w) off such a map, Section 5).
Synthetic seeded weights and prompt; one GPU.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="7b")
    ap.add_argument("--ctx", default="25,100,500,2048")
    ap.add_argument("--k", default="1,2,4,8,10,16,25,32")
    ap.add_argument("--w", default="0,1,2,3,5,8,10,15")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    ctxs = [int(x) for x in args.ctx.split(",")]
    ks = [int(x) for x in args.k.split(",")]
    ws = [int(x) for x in args.w.split(",")]

    import torch
    import synth_inputs as si
    import paper_2411_03786_amd as ngg

    m = si.MODELS[args.model]
    torch.cuda.set_device(0)
    dev_w = si.make_weights_device(m, seed=0)
    ctx = ngg.Context(m, dev_w, max_seq=max(ctxs) + 64, max_k=max(ks), max_w=max(ws))
    lines = [f"# verify-call slowdown map, {args.model}-shaped {m['dtype']} decoder ({m['n_layers']} layers, d_model {m['d_model']}, "
             f"vocab {m['vocab']}), one MI355X", f"# command: python -m paper_2411_03786_amd.slowdown_map {' '.join(sys.argv[1:])}",
             f"# entry = latency of ngg_verify_step on a (k, w+1) block / latency of the (1, 1) call at the same context; "
             f"mean of {args.reps} calls after 3 warm-up calls", ""]

    def timed(k, w):
        for _ in range(3):
            ctx.verify_step(None, k, w, fetch=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.reps):
            ctx.verify_step(None, k, w, fetch=False)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.reps

    for n_ctx in ctxs:
        prompt = si.prompt_spans(m["vocab"], n_ctx, 0.30, seed=1)
        ctx.prefill(prompt)
        base = timed(1, 0)
        lines.append(f"## context {n_ctx} tokens: single-token call {base * 1e3:.3f} ms")
        lines.append("")
        lines.append("| k \\ w | " + " | ".join(str(w) for w in ws) + " |")
        lines.append("|---|" + "---|" * len(ws))
        best = {1.15: (0, None), 1.25: (0, None), 1.5: (0, None)}
        for k in ks:
            row = []
            for w in ws:
                # drafts on the device: any valid tokens do for timing (bigram rows of the current state)
                if w > 0:
                    ctx.build_drafts(dict(k=k, w=w, k_ctx_max=0, q_min=1, q_max=1), fetch=False)
                s = timed(k, w) / base
                row.append(f"{s:.2f}")
                for lim in best:
                    if s <= lim and k * w > best[lim][0]:
                        best[lim] = (k * w, (k, w, s))
            lines.append(f"| {k} | " + " | ".join(row) + " |")
            print(lines[-1], flush=True)
        lines.append("")
        for lim, (kw, arg) in best.items():
            if arg:
                lines.append(f"largest k*w with slowdown <= {lim}: k={arg[0]}, w={arg[1]} (k*w = {kw}, slowdown {arg[2]:.2f})")
        lines.append("")
    ctx.close()
    text = "\n".join(lines)
    print(text)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text + "\n")


if __name__ == "__main__":
    main()
