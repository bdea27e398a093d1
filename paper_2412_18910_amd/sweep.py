"""Table-2-style breakdown on synthetic scripted acceptance (python -m paper_2412_18910_amd.sweep).

For one model shape and one seeded acceptance trace, compares plain autoregressive decoding,
fixed draft lengths, the draft-length oracle (k = the scripted acceptance length) and the
LDLP-chosen length: tau, tokens/s, time in the draft and target phases, N_draft / N_target /
N_waste as defined for Table 2 of arxiv 2412.18910.  Only the shape of the trade-off is
comparable with the paper: weights are random and acceptance is scripted.

Two more rows run AdaEAGLE-DDD (Sec. 3.4: LDLP length, then keep drafting while the draft
sequence's log-probability stays above a threshold) with the exit rule evaluated on the host
(one synchronisation per decision past k) and on the device (no synchronisation inside the
draft, skipped tokens cost empty launches, padded verify block).  The random-init head gives
every token a near-uniform probability, so the paper's threshold of -0.6 would never extend a
draft; the default threshold here is the log-probability of 3.5 tokens at the uniform rate,
which extends short predicted lengths to 3-4 tokens.
"""
import argparse
import sys
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--preset", default="7b")
    ap.add_argument("--context", type=int, default=2048)
    ap.add_argument("--tokens", type=int, default=256)
    ap.add_argument("--mean-accept", type=float, default=3.5)
    ap.add_argument("--ddd-threshold", type=float, default=None,
                    help="log-probability threshold of the DDD rows (default: -3.5 * ln(vocab))")
    ap.add_argument("--no-ddd", action="store_true")
    args = ap.parse_args()

    import torch
    from . import synth
    from .binding import Engine
    from .config import PRESETS
    from .loop import Counters, scripted_override

    cfg = PRESETS[args.preset].with_(temperature=0.0)
    n_formal = args.tokens + 2 * (cfg.k_max + 2)
    cfg = cfg.with_(n_ctx_max=args.context + n_formal + 64)
    w = synth.make_weights(cfg, 1, device="cuda:0")
    eng = Engine(cfg, w)
    ctx_ids = synth.token_ids(args.context, cfg.vocab, 11)
    script = synth.truncated_geometric(4 * args.tokens, args.mean_accept, cfg.k_max, 5)

    eng.prefill(ctx_ids)
    formal = np.zeros(n_formal, np.int64)
    torch.cuda.synchronize(); t0 = time.perf_counter()
    for i in range(n_formal):
        eng.verify([eng.pending]); formal[i] = eng.accept()[1]
    torch.cuda.synchronize()
    ar_tok_s = n_formal / (time.perf_counter() - t0)

    rows = [("Vanilla AR", "-", 1.0, ar_tok_s, None, None, None, 0, n_formal, 0)]
    modes = [("fixed", k) for k in (2, 3, 4, 5, 6)] + [("oracle", None), ("ldlp", None)]
    theta = args.ddd_threshold if args.ddd_threshold is not None else -3.5 * float(np.log(cfg.vocab))
    if not args.no_ddd:
        modes += [("ddd-host", None), ("ddd-device", None)]
    for mode, kf in modes:
        if mode == "ddd-host":     # same weights, exit rule switched on
            eng.close()
            eng = Engine(cfg.with_(ddd_enabled=1, ddd_threshold=theta), w)
        if mode.startswith("ddd"):
            eng.set_ddd_mode(Engine.DDD_DEVICE if mode == "ddd-device" else Engine.DDD_HOST)
        eng.prefill(ctx_ids)
        eng.set_profiling(True)
        cnt, pos, r = Counters(), 0, 0
        t_draft = t_target = 0.0
        torch.cuda.synchronize(); t0 = time.perf_counter()
        while pos < args.tokens:
            k = kf if mode == "fixed" else (int(script[r]) if mode == "oracle" else eng.ldlp()[0])
            # the DDD rule may extend the draft up to k_max tokens: script all of them
            ov = scripted_override(formal, pos, cfg.k_max if mode.startswith("ddd") else k, int(script[r]), cfg.vocab)
            kk, na, toks = eng.step(k_force=k, override_ids=ov)
            assert np.array_equal(toks, formal[pos:pos + na + 1]), "speculative output left the AR sequence"
            pt = eng.phase_times()
            t_draft += pt["draft"]; t_target += pt["verify"]
            cnt.add(kk, na); pos += na + 1; r += 1
        torch.cuda.synchronize(); total = time.perf_counter() - t0
        eng.set_profiling(False)
        s = cnt.summary()
        name = {"fixed": "fixed length", "oracle": "draft-length oracle", "ldlp": "LDLP (random weights)",
                "ddd-host": f"LDLP + DDD rule (theta {theta:.1f}), decided on the host",
                "ddd-device": f"LDLP + DDD rule (theta {theta:.1f}), decided on the device"}[mode]
        rows.append((name, kf if kf else "dyn.", s["tau"], s["tokens"] / total, total * 1e3, t_draft / 1e3, t_target / 1e3,
                     s["N_draft"], s["N_target"], s["N_waste"]))
    eng.close()

    print(f"# Table-2-style breakdown, {args.preset} shape, bf16, bs=1, context {args.context}, {args.tokens} tokens, "
          f"scripted acceptance (truncated geometric, mean {args.mean_accept})\n")
    print("| method | draft len | tau | tok/s | T_total ms | T_draft ms | T_target ms | N_draft | N_target | N_waste |")
    print("|---|---|---:|---:|---:|---:|---:|---:|---:|---:|")
    for name, k, tau, toks, tt, td, tg, nd, nt, nw in rows:
        f = lambda v: "-" if v is None else f"{v:.1f}"
        print(f"| {name} | {k} | {tau:.2f} | {toks:.1f} | {f(tt)} | {f(td)} | {f(tg)} | {nd} | {nt} | {nw} |")


if __name__ == "__main__":
    sys.exit(main())
