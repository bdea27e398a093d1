"""Times the prompt pass (first iteration of Alg. 1) on one MI355X: dense chunk kernels against
16-row blocks through the decode kernels, on a synthetic random-init model.

    python3 prefill_bench.py [--preset 7b] [--tokens 2048] [--layers N] [--modes dense,blocks] [--reps 3] [--chunk 2048]

Prints one line per mode and a JSON summary.  Also the workload of the rocprofv3 summaries of
the dense kernels under profiles/.
"""
import argparse
import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def model_flops(cfg, n):
    """Multiply-add flops (x2) of the prompt pass: target GEMMs, the draft head's fc and K/V
    projections, causal attention."""
    d, f, L = cfg.d_model, cfg.d_ffn, cfg.n_layers
    dq, dkv = cfg.n_heads * cfg.head_dim, cfg.d_kv
    gemm = 2 * n * (L * (2 * d * dq + 2 * d * dkv + 3 * d * f) + (2 * d * d + d * (dq + 2 * dkv)))
    attn = 4 * L * dq * n * (n + 1) // 2
    return gemm + attn


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--preset", default="7b")
    ap.add_argument("--tokens", type=int, default=2048)
    ap.add_argument("--layers", type=int, default=0, help="override the number of target layers")
    ap.add_argument("--modes", default="dense,blocks")
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--chunk", type=int, default=0, help="rows per dense pass (multiple of 128)")
    args = ap.parse_args()

    import numpy as np
    import torch
    from paper_2412_18910_amd import synth
    from paper_2412_18910_amd.binding import Engine
    from paper_2412_18910_amd.config import PRESETS

    cfg = PRESETS[args.preset].with_(n_ctx_max=args.tokens + 64)
    if args.layers:
        cfg = cfg.with_(n_layers=args.layers)
    torch.cuda.set_device(0)
    eng = Engine(cfg, synth.make_weights(cfg, 1, device="cuda:0"))
    ids = synth.token_ids(args.tokens, cfg.vocab, 11)
    flops = model_flops(cfg, args.tokens)
    out = {"preset": args.preset, "tokens": args.tokens, "n_layers": cfg.n_layers}
    logits = {}
    for name in args.modes.split(","):
        mode = {"dense": Engine.PREFILL_DENSE, "blocks": Engine.PREFILL_BLOCKS}[name]
        eng.set_prefill_mode(mode, args.chunk if name == "dense" else 0)
        eng.prefill(ids)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.reps):
            eng.prefill(ids)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.reps * 1e3
        logits[name] = eng.logits(0)
        out[name] = {"ms": round(ms, 2), "tokens_per_s": round(args.tokens / ms * 1e3, 1),
                     "model_tflops": round(flops / ms / 1e9, 1)}
        print(f"{name}: {ms:.2f} ms  {args.tokens / ms * 1e3:.0f} tokens/s  {flops / ms / 1e9:.1f} model TFLOP/s "
              f"({2 * flops / ms / 1e9:.1f} issued on the matrix cores: bf16 hi and lo halves)", flush=True)
    if len(logits) == 2:
        out["max_logit_diff"] = float(np.max(np.abs(logits["dense"] - logits["blocks"])))
    eng.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
