"""Seeded synthetic inputs shared by the HIP path and the CPU oracle.

Holds no arithmetic of the decode step: it only draws random weights, token ids,
K/V fill values and uniforms, so that both sides can be fed identical bytes.
All 2-D matrices are iid N(0, 0.02^2) in the configuration's dtype, norm gains are
1 + 0.1 N(0,1), biases 0.02 N(0,1) (all 1-D vectors are float32).
"""
import math

import numpy as np
import torch

from .config import BF16, Config

_LAYER_MATS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_weights(cfg: Config, seed: int, device="cpu"):
    """Dict of torch tensors in a fixed draw order (tok_emb, lm_head, final_norm,
    target layers, draft layer, draft fc, LDLP)."""
    g = _gen(seed, device)
    mdt = torch.bfloat16 if cfg.dtype == BF16 else torch.float32

    def mat(*shape, std=0.02):
        return (torch.randn(*shape, generator=g, device=device, dtype=torch.float32) * std).to(mdt)

    def gain(n):
        return 1.0 + 0.1 * torch.randn(n, generator=g, device=device, dtype=torch.float32)

    def bias(n, std=0.02):
        return std * torch.randn(n, generator=g, device=device, dtype=torch.float32)

    d, f, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    dq, dkv = cfg.n_heads * cfg.head_dim, cfg.d_kv

    def layer():
        return {"attn_norm": gain(d), "wq": mat(dq, d), "wk": mat(dkv, d), "wv": mat(dkv, d),
                "wo": mat(d, dq), "ffn_norm": gain(d), "w_gate": mat(f, d), "w_up": mat(f, d),
                "w_down": mat(d, f)}

    w = {"tok_emb": mat(V, d), "lm_head": mat(V, d), "final_norm": gain(d)}
    w["layers"] = [layer() for _ in range(cfg.n_layers)]
    w["draft_layer"] = layer()
    w["draft_fc_w"] = mat(d, 2 * d)
    w["draft_fc_b"] = bias(d)
    h = cfg.ldlp_hidden
    lin = 2 * d if cfg.ldlp_in_mode == 0 else d
    w["ldlp_w_in"] = mat(h, lin)
    w["ldlp_b_in"] = bias(h)
    if cfg.ldlp_n_res > 0:
        w["ldlp_w_res"] = mat(cfg.ldlp_n_res, h, h, std=1.0 / math.sqrt(h))
        w["ldlp_b_res"] = bias(cfg.ldlp_n_res * h).reshape(cfg.ldlp_n_res, h)
    else:
        w["ldlp_w_res"] = None
        w["ldlp_b_res"] = None
    # spread the predicted length over 0..k_max instead of collapsing on one value
    s_out = (cfg.k_max / 4.0) / (math.sqrt(h) * 0.02 * math.sqrt(d) * 0.6)
    if cfg.ldlp_cls:
        # one score row per candidate length; comparable spread so that every class wins sometimes
        w["ldlp_w_out"] = s_out * torch.randn(cfg.k_max + 1, h, generator=g, device=device, dtype=torch.float32)
        w["ldlp_b_out"] = 0.1 * torch.randn(cfg.k_max + 1, generator=g, device=device, dtype=torch.float32)
    else:
        w["ldlp_w_out"] = s_out * torch.randn(h, generator=g, device=device, dtype=torch.float32)
        w["ldlp_b_out"] = torch.full((1,), (cfg.k_max + 1) / 2.0, device=device, dtype=torch.float32)
    return w


def to_numpy(t):
    """torch tensor -> numpy (bf16 as uint16 bit patterns), on the host."""
    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def weights_to_numpy(w):
    def conv(v):
        if isinstance(v, dict):
            return {k: conv(x) for k, x in v.items()}
        if isinstance(v, list):
            return [conv(x) for x in v]
        return to_numpy(v)
    return conv(w)


def token_ids(n, vocab, seed):
    g = _gen(seed, "cpu")
    return torch.randint(0, vocab, (n,), generator=g, dtype=torch.int32).numpy()


def kv_fill(cfg: Config, n, seed, layer):
    """K and V rows [n, d_kv] ~ N(0,1), already rounded to the cache dtype, as float32."""
    g = _gen(seed * 1000003 + layer, "cpu")
    k = torch.randn(n, cfg.d_kv, generator=g, dtype=torch.float32)
    v = torch.randn(n, cfg.d_kv, generator=g, dtype=torch.float32)
    if cfg.dtype == BF16:
        k, v = k.to(torch.bfloat16).float(), v.to(torch.bfloat16).float()
    return k.numpy(), v.numpy()


def feature_row(cfg: Config, seed):
    g = _gen(seed, "cpu")
    return torch.randn(cfg.d_model, generator=g, dtype=torch.float32).numpy()


def uniforms(n, seed):
    """n doubles in [0, 1) from a counter-based generator (Philox)."""
    return np.random.Generator(np.random.Philox(int(seed))).random(n)


def truncated_geometric(n, mean, k_max, seed):
    """n acceptance lengths in [0, k_max] ~ geometric truncated at k_max whose mean is
    `mean` (the success ratio is found by bisection on the closed-form mean)."""
    def tmean(r):
        p = np.array([r ** i for i in range(k_max + 1)], dtype=np.float64)
        p /= p.sum()
        return float((p * np.arange(k_max + 1)).sum())
    lo, hi = 1e-6, 50.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if tmean(mid) < mean:
            lo = mid
        else:
            hi = mid
    r = 0.5 * (lo + hi)
    p = np.array([r ** i for i in range(k_max + 1)], dtype=np.float64)
    p /= p.sum()
    rng = np.random.Generator(np.random.Philox(int(seed)))
    return rng.choice(k_max + 1, size=n, p=p).astype(np.int32)
