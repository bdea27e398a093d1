"""Whole-forward pins: a float64 library re-expression, block == sequential, accumulator width."""

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from paper_2412_18910_amd import synth
from paper_2412_18910_amd.config import BF16, FP32, Config, TINY

from .helpers import make_oracle

SMALL_BF16 = Config(3, 128, 4, 2, 32, 192, 512, dtype=BF16, k_max=6, n_ctx_max=96, ldlp_hidden=32,
                    rope_base=500000.0, rms_eps=1e-5)


def _rope64(x, pos, hd, base):
    half = hd // 2
    inv = base ** (-torch.arange(half, dtype=torch.float64) * 2 / hd)
    ang = pos.double()[:, None] * inv[None]
    c, s = ang.cos()[:, None, :], ang.sin()[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return torch.cat([a * c - b * s, b * c + a * s], -1)


def _layer64(cfg, lw, x, pos):
    """Llama-style pre-norm layer over a whole sequence with library ops, float64."""
    n, H, Hk, hd = x.shape[0], cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    W = {k: v.double() for k, v in lw.items()}
    rms = lambda t, g: t / torch.sqrt((t * t).mean(-1, keepdim=True) + cfg.rms_eps) * g
    h = rms(x, W["attn_norm"])
    q = _rope64((h @ W["wq"].T).view(n, H, hd), pos, hd, cfg.rope_base)
    k = _rope64((h @ W["wk"].T).view(n, Hk, hd), pos, hd, cfg.rope_base)
    v = (h @ W["wv"].T).view(n, Hk, hd)
    if cfg.dtype == BF16:
        k, v = k.float().bfloat16().double(), v.float().bfloat16().double()
    g = H // Hk
    a = Fn.scaled_dot_product_attention(q.permute(1, 0, 2), k.permute(1, 0, 2).repeat_interleave(g, 0),
                                        v.permute(1, 0, 2).repeat_interleave(g, 0), is_causal=True)
    x = x + a.permute(1, 0, 2).reshape(n, H * hd) @ W["wo"].T
    h = rms(x, W["ffn_norm"])
    return x + (Fn.silu(h @ W["w_gate"].T) * (h @ W["w_up"].T)) @ W["w_down"].T


def _target64(cfg, w, ids):
    x = w["tok_emb"].double()[torch.as_tensor(ids).long()]
    pos = torch.arange(len(ids))
    for lw in w["layers"]:
        x = _layer64(cfg, lw, x, pos)
    F = x / torch.sqrt((x * x).mean(-1, keepdim=True) + cfg.rms_eps) * w["final_norm"].double()
    return F, F @ w["lm_head"].double().T


@pytest.mark.parametrize("cfg", [TINY, SMALL_BF16], ids=["tiny-fp32", "small-bf16-gqa"])
def test_target_forward_matches_float64_library(cfg):
    m, w = make_oracle(cfg, 0)
    ids = synth.token_ids(24, cfg.vocab, 11)
    block = synth.token_ids(5, cfg.vocab, 12)
    m.prefill(ids)
    F64, lg64 = _target64(cfg, w, np.concatenate([ids, block]))
    assert m.pending == int(lg64[23].argmax())
    m.verify(block)
    # bf16 caches round K/V: a float32-vs-float64 difference can flip a rounding, so allow more
    tol = 2e-5 if cfg.dtype == FP32 else 2e-3
    for r in range(5):
        np.testing.assert_allclose(m.logits(r), lg64[24 + r].numpy(), atol=tol, rtol=0)
        np.testing.assert_allclose(m.feature(r), F64[24 + r].numpy(), atol=10 * tol, rtol=0)


def test_draft_head_matches_float64_library():
    cfg = TINY
    m, w = make_oracle(cfg, 0)
    ids = synth.token_ids(20, cfg.vocab, 21)
    m.prefill(ids)
    F64, lg64 = _target64(cfg, w, ids)
    first = int(lg64[-1].argmax())
    # slot s pairs the feature of token s with the embedding of token s+1
    nxt = np.concatenate([ids[1:], [first]])
    emb = w["tok_emb"].double()[torch.as_tensor(nxt).long()]
    x = torch.cat([F64, emb], -1) @ w["draft_fc_w"].double().T + w["draft_fc_b"].double()
    fh = _layer64(cfg, w["draft_layer"], x, torch.arange(20))
    dl = fh[-1] @ w["lm_head"].double().T
    got = m.draft(1)
    np.testing.assert_allclose(m.draft_logits(0), dl.numpy(), atol=2e-5, rtol=0)
    assert got[0] == int(dl.argmax())
    # second chained token: the head's own output replaces the feature
    m2, _ = make_oracle(cfg, 0)
    m2.prefill(ids)
    got2 = m2.draft(2)
    x2 = torch.cat([fh[-1], w["tok_emb"].double()[int(got2[0])]]) @ w["draft_fc_w"].double().T + w["draft_fc_b"].double()
    fh2 = _layer64(cfg, w["draft_layer"], torch.cat([x, x2[None]]), torch.arange(21))
    np.testing.assert_allclose(m2.draft_logits(1), (fh2[-1] @ w["lm_head"].double().T).numpy(), atol=2e-5, rtol=0)
    # third token: chained from the second token and the second output, not from the first
    m3, _ = make_oracle(cfg, 0)
    m3.prefill(ids)
    forced = np.array([int(got2[0]), (int(got2[0]) + 1234) % cfg.vocab, -1], np.int32)
    got3 = m3.draft(3, override_ids=forced)
    assert list(got3[:2]) == list(forced[:2])
    x2b = torch.cat([fh[-1], w["tok_emb"].double()[int(forced[0])]]) @ w["draft_fc_w"].double().T + w["draft_fc_b"].double()
    fh2b = _layer64(cfg, w["draft_layer"], torch.cat([x, x2b[None]]), torch.arange(21))
    x3 = torch.cat([fh2b[-1], w["tok_emb"].double()[int(forced[1])]]) @ w["draft_fc_w"].double().T + w["draft_fc_b"].double()
    fh3 = _layer64(cfg, w["draft_layer"], torch.cat([x, x2b[None], x3[None]]), torch.arange(22))
    np.testing.assert_allclose(m3.draft_logits(2), (fh3[-1] @ w["lm_head"].double().T).numpy(), atol=3e-5, rtol=0)


def test_draft_catch_up_over_several_rows_hands_on_the_last_row():
    """Eq. 2 after a step that validated tokens: the head first recomputes the slots of the accepted
    tokens from their true features; its next-token logits come from the LAST of those rows."""
    cfg = TINY
    m, w = make_oracle(cfg, 0)
    ids = synth.token_ids(20, cfg.vocab, 21)
    ar, _ = make_oracle(cfg, 0, weights=w)
    ar.prefill(ids)
    t1 = ar.pending
    t234 = ar.ar_greedy(3)                       # tokens after t1 under the target alone
    m.prefill(ids)
    m.draft(2, override_ids=t234[:2])             # a draft the target will accept in full
    m.verify(n_rows=3)
    na, bonus = m.accept()
    assert (na, bonus) == (2, int(t234[2]))
    m.draft(1)                                    # catch-up over slots 20, 21, 22, then one token
    seq = np.concatenate([ids, [t1], t234])       # 24 tokens; slot s pairs feature s with token s + 1
    F64, _ = _target64(cfg, w, seq[:23])
    emb = w["tok_emb"].double()[torch.as_tensor(seq[1:24]).long()]
    x = torch.cat([F64, emb], -1) @ w["draft_fc_w"].double().T + w["draft_fc_b"].double()
    fh = _layer64(cfg, w["draft_layer"], x, torch.arange(23))
    want = (fh[-1] @ w["lm_head"].double().T).numpy()
    np.testing.assert_allclose(m.draft_logits(0), want, atol=3e-5, rtol=0)
    wrong = (fh[-3] @ w["lm_head"].double().T).numpy()   # the first catch-up row would give this
    assert np.max(np.abs(wrong - want)) > 1e-2
    # the sequence log-probability starts afresh with every draft
    lp = torch.log_softmax(torch.from_numpy(m.draft_logits(0)).double(), -1)
    assert abs(m.draft_logprob - float(lp.max())) < 1e-6


@pytest.mark.parametrize("cfg", [TINY, SMALL_BF16], ids=["tiny-fp32", "small-bf16-gqa"])
def test_block_verify_equals_sequential_bit_exact(cfg):
    """A (k+1)-row verify is the same computation as k+1 one-row forwards (Sec. 2.1, 3.1)."""
    ids = synth.token_ids(17, cfg.vocab, 31)
    block = synth.token_ids(cfg.k_max + 1, cfg.vocab, 32)
    a, _ = make_oracle(cfg, 3)
    b, _ = make_oracle(cfg, 3)
    a.prefill(ids)
    b.prefill(ids)
    a.verify(block)
    for r, t in enumerate(block):
        b.verify([t])
        assert np.array_equal(a.logits(r), b.logits(0))
        assert np.array_equal(a.feature(r), b.feature(0))
        b.accept()
    for l in range(cfg.n_layers):
        for s in (0, 16, 17, 17 + cfg.k_max):
            assert np.array_equal(a.kv_row(l, 0, s), b.kv_row(l, 0, s))
            assert np.array_equal(a.kv_row(l, 1, s), b.kv_row(l, 1, s))


def test_prefill_chunking_equals_one_row_prefill():
    cfg = TINY
    ids = synth.token_ids(21, cfg.vocab, 41)
    a, _ = make_oracle(cfg, 4)
    a.prefill(ids)
    b, _ = make_oracle(cfg, 4)
    b.prefill(ids[:1])
    for t in ids[1:]:
        b.verify([t])
        b.accept()
    # same cache => same next-token logits
    a.verify([int(ids[3])])
    b.verify([int(ids[3])])
    assert np.array_equal(a.logits(0), b.logits(0))


def test_float_and_double_accumulators_agree():
    cfg = TINY
    ids = synth.token_ids(32, cfg.vocab, 51)
    a, w = make_oracle(cfg, 5)
    b, _ = make_oracle(cfg, 5, acc_double=True, weights=w)
    a.prefill(ids)
    b.prefill(ids)
    blk = synth.token_ids(4, cfg.vocab, 52)
    a.verify(blk)
    b.verify(blk)
    for r in range(4):
        assert np.max(np.abs(a.logits(r) - b.logits(r))) < 2e-5


def test_bf16_cache_rows_are_bf16_values():
    cfg = SMALL_BF16
    m, _ = make_oracle(cfg, 6)
    m.prefill(synth.token_ids(9, cfg.vocab, 61))
    for which in (0, 1):
        row = m.kv_row(1, which, 5)
        assert np.array_equal(row, torch.from_numpy(row).bfloat16().float().numpy())
        assert np.any(row != 0)
    # rows installed from outside are held to the same 8 significant bits (round to nearest even)
    k = np.random.default_rng(3).standard_normal((4, cfg.n_kv_heads * cfg.head_dim)).astype(np.float32)
    m.kv_import(0, k, -k)
    want = torch.from_numpy(k).bfloat16().float().numpy()
    assert np.any(want != k)
    assert np.array_equal(m.kv_row(0, 0, 2), want[2]) and np.array_equal(m.kv_row(0, 1, 3), -want[3])


def test_kv_import_and_set_state_reproduce_prefill_state():
    """Installing K/V + feature by hand must be equivalent to having computed them."""
    cfg = TINY
    ids = synth.token_ids(12, cfg.vocab, 71)
    a, w = make_oracle(cfg, 7)
    a.prefill(ids)
    b, _ = make_oracle(cfg, 7, weights=w)
    L = cfg.n_layers
    for l in range(L + 1):
        n = 12 if l < L else 11
        k = np.stack([a.kv_row(l, 0, s) for s in range(n)])
        v = np.stack([a.kv_row(l, 1, s) for s in range(n)])
        b.kv_import(l, k, v)
    b.set_state(12, int(ids[-1]), a.pending, a.feature((12 - 1) % (cfg.k_max + 1)))
    assert a.ldlp() == b.ldlp()
    da, db = a.draft(3), b.draft(3)
    assert np.array_equal(da, db)
    a.verify(n_rows=4)
    b.verify(n_rows=4)
    assert np.array_equal(a.logits(3), b.logits(3))
