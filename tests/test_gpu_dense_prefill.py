"""Dense prompt pass (Alg. 1, first iteration on a long prompt) against the oracle (needs an MI355X).

The oracle runs the prompt in blocks of k_max+1 rows; the dense pass runs it in chunks of
128..8192 rows with other kernels.  Both must leave the same state up to rounding: first
token, last-position logits and feature, K/V rows of every layer and of the draft head, and
the decode steps that follow.
"""
import numpy as np
import pytest

from paper_2412_18910_amd import synth
from paper_2412_18910_amd.binding import AE_EINVAL, AE_EUNSUPPORTED, AdaEagleError, Engine
from paper_2412_18910_amd.config import BF16, Config, TINY

from .gpu_helpers import make_pair, top2_margin
from .test_gpu_parity import MARGIN, MED_BF16, SMALL_BF16

pytestmark = pytest.mark.gpu

TOL = 2e-2
GQA4_BF16 = Config(2, 512, 8, 2, 64, 1024, 4096, dtype=BF16, k_max=7, n_ctx_max=1024, ldlp_hidden=64)


def check_state(cfg, eng, orc, n, slots):
    assert eng.kv_len == orc.kv_len == n
    lo, lg = orc.logits(0), eng.logits(0)
    assert np.max(np.abs(lo - lg)) <= TOL, float(np.max(np.abs(lo - lg)))
    if top2_margin(lo) > MARGIN:
        assert eng.pending == orc.pending
    fo = orc.feature((n - 1) % (cfg.k_max + 1))
    fg = eng.feature((n - 1) % 16)
    assert np.max(np.abs(fo - fg)) <= 0.1
    for layer in sorted({0, cfg.n_layers - 1, cfg.n_layers}):
        for which in (0, 1):
            for slot in slots:
                if layer == cfg.n_layers and slot >= n - 1:
                    continue   # the draft head's slot n-1 needs the first new token
                a, b = orc.kv_row(layer, which, slot), eng.kv_row(layer, which, slot)
                assert np.max(np.abs(a - b)) <= np.max(np.abs(a)) * 2 ** -7 + 1e-6, (layer, which, slot)
                assert np.mean(a != b) < (0.02 if layer == 0 else 0.3), (layer, which, slot)


def steps_after(cfg, eng, orc, n_steps=4):
    """A few decode steps from the prefilled state, GPU drafts forced to the oracle's."""
    for r in range(n_steps):
        k = min(cfg.k_max, 2 + r)
        d_o = orc.draft(k)
        d_g = eng.draft(k, override_ids=d_o)
        assert np.array_equal(d_o, d_g)
        for i in range(k):
            assert np.max(np.abs(orc.draft_logits(i) - eng.draft_logits(i))) <= TOL, (r, i)
        orc.verify(n_rows=k + 1)
        eng.verify(n_rows=k + 1)
        clear = True
        for row in range(k + 1):
            lo = orc.logits(row)
            assert np.max(np.abs(lo - eng.logits(row))) <= TOL, (r, row)
            clear = clear and top2_margin(lo) > MARGIN
        ao, ag = orc.accept(), eng.accept()
        if not clear and ao != ag:
            return
        assert ao == ag


@pytest.mark.parametrize("cfg,n,chunk", [
    (SMALL_BF16, 100, 0),      # one ragged 128-row tile, GQA group 4, head_dim 64
    (SMALL_BF16, 300, 128),    # three chunks: attention reads the earlier chunks' cache rows
    (SMALL_BF16, 257, 256),    # a one-row last chunk (no draft rows in it)
    (GQA4_BF16, 450, 256),     # group 4 with two chunks, ragged tail
    (MED_BF16, 200, 0),        # head_dim 128, multi-head, two row tiles in one chunk
])
def test_dense_prefill_state_matches_oracle(cfg, n, chunk):
    eng, orc, _ = make_pair(cfg, 31)
    ids = synth.token_ids(n, cfg.vocab, 300 + n)
    orc.prefill(ids)
    eng.set_prefill_mode(Engine.PREFILL_DENSE, chunk)
    eng.prefill(ids)
    check_state(cfg, eng, orc, n, slots=sorted({0, 15, 16, 63, 64, 127, min(128, n - 2), n - 2, n - 1}))
    steps_after(cfg, eng, orc)
    eng.close()


def test_dense_and_block_prefill_agree_and_auto_picks_by_length():
    cfg = SMALL_BF16
    eng, orc, w = make_pair(cfg, 32)
    ids = synth.token_ids(96, cfg.vocab, 7)
    eng.set_prefill_mode(Engine.PREFILL_BLOCKS)
    eng.prefill(ids)
    lb, fb = eng.logits(0), eng.feature(95 % 16)
    kb = eng.kv_row(cfg.n_layers, 0, 50)
    eng.set_prefill_mode(Engine.PREFILL_AUTO)     # more than one 16-row block: the dense pass
    eng.prefill(ids)
    ld, fd = eng.logits(0), eng.feature(95 % 16)
    kd = eng.kv_row(cfg.n_layers, 0, 50)
    assert np.max(np.abs(lb - ld)) <= TOL and np.max(np.abs(fb - fd)) <= 0.1
    assert np.max(np.abs(kb - kd)) <= np.max(np.abs(kb)) * 2 ** -7
    assert not np.array_equal(lb, ld)             # different kernels, different rounding order
    # a prompt of one block keeps the 16-row path under AUTO: bit-identical to BLOCKS
    short = synth.token_ids(16, cfg.vocab, 8)
    eng.prefill(short)
    la = eng.logits(0)
    eng.set_prefill_mode(Engine.PREFILL_BLOCKS)
    eng.prefill(short)
    assert np.array_equal(la, eng.logits(0))
    # a dense prefill of a short prompt (forced) still matches the oracle
    eng.set_prefill_mode(Engine.PREFILL_DENSE)
    for n in (1, 2, 17):
        p = synth.token_ids(n, cfg.vocab, 9 + n)
        orc.prefill(p)
        eng.prefill(p)
        assert np.max(np.abs(orc.logits(0) - eng.logits(0))) <= TOL, n
        steps_after(cfg, eng, orc, 2)
    eng.close()


def test_dense_prefill_then_lossless_greedy_run():
    """After a dense prefill the speculative loop still reproduces plain greedy decoding of
    the same engine (validated tokens are the target's argmax whatever the draft proposes)."""
    cfg = SMALL_BF16
    eng, _, _ = make_pair(cfg, 33)
    ids = synth.token_ids(200, cfg.vocab, 11)
    eng.set_prefill_mode(Engine.PREFILL_DENSE, 128)
    eng.prefill(ids)
    out = [eng.pending]
    while len(out) < 40:
        k, na, toks = eng.step()
        out.extend(int(t) for t in toks)
    eng.prefill(ids)
    ar = [eng.pending]
    while len(ar) < len(out):
        eng.verify(block_ids=[ar[-1]])
        _, b = eng.accept()
        ar.append(int(b))
    assert out == ar
    eng.close()


def test_prefill_mode_argument_errors():
    cfg = SMALL_BF16
    eng, _, _ = make_pair(cfg, 34)
    for mode, chunk in ((3, 0), (-1, 0), (2, 100), (2, 64), (2, 8320)):
        with pytest.raises(AdaEagleError) as e:
            eng.set_prefill_mode(mode, chunk)
        assert e.value.code == AE_EINVAL
    eng.close()
    eng, _, _ = make_pair(TINY, 35)     # fp32 weights have no dense pass
    with pytest.raises(AdaEagleError) as e:
        eng.set_prefill_mode(Engine.PREFILL_DENSE)
    assert e.value.code == AE_EUNSUPPORTED
    eng.close()


def test_7b_shape_dense_prefill_matches_oracle():
    """Full 7B shape (32 layers): a 160-token prompt (one full 128-row tile plus a ragged one)
    through the dense pass against the oracle's block-wise prompt pass."""
    from paper_2412_18910_amd.config import LLAMA_7B
    cfg = LLAMA_7B.with_(n_ctx_max=256)
    eng, orc, _ = make_pair(cfg, 1)
    n = 160
    ids = synth.token_ids(n, cfg.vocab, 77)
    orc.prefill(ids)
    eng.set_prefill_mode(Engine.PREFILL_DENSE)
    eng.prefill(ids)
    lo, lg = orc.logits(0), eng.logits(0)
    assert np.max(np.abs(lo - lg)) <= TOL, float(np.max(np.abs(lo - lg)))
    if top2_margin(lo) > MARGIN:
        assert eng.pending == orc.pending
    for layer in (0, 31, 32):
        for slot in (0, 127, 128, 158):
            a, b = orc.kv_row(layer, 0, slot), eng.kv_row(layer, 0, slot)
            assert np.max(np.abs(a - b)) <= np.max(np.abs(a)) * 2 ** -7 + 1e-6, (layer, slot)
    # one decode step on top of the dense-prefilled caches (draft head included)
    d_o = orc.draft(3)
    d_g = eng.draft(3, override_ids=d_o)
    assert np.array_equal(d_o, d_g)
    orc.verify(n_rows=4)
    eng.verify(n_rows=4)
    for row in range(4):
        assert np.max(np.abs(orc.logits(row) - eng.logits(row))) <= TOL, row
    eng.close()


def test_7b_shape_2048_token_prompt_dense_agrees_with_block_pass():
    """The benchmark's prompt (2048 tokens, 7B shape, one 2048-row chunk) is too long for the
    oracle; at that size the dense pass is checked against the 16-row pass of the decode
    kernels, which the other tests tie to the oracle: last-position logits and feature, first
    token, and sampled cache rows of the first / last target layer and of the draft head."""
    from paper_2412_18910_amd.config import LLAMA_7B
    cfg = LLAMA_7B.with_(n_ctx_max=2048 + 64)
    w = synth.make_weights(cfg, 1, device="cuda:0")
    eng = Engine(cfg, w)
    ids = synth.token_ids(2048, cfg.vocab, 11)
    res = {}
    for mode in (Engine.PREFILL_BLOCKS, Engine.PREFILL_DENSE):
        eng.set_prefill_mode(mode)
        eng.prefill(ids)
        res[mode] = dict(logits=eng.logits(0), feat=eng.feature(2047 % 16), pending=eng.pending,
                         kv={(l, wh, s): eng.kv_row(l, wh, s) for l in (0, 31, 32) for wh in (0, 1)
                             for s in (0, 1, 1023, 1024, 2046)})
    b, d = res[Engine.PREFILL_BLOCKS], res[Engine.PREFILL_DENSE]
    assert np.max(np.abs(b["logits"] - d["logits"])) <= TOL
    assert np.max(np.abs(b["feat"] - d["feat"])) <= 0.1
    if top2_margin(b["logits"]) > MARGIN:
        assert b["pending"] == d["pending"]
    for key, a in b["kv"].items():
        assert np.max(np.abs(a - d["kv"][key])) <= np.max(np.abs(a)) * 2 ** -6 + 1e-6, key
    eng.close()


def test_8b_gqa_shape_long_prompt_dense_agrees_with_block_pass():
    """8B-GQA shape at reduced depth, 8192-token prompt in four 2048-row chunks (group size 4,
    vocabulary 128256, rope base 5e5): dense pass against the 16-row pass of the decode kernels."""
    from paper_2412_18910_amd.config import LLAMA_8B_GQA
    n = 8192
    cfg = LLAMA_8B_GQA.with_(n_layers=2, n_ctx_max=n + 64, temperature=0.0)
    w = synth.make_weights(cfg, 2, device="cuda:0")
    eng = Engine(cfg, w)
    ids = synth.token_ids(n, cfg.vocab, 13)
    res = {}
    for mode in (Engine.PREFILL_BLOCKS, Engine.PREFILL_DENSE):
        eng.set_prefill_mode(mode)
        eng.prefill(ids)
        res[mode] = dict(logits=eng.logits(0), pending=eng.pending,
                         kv={(l, wh, s): eng.kv_row(l, wh, s) for l in (0, 1, 2) for wh in (0, 1)
                             for s in (0, 2047, 2048, 6143, 8190)})
    b, d = res[Engine.PREFILL_BLOCKS], res[Engine.PREFILL_DENSE]
    assert np.max(np.abs(b["logits"] - d["logits"])) <= TOL
    if top2_margin(b["logits"]) > MARGIN:
        assert b["pending"] == d["pending"]
    for key, a in b["kv"].items():
        assert np.max(np.abs(a - d["kv"][key])) <= np.max(np.abs(a)) * 2 ** -6 + 1e-6, key
    eng.close()
