"""GPU <-> oracle parity through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

from paper_2412_18910_amd import synth
from paper_2412_18910_amd.binding import AE_EINVAL, AE_ESTATE, AdaEagleError
from paper_2412_18910_amd.config import BF16, FP32, Config, TINY

from .gpu_helpers import make_pair, top2_margin
from .helpers import make_oracle

pytestmark = pytest.mark.gpu

SMALL_BF16 = Config(3, 256, 8, 2, 32 * 2, 512, 2048, dtype=BF16, k_max=6, n_ctx_max=640, ldlp_hidden=64,
                    rope_base=500000.0, rms_eps=1e-5)
MED_BF16 = Config(4, 1024, 8, 8, 128, 2816, 8192, dtype=BF16, k_max=8, n_ctx_max=1024, ldlp_hidden=128)
TOL = {FP32: 1e-4, BF16: 2e-2}
MARGIN = 5e-2


def run_teacher_forced(cfg, seed, prompt_len, n_steps, script_mean=2.5):
    """Both sides get the same ids at every step; logits, features, LDLP scalar, draft
    logits, accepted lengths and tokens are compared step by step."""
    eng, orc, w = make_pair(cfg, seed)
    ids = synth.token_ids(prompt_len, cfg.vocab, seed + 100)
    orc.prefill(ids)
    eng.prefill(ids)
    tol = TOL[cfg.dtype]
    assert eng.kv_len == orc.kv_len == prompt_len
    assert eng.pending == orc.pending
    # Acceptance is scripted (a random-init head is almost never accepted on its own): the first
    # a draft tokens of a step are the target's own next tokens, the next one is guaranteed wrong,
    # so the steps that follow start from several validated rows (multi-row draft catch-up,
    # LDLP on the last accepted token) on both sides.
    script = synth.truncated_geometric(n_steps, script_mean, cfg.k_max, seed + 7)
    ar_orc, _ = make_oracle(cfg, seed, weights=w)
    ar_orc.prefill(ids)
    formal = np.concatenate([[ar_orc.pending], ar_orc.ar_greedy(n_steps * (cfg.k_max + 1) + 1)])
    pos = 1                                   # formal[pos] = token that follows the pending one
    worst = 0.0
    stats = dict(steps=0, submargin=0, accepted=0, draft_rows=0, free_tokens=0, verify_rows=0)
    for r in range(n_steps):
        ko, yo = orc.ldlp()
        kg, yg = eng.ldlp()
        assert abs(yo - yg) < 50 * tol, (r, yo, yg)
        if abs(yo - (np.floor(yo) + 0.5)) > 1e-2:
            assert ko == kg
        k = ko
        a = min(int(script[r]), k)
        ov = -np.ones(max(k, 1), np.int32)
        ov[:a] = formal[pos:pos + a]
        if a < k:
            ov[a] = (int(formal[pos + a]) + 1) % cfg.vocab
        # both sides get the SAME scripted table: entries >= 0 are forced, the tokens behind them
        # (-1) are the ones each side picks itself; those must agree wherever the oracle's draft
        # logits have a clear winner
        d_o = orc.draft(k, override_ids=ov[:k] if k else None)
        d_g = eng.draft(k, override_ids=ov[:k] if k else None)
        parted = False
        for i in range(k):
            lo, lg = orc.draft_logits(i), eng.draft_logits(i)
            worst = max(worst, float(np.max(np.abs(lo - lg))))
            assert np.max(np.abs(lo - lg)) <= tol, (r, i)
            stats["draft_rows"] += 1
            if ov[i] >= 0:
                assert int(d_g[i]) == int(d_o[i]) == int(ov[i])
            elif top2_margin(lo) > MARGIN:   # a token the head chose itself, on the device
                assert int(d_g[i]) == int(d_o[i]), (r, i)
                stats["free_tokens"] += 1
            elif int(d_g[i]) != int(d_o[i]):
                parted = True                # sub-margin pick: the two chains legitimately part here
                break
        if parted:
            stats["submargin"] += 1
            break
        assert np.array_equal(d_g, d_o)
        orc.verify(n_rows=k + 1)
        eng.verify(n_rows=k + 1)
        clear = True
        for row in range(k + 1):
            lo, lg = orc.logits(row), eng.logits(row)
            worst = max(worst, float(np.max(np.abs(lo - lg))))
            assert np.max(np.abs(lo - lg)) <= tol, (r, row, float(np.max(np.abs(lo - lg))))
            assert np.max(np.abs(orc.feature(row) - eng.feature(row))) <= 50 * tol
            clear = clear and top2_margin(lo) > MARGIN
            stats["verify_rows"] += 1
        na_o, b_o = orc.accept()
        na_g, b_g = eng.accept()
        stats["steps"] += 1
        stats["accepted"] += na_o
        pos += na_o + 1
        if clear:
            assert (na_g, b_g) == (na_o, b_o), r
            assert na_o == a and b_o == int(formal[pos - 1]), r
        elif (na_g, b_g) != (na_o, b_o):
            stats["submargin"] += 1
            break   # the two sequences legitimately part ways on a sub-margin row
        assert eng.kv_len == orc.kv_len and eng.pending == orc.pending
    eng.close()
    return worst, stats


def test_tiny_fp32_teacher_forced_steps():
    worst, st = run_teacher_forced(TINY, 0, 64, 24)
    assert st["submargin"] == 0 and st["accepted"] >= 24
    assert worst < 1e-4


@pytest.mark.parametrize("cfg,seed,prompt", [(SMALL_BF16, 1, 300), (MED_BF16, 2, 70)], ids=["small-gqa", "medium-mha"])
def test_bf16_teacher_forced_steps(cfg, seed, prompt):
    worst, st = run_teacher_forced(cfg, seed, prompt, 16)
    print(st)
    assert worst < 2e-2
    # the run may stop early only on a sub-margin row; it must have covered real ground before
    # (free picks are rare here, the script forces most tokens: test_bf16_free_draft_tokens_match_oracle covers them)
    assert st["steps"] >= 12 and st["verify_rows"] >= 40 and st["draft_rows"] >= 30 and st["accepted"] >= 12


@pytest.mark.parametrize("cfg,seed,prompt,floor", [(SMALL_BF16, 31, 200, 10), (MED_BF16, 32, 90, 20)],
                         ids=["small-gqa", "medium-mha"])
def test_bf16_free_draft_tokens_match_oracle(cfg, seed, prompt, floor):
    """No override table at all: every draft token is the device-side pick of the bf16 path (argmax
    partials in the LM-head epilogue + the finishing kernel).  It must equal the oracle's token
    wherever the oracle's draft logits have a clear winner (top-2 margin > 5e-2)."""
    eng, orc, _ = make_pair(cfg, seed)
    ids = synth.token_ids(prompt, cfg.vocab, seed + 100)
    orc.prefill(ids)
    eng.prefill(ids)
    compared = steps = 0
    for r in range(12):
        k = cfg.k_max if r % 3 else 1 + r % cfg.k_max
        d_o, d_g = orc.draft(k), eng.draft(k)
        assert len(d_o) == len(d_g) == k
        parted = False
        for i in range(k):
            lo, lg = orc.draft_logits(i), eng.draft_logits(i)
            assert np.max(np.abs(lo - lg)) <= 2e-2 * max(1.0, float(np.std(lo)) / 1.28), (r, i)
            if top2_margin(lo) > MARGIN:
                assert int(d_g[i]) == int(d_o[i]) == int(np.argmax(lo)), (r, i)
                compared += 1
            elif int(d_g[i]) != int(d_o[i]):
                parted = True
                break
        if parted:
            break
        orc.verify(n_rows=k + 1)
        eng.verify(n_rows=k + 1)
        clear = all(top2_margin(orc.logits(row)) > MARGIN for row in range(k + 1))
        ao, ag = orc.accept(), eng.accept()
        if clear:
            assert ao == ag, r
        if ao != ag:
            break
        steps += 1
    print("free draft tokens compared:", compared, "steps:", steps)
    assert compared >= floor and steps >= 6
    eng.close()


def test_tiny_lossless_run_matches_oracle_and_autoregressive():
    """Configuration 1: 64 prompt ids, 128 generated tokens, greedy; speculative output ==
    oracle speculative output == autoregressive output, token for token."""
    cfg = TINY
    eng, orc, w = make_pair(cfg, 0)
    ids = synth.token_ids(64, cfg.vocab, 100)
    orc.prefill(ids)
    ar = orc.ar_greedy(128)
    eng.prefill(ids)
    out, ks = [], []
    while len(out) < 128:
        k, na, toks = eng.step()
        assert len(toks) == na + 1 and 0 <= k <= cfg.k_max
        out.extend(int(t) for t in toks)
        ks.append(k)
    assert np.array_equal(np.array(out[:128]), ar)
    assert len(set(ks)) > 2
    # plain autoregressive decoding on the same kernels gives the same tokens
    eng2, _, _ = make_pair(cfg, 0)
    eng2.prefill(ids)
    ar_gpu = []
    for _ in range(128):
        eng2.verify([eng2.pending])
        ar_gpu.append(eng2.accept()[1])
    assert np.array_equal(np.array(ar_gpu), ar)
    eng.close()
    eng2.close()


def test_scripted_acceptance_exercises_rollback():
    cfg = TINY
    eng, orc, _ = make_pair(cfg, 0)
    ids = synth.token_ids(64, cfg.vocab, 100)
    orc.prefill(ids)
    ar = orc.ar_greedy(160)
    eng.prefill(ids)
    script = synth.truncated_geometric(400, 3.5, cfg.k_max, 3)
    out, r = [], 0
    n_draft = n_waste = n_target = 0
    while len(out) < 128:
        k, _ = eng.ldlp()
        a = min(int(script[r]), k)
        ov = -np.ones(max(k, 1), np.int32)
        pos = len(out)
        ov[:a] = ar[pos:pos + a]
        if a < k:
            ov[a] = (int(ar[pos + a]) + 1) % cfg.vocab
        kk, na, toks = eng.step(k_force=k, override_ids=ov[:k] if k else None)
        assert na == a
        out.extend(int(t) for t in toks)
        n_draft += k; n_waste += k - na; n_target += 1
        r += 1
    assert np.array_equal(np.array(out[:128]), ar[:128])
    assert len(out) == n_draft - n_waste + n_target
    assert eng.kv_len == 64 + len(out)
    eng.close()


@pytest.mark.parametrize("cfg", [TINY, SMALL_BF16], ids=["fp32", "bf16-gqa"])
def test_block_verify_equals_sequential_on_gpu_bit_exact(cfg):
    eng_a, _, _ = make_pair(cfg, 3)
    eng_b, _, _ = make_pair(cfg, 3)
    ids = synth.token_ids(250 if cfg.n_ctx_max > 600 else 40, cfg.vocab, 31)
    block = synth.token_ids(cfg.k_max + 1, cfg.vocab, 32)
    eng_a.prefill(ids)
    eng_b.prefill(ids)
    eng_a.verify(block)
    for r, t in enumerate(block):
        eng_b.verify([int(t)])
        assert np.array_equal(eng_a.logits(r), eng_b.logits(0)), r
        assert np.array_equal(eng_a.feature(r), eng_b.feature(0))
        eng_b.accept()
    eng_a.close()
    eng_b.close()


def test_kv_rows_match_oracle():
    cfg = SMALL_BF16
    eng, orc, _ = make_pair(cfg, 4)
    ids = synth.token_ids(33, cfg.vocab, 41)
    orc.prefill(ids)
    eng.prefill(ids)
    for layer in (0, cfg.n_layers - 1):
        for which in (0, 1):
            for slot in (0, 15, 16, 32):
                a, b = orc.kv_row(layer, which, slot), eng.kv_row(layer, which, slot)
                # identical up to flipped bf16 roundings (1 part in 256); layer 0 sees identical
                # inputs on both sides, deeper layers inherit the flips of the layers before
                assert np.max(np.abs(a - b)) <= np.max(np.abs(a)) * 2 ** -7
                assert np.mean(a != b) < (0.02 if layer == 0 else 0.3)
    eng.close()


def test_rollback_dead_rows_are_never_read():
    """Rollback (Sec. 2.1: the successors of a rejected token are discarded): cache rows at and
    beyond kv_len are dead.  Here they hold large finite junk (+-1e30) on the GPU only, a step
    rejects most of its draft so that rejected tokens' K/V rows stay behind as well, and the
    steps that follow must still match the oracle, which never had those rows.
    (Finite junk: the matrix-core attention multiplies masked keys' V rows by an exact zero.)"""
    cfg = MED_BF16
    eng, orc, w = make_pair(cfg, 14)
    ar, _ = make_oracle(cfg, 14, weights=w)
    n, junk = 200, 60
    sign = np.where(np.arange(cfg.d_kv) % 2 == 0, 1.0, -1.0).astype(np.float32)
    jk = np.tile(1e30 * sign, (junk, 1)).astype(np.float32)
    for layer in range(cfg.n_layers + 1):
        k, v = synth.kv_fill(cfg, n, 15, layer)
        orc.kv_import(layer, k, v)
        ar.kv_import(layer, k, v)
        eng.kv_import(layer, np.concatenate([k, jk]), np.concatenate([v, -jk]))
    assert float(eng.kv_row(0, 1, n + 5)[0]) < -9e29
    feat = synth.feature_row(cfg, 16)
    for m in (orc, ar, eng):
        m.set_state(n, 5, 7, feat)
    formal = ar.ar_greedy(24)            # formal[0] follows the pending token
    pos, compared = 0, 0
    # (k, accepted): reject most of a long draft, then short blocks that leave rejected rows
    # and junk rows inside the 64-key span the attention waves load
    for r, (k, a) in enumerate([(6, 2), (1, 1), (3, 0), (8, 8), (2, 1)]):
        ov = -np.ones(k, np.int32)
        ov[:a] = formal[pos:pos + a]
        if a < k:
            ov[a] = (int(formal[pos + a]) + 1) % cfg.vocab
        d_o = orc.draft(k, override_ids=ov)
        d_g = eng.draft(k, override_ids=d_o)
        orc.verify(n_rows=k + 1)
        eng.verify(n_rows=k + 1)
        clear = True
        for row in range(k + 1):
            lo, lg = orc.logits(row), eng.logits(row)
            assert np.all(np.isfinite(lg))
            assert np.max(np.abs(lo - lg)) <= 2e-2, (r, row)
            clear = clear and top2_margin(lo) > MARGIN
            compared += 1
        ao, ag = orc.accept(), eng.accept()
        if clear:
            assert ao == ag == (a, int(formal[pos + a])), r
        if ao != ag:
            break
        pos += a + 1
        assert eng.kv_len == orc.kv_len == n + pos
    assert compared >= 12
    # the junk that no block has overwritten is still there: nothing cleared it behind our back
    assert float(eng.kv_row(0, 1, n + junk - 1)[0]) < -9e29
    eng.close()


def test_kv_import_rejects_non_finite_values():
    cfg = SMALL_BF16
    eng, _, _ = make_pair(cfg, 4)
    k, v = synth.kv_fill(cfg, 8, 1, 0)
    bad = k.copy()
    bad[3, 5] = np.inf
    with pytest.raises(AdaEagleError) as e:
        eng.kv_import(0, bad, v)
    assert e.value.code == AE_EINVAL
    bad[3, 5] = np.nan
    with pytest.raises(AdaEagleError) as e:
        eng.kv_import(0, k, bad)
    assert e.value.code == AE_EINVAL
    with pytest.raises(AdaEagleError) as e:
        eng.kv_import_static(0, k, bad)
    assert e.value.code == AE_EINVAL
    eng.kv_import(0, k, v)
    eng.close()


@pytest.mark.parametrize("cfg0,seed", [(TINY, 17), (SMALL_BF16, 18), (MED_BF16, 19)], ids=["fp32", "bf16-small", "bf16-medium"])
def test_ldlp_feature_only_input_matches_oracle(cfg0, seed):
    """LDLP fed the hidden state alone (ldlp_in_mode = 1, input width d): scalar and length
    through ae_ldlp against the oracle, after the prompt and after steps with accepted tokens
    (the row behind the last validated token moves with the accepted length)."""
    cfg = cfg0.with_(ldlp_in_mode=1)
    eng, orc, w = make_pair(cfg, seed)
    assert w["ldlp_w_in"].shape[1] == cfg.d_model
    ids = synth.token_ids(50, cfg.vocab, seed + 60)
    orc.prefill(ids)
    eng.prefill(ids)
    ar, _ = make_oracle(cfg, seed, weights=w)
    ar.prefill(ids)
    formal = ar.ar_greedy(60)
    ytol = 1e-3 if cfg.dtype == FP32 else 5e-2
    pos = compared = 0
    ks = []
    for r, a in enumerate([0, 2, 1, 3, 0, 2]):
        ko, yo = orc.ldlp()
        kg, yg = eng.ldlp()
        assert abs(yo - yg) < ytol, (r, yo, yg)
        if abs(yo - (np.floor(yo) + 0.5)) > ytol:
            assert ko == kg, r
            compared += 1
        ks.append(ko)
        k = 3
        ov = -np.ones(k, np.int32)
        ov[:a] = formal[pos:pos + a]
        if a < k:
            ov[a] = (int(formal[pos + a]) + 1) % cfg.vocab
        d_o = orc.draft(k, override_ids=ov)
        eng.draft(k, override_ids=d_o)
        orc.verify(n_rows=k + 1)
        eng.verify(n_rows=k + 1)
        clear = all(top2_margin(orc.logits(row)) > MARGIN for row in range(k + 1))
        ao, ag = orc.accept(), eng.accept()
        if clear:
            assert ao == ag, r
        if ao != ag:
            break
        pos += ao[0] + 1
    assert compared >= 3
    eng.close()


def test_ldlp_loss_kernel_matches_oracle():
    """The LDLP's training criterion (Sec. 3.3) as an evaluation function, device side vs oracle."""
    from oracle import binding as ob
    from .helpers import f32, fp, ip
    lib = ob.load()
    eng, _, _ = make_pair(TINY, 0)
    rng = np.random.default_rng(3)
    for n in (0, 1, 5, 255, 256, 257, 10000):
        pred = f32(rng.uniform(-1, 9, n))
        truth = rng.integers(0, 9, n).astype(np.int32)
        for lam in (1.0, 2.0, 3.5):
            want = lib.orc_ldlp_loss(fp(pred), ip(truth), n, lam) if n else 0.0
            got = eng.ldlp_loss(pred, truth, lam)
            assert abs(got - want) <= 1e-12 * max(1.0, abs(want)), (n, lam, got, want)
    with pytest.raises(AdaEagleError) as e:
        eng.ldlp_loss(f32([1.0]), np.array([1], np.int32), -1.0)
    assert e.value.code == AE_EINVAL
    eng.close()


def test_kv_import_and_set_state_round_trip():
    cfg = MED_BF16
    eng, orc, _ = make_pair(cfg, 5)
    n = 600
    for layer in range(cfg.n_layers + 1):
        k, v = synth.kv_fill(cfg, n, 9, layer)
        orc.kv_import(layer, k, v)
        eng.kv_import(layer, k, v)
        if layer in (0, cfg.n_layers):
            assert np.array_equal(eng.kv_row(layer, 0, 517), k[517])
            assert np.array_equal(eng.kv_row(layer, 1, 3), v[3])
    # values with more than 8 significant bits are rounded to nearest even on the way in, both sides
    rng = np.random.default_rng(11)
    k2 = rng.standard_normal((8, cfg.n_kv_heads * cfg.head_dim)).astype(np.float32)
    k2[0, :4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-39]      # two ties (to even), a negative tie, a subnormal
    scratch = cfg.n_layers                                            # the draft layer's cache, re-imported below
    orc.kv_import(scratch, k2, -k2)
    eng.kv_import(scratch, k2, -k2)
    for slot in (0, 5):
        assert np.array_equal(eng.kv_row(scratch, 0, slot), orc.kv_row(scratch, 0, slot))
        assert np.array_equal(eng.kv_row(scratch, 1, slot), orc.kv_row(scratch, 1, slot))
    assert list(orc.kv_row(scratch, 0, 0)[:3]) == [1.0, 1.015625, -1.0]
    k, v = synth.kv_fill(cfg, n, 9, scratch)
    orc.kv_import(scratch, k, v)
    eng.kv_import(scratch, k, v)
    feat = synth.feature_row(cfg, 5)
    orc.set_state(n, 17, 23, feat)
    eng.set_state(n, 17, 23, feat)
    ko, yo = orc.ldlp()
    kg, yg = eng.ldlp()
    assert abs(yo - yg) < 1e-2
    d_o = orc.draft(4)
    eng.draft(4, override_ids=d_o)
    orc.verify(n_rows=5)
    eng.verify(n_rows=5)
    for row in range(5):
        assert np.max(np.abs(orc.logits(row) - eng.logits(row))) < 2e-2
    eng.close()


def test_edge_cases_and_errors():
    cfg = TINY
    eng, orc, _ = make_pair(cfg, 6)
    with pytest.raises(AdaEagleError) as e:
        eng.ldlp()
    assert e.value.code == AE_ESTATE
    with pytest.raises(AdaEagleError) as e:
        eng.prefill([])
    assert e.value.code == AE_EINVAL
    with pytest.raises(AdaEagleError) as e:
        eng.prefill([cfg.vocab])
    assert e.value.code == AE_EINVAL
    with pytest.raises(AdaEagleError):
        eng.prefill(np.zeros(cfg.n_ctx_max, np.int32))     # does not leave room for a block
    ids = synth.token_ids(1, cfg.vocab, 1)                   # single-token prompt
    orc.prefill(ids)
    eng.prefill(ids)
    assert eng.pending == orc.pending
    with pytest.raises(AdaEagleError) as e:
        eng.verify(n_rows=1)                                 # no draft yet
    assert e.value.code == AE_ESTATE
    with pytest.raises(AdaEagleError) as e:
        eng.draft(cfg.k_max + 1)
    assert e.value.code == AE_EINVAL
    with pytest.raises(AdaEagleError) as e:
        eng.accept()
    assert e.value.code == AE_ESTATE
    # k = 0: a plain autoregressive step through ae_step; k = k_max: the widest block
    for k in (0, cfg.k_max, 0, 3):
        ko, nao, to = orc.step(k_force=k)
        kg, nag, tg = eng.step(k_force=k)
        assert (ko, nao) == (kg, nag) and np.array_equal(to, tg)
    # autoregressive verify steps leave the draft cache behind: drafting must refuse
    eng.verify([eng.pending]); eng.accept()
    eng.verify([eng.pending]); eng.accept()
    with pytest.raises(AdaEagleError) as e:
        eng.draft(2)
    assert e.value.code == AE_ESTATE
    eng.close()


def test_tiny_fp32_sampling_steps_match_oracle():
    """temperature > 0: same uniforms on both sides => same sampled drafts, accepted lengths,
    resampled / bonus tokens (float32 model: logits agree to ~1e-6, so no draw sits on an edge)."""
    cfg = TINY.with_(temperature=0.8)
    eng, orc, _ = make_pair(cfg, 8)
    ids = synth.token_ids(48, cfg.vocab, 81)
    orc.prefill(ids)
    eng.prefill(ids)
    assert eng.pending == orc.pending
    accepted = 0
    for r in range(24):
        k = orc.ldlp()[0] if r % 3 else (r // 3) % (cfg.k_max + 1)
        ud, ua = synth.uniforms(cfg.k_max, 1000 + r), synth.uniforms(cfg.k_max + 1, 2000 + r)
        if r in (7, 16):      # uniforms at the two ends of [0, 1): first / last token that carries mass
            edge = 0.0 if r == 7 else float(np.nextafter(1.0, 0.0))
            ud, ua = np.full_like(ud, edge), np.full_like(ua, edge)
        ko, nao, to = orc.step(k_force=k, u_draft=ud, u_accept=ua)
        kg, nag, tg = eng.step(k_force=k, u_draft=ud, u_accept=ua)
        assert (ko, nao) == (kg, nag) and np.array_equal(to, tg), r
        accepted += nao
    assert eng.kv_len == orc.kv_len
    assert accepted >= 30          # accepted prefixes of several tokens, partial rejections and full rejections all occur
    eng.close()


def test_set_temperature_equals_an_engine_built_at_that_temperature():
    """The temperature is a per-step parameter: an engine switched from greedy to T = 0.8 and on
    to T = 5 produces, step for step, what the oracle built at that temperature produces."""
    base = TINY
    w = synth.make_weights(base, 8)
    from paper_2412_18910_amd.binding import Engine
    from .gpu_helpers import to_device
    from .helpers import make_oracle
    eng = Engine(base.with_(temperature=0.0), to_device(w))
    ids = synth.token_ids(40, base.vocab, 83)
    with pytest.raises(AdaEagleError) as e:
        eng.set_temperature(-1.0)
    assert e.value.code == AE_EINVAL
    with pytest.raises(AdaEagleError) as e:
        eng.set_temperature(float("nan"))
    assert e.value.code == AE_EINVAL
    for T in (0.8, 5.0):
        orc, _ = make_oracle(base.with_(temperature=T), 8, weights=w)
        orc.prefill(ids)
        eng.set_temperature(T)
        eng.prefill(ids)
        for r in range(8):
            k = 1 + (3 * r) % base.k_max
            ud, ua = synth.uniforms(base.k_max, 500 + r), synth.uniforms(base.k_max + 1, 600 + r)
            ko, nao, to = orc.step(k_force=k, u_draft=ud, u_accept=ua)
            kg, nag, tg = eng.step(k_force=k, u_draft=ud, u_accept=ua)
            assert (ko, nao) == (kg, nag) and np.array_equal(to, tg), (T, r)
        assert eng.kv_len == orc.kv_len
    # a draft sampled at one temperature must be judged at the same one
    eng.draft(2, u_draft=[0.3, 0.6])
    with pytest.raises(AdaEagleError) as e:
        eng.set_temperature(1.0)
    assert e.value.code == AE_ESTATE
    eng.verify(n_rows=3)
    eng.accept([0.1, 0.2, 0.3])
    eng.set_temperature(0.0)      # back to greedy: no uniforms needed
    orc0, _ = make_oracle(base, 8, weights=w)
    orc0.prefill(ids)
    eng.prefill(ids)
    for r in range(4):
        ko, nao, to = orc0.step(k_force=3)
        kg, nag, tg = eng.step(k_force=3)
        assert (ko, nao) == (kg, nag) and np.array_equal(to, tg), r
    eng.close()


def _sampling_cfgs():
    from paper_2412_18910_amd.config import LLAMA_8B_GQA
    return [(SMALL_BF16.with_(temperature=1.0), 16, 0),
            # the largest vocabulary of the workloads: 126 segments of 1024 tokens, the last one ragged
            (LLAMA_8B_GQA.with_(n_layers=1, n_ctx_max=128, temperature=0.7), 6, 0),
            # both laws flattened until the random-init head is mostly accepted (the temperature scale of the
            # 8B-GQA workload): accepted prefixes of several tokens and bonus draws from the last row
            (LLAMA_8B_GQA.with_(n_layers=1, n_ctx_max=128, temperature=26.0), 8, 8)]


@pytest.mark.parametrize("cfg,n_steps,min_accepted", _sampling_cfgs(), ids=["small", "vocab128256", "vocab128256_T26"])
def test_bf16_sampling_kernels_match_oracle_rule_on_gpu_logits(cfg, n_steps, min_accepted):
    """Accept-kernel parity: the oracle's rule applied to the logits the GPU produced must give
    the GPU's own (n_accepted, bonus) and draft samples, for the same uniforms."""
    import ctypes as C
    from oracle import binding as ob
    from paper_2412_18910_amd.binding import Engine
    from .gpu_helpers import to_device
    from .helpers import dp, fp, ip
    eng = Engine(cfg, to_device(synth.make_weights(cfg, 9)))
    lib = ob.load()
    ids = synth.token_ids(40, cfg.vocab, 91)
    eng.prefill(ids)
    V, T = cfg.vocab, float(cfg.temperature)
    n_acc_hist = []
    for r in range(n_steps):
        k = 1 + r % cfg.k_max
        ud, ua = synth.uniforms(cfg.k_max, 3000 + r), synth.uniforms(cfg.k_max + 1, 4000 + r)
        d = eng.draft(k, u_draft=ud)
        dl = np.stack([eng.draft_logits(i) for i in range(k)])
        for i in range(k):   # the sampled draft token is the inverse CDF of softmax(draft logits / T)
            p = np.exp((dl[i].astype(np.float64) - dl[i].max()) / T)
            assert lib.orc_sample_inverse_cdf(dp(np.ascontiguousarray(p)), V, float(ud[i])) == d[i], (r, i)
        eng.verify(n_rows=k + 1)
        tl = np.stack([eng.logits(i) for i in range(k + 1)])
        na, b = C.c_int(), C.c_int32()
        dd = np.ascontiguousarray(d, np.int32)
        uu = np.ascontiguousarray(ua[:k + 1], np.float64)
        lib.orc_accept_sample(fp(np.ascontiguousarray(tl)), fp(np.ascontiguousarray(dl)), V, k, ip(dd), T, dp(uu),
                              C.byref(na), C.byref(b))
        got = eng.accept(ua[:k + 1])
        assert got == (na.value, b.value), r
        n_acc_hist.append(got[0])
    assert eng.kv_len == 40 + sum(n_acc_hist) + len(n_acc_hist)
    assert sum(n_acc_hist) >= min_accepted, n_acc_hist
    eng.close()


def test_sampling_argument_errors():
    cfg = TINY.with_(temperature=0.5)
    eng, _, _ = make_pair(cfg, 10)
    eng.prefill(synth.token_ids(8, cfg.vocab, 3))
    with pytest.raises(AdaEagleError) as e:
        eng.draft(2)                                   # uniforms missing
    assert e.value.code == AE_EINVAL
    eng.draft(2, u_draft=[0.1, 0.7])
    eng.verify(n_rows=3)
    with pytest.raises(AdaEagleError) as e:
        eng.accept()                                   # uniforms missing
    assert e.value.code == AE_EINVAL
    with pytest.raises(AdaEagleError) as e:
        eng.accept([0.1, 1.0, 0.2])                    # 1.0 is outside [0, 1)
    assert e.value.code == AE_EINVAL
    na, b = eng.accept([0.1, 0.2, 0.3])
    assert 0 <= na <= 2 and 0 <= b < cfg.vocab
    eng.close()


def _full_size_step(cfg, seed, n_ctx, ks, tol=2e-2, sampling=False):
    """One or more teacher-forced steps at a full-width shape: weights drawn on the GPU and
    copied to the host for the oracle, K/V of every layer imported from the seeded generator,
    so the oracle only has to run the step itself."""
    import torch
    from paper_2412_18910_amd.binding import Engine
    from .helpers import make_oracle
    w = synth.make_weights(cfg, seed, device="cuda:0")
    eng = Engine(cfg, w)
    orc, _ = make_oracle(cfg, seed, weights=w)      # converts to host numpy (bf16 bit patterns)
    for layer in range(cfg.n_layers + 1):
        k, v = synth.kv_fill(cfg, n_ctx, seed, layer)
        orc.kv_import(layer, k, v)
        eng.kv_import(layer, k, v)
    feat = synth.feature_row(cfg, seed + 1)
    orc.set_state(n_ctx, 5, 7, feat)
    eng.set_state(n_ctx, 5, 7, feat)
    worst = 0.0
    for r, k in enumerate(ks):
        yo, yg = orc.ldlp()[1], eng.ldlp()[1]
        assert abs(yo - yg) < 0.05, (yo, yg)
        ud = synth.uniforms(cfg.k_max, 50 + r) if sampling else None
        ua = synth.uniforms(cfg.k_max + 1, 60 + r) if sampling else None
        d_o = orc.draft(k, u_draft=ud)
        d_g = eng.draft(k, override_ids=d_o, u_draft=ud)
        errs_d = [float(np.max(np.abs(orc.draft_logits(i) - eng.draft_logits(i)))) for i in range(k)]
        orc.verify(n_rows=k + 1)
        eng.verify(n_rows=k + 1)
        errs_v = [float(np.max(np.abs(orc.logits(row) - eng.logits(row)))) for row in range(k + 1)]
        stds_d = [float(np.std(orc.draft_logits(i))) for i in range(k)]
        print(f"step {r}: k={k} draft-chain max|dlogit| {['%.1e' % e for e in errs_d]} (logit std {['%.1f' % v for v in stds_d]}) "
              f"verify rows {['%.1e' % e for e in errs_v]}", flush=True)
        clear = True
        for i, e in enumerate(errs_d):
            # The random-init draft head is not norm-preserving: chained outputs (and their logits)
            # grow with the chain depth, so the bound scales with the row's own logit spread
            # relative to the 1.28 of a target row (0.02 * sqrt(4096)).
            assert e <= tol * max(1.0, stds_d[i] / 1.28), ("draft", r, i, e, stds_d[i])
        for row in range(k + 1):
            lo = orc.logits(row)
            e = errs_v[row]
            worst = max(worst, e)
            assert e <= tol, ("verify", r, row, e)
            clear = clear and top2_margin(lo) > MARGIN
        ao, ag = orc.accept(ua[:k + 1] if sampling else None), eng.accept(ua[:k + 1] if sampling else None)
        if clear and not sampling:
            assert ao == ag
        if ao != ag:
            break
    eng.close()
    orc.close()
    del w
    torch.cuda.empty_cache()
    return worst


def test_7b_shape_full_size_step_matches_oracle():
    """The benchmark's own shape and launch configuration: 32 layers, d 4096, 1024 cached tokens."""
    from paper_2412_18910_amd.config import LLAMA_7B
    cfg = LLAMA_7B.with_(n_ctx_max=1024 + 64)
    worst = _full_size_step(cfg, 1, 1024, ks=[4, 8])
    print("7B full-size max |dlogit| =", worst)
    assert worst < 2e-2


def test_8b_gqa_shape_reduced_depth_step_matches_oracle():
    """Grouped-query attention (32 query / 8 KV heads), 128256-token vocabulary, rope base 5e5,
    at full width with 2 layers; 1100 cached tokens span several attention chunks."""
    from paper_2412_18910_amd.config import LLAMA_8B_GQA
    cfg = LLAMA_8B_GQA.with_(n_layers=2, n_ctx_max=1100 + 64, temperature=0.0)
    worst = _full_size_step(cfg, 2, 1100, ks=[8, 3])
    assert worst < 2e-2
    cfg = cfg.with_(temperature=1.0)
    _full_size_step(cfg, 3, 300, ks=[5], sampling=True)


def test_13b_shape_reduced_depth_step_matches_oracle():
    """13B width (d 5120, 40 heads, FFN 13824) at 2 layers with k_max = 10: 11-row verify blocks,
    a 3000-slot cache (12 attention chunks) and the ragged-tail GEMM shapes of this model."""
    from paper_2412_18910_amd.config import LLAMA_13B
    cfg = LLAMA_13B.with_(n_layers=2, n_ctx_max=3000 + 64)
    worst = _full_size_step(cfg, 4, 3000, ks=[10, 0, 6])
    assert worst < 2e-2


def test_13b_shape_full_depth_step_matches_oracle():
    """All 40 layers of the 13B shape at its workload context (4096 cached tokens, 16 attention
    chunks), one teacher-forced step with the widest block (k = k_max = 10, 11 rows)."""
    from paper_2412_18910_amd.config import LLAMA_13B
    cfg = LLAMA_13B.with_(n_ctx_max=4096 + 64)
    worst = _full_size_step(cfg, 5, 4096, ks=[10])
    print("13B full-depth max |dlogit| =", worst)
    assert worst < 2e-2


def test_8b_gqa_shape_full_depth_step_matches_oracle():
    """All 32 layers of the 8B-GQA shape (4 query heads per KV head, 128256-token vocabulary) at
    its workload context (8192 cached tokens, 32 attention chunks), greedy, k = k_max = 8."""
    from paper_2412_18910_amd.config import LLAMA_8B_GQA
    cfg = LLAMA_8B_GQA.with_(n_ctx_max=8192 + 64, temperature=0.0)
    worst = _full_size_step(cfg, 6, 8192, ks=[8])
    print("8B-GQA full-depth max |dlogit| =", worst)
    assert worst < 2e-2


@pytest.mark.parametrize("cfg0,seed", [(TINY, 12), (MED_BF16, 13)], ids=["fp32", "bf16"])
def test_ddd_exit_rule_matches_oracle(cfg0, seed):
    """AdaEAGLE-DDD: the draft keeps going past the predicted length while the sequence
    log-probability stays above the threshold; lengths, tokens and the log-probability match."""
    probe_cfg = cfg0.with_(ddd_enabled=1, ddd_threshold=-1e9)
    eng, orc, w = make_pair(probe_cfg, seed)
    ids = synth.token_ids(40, probe_cfg.vocab, seed + 200)
    orc.prefill(ids)
    eng.prefill(ids)
    d_o = orc.draft(0)
    d_g = eng.draft(0, override_ids=np.concatenate([d_o, -np.ones(probe_cfg.k_max, np.int32)])[:probe_cfg.k_max])
    assert len(d_o) == len(d_g) == probe_cfg.k_max            # threshold -1e9: always k_max tokens
    assert abs(orc.draft_logprob - eng.draft_logprob) < (1e-3 if cfg0.dtype == FP32 else 5e-2)
    cums = np.cumsum([float(np.log(np.exp(orc.draft_logits(i).astype(np.float64) - orc.draft_logits(i).max()).sum()) * -1
                            + orc.draft_logits(i)[int(t)] - orc.draft_logits(i).max()) for i, t in enumerate(d_o)])
    eng.close()
    # thresholds half way between consecutive cumulative log-probabilities: no decision near a tie
    for cut, k in [(1, 0), (3, 2), (5, 5), (2, 6)]:
        theta = float(0.5 * (cums[cut] + cums[cut + 1]))
        cfg = cfg0.with_(ddd_enabled=1, ddd_threshold=theta)
        eng, orc, _ = make_pair(cfg, seed)
        orc.prefill(ids)
        eng.prefill(ids)
        want = orc.draft(k)
        got = eng.draft(k, override_ids=np.concatenate([want, -np.ones(cfg.k_max, np.int32)])[:cfg.k_max])
        assert len(want) == max(k, cut + 2), (cut, k, len(want))
        assert np.array_equal(got, want)
        # a full step: verify block of (drafted + 1) rows, accept, next prediction
        orc.verify(n_rows=len(want) + 1)
        eng.verify(n_rows=len(got) + 1)
        lo, lg = orc.logits(len(want)), eng.logits(len(got))
        assert np.max(np.abs(lo - lg)) <= TOL[cfg.dtype]
        clear = all(top2_margin(orc.logits(r)) > MARGIN for r in range(len(want) + 1))
        acc_o, acc_g = orc.accept(), eng.accept()
        assert acc_o == acc_g or not clear
        if acc_o == acc_g:
            # next step: the statistic starts from zero again
            w2 = orc.draft(1)
            g2 = eng.draft(1, override_ids=np.concatenate([w2, -np.ones(cfg.k_max, np.int32)])[:cfg.k_max])
            assert np.array_equal(w2, g2)
            assert abs(orc.draft_logprob - eng.draft_logprob) < (1e-3 if cfg0.dtype == FP32 else 5e-2)
        eng.close()
    # tokens forced by the caller: the statistic is the log-probability of THOSE tokens, on both sides
    cfg = cfg0.with_(ddd_enabled=1, ddd_threshold=-1e9)      # never reached: k_max tokens, no decision near a tie
    eng, orc, _ = make_pair(cfg, seed)
    orc.prefill(ids)
    eng.prefill(ids)
    forced = -np.ones(cfg.k_max, np.int32)
    forced[:3] = [5, (int(d_o[1]) + 77) % cfg.vocab, 9]
    want = orc.draft(1, override_ids=forced)
    got = eng.draft(1, override_ids=np.where(forced >= 0, forced, np.concatenate([want, forced])[:cfg.k_max]))
    assert np.array_equal(want, got) and list(want[:3]) == list(forced[:3]) and len(want) == cfg.k_max
    assert orc.draft_logprob < -10.0       # three unlikely tokens
    assert abs(orc.draft_logprob - eng.draft_logprob) < (1e-3 if cfg0.dtype == FP32 else 0.1)
    eng.close()


def _logp64(logits, tok, T=1.0):
    z = logits.astype(np.float64) / T
    return float(z[int(tok)] - z.max() - np.log(np.exp(z - z.max()).sum()))


@pytest.mark.parametrize("temperature", [0.0, 0.8], ids=["greedy", "T0.8"])
def test_ddd_device_rule_matches_host_rule_and_oracle_fp32(temperature):
    """AdaEAGLE-DDD with the exit rule evaluated on the device (no synchronisation inside the
    draft, padded verify block, drafted length taken from the device by the accept kernels)
    against the host-evaluated rule and the oracle: whole steps, greedy and temperature > 0
    (the statistic is then the log-probability of the SAMPLED tokens under softmax(logits/T))."""
    base = TINY.with_(temperature=temperature, ddd_enabled=1)
    ids = synth.token_ids(40, base.vocab, 300)
    n_steps = 10

    def uni(r):
        if temperature == 0.0:
            return None, None
        return synth.uniforms(base.k_max, 5000 + r), synth.uniforms(base.k_max + 1, 6000 + r)

    # probe: cumulative log-probabilities at every depth with the rule switched off (-1e9)
    probe, _ = make_oracle(base.with_(ddd_threshold=-1e9), 50)
    probe.prefill(ids)
    depth3 = []
    for r in range(n_steps):
        ud, ua = uni(r)
        d = probe.draft(0, u_draft=ud)
        assert len(d) == base.k_max
        T = temperature if temperature > 0 else 1.0
        depth3.append(sum(_logp64(probe.draft_logits(i), d[i], T) for i in range(3)))
        probe.verify(n_rows=len(d) + 1)
        probe.accept(ua[:len(d) + 1] if ua is not None else None)
    srt = sorted(depth3)
    theta = 0.5 * (srt[n_steps // 2 - 1] + srt[n_steps // 2])     # about half of the steps pass depth 3
    assert min(abs(v - theta) for v in depth3) > 1e-3
    cfg = base.with_(ddd_threshold=float(theta))
    eng_h, orc, w = make_pair(cfg, 50)
    from paper_2412_18910_amd.binding import Engine
    from .gpu_helpers import to_device
    eng_d = Engine(cfg, to_device(w))
    eng_d.set_ddd_mode(Engine.DDD_DEVICE)
    for m in (orc, eng_h, eng_d):
        m.prefill(ids)
    lens = []
    for r in range(n_steps):
        k = r % 4                                  # predicted lengths 0..3: the rule decides the rest
        ud, ua = uni(r)
        so = orc.step(k_force=k, u_draft=ud, u_accept=ua)
        sh = eng_h.step(k_force=k, u_draft=ud, u_accept=ua)
        sd = eng_d.step(k_force=k, u_draft=ud, u_accept=ua)
        for got in (sh, sd):
            assert got[:2] == so[:2] and np.array_equal(got[2], so[2]), (r, so, got)
        lens.append(so[0])
        assert abs(eng_d.draft_logprob - orc.draft_logprob) < 1e-3
        assert eng_h.kv_len == eng_d.kv_len == orc.kv_len
    assert any(l > (r % 4) for r, l in enumerate(lens)) and any(l < base.k_max for l in lens), lens
    # un-padded use of the device rule: ae_draft with an id output synchronises and reports the length
    ud, ua = uni(99)
    want = orc.draft(1, u_draft=ud)
    got = eng_d.draft(1, u_draft=ud)
    assert np.array_equal(want, got)
    orc.verify(n_rows=len(want) + 1)
    eng_d.verify(n_rows=len(got) + 1)
    assert orc.accept(ua[:len(want) + 1] if ua is not None else None) == \
        eng_d.accept(ua[:len(got) + 1] if ua is not None else None)
    with pytest.raises(AdaEagleError) as e:
        eng_d.set_ddd_mode(7)
    assert e.value.code == AE_EINVAL
    for m in (eng_h, eng_d):
        m.close()


def test_ddd_device_rule_equals_host_rule_bf16_and_decides_next_to_the_threshold():
    """bf16 path: (1) device-evaluated rule == host-evaluated rule, step for step (same kernels,
    so tokens, lengths and logits are bit-identical); (2) the statistic the kernels keep equals a
    float64 evaluation of the GPU's own draft logits to 1e-3; (3) thresholds placed 2e-3 below /
    above that value make the chain continue / stop exactly there."""
    from paper_2412_18910_amd.binding import Engine
    from .gpu_helpers import to_device
    base = MED_BF16.with_(ddd_enabled=1)
    w = to_device(synth.make_weights(base, 60))
    ids = synth.token_ids(60, base.vocab, 301)
    probe = Engine(base.with_(ddd_threshold=-1e9), w)
    probe.prefill(ids)
    d = probe.draft(0)
    assert len(d) == base.k_max
    lps = [_logp64(probe.draft_logits(i), d[i]) for i in range(base.k_max)]
    cums = np.cumsum(lps)
    assert abs(probe.draft_logprob - cums[-1]) < 1e-3 * max(1.0, abs(cums[-1]) / 10)
    probe.close()
    for mode in (Engine.DDD_HOST, Engine.DDD_DEVICE):
        for j in (0, 2, 4):                       # decision taken behind token j+1
            for sign, want_len in ((-1, None), (+1, j + 1)):
                theta = float(cums[j] + sign * 2e-3)
                eng = Engine(base.with_(ddd_threshold=theta), w)
                eng.set_ddd_mode(mode)
                eng.prefill(ids)
                got = eng.draft(1)
                if want_len is None:              # threshold just below: the chain goes past token j+1
                    assert len(got) >= j + 2, (mode, j, len(got))
                    nxt = next((i for i in range(j + 1, base.k_max) if cums[i] < theta), base.k_max - 1)
                    assert len(got) == min(nxt + 1, base.k_max)
                else:                             # threshold just above: token j+1 is the last one
                    assert len(got) == max(want_len, 1), (mode, j, len(got))
                assert np.array_equal(got, d[:len(got)])
                eng.close()
    # whole steps, natural drafts: the two modes agree bit for bit
    theta = float(np.median(cums[1:4]))
    cfg = base.with_(ddd_threshold=theta)
    eng_h, eng_d = Engine(cfg, w), Engine(cfg, w)
    eng_d.set_ddd_mode(Engine.DDD_DEVICE)
    eng_h.prefill(ids)
    eng_d.prefill(ids)
    lens = []
    for r in range(10):
        k = r % 5
        sh, sd = eng_h.step(k_force=k), eng_d.step(k_force=k)
        assert sh[:2] == sd[:2] and np.array_equal(sh[2], sd[2]), (r, sh, sd)
        assert np.array_equal(eng_h.logits(sh[1]), eng_d.logits(sd[1]))
        assert eng_h.draft_logprob == eng_d.draft_logprob
        lens.append(sh[0])
    assert len(set(l - r % 5 for r, l in enumerate(lens))) > 1, lens     # some steps extended, by different amounts
    eng_h.close()
    eng_d.close()


def test_ddd_device_rule_equals_host_rule_bf16_sampling():
    """bf16 path at temperature > 0 with the exit rule on: sampled drafts, rejection sampling on a
    padded block (the accept kernels take the drafted length from the device) - the two modes agree
    bit for bit, and the statistic is the log-probability of the SAMPLED tokens under softmax(l/T)."""
    from paper_2412_18910_amd.binding import Engine
    from .gpu_helpers import to_device
    T = 0.7
    cfg = SMALL_BF16.with_(temperature=T, ddd_enabled=1, ddd_threshold=-14.0)
    w = to_device(synth.make_weights(cfg, 61))
    ids = synth.token_ids(80, cfg.vocab, 302)
    eng_h, eng_d = Engine(cfg, w), Engine(cfg, w)
    eng_h.set_ddd_mode(Engine.DDD_HOST)
    eng_d.set_ddd_mode(Engine.DDD_DEVICE)
    eng_h.prefill(ids)
    eng_d.prefill(ids)
    lens = []
    for r in range(12):
        k = r % 3
        ud, ua = synth.uniforms(cfg.k_max, 7000 + r), synth.uniforms(cfg.k_max + 1, 8000 + r)
        if r % 4 == 3:      # un-padded use: the id output synchronises, then verify / accept with the real length
            dh, dd = eng_h.draft(k, u_draft=ud), eng_d.draft(k, u_draft=ud)
            assert np.array_equal(dh, dd)
            lp = sum(_logp64(eng_d.draft_logits(i), dd[i], T) for i in range(len(dd)))
            assert abs(eng_d.draft_logprob - lp) < 1e-3 * max(1.0, abs(lp) / 10)
            eng_h.verify(n_rows=len(dh) + 1)
            eng_d.verify(n_rows=len(dd) + 1)
            assert eng_h.accept(ua[:len(dh) + 1]) == eng_d.accept(ua[:len(dd) + 1])
            lens.append(len(dd))
        else:
            sh = eng_h.step(k_force=k, u_draft=ud, u_accept=ua)
            sd = eng_d.step(k_force=k, u_draft=ud, u_accept=ua)
            assert sh[:2] == sd[:2] and np.array_equal(sh[2], sd[2]), (r, sh, sd)
            assert eng_h.draft_logprob == eng_d.draft_logprob
            lens.append(sh[0])
        assert eng_h.kv_len == eng_d.kv_len and eng_h.pending == eng_d.pending
    assert min(lens) < cfg.k_max and max(l - r % 3 for r, l in enumerate(lens)) > 0, lens   # the rule both stopped and extended
    eng_h.close()
    eng_d.close()


EDGE_BF16 = Config(2, 256, 4, 2, 64, 512, 1024, dtype=BF16, k_max=15, n_ctx_max=1024, ldlp_hidden=64)


@pytest.mark.parametrize("n_ctx,cap", [(n, 1024) for n in (1, 15, 16, 17, 255, 256, 257, 511, 513)] +
                         [(n, 2304) for n in (31, 33, 127, 128, 129, 383, 385)])
def test_context_lengths_around_tile_and_chunk_boundaries(n_ctx, cap):
    """Cached lengths next to the 16/32-slot cache tiles, the 64-key spans of the attention waves
    and the 256-key attention chunks, at two cache capacities, with the widest block (k_max = 15:
    16 rows, group size 2) so that blocks straddle the boundaries."""
    cfg = EDGE_BF16.with_(n_ctx_max=cap)
    eng, orc, _ = make_pair(cfg, 20)
    for layer in range(cfg.n_layers + 1):
        k, v = synth.kv_fill(cfg, n_ctx, 30 + n_ctx, layer)
        orc.kv_import(layer, k, v)
        eng.kv_import(layer, k, v)
    feat = synth.feature_row(cfg, 21)
    orc.set_state(n_ctx, 3, 4, feat)
    eng.set_state(n_ctx, 3, 4, feat)
    done = 0
    for k in (15, 0, 7):
        d_o = orc.draft(k)
        d_g = eng.draft(k, override_ids=d_o if k else None)
        assert np.array_equal(d_o, d_g)
        orc.verify(n_rows=k + 1)
        eng.verify(n_rows=k + 1)
        for row in range(k + 1):
            assert np.max(np.abs(orc.logits(row) - eng.logits(row))) <= 2e-2, (n_ctx, k, row)
        clear = all(top2_margin(orc.logits(row)) > MARGIN for row in range(k + 1))
        ao, ag = orc.accept(), eng.accept()
        if clear:
            assert ao == ag, (n_ctx, k)
        done += 1
        if ao != ag:      # only possible on a row without a clear winner
            break
    assert done >= 1
    eng.close()


def test_read_stream_probe_reports_a_plausible_rate():
    """The diagnostic yardstick of the bandwidth figures: a chain of read-only kernels."""
    from paper_2412_18910_amd.binding import load_library, probe_read_stream
    import ctypes as C
    us = probe_read_stream(32 << 20, launches=16, repeats=2)
    gbps = (32 << 20) / us / 1e3
    assert 1000.0 < gbps < 8000.0, gbps          # between a seventh of the published HBM peak and the peak itself
    out = C.c_double()
    assert load_library().ae_probe_read_stream(None, 1000, 4, 1, C.byref(out)) == AE_EINVAL   # not a multiple of 4096


def test_capacity_limits_are_enforced():
    cfg = EDGE_BF16.with_(n_ctx_max=64, k_max=7)
    eng, _, _ = make_pair(cfg, 22)
    with pytest.raises(AdaEagleError) as e:
        eng.prefill(np.zeros(57, np.int32))        # 57 + k_max + 1 > 64
    assert e.value.code == AE_EINVAL
    eng.prefill(np.zeros(56, np.int32))            # exactly fits one more widest block
    assert eng.kv_len == 56
    k, na, toks = eng.step(k_force=7)
    assert eng.kv_len == 56 + na + 1
    with pytest.raises(AdaEagleError) as e:        # the next widest block would overflow the cache
        eng.step(k_force=7)
    assert e.value.code == AE_EINVAL
    eng.close()


def test_two_contexts_are_independent():
    cfg = TINY
    eng_a, orc, w = make_pair(cfg, 23)
    from .gpu_helpers import to_device
    from paper_2412_18910_amd.binding import Engine
    eng_b = Engine(cfg, to_device(w))
    ids_a, ids_b = synth.token_ids(20, cfg.vocab, 1), synth.token_ids(31, cfg.vocab, 2)
    eng_a.prefill(ids_a)
    eng_b.prefill(ids_b)
    orc.prefill(ids_a)
    for _ in range(6):                              # interleave the two sequences
        ta = eng_a.step(k_force=3)
        eng_b.step(k_force=5)
        to = orc.step(k_force=3)
        assert ta[1] == to[1] and np.array_equal(ta[2], to[2])
    eng_a.close()
    eng_b.close()


@pytest.mark.parametrize("cfg0,seed", [(TINY, 0), (SMALL_BF16, 6)])
def test_ldlp_classification_head_matches_oracle(cfg0, seed):
    """Classification variant of the LDLP (Sec. 4.3 ablation): k_max+1 class scores, k = the
    best-scoring length.  The winning score is compared always; the class wherever the top two
    scores (float64 re-expression of the MLP on the oracle's own feature row) are clearly apart."""
    import torch
    F = torch.nn.functional
    cfg = cfg0.with_(ldlp_cls=1, ldlp_n_res=1)
    eng, orc, w = make_pair(cfg, seed)
    n = 24
    ids = synth.token_ids(n, cfg.vocab, seed + 50)
    orc.prefill(ids)
    eng.prefill(ids)
    ytol = 1e-3 if cfg.dtype == FP32 else 0.1    # class scores have a spread of ~k_max/4
    last_tok, f_row = int(ids[-1]), (n - 1) % (cfg.k_max + 1)
    compared = 0
    for r in range(10):
        ko, yo = orc.ldlp()
        kg, yg = eng.ldlp()
        assert abs(yo - yg) < ytol, (r, yo, yg)
        u = torch.cat([w["tok_emb"].double()[last_tok], torch.from_numpy(orc.feature(f_row)).double()])
        z = F.linear(u, w["ldlp_w_in"].double(), w["ldlp_b_in"].double())
        z = z + F.silu(F.linear(z, w["ldlp_w_res"][0].double(), w["ldlp_b_res"][0].double()))
        scores = F.linear(F.silu(z), w["ldlp_w_out"].double(), w["ldlp_b_out"].double()).numpy()
        assert ko == int(np.argmax(scores))
        if top2_margin(scores) > 3 * ytol:
            assert kg == ko, (r, scores)
            compared += 1
        k = min(ko, 3)
        pend = orc.pending
        d_o = orc.draft(k)
        d_g = eng.draft(k, override_ids=d_o if k else None)
        assert np.array_equal(d_o, d_g)
        orc.verify(n_rows=k + 1)
        eng.verify(n_rows=k + 1)
        clear = all(top2_margin(orc.logits(row)) > MARGIN for row in range(k + 1))
        ao, ag = orc.accept(), eng.accept()
        if clear:
            assert ao == ag, r
        if ao != ag:
            break
        last_tok, f_row = (pend if ao[0] == 0 else int(d_o[ao[0] - 1])), ao[0]
    assert compared >= 3
    eng.close()


def test_ldlp_classification_reaches_every_length_including_k_max():
    """Zero input layer and equal output rows: the bias alone names the class, on both sides."""
    import torch
    from paper_2412_18910_amd.binding import Engine
    from .gpu_helpers import to_device
    cfg = TINY.with_(ldlp_cls=1)
    w = dict(synth.make_weights(cfg, 0))
    w["ldlp_w_in"] = torch.zeros_like(w["ldlp_w_in"])
    w["ldlp_b_in"] = torch.full_like(w["ldlp_b_in"], 0.5)
    w["ldlp_w_out"] = torch.ones_like(w["ldlp_w_out"])
    ids = synth.token_ids(8, cfg.vocab, 5)
    for want_k in (0, 3, cfg.k_max):
        bias = torch.zeros(cfg.k_max + 1)
        bias[want_k] = 2.0
        w["ldlp_b_out"] = bias
        orc, _ = make_oracle(cfg, 0, weights=w)
        eng = Engine(cfg, to_device(w))
        orc.prefill(ids)
        eng.prefill(ids)
        (ko, yo), (kg, yg) = orc.ldlp(), eng.ldlp()
        assert ko == kg == want_k and abs(yo - yg) < 1e-3
        eng.close()


def test_runs_are_bit_reproducible():
    """No atomics on floating-point data and fixed reduction orders everywhere: two engines fed the
    same bytes produce bit-identical logits, features and cache rows (dense prompt pass, greedy
    steps, and a temperature > 0 configuration with the same uniforms)."""
    from paper_2412_18910_amd.binding import Engine
    from .gpu_helpers import to_device
    for cfg in (MED_BF16, SMALL_BF16.with_(temperature=0.8)):
        w = to_device(synth.make_weights(cfg, 40))
        ids = synth.token_ids(130, cfg.vocab, 41)
        runs = []
        for rep in range(2):
            eng = Engine(cfg, w)
            eng.set_prefill_mode(Engine.PREFILL_DENSE)
            eng.prefill(ids)
            rec = [eng.logits(0).tobytes(), eng.kv_row(cfg.n_layers, 0, 100).tobytes()]
            for r in range(4):
                k = 2 + r
                ud = synth.uniforms(cfg.k_max, 70 + r) if cfg.temperature > 0 else None
                ua = synth.uniforms(cfg.k_max + 1, 80 + r) if cfg.temperature > 0 else None
                kk, na, toks = eng.step(k_force=k, u_draft=ud, u_accept=ua)
                rec += [toks.tobytes(), eng.logits(min(na, k)).tobytes(), eng.feature(0).tobytes(),
                        eng.draft_logits(k - 1).tobytes()]
            runs.append(rec)
            eng.close()
        assert runs[0] == runs[1]


def test_largest_supported_context():
    """n_ctx_max = 16384 is the largest cache the attention kernels accept (64 chunks of 256 keys):
    a step right at the end of that cache, against the oracle; one slot more is refused."""
    from paper_2412_18910_amd.binding import AE_EUNSUPPORTED, Engine
    from .gpu_helpers import to_device
    cfg = EDGE_BF16.with_(n_ctx_max=16384, k_max=7)
    eng, orc, _ = make_pair(cfg, 23)
    n = 16384 - 8 - 3                       # room for one 8-row block and a few accepted tokens
    for layer in range(cfg.n_layers + 1):
        k, v = synth.kv_fill(cfg, n, 77, layer)
        orc.kv_import(layer, k, v)
        eng.kv_import(layer, k, v)
    feat = synth.feature_row(cfg, 24)
    orc.set_state(n, 3, 4, feat)
    eng.set_state(n, 3, 4, feat)
    d_o = orc.draft(7)
    assert np.array_equal(d_o, eng.draft(7, override_ids=d_o))
    orc.verify(n_rows=8)
    eng.verify(n_rows=8)
    for row in range(8):
        assert np.max(np.abs(orc.logits(row) - eng.logits(row))) <= 2e-2, row
    eng.close()
    with pytest.raises(AdaEagleError) as e:
        Engine(cfg.with_(n_ctx_max=16385), to_device(synth.make_weights(cfg, 23)))
    assert e.value.code == AE_EUNSUPPORTED


def test_generate_until_terminator_matches_autoregressive_oracle():
    """Alg. 1 end to end on the GPU (LDLP-chosen lengths, natural drafts, fp32): generation stops
    right behind the first terminator and equals the oracle's plain greedy decoding up to there."""
    from paper_2412_18910_amd.loop import generate
    eng, orc, _ = make_pair(TINY, 0)
    ids = synth.token_ids(64, TINY.vocab, 100)
    orc.prefill(ids)
    ref = [int(orc.pending)] + [int(t) for t in orc.ar_greedy(90)]
    # a terminator whose first occurrence lies well inside the run (the sequence has repeats)
    j = next(i for i in range(12, len(ref)) if ref[i] not in ref[:i])
    eos, cut = ref[j], j + 1
    eng.prefill(ids)
    toks, cnt = generate(eng, 200, eos_id=eos)
    assert list(toks) == ref[:cut]
    assert cnt.tokens >= cut - 1 and cnt.n_target >= 1
    eng.prefill(ids)
    toks, _ = generate(eng, 33)                      # no terminator: the token budget ends it
    assert list(toks) == ref[:33]
    eng.close()
