"""Pins for the decode loop: losslessness, counters, LDLP (Alg. 1, Eq. 1-3, Table 2)."""
import os

import numpy as np
import pytest
import torch

from paper_2412_18910_amd import synth
from paper_2412_18910_amd.config import TINY

from .helpers import make_oracle

PROMPT, NGEN = 64, 128   # the tiny lossless configuration: 64 prompt ids, 128 generated tokens


@pytest.fixture(scope="module")
def ar_reference():
    m, w = make_oracle(TINY, 0)
    ids = synth.token_ids(PROMPT, TINY.vocab, 100)
    m.prefill(ids)
    first = m.pending
    return ids, w, first, m.ar_greedy(NGEN)


def _run_spec(w, ids, n_gen, k_of_step, script=None, formal=None):
    """Loop of Alg. 1 on the oracle.  script[r] = number of leading draft tokens forced to
    equal the formal sequence (the next one is forced to mismatch); None = natural draft."""
    m, _ = make_oracle(TINY, 0, weights=w)
    m.prefill(ids)
    out, stats = [], dict(N_draft=0, N_target=0, N_waste=0, steps=[])
    r = 0
    while len(out) < n_gen:
        k = k_of_step(r, m)
        ov = None
        if script is not None and k > 0:
            a = min(int(script[r]), k)
            ov = -np.ones(k, np.int32)
            pos = len(out)
            ov[:a] = formal[pos:pos + a]
            if a < k:
                ov[a] = (int(formal[pos + a]) + 1) % TINY.vocab
        kk, na, toks = m.step(k_force=k, override_ids=ov)
        assert kk == k and len(toks) == na + 1
        out.extend(int(t) for t in toks)
        stats["N_draft"] += k
        stats["N_target"] += 1
        stats["N_waste"] += k - na
        stats["steps"].append((k, na))
        r += 1
    return np.array(out[:n_gen], np.int32), stats, len(out)


def test_greedy_speculative_equals_autoregressive_natural_draft(ar_reference):
    ids, w, _, ar = ar_reference
    out, st, _ = _run_spec(w, ids, NGEN, lambda r, m: m.ldlp()[0])
    assert np.array_equal(out, ar)
    ks = {k for k, _ in st["steps"]}
    assert len(ks) > 2, "LDLP of the synthetic weights should spread over several lengths"


def test_greedy_speculative_equals_autoregressive_scripted_acceptance(ar_reference):
    ids, w, _, ar = ar_reference
    formal = np.concatenate([ar, ar[:32]])  # padding so slices past the end stay defined
    script = synth.truncated_geometric(4 * NGEN, 3.5, TINY.k_max, 7)
    out, st, total = _run_spec(w, ids, NGEN, lambda r, m: m.ldlp()[0], script, formal)
    assert np.array_equal(out, ar)
    # forced prefix => accepted length is at least the script (the forced mismatch stops it
    # unless k was shorter than the script)
    for (k, na), a in zip(st["steps"], script):
        assert na == min(int(a), k)
    assert total == st["N_draft"] - st["N_waste"] + st["N_target"]


@pytest.mark.parametrize("sched", ["zeros", "kmax", "cycle"])
def test_greedy_lossless_under_adversarial_lengths(ar_reference, sched):
    ids, w, _, ar = ar_reference
    f = {"zeros": lambda r, m: 0, "kmax": lambda r, m: TINY.k_max, "cycle": lambda r, m: r % (TINY.k_max + 1)}[sched]
    out, st, total = _run_spec(w, ids, 48, f)
    assert np.array_equal(out, ar[:48])
    if sched == "zeros":  # k = 0 is a plain autoregressive step: one token per target forward
        assert st["N_target"] == 48 and st["N_draft"] == 0


def test_counter_identities_fixed_and_oracle_lengths(ar_reference):
    ids, w, _, ar = ar_reference
    formal = np.concatenate([ar, ar[:32]])
    script = synth.truncated_geometric(4 * NGEN, 3.5, TINY.k_max, 8)
    # fixed length k: N_draft = k * N_target (Table 2, EAGLE rows)
    for k in (2, 5):
        out, st, total = _run_spec(w, ids, 64, lambda r, m: k, script, formal)
        assert st["N_draft"] == k * st["N_target"]
        assert st["N_waste"] == sum(kk - na for kk, na in st["steps"])
        assert total == sum(na + 1 for _, na in st["steps"])
    # draft-length oracle: k = the scripted acceptance length => nothing wasted (Sec. 2.4)
    out, st, total = _run_spec(w, ids, 64, lambda r, m: int(script[r]), script, formal)
    assert st["N_waste"] == 0
    assert np.array_equal(out, ar[:64])


def test_table2_rows_obey_the_counter_definitions():
    path = os.path.join(os.path.dirname(__file__), "golden", "table2_counts.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 7
    for name, tau, toks, nd, nt, nw in rows:
        nd, nt, nw = int(nd), int(nt), int(nw)
        if name.isdigit():
            assert nd == int(name) * nt          # fixed length: k drafts per target forward
        if name == "dyn_oracle":
            assert nw == 0
        # tokens per target forward = accepted drafts + 1 bonus; tau is its per-sample average,
        # so the pooled ratio only has to be close
        assert abs((nd - nw + nt) / nt - float(tau)) < 0.12


def test_ldlp_closed_forms():
    cfg = TINY
    w = synth.make_weights(cfg, 0)
    ids = synth.token_ids(8, cfg.vocab, 5)
    # zero input layer => z = b_in, y = sum w_out silu(b_in) + b_out
    w0 = dict(w)
    w0["ldlp_w_in"] = torch.zeros_like(w["ldlp_w_in"])
    w0["ldlp_b_in"] = torch.full_like(w["ldlp_b_in"], 0.75)
    m, _ = make_oracle(cfg, 0, weights=w0)
    m.prefill(ids)
    k, y = m.ldlp()
    s = 0.75 / (1 + np.exp(-0.75))
    want = float(w["ldlp_w_out"].double().sum() * s + w["ldlp_b_out"].double()[0])
    assert abs(y - want) < 1e-4 * max(1, abs(want))
    assert k == min(cfg.k_max, max(0, int(np.rint(want))))


@pytest.mark.parametrize("mode,n_res", [(0, 0), (1, 0), (0, 2)])
def test_ldlp_matches_library_expression(mode, n_res):
    cfg = TINY.with_(ldlp_in_mode=mode, ldlp_n_res=n_res)
    m, w = make_oracle(cfg, 9)
    ids = synth.token_ids(10, cfg.vocab, 6)
    m.prefill(ids)
    k, y = m.ldlp()
    f = torch.from_numpy(m.feature((10 - 1) % (cfg.k_max + 1))).double()   # last prompt row (prefill runs in k_max+1 row chunks)
    e = w["tok_emb"].double()[int(ids[-1])]               # embedding of the SAME token, not the bonus
    u = torch.cat([e, f]) if mode == 0 else f
    z = torch.nn.functional.linear(u, w["ldlp_w_in"].double(), w["ldlp_b_in"].double())
    for r in range(n_res):
        z = z + torch.nn.functional.silu(torch.nn.functional.linear(z, w["ldlp_w_res"][r].double(), w["ldlp_b_res"][r].double()))
    want = float(torch.nn.functional.silu(z) @ w["ldlp_w_out"].double() + w["ldlp_b_out"].double()[0])
    assert abs(y - want) < 1e-4
    assert k == int(min(cfg.k_max, max(0, np.rint(want))))


def test_ldlp_uses_feature_of_last_accepted_row(ar_reference):
    """After a step with k° accepted, Eq. 3 reads row k° of the verify block (Sec. 3.2)."""
    ids, w, _, ar = ar_reference
    m, _ = make_oracle(TINY, 0, weights=w)
    m.prefill(ids)
    ov = np.array([ar[0], ar[1], (int(ar[2]) + 1) % TINY.vocab, -1], np.int32)
    k, na, toks = m.step(k_force=4, override_ids=ov)
    assert na == 2 and list(toks) == [ar[0], ar[1], ar[2]]
    f_row2 = m.feature(2)
    _, y = m.ldlp()
    e = w["tok_emb"].double()[int(ar[1])]                 # last validated token, not the bonus ar[2]
    u = torch.cat([e, torch.from_numpy(f_row2).double()])
    z = torch.nn.functional.linear(u, w["ldlp_w_in"].double(), w["ldlp_b_in"].double())
    want = float(torch.nn.functional.silu(z) @ w["ldlp_w_out"].double() + w["ldlp_b_out"].double()[0])
    assert abs(y - want) < 1e-4


def test_state_errors():
    from oracle.binding import OracleError
    m, _ = make_oracle(TINY, 0)
    with pytest.raises(OracleError):
        m.ldlp()                      # nothing prefetched yet
    m.prefill(synth.token_ids(4, TINY.vocab, 1))
    with pytest.raises(OracleError):
        m.verify(n_rows=1)            # no draft to verify
    with pytest.raises(OracleError):
        m.draft(TINY.k_max + 1)
    with pytest.raises(OracleError):
        m.verify([TINY.vocab])        # id out of range


# ---------------------------------------------------------------- AdaEAGLE-DDD exit rule (Sec. 3.4, 4.2)

def _ddd_model(theta, w=None, seed=0):
    cfg = TINY.with_(ddd_enabled=1, ddd_threshold=theta)
    m, w = make_oracle(cfg, seed, weights=w)
    m.prefill(synth.token_ids(24, cfg.vocab, 300))
    return cfg, m, w


def test_ddd_sequence_logprob_matches_library_log_softmax():
    cfg, m, w = _ddd_model(-1e9)            # threshold never reached: always drafts k_max tokens
    ids = m.draft(2)
    assert len(ids) == cfg.k_max
    want = 0.0
    for i, t in enumerate(ids):
        lp = torch.log_softmax(torch.from_numpy(m.draft_logits(i)).double(), -1)
        want += float(lp[int(t)])
        assert int(t) == int(lp.argmax())   # greedy draft token
    assert abs(m.draft_logprob - want) < 1e-6


def test_ddd_keeps_the_longer_of_the_two_lengths():
    # reference lengths from an unconstrained run: cumulative log-probabilities c_1 > c_2 > ...
    cfg, m, w = _ddd_model(-1e9)
    ids = m.draft(0)
    cums = np.cumsum([float(torch.log_softmax(torch.from_numpy(m.draft_logits(i)).double(), -1)[int(t)])
                      for i, t in enumerate(ids)])
    assert np.all(np.diff(cums) < 0)
    # threshold between c_3 and c_4: the rule stops before token s iff s > k and c_{s-1} < theta,
    # so the DDD length is 4 (c_3 >= theta lets token 4 through, c_4 < theta stops token 5)
    theta = 0.5 * (cums[2] + cums[3])
    for k, want in [(0, 4), (2, 4), (4, 4), (6, 6), (cfg.k_max, cfg.k_max)]:
        _, m2, _ = _ddd_model(theta, w)
        got = m2.draft(k)
        assert len(got) == want, (k, len(got))
        assert np.array_equal(got, ids[:want])
        assert abs(m2.draft_logprob - cums[want - 1]) < 1e-6
    # a threshold above 0 can never be met by a log-probability: only the predicted length remains,
    # except that the empty sequence (log-probability 0) is compared too
    _, m3, _ = _ddd_model(1e-3, w)
    assert len(m3.draft(3)) == 3
    _, m4, _ = _ddd_model(1e-3, w)
    assert len(m4.draft(0)) == 0
    _, m5, _ = _ddd_model(-1e-9, w)          # empty sequence passes (0 >= theta): at least one token
    assert len(m5.draft(0)) == 1


def test_ddd_equality_with_the_threshold_continues():
    """Sec. 4.1: the AdaEAGLE-DDD exit needs the sequence probability to be LOWER than the threshold.
    With a one-token vocabulary every draft sequence has probability exactly 1 (log 0): at
    threshold 0 nothing is lower, the draft runs to k_max; any threshold above 0 ends it at k."""
    cfg = TINY.with_(vocab=1, ddd_enabled=1, ddd_threshold=0.0)
    m, w = make_oracle(cfg, 0)
    m.prefill(np.zeros(8, np.int32))
    assert len(m.draft(2)) == cfg.k_max and m.draft_logprob == 0.0
    m2, _ = make_oracle(cfg.with_(ddd_threshold=1e-6), 0, weights=w)
    m2.prefill(np.zeros(8, np.int32))
    assert len(m2.draft(2)) == 2


def test_sampled_and_overridden_draft_tokens_and_their_logprob():
    """The draft token at temperature T is the inverse-CDF draw from softmax(logits / T) with the
    caller's uniform, and the DDD statistic is the log-probability of the tokens actually chained
    (drawn or overridden) under that same law -- not of the most likely ones."""
    T = 0.7
    cfg = TINY.with_(temperature=T, ddd_enabled=1, ddd_threshold=-1e9)
    m, w = make_oracle(cfg, 0)
    ids = synth.token_ids(24, cfg.vocab, 300)
    m.prefill(ids)
    u = np.random.default_rng(5).random(cfg.k_max)
    got = m.draft(2, u_draft=u)
    assert len(got) == cfg.k_max
    want_lp, n_off_mode = 0.0, 0
    for i, t in enumerate(got):
        z = m.draft_logits(i).astype(np.float64) / T
        p = np.exp(z - z.max())
        c = np.cumsum(p)
        assert int(t) == int(np.searchsorted(c, u[i] * c[-1], side="right"))
        want_lp += z[int(t)] - z.max() - np.log(c[-1])
        n_off_mode += int(t) != int(z.argmax())
    assert n_off_mode >= 1                       # the draws really left the mode
    assert abs(m.draft_logprob - want_lp) < 1e-6
    # greedy head, tokens forced by the caller: their log-probability, not the mode's
    cfg0 = TINY.with_(ddd_enabled=1, ddd_threshold=-1e9)
    m0, _ = make_oracle(cfg0, 0, weights=w)
    m0.prefill(ids)
    forced = np.array([7, 7, 1900, 3, -1, -1, 42, 0], np.int32)[:cfg.k_max]
    got0 = m0.draft(0, override_ids=forced)
    want0 = 0.0
    for i, t in enumerate(got0):
        lp = torch.log_softmax(torch.from_numpy(m0.draft_logits(i)).double(), -1)
        assert int(t) == (int(forced[i]) if forced[i] >= 0 else int(lp.argmax()))
        want0 += float(lp[int(t)])
    assert abs(m0.draft_logprob - want0) < 1e-6


def test_ddd_run_stays_lossless(ar_reference):
    ids, w, _, ar = ar_reference
    cfg = TINY.with_(ddd_enabled=1, ddd_threshold=-8.0)
    m, _ = make_oracle(cfg, 0, weights=w)
    m.prefill(ids)
    out, ks = [], []
    while len(out) < 64:
        k, na, toks = m.step()
        out.extend(int(t) for t in toks)
        ks.append(k)
    assert np.array_equal(np.array(out[:64]), ar[:64])
    assert max(ks) >= 1


# ---- LDLP variants of the Sec. 4.3 ablation: classification head; the Sec. 3.3 criterion ----

def test_ldlp_classification_matches_library_expression_and_picks_the_best_class():
    cfg = TINY.with_(ldlp_cls=1, ldlp_n_res=1)
    m, w = make_oracle(cfg, 12)
    ids = synth.token_ids(10, cfg.vocab, 6)
    m.prefill(ids)
    k, y = m.ldlp()
    f = torch.from_numpy(m.feature((10 - 1) % (cfg.k_max + 1))).double()
    e = w["tok_emb"].double()[int(ids[-1])]
    z = torch.nn.functional.linear(torch.cat([e, f]), w["ldlp_w_in"].double(), w["ldlp_b_in"].double())
    z = z + torch.nn.functional.silu(torch.nn.functional.linear(z, w["ldlp_w_res"][0].double(), w["ldlp_b_res"][0].double()))
    scores = torch.nn.functional.linear(torch.nn.functional.silu(z), w["ldlp_w_out"].double(), w["ldlp_b_out"].double())
    assert scores.shape == (cfg.k_max + 1,)
    assert k == int(torch.argmax(scores)) and abs(y - float(scores.max())) < 1e-4


def test_ldlp_classification_closed_form_and_ties():
    """Zero input layer: silu(z) is a constant vector, so class c scores s * sum(w_out[c]) + b_out[c];
    with equal rows the bias alone decides and the lowest length wins a tie."""
    cfg = TINY.with_(ldlp_cls=1)
    w = dict(synth.make_weights(cfg, 0))
    w["ldlp_w_in"] = torch.zeros_like(w["ldlp_w_in"])
    w["ldlp_b_in"] = torch.full_like(w["ldlp_b_in"], 0.5)
    w["ldlp_w_out"] = torch.ones_like(w["ldlp_w_out"])
    ids = synth.token_ids(8, cfg.vocab, 5)
    s = 0.5 / (1 + np.exp(-0.5)) * cfg.ldlp_hidden
    for bias, want_k in (([0, 0, 0, 0, 0, 3, 0, 0, 0], 5), ([1, 0, 0, 2, 0, 2, 0, 0, 1], 3), ([0] * 9, 0),
                         ([0, 0, 0, 0, 0, 0, 0, 1, 2], 8)):   # k_max itself is a class
        w["ldlp_b_out"] = torch.tensor(bias, dtype=torch.float32)
        m, _ = make_oracle(cfg, 0, weights=w)
        m.prefill(ids)
        k, y = m.ldlp()
        assert k == want_k and abs(y - (s + max(bias))) < 1e-3


def test_ldlp_classification_drives_the_loop_losslessly(ar_reference):
    """Same target and draft weights as the regression runs (the LDLP output layer is drawn
    last), lengths now chosen by the classifier: the output is still the greedy sequence."""
    ids, _, first, ar = ar_reference
    cfg = TINY.with_(ldlp_cls=1)
    m, _ = make_oracle(cfg, 0)
    m.prefill(ids)
    assert m.pending == first
    out, ks = [], []
    while len(out) < 64:
        k, na, toks = m.step()
        ks.append(k)
        out.extend(int(t) for t in toks)
    assert out[:64] == [int(t) for t in ar[:64]]
    assert len(set(ks)) >= 2 and 0 <= min(ks) and max(ks) <= cfg.k_max


def test_ldlp_loss_criterion():
    """Sec. 3.3: |pred - truth|, times lambda when the prediction is too short."""
    from oracle import binding as ob
    from .helpers import f32, fp, ip
    lib = ob.load()
    pred = f32([3.0, 1.0, 5.0, 2.5, 0.0])
    truth = np.array([3, 4, 2, 3, 0], np.int32)
    # per pair: 0, 3*lam (short by 3), 3 (long by 3), 0.5*lam, 0
    for lam in (1.0, 2.0, 3.5):
        want = (0 + 3 * lam + 3 + 0.5 * lam + 0) / 5
        assert abs(lib.orc_ldlp_loss(fp(pred), ip(truth), 5, lam) - want) < 1e-12
    assert lib.orc_ldlp_loss(fp(pred), ip(truth), 0, 2.0) == 0.0
    # lambda = 1 is plain L1; the penalty only ever raises the loss, and only on short predictions
    rng = np.random.default_rng(0)
    p, t = f32(rng.uniform(0, 8, 1000)), rng.integers(0, 9, 1000).astype(np.int32)
    l1 = float(np.mean(np.abs(p.astype(np.float64) - t)))
    assert abs(lib.orc_ldlp_loss(fp(p), ip(t), 1000, 1.0) - l1) < 1e-12
    short = float(np.mean(np.clip(t - p.astype(np.float64), 0, None)))
    assert abs(lib.orc_ldlp_loss(fp(p), ip(t), 1000, 3.0) - (l1 + 2.0 * short)) < 1e-12
