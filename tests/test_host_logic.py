"""Host-side logic (no GPU): Table-2 counters, the acceptance script, seeded inputs, and the
byte / flop accounting the benchmark divides by."""
import importlib.util
import os

import numpy as np

from paper_2412_18910_amd import synth
from paper_2412_18910_amd.config import LLAMA_13B, LLAMA_7B, LLAMA_8B_GQA, TINY
from paper_2412_18910_amd.loop import Counters, generate, run_scripted, scripted_override

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _script(name):
    spec = importlib.util.spec_from_file_location(name + "_mod", os.path.join(ROOT, name + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _bench():
    return _script("bench")


def test_counters_follow_the_table2_definitions():
    """Table 2: N_draft = drafted tokens, N_target = target forwards, N_waste = drafted but
    rejected, tau = tokens per target forward (accepted + bonus)."""
    c = Counters()
    for k, acc in ((4, 4), (4, 0), (0, 0), (6, 3)):
        c.add(k, acc)
    s = c.summary()
    assert (s["N_draft"], s["N_target"], s["N_waste"], s["tokens"]) == (14, 4, 7, 11)
    assert s["tau"] == 11 / 4 and s["mean_accepted"] == 7 / 4 and s["mean_k"] == 14 / 4
    assert s["N_draft"] - s["N_waste"] + s["N_target"] == s["tokens"]


def test_scripted_override_matches_then_breaks():
    formal = np.arange(100, 120)
    ov = scripted_override(formal, 3, 5, 2, 1000)
    assert list(ov) == [103, 104, 106, -1, -1]          # 2 matches, a guaranteed mismatch, then free
    assert list(scripted_override(formal, 0, 3, 7, 1000)) == [100, 101, 102]   # script longer than the draft
    assert scripted_override(formal, 0, 0, 3, 1000) is None
    wrap = scripted_override(np.array([9, 9]), 0, 1, 0, 10)
    assert list(wrap) == [0]                             # (9 + 1) mod vocab still differs from 9


def test_truncated_geometric_mean_range_and_determinism():
    a = synth.truncated_geometric(20000, 3.5, 8, 5)
    assert a.min() >= 0 and a.max() <= 8
    assert abs(a.mean() - 3.5) < 0.06
    assert np.array_equal(a, synth.truncated_geometric(20000, 3.5, 8, 5))
    assert not np.array_equal(a, synth.truncated_geometric(20000, 3.5, 8, 6))
    # geometric shape: successive ratios of the bin counts are constant
    cnt = np.bincount(a, minlength=9).astype(float)
    ratios = cnt[1:] / cnt[:-1]
    assert np.max(np.abs(ratios - ratios.mean())) < 0.08


class _FakeEngine:
    """Accepts exactly the scripted prefix (what the target does with override ids)."""

    def __init__(self, formal, vocab):
        self.formal, self.pos = formal, 0

        class _C:
            pass
        self.cfg = _C()
        self.cfg.vocab = vocab
        self.k_seq = iter([3, 0, 8, 5, 2, 7, 1, 4] * 8)

    def ldlp(self):
        return next(self.k_seq), 0.0

    def step(self, k_force=-1, override_ids=None, **_):
        acc = 0
        while acc < k_force and override_ids[acc] == self.formal[self.pos + acc]:
            acc += 1
        toks = self.formal[self.pos:self.pos + acc + 1].copy()
        self.pos += acc + 1
        return k_force, acc, toks


def test_run_scripted_realises_min_of_script_and_k():
    formal = np.arange(7, 7 + 400) % 50
    script = synth.truncated_geometric(40, 3.5, 8, 1)
    eng = _FakeEngine(formal, 50)
    cnt = Counters()
    emitted, pos = run_scripted(eng, formal, 0, 40, script, counters=cnt)
    assert emitted == pos == cnt.tokens
    assert cnt.accs == [min(int(g), k) for g, k in zip(script, cnt.ks)]
    assert cnt.n_waste == sum(k - a for k, a in zip(cnt.ks, cnt.accs))


def test_token_ids_and_kv_fill_are_seeded():
    a, b = synth.token_ids(64, 32000, 11), synth.token_ids(64, 32000, 11)
    assert np.array_equal(a, b) and a.min() >= 0 and a.max() < 32000
    assert not np.array_equal(a, synth.token_ids(64, 32000, 12))
    k1, v1 = synth.kv_fill(TINY, 10, 3, 0)
    k2, v2 = synth.kv_fill(TINY, 10, 3, 0)
    assert np.array_equal(k1, k2) and np.array_equal(v1, v2) and k1.shape == (10, TINY.d_kv)


def test_verify_bytes_match_the_shape_table():
    """Weight and KV bytes of one verify forward: 2 bytes x (L(2 d dq + 2 d dkv + 3 d f) + V d)
    plus 2 x 2 bytes x L n dkv; the figures every GB/s in the benchmark is divided by."""
    b = _bench()
    total, weights = b.verify_bytes(LLAMA_7B, 1024)
    assert abs(weights / 1e9 - 13.214) < 0.001 and abs((total - weights) / 1e9 - 0.537) < 0.001
    total, weights = b.verify_bytes(LLAMA_13B, 4096)
    assert abs(weights / 1e9 - 25.703) < 0.001 and abs((total - weights) / 1e9 - 3.355) < 0.001
    total, weights = b.verify_bytes(LLAMA_8B_GQA, 8192)
    assert abs(weights / 1e9 - 15.009) < 0.001 and abs((total - weights) / 1e9 - 1.074) < 0.001
    assert abs(b.draft_bytes(LLAMA_7B, 0) / 1e9 - 0.734) < 0.001
    # the dominant kernel's bytes: gate and up matrices, bf16
    assert 2 * 2 * LLAMA_7B.d_ffn * LLAMA_7B.d_model == 180355072


def test_prompt_pass_flops():
    """2 x rows x parameters of the GEMMs it runs, plus causal attention (QK^T and PV)."""
    c = LLAMA_7B
    n = 2048
    per_layer = 4 * c.d_model * c.d_model + 3 * c.d_model * c.d_ffn
    draft = 2 * c.d_model * c.d_model + 3 * c.d_model * c.d_model      # fc [d, 2d] + fused q, k, v
    attn = 4 * c.n_layers * c.d_model * n * (n + 1) // 2
    model_flops = _script("prefill_bench").model_flops
    assert model_flops(c, n) == 2 * n * (c.n_layers * per_layer + draft) + attn
    assert 26e12 < model_flops(c, n) < 29e12


class _ScriptedEngine:
    """Emits a fixed token sequence in steps of varying size, like an engine after prefill."""

    def __init__(self, seq, sizes):
        self.seq, self.sizes, self.pos, self.i = list(seq), sizes, 1, 0
        self.pending = seq[0]

        class _C:
            k_max = 8
        self.cfg = _C()

    def step(self, u_draft=None, u_accept=None):
        n = self.sizes[self.i % len(self.sizes)]
        self.i += 1
        toks = np.array(self.seq[self.pos:self.pos + n], np.int32)
        self.pos += n
        return n + 1, n - 1, toks


def test_generate_stops_at_the_terminator_or_the_budget():
    """Alg. 1 runs until a terminator is generated; the output ends right behind it even when the
    step that produced it validated more tokens."""
    seq = list(range(100, 160))
    toks, cnt = generate(_ScriptedEngine(seq, [3, 1, 4]), 20)
    assert list(toks) == seq[:20]
    toks, cnt = generate(_ScriptedEngine(seq, [3, 1, 4]), 50, eos_id=106)     # 106 sits mid-step
    assert list(toks) == seq[:7] and toks[-1] == 106 and cnt.n_target == 3
    toks, _ = generate(_ScriptedEngine(seq, [3, 1, 4]), 50, eos_id=100)       # the first token already ends it
    assert list(toks) == [100]
    toks, _ = generate(_ScriptedEngine(seq, [2]), 9, eos_id=999)              # never generated: the budget ends it
    assert list(toks) == seq[:9]
