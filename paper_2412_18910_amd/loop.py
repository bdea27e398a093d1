"""Host loop over ae_step (Algorithm 1) with the counters of the paper's Table 2."""
import numpy as np


class Counters:
    """N_draft / N_target / N_waste, tokens, tau as defined for Table 2."""

    def __init__(self):
        self.n_draft = self.n_target = self.n_waste = self.tokens = 0
        self.ks, self.accs = [], []

    def add(self, k, n_accepted):
        self.n_draft += k
        self.n_target += 1
        self.n_waste += k - n_accepted
        self.tokens += n_accepted + 1
        self.ks.append(k)
        self.accs.append(n_accepted)

    def summary(self):
        nt = max(self.n_target, 1)
        return {"N_draft": self.n_draft, "N_target": self.n_target, "N_waste": self.n_waste,
                "tokens": self.tokens, "tau": self.tokens / nt, "mean_accepted": float(np.mean(self.accs)) if self.accs else 0.0,
                "mean_k": float(np.mean(self.ks)) if self.ks else 0.0}


def scripted_override(formal, pos, k, n_match, vocab):
    """Override table that makes the first n_match draft tokens equal the formal
    (autoregressive) sequence and the next one differ from it; the draft head still runs
    all its forwards.  formal[pos] is the token the target will emit next."""
    if k == 0:
        return None
    ov = -np.ones(k, np.int32)
    a = min(n_match, k)
    ov[:a] = formal[pos:pos + a]
    if a < k:
        ov[a] = (int(formal[pos + a]) + 1) % vocab
    return ov


def run_scripted(engine, formal, pos, n_steps, script, k_mode="ldlp", k_fixed=4, counters=None, check=True):
    """n_steps iterations of Alg. 1 with scripted acceptance.  Returns (tokens emitted, new pos).
    k_mode: 'ldlp' (Eq. 3), 'fixed', or 'oracle' (k = scripted acceptance length)."""
    vocab = engine.cfg.vocab
    emitted = 0
    for r in range(n_steps):
        if k_mode == "ldlp":
            k, _ = engine.ldlp()
        elif k_mode == "fixed":
            k = k_fixed
        else:
            k = int(script[r])
        ov = scripted_override(formal, pos, k, int(script[r]), vocab)
        kk, na, toks = engine.step(k_force=k, override_ids=ov)
        if check and not np.array_equal(toks, formal[pos:pos + na + 1]):
            raise RuntimeError(f"speculative output left the autoregressive sequence at token {pos}")
        pos += na + 1
        emitted += na + 1
        if counters is not None:
            counters.add(kk, na)
    return emitted, pos


def generate(engine, max_tokens, eos_id=None, u_stream=None):
    """Algorithm 1 as a generation loop: after a prefill, repeat ae_step (LDLP -> draft ->
    verify -> accept) until max_tokens tokens exist or the terminator eos_id was generated;
    the output is cut right behind the terminator (tokens a step validated after it are
    dropped).  Returns (tokens, Counters).  u_stream(step, n) supplies n uniforms for the
    step's draws when the engine runs at temperature > 0 (draft draws first, then accept)."""
    out = [int(engine.pending)]
    cnt = Counters()
    k_max = engine.cfg.k_max
    step = 0
    while len(out) < max_tokens and (eos_id is None or out[-1] != eos_id):
        ud = ua = None
        if u_stream is not None:
            u = np.asarray(u_stream(step, 2 * k_max + 1), np.float64)
            ud, ua = u[:k_max], u[k_max:]
        k, na, toks = engine.step(u_draft=ud, u_accept=ua)
        cnt.add(k, na)
        for t in toks:
            out.append(int(t))
            if len(out) >= max_tokens or (eos_id is not None and int(t) == eos_id):
                break
        step += 1
    return np.array(out, np.int64), cnt
