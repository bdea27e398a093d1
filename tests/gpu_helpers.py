"""GPU-side test helpers: engines fed the same bytes as the oracle."""
import numpy as np

from paper_2412_18910_amd import synth
from paper_2412_18910_amd.binding import Engine

from .helpers import make_oracle


def to_device(w, dev="cuda:0"):
    def conv(v):
        if isinstance(v, dict):
            return {k: conv(x) for k, x in v.items()}
        if isinstance(v, list):
            return [conv(x) for x in v]
        return None if v is None else v.to(dev).contiguous()
    return conv(w)


def make_pair(cfg, seed):
    """(engine, oracle) built from identical weight bytes."""
    w = synth.make_weights(cfg, seed)
    orc, _ = make_oracle(cfg, seed, weights=w)
    eng = Engine(cfg, to_device(w))
    return eng, orc, w


def top2_margin(logits):
    p = np.partition(logits, -2)
    return float(p[-1] - p[-2])
