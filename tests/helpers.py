"""Test-side helpers: build oracle models from the seeded generators."""
import ctypes as C

import numpy as np

from oracle import binding
from paper_2412_18910_amd import synth
from paper_2412_18910_amd.config import Config


def orc_cfg(cfg: Config):
    d = cfg.dict()
    d["wdtype"] = d.pop("dtype")
    return d


def make_oracle(cfg: Config, seed, acc_double=False, weights=None):
    w = weights if weights is not None else synth.make_weights(cfg, seed)
    return binding.OracleModel(orc_cfg(cfg), synth.weights_to_numpy(w), acc_double=acc_double), w


def fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)
