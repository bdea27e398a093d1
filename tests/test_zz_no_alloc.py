"""ae_kv_import_static (the entry point that allocates nothing) against ae_kv_import, through
the C ABI: cache rows bit for bit, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from paper_2412_18910_amd import synth
from paper_2412_18910_amd.binding import AE_EINVAL, AdaEagleError, Engine
from paper_2412_18910_amd.config import BF16, Config, TINY

from .gpu_helpers import to_device

pytestmark = pytest.mark.gpu

MED_BF16 = Config(4, 1024, 8, 8, 128, 2816, 8192, dtype=BF16, k_max=8, n_ctx_max=1024, ldlp_hidden=128)
STAGE_FLOATS = 2 * 1024 * 1024


def _rows(eng, cfg, layer, slots):
    return [eng.kv_row(layer, which, s).tobytes() for which in (0, 1) for s in slots]


@pytest.mark.parametrize("cfg", [MED_BF16, TINY], ids=["bf16-tiled", "fp32"])
def test_static_import_equals_allocating_import_twice_in_a_row(cfg):
    w = to_device(synth.make_weights(cfg, 3))
    ref, sta = Engine(cfg, w), Engine(cfg, w)
    n1, n2 = 300, 37                                    # 300 rows span tiles and a ragged tail; then fewer rows
    assert 2 * n1 * cfg.d_kv <= STAGE_FLOATS
    rng = np.random.default_rng(5)
    for layer in (0, cfg.n_layers):                       # a target layer and the draft head's cache
        k1, v1 = synth.kv_fill(cfg, n1, 9, layer)
        ref.kv_import(layer, k1, v1)
        sta.kv_import_static(layer, k1, v1)
        slots = [0, 1, 15, 16, 31, 32, 255, 256, n1 - 1]
        assert _rows(sta, cfg, layer, slots) == _rows(ref, cfg, layer, slots)
        # second call, smaller input, values that need rounding in the bf16 cache
        k2 = rng.standard_normal((n2, cfg.d_kv)).astype(np.float32)
        v2 = rng.standard_normal((n2, cfg.d_kv)).astype(np.float32)
        ref.kv_import(layer, k2, v2)
        sta.kv_import_static(layer, k2, v2)
        slots = [0, 15, 16, n2 - 1, n2, 255, n1 - 1]     # rows >= n2 keep the first call's values
        got, want = _rows(sta, cfg, layer, slots), _rows(ref, cfg, layer, slots)
        assert got == want
        assert np.array_equal(np.frombuffer(got[3], np.float32) != 0, np.ones(cfg.d_kv, bool))
    # an engine fed through the static import decodes like one fed through the allocating import
    feat = synth.feature_row(cfg, 4)
    for layer in range(cfg.n_layers + 1):
        k, v = synth.kv_fill(cfg, 100, 21, layer)
        ref.kv_import(layer, k, v)
        sta.kv_import_static(layer, k, v)
    ref.set_state(100, 3, 4, feat)
    sta.set_state(100, 3, 4, feat)
    ta, tb = ref.step(k_force=4), sta.step(k_force=4)
    assert ta[:2] == tb[:2] and np.array_equal(ta[2], tb[2])
    assert np.array_equal(ref.logits(0), sta.logits(0))
    ref.close()
    sta.close()


def test_static_import_rejects_what_does_not_fit():
    cfg = MED_BF16
    eng = Engine(cfg, to_device(synth.make_weights(cfg, 3)))
    n_fit = STAGE_FLOATS // (2 * cfg.d_kv)                # 1024 rows of 1024 floats
    assert n_fit == cfg.n_ctx_max
    big = cfg.with_(n_ctx_max=2048)
    eng2 = Engine(big, to_device(synth.make_weights(big, 3)))
    z = np.zeros((n_fit + 1, cfg.d_kv), np.float32)
    with pytest.raises(AdaEagleError) as e:
        eng2.kv_import_static(0, z, z)
    assert e.value.code == AE_EINVAL and "staging" in str(e.value)
    eng2.kv_import_static(0, z[:n_fit], z[:n_fit])       # exactly the limit
    with pytest.raises(AdaEagleError) as e:
        eng.kv_import_static(cfg.n_layers + 1, z[:4], z[:4])
    assert e.value.code == AE_EINVAL
    eng.kv_import_static(0, z[:0], z[:0])                 # empty input: nothing to do
    eng.close()
    eng2.close()
