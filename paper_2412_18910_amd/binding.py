"""Thin ctypes binding of libadaeagle.so: argument marshalling only.

Every step of the decode path runs inside the library's HIP kernels; PyTorch is used
by callers only to own device memory (weights) and streams.  Importing this module
does not need a GPU; creating an Engine does, and raises if the library is missing.
"""
import ctypes as C
import os

import numpy as np

from .config import Config

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadaeagle.so")

AE_OK, AE_EINVAL, AE_ESTATE, AE_ENOMEM, AE_EHIP, AE_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
_CODES = {AE_EINVAL: "AE_EINVAL", AE_ESTATE: "AE_ESTATE", AE_ENOMEM: "AE_ENOMEM", AE_EHIP: "AE_EHIP",
          AE_EUNSUPPORTED: "AE_EUNSUPPORTED"}

EXPORTS = ("ae_init", "ae_free", "ae_last_error", "ae_prefill", "ae_kv_import", "ae_set_state", "ae_ldlp",
           "ae_draft", "ae_verify", "ae_accept", "ae_step", "ae_kv_len", "ae_pending", "ae_get_logits",
           "ae_get_feature", "ae_get_draft_logits", "ae_get_kv_row", "ae_set_profiling", "ae_get_phase_times",
           "ae_set_kernel_timing", "ae_get_kernel_timing", "ae_last_draft_len", "ae_get_draft_logprob", "ae_set_prefill_mode", "ae_version",
           "ae_kv_import_static", "ae_ldlp_loss", "ae_set_ddd_mode", "ae_set_temperature", "ae_probe_read_stream")


class AeConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + [
        ("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32), ("k_max", C.c_int32),
        ("n_ctx_max", C.c_int32), ("ldlp_in_mode", C.c_int32), ("ldlp_hidden", C.c_int32),
        ("ldlp_n_res", C.c_int32), ("temperature", C.c_float), ("ddd_enabled", C.c_int32),
        ("ddd_threshold", C.c_float), ("ldlp_cls", C.c_int32)]


class AeLayerW(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class AeWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(AeLayerW)), ("draft_layer", AeLayerW),
                ("draft_fc_w", C.c_void_p), ("draft_fc_b", C.c_void_p),
                ("ldlp_w_in", C.c_void_p), ("ldlp_b_in", C.c_void_p), ("ldlp_w_res", C.c_void_p),
                ("ldlp_b_res", C.c_void_p), ("ldlp_w_out", C.c_void_p), ("ldlp_b_out", C.c_void_p)]


class AeStepIO(C.Structure):
    _fields_ = [("k_force", C.c_int32), ("override_ids", C.POINTER(C.c_int32)), ("u_draft", C.POINTER(C.c_double)),
                ("u_accept", C.POINTER(C.c_double)), ("k", C.c_int32), ("n_accepted", C.c_int32),
                ("n_tokens", C.c_int32), ("tokens", C.c_int32 * 16), ("us_total", C.c_float)]


class AePhaseTimes(C.Structure):
    _fields_ = [("us_ldlp", C.c_float), ("us_draft", C.c_float), ("us_verify", C.c_float), ("us_accept", C.c_float)]


class AdaEagleError(RuntimeError):
    def __init__(self, code, what, msg):
        super().__init__(f"{what}: {_CODES.get(code, code)}: {msg}")
        self.code = code


_lib = None


def load_library(path=LIB_PATH):
    """dlopen the HIP library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2412_18910_amd.build` "
                           "(hipcc, gfx950); there is no fallback path")
    lib = C.CDLL(path)
    P, I = C.c_void_p, C.c_int
    i32p, f32p, f64p = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_double)
    sig = {
        "ae_init": (I, [C.POINTER(AeConfig), C.POINTER(AeWeights), P, C.POINTER(P)]),
        "ae_free": (None, [P]),
        "ae_last_error": (C.c_char_p, [P]),
        "ae_prefill": (I, [P, i32p, I]),
        "ae_kv_import": (I, [P, I, f32p, f32p, I]),
        "ae_kv_import_static": (I, [P, I, f32p, f32p, I]),
        "ae_ldlp_loss": (I, [P, f32p, i32p, I, C.c_double, f64p]),
        "ae_set_state": (I, [P, I, C.c_int32, C.c_int32, f32p]),
        "ae_ldlp": (I, [P, C.POINTER(I), f32p]),
        "ae_draft": (I, [P, I, i32p, f64p, i32p]),
        "ae_verify": (I, [P, i32p, I]),
        "ae_accept": (I, [P, f64p, C.POINTER(I), i32p]),
        "ae_step": (I, [P, C.POINTER(AeStepIO)]),
        "ae_kv_len": (I, [P]),
        "ae_last_draft_len": (I, [P]),
        "ae_get_draft_logprob": (I, [P, f32p]),
        "ae_pending": (C.c_int32, [P]),
        "ae_get_logits": (I, [P, I, f32p]),
        "ae_get_feature": (I, [P, I, f32p]),
        "ae_get_draft_logits": (I, [P, I, f32p]),
        "ae_get_kv_row": (I, [P, I, I, I, f32p]),
        "ae_set_profiling": (I, [P, I]),
        "ae_get_phase_times": (I, [P, C.POINTER(AePhaseTimes)]),
        "ae_set_kernel_timing": (I, [P, I]),
        "ae_set_prefill_mode": (I, [P, I, I]),
        "ae_set_ddd_mode": (I, [P, I]),
        "ae_set_temperature": (I, [P, C.c_float]),
        "ae_get_kernel_timing": (I, [P, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
        "ae_version": (C.c_char_p, []),
        "ae_probe_read_stream": (I, [P, C.c_size_t, I, I, f64p]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def probe_read_stream(bytes_per_launch, launches=64, repeats=5, stream=None):
    """Microseconds per launch of a dependent chain of read-only streaming kernels (diagnostic)."""
    lib = load_library()
    us = C.c_double()
    rc = lib.ae_probe_read_stream(stream.cuda_stream if stream is not None else None, int(bytes_per_launch), launches,
                                  repeats, C.byref(us))
    if rc != AE_OK:
        raise AdaEagleError(rc, "ae_probe_read_stream", "probe failed")
    return us.value


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


_LAYER_KEYS = [n for n, _ in AeLayerW._fields_]


class Engine:
    """One sequence on the GPU.  `weights` is the dict layout of synth.make_weights holding
    torch tensors on the target device (matrices in cfg.dtype, vectors float32)."""

    def __init__(self, cfg: Config, weights, stream=None):
        import torch
        self.lib = load_library()
        self.cfg = cfg
        self._weights = weights  # keep the device memory alive
        self.c = AeConfig(**cfg.dict())
        mdt = torch.bfloat16 if cfg.dtype == 0 else torch.float32

        def ptr(t, dt):
            if t is None:
                return None
            if not t.is_cuda or t.dtype != dt or not t.is_contiguous():
                raise TypeError(f"weight must be a contiguous {dt} device tensor, got {t.dtype} on {t.device}")
            return t.data_ptr()

        def layer(d):
            return AeLayerW(**{k: ptr(d[k], torch.float32 if k.endswith("norm") else mdt) for k in _LAYER_KEYS})

        self._layers = (AeLayerW * cfg.n_layers)(*[layer(d) for d in weights["layers"]])
        w = AeWeights()
        w.tok_emb, w.final_norm, w.lm_head = ptr(weights["tok_emb"], mdt), ptr(weights["final_norm"], torch.float32), ptr(weights["lm_head"], mdt)
        w.layers = C.cast(self._layers, C.POINTER(AeLayerW))
        w.draft_layer = layer(weights["draft_layer"])
        w.draft_fc_w, w.draft_fc_b = ptr(weights["draft_fc_w"], mdt), ptr(weights.get("draft_fc_b"), torch.float32)
        w.ldlp_w_in, w.ldlp_b_in = ptr(weights["ldlp_w_in"], mdt), ptr(weights["ldlp_b_in"], torch.float32)
        w.ldlp_w_res, w.ldlp_b_res = ptr(weights.get("ldlp_w_res"), mdt), ptr(weights.get("ldlp_b_res"), torch.float32)
        w.ldlp_w_out, w.ldlp_b_out = ptr(weights["ldlp_w_out"], torch.float32), ptr(weights["ldlp_b_out"], torch.float32)
        self._w = w
        self.stream = stream
        h = C.c_void_p()
        rc = self.lib.ae_init(C.byref(self.c), C.byref(w), stream.cuda_stream if stream is not None else None, C.byref(h))
        if rc != AE_OK:
            raise AdaEagleError(rc, "ae_init", self.lib.ae_last_error(None).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.ae_free(self.h)
            self.h = None

    __del__ = close

    def _chk(self, rc, what):
        if rc != AE_OK:
            raise AdaEagleError(rc, what, self.lib.ae_last_error(self.h).decode())

    def prefill(self, ids):
        ids = _i32(ids)
        self._chk(self.lib.ae_prefill(self.h, _p(ids, C.c_int32), len(ids)), "ae_prefill")

    def kv_import(self, layer, k, v):
        k, v = _f32(k), _f32(v)
        self._chk(self.lib.ae_kv_import(self.h, layer, _p(k, C.c_float), _p(v, C.c_float), k.shape[0]), "ae_kv_import")

    def kv_import_static(self, layer, k, v):
        k, v = _f32(k), _f32(v)
        self._chk(self.lib.ae_kv_import_static(self.h, layer, _p(k, C.c_float), _p(v, C.c_float), k.shape[0]),
                  "ae_kv_import_static")

    def set_state(self, kv_len, last_tok, pending, feat):
        feat = _f32(feat)
        self._chk(self.lib.ae_set_state(self.h, kv_len, last_tok, pending, _p(feat, C.c_float)), "ae_set_state")

    def ldlp(self):
        k, y = C.c_int(), C.c_float()
        self._chk(self.lib.ae_ldlp(self.h, C.byref(k), C.byref(y)), "ae_ldlp")
        return k.value, y.value

    def ldlp_loss(self, pred, truth, lam):
        pred, truth = _f32(pred), _i32(truth)
        out = C.c_double()
        self._chk(self.lib.ae_ldlp_loss(self.h, _p(pred, C.c_float), _p(truth, C.c_int32), len(pred), float(lam),
                                        C.byref(out)), "ae_ldlp_loss")
        return out.value

    def draft(self, k, override_ids=None, u_draft=None, want_ids=True):
        out = np.zeros(self.cfg.k_max + 1, np.int32)
        ov, ud = _i32(override_ids), _f64(u_draft)
        self._chk(self.lib.ae_draft(self.h, k, _p(ov, C.c_int32), _p(ud, C.c_double),
                                    _p(out, C.c_int32) if want_ids else None), "ae_draft")
        return out[:self.lib.ae_last_draft_len(self.h)]

    @property
    def draft_logprob(self):
        v = C.c_float()
        self._chk(self.lib.ae_get_draft_logprob(self.h, C.byref(v)), "ae_get_draft_logprob")
        return v.value

    def verify(self, block_ids=None, n_rows=None):
        b = _i32(block_ids)
        n = len(b) if b is not None else n_rows
        self._chk(self.lib.ae_verify(self.h, _p(b, C.c_int32), n), "ae_verify")

    def accept(self, u=None):
        u = _f64(u)
        na, bonus = C.c_int(), C.c_int32()
        self._chk(self.lib.ae_accept(self.h, _p(u, C.c_double), C.byref(na), C.byref(bonus)), "ae_accept")
        return na.value, bonus.value

    def step(self, k_force=-1, override_ids=None, u_draft=None, u_accept=None):
        ov, ud, ua = _i32(override_ids), _f64(u_draft), _f64(u_accept)
        io = AeStepIO()
        io.k_force = k_force
        io.override_ids, io.u_draft, io.u_accept = _p(ov, C.c_int32), _p(ud, C.c_double), _p(ua, C.c_double)
        self._chk(self.lib.ae_step(self.h, C.byref(io)), "ae_step")
        self.last_us = io.us_total
        return io.k, io.n_accepted, np.array(io.tokens[:io.n_tokens], np.int32)

    @property
    def kv_len(self):
        return self.lib.ae_kv_len(self.h)

    @property
    def pending(self):
        return self.lib.ae_pending(self.h)

    def _get(self, fn, what, n, *args):
        out = np.zeros(n, np.float32)
        self._chk(fn(self.h, *args, _p(out, C.c_float)), what)
        return out

    def logits(self, row):
        return self._get(self.lib.ae_get_logits, "ae_get_logits", self.cfg.vocab, row)

    def feature(self, row):
        return self._get(self.lib.ae_get_feature, "ae_get_feature", self.cfg.d_model, row)

    def draft_logits(self, i):
        return self._get(self.lib.ae_get_draft_logits, "ae_get_draft_logits", self.cfg.vocab, i)

    def kv_row(self, layer, which, slot):
        return self._get(self.lib.ae_get_kv_row, "ae_get_kv_row", self.cfg.d_kv, layer, which, slot)

    def set_profiling(self, on=True):
        self._chk(self.lib.ae_set_profiling(self.h, int(on)), "ae_set_profiling")

    PREFILL_AUTO, PREFILL_BLOCKS, PREFILL_DENSE = 0, 1, 2

    def set_prefill_mode(self, mode, chunk_rows=0):
        self._chk(self.lib.ae_set_prefill_mode(self.h, int(mode), int(chunk_rows)), "ae_set_prefill_mode")

    DDD_HOST, DDD_DEVICE = 0, 1

    def set_ddd_mode(self, mode):
        self._chk(self.lib.ae_set_ddd_mode(self.h, int(mode)), "ae_set_ddd_mode")

    def set_temperature(self, temperature):
        self._chk(self.lib.ae_set_temperature(self.h, float(temperature)), "ae_set_temperature")
        self.cfg = self.cfg.with_(temperature=float(temperature))

    def set_kernel_timing(self, on=True):
        self._chk(self.lib.ae_set_kernel_timing(self.h, int(on)), "ae_set_kernel_timing")

    def kernel_timing(self):
        """(total microseconds, launches) of the gate/up GEMM since timing was enabled."""
        t, n = C.c_double(), C.c_int64()
        self._chk(self.lib.ae_get_kernel_timing(self.h, C.byref(t), C.byref(n)), "ae_get_kernel_timing")
        return t.value, n.value

    def phase_times(self):
        t = AePhaseTimes()
        self._chk(self.lib.ae_get_phase_times(self.h, C.byref(t)), "ae_get_phase_times")
        return {"ldlp": t.us_ldlp, "draft": t.us_draft, "verify": t.us_verify, "accept": t.us_accept}
