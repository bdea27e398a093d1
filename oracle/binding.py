"""ctypes binding of the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Loaded by tests, the smoke check and the CPU-baseline leg of the benchmark; the
product path never imports this module.  It takes plain dicts and numpy arrays
(bf16 matrices as uint16 bit patterns) and imports nothing from the HIP package.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
BF16, FP32 = 0, 1


class OrcConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + [
        ("rope_base", C.c_float), ("rms_eps", C.c_float), ("wdtype", C.c_int32),
        ("k_max", C.c_int32), ("n_ctx_max", C.c_int32), ("ldlp_in_mode", C.c_int32),
        ("ldlp_hidden", C.c_int32), ("ldlp_n_res", C.c_int32), ("temperature", C.c_float),
        ("ddd_enabled", C.c_int32), ("ddd_threshold", C.c_float), ("ldlp_cls", C.c_int32)]


class OrcLayer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class OrcWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(OrcLayer)), ("draft_layer", OrcLayer),
                ("draft_fc_w", C.c_void_p), ("draft_fc_b", C.c_void_p),
                ("ldlp_w_in", C.c_void_p), ("ldlp_b_in", C.c_void_p), ("ldlp_w_res", C.c_void_p),
                ("ldlp_b_res", C.c_void_p), ("ldlp_w_out", C.c_void_p), ("ldlp_b_out", C.c_void_p)]


_LAYER_KEYS = [n for n, _ in OrcLayer._fields_]


def build(force=False):
    """Compile the oracle libraries with gcc (make) if they are missing."""
    if force or not all(os.path.exists(os.path.join(_HERE, n)) for n in ("liboracle.so", "liboracle_f64.so")):
        subprocess.check_call(["make", "-C", _HERE, "-B" if force else "-s"])


_libs = {}


def load(acc_double=False):
    name = "liboracle_f64.so" if acc_double else "liboracle.so"
    if name in _libs:
        return _libs[name]
    build()
    lib = C.CDLL(os.path.join(_HERE, name))
    P, I, F, D = C.c_void_p, C.c_int, C.c_float, C.c_double
    i32p, f32p, f64p = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_double)
    sig = {
        "orc_create": (P, [C.POINTER(OrcConfig), C.POINTER(OrcWeights)]),
        "orc_destroy": (None, [P]),
        "orc_prefill": (I, [P, i32p, I]),
        "orc_kv_import": (I, [P, I, f32p, f32p, I]),
        "orc_set_state": (I, [P, I, C.c_int32, C.c_int32, f32p]),
        "orc_ldlp": (I, [P, C.POINTER(I), f32p]),
        "orc_draft": (I, [P, I, i32p, f64p, i32p]),
        "orc_verify": (I, [P, i32p, I]),
        "orc_accept": (I, [P, f64p, C.POINTER(I), i32p]),
        "orc_step": (I, [P, I, i32p, f64p, f64p, C.POINTER(I), C.POINTER(I), i32p]),
        "orc_ar_greedy": (I, [P, I, i32p]),
        "orc_kv_len": (I, [P]),
        "orc_last_draft_len": (I, [P]),
        "orc_draft_logprob": (D, [P]),
        "orc_pending": (C.c_int32, [P]),
        "orc_logits": (f32p, [P, I]),
        "orc_feature": (f32p, [P, I]),
        "orc_draft_logits": (f32p, [P, I]),
        "orc_kv_row": (f32p, [P, I, I, I]),
        "orc_rmsnorm": (None, [f32p, f32p, I, F, f32p]),
        "orc_rope": (None, [f32p, I, I, I, F]),
        "orc_attention_row": (None, [f32p, f32p, f32p, I, I, I, I, I, f32p]),
        "orc_round_clamp": (I, [F, I]),
        "orc_bf16_round": (F, [F]),
        "orc_argmax": (I, [f32p, I]),
        "orc_accept_sample": (I, [f32p, f32p, I, I, i32p, D, f64p, C.POINTER(I), i32p]),
        "orc_accept_greedy": (I, [f32p, I, I, i32p, C.POINTER(I), i32p]),
        "orc_sample_inverse_cdf": (C.c_int32, [f64p, I, D]),
        "orc_ldlp_loss": (D, [f32p, i32p, I, D]),
    }
    for name_, (res, args) in sig.items():
        fn = getattr(lib, name_)
        fn.restype, fn.argtypes = res, args
    _libs[name] = lib
    return lib


def _ptr(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


class OracleError(RuntimeError):
    pass


class OracleModel:
    """One sequence on the CPU oracle.

    cfg: dict with the OrcConfig fields (wdtype BF16/FP32).
    weights: dict -- matrices as numpy uint16 (bf16 bits) or float32, vectors float32:
      tok_emb, final_norm, lm_head, layers=[{attn_norm,wq,wk,wv,wo,ffn_norm,w_gate,w_up,w_down}],
      draft_layer={...}, draft_fc_w, draft_fc_b, ldlp_w_in, ldlp_b_in, ldlp_w_res, ldlp_b_res,
      ldlp_w_out, ldlp_b_out.
    """

    def __init__(self, cfg, weights, acc_double=False):
        self.lib = load(acc_double)
        self.cfg = dict(cfg)
        self.c = OrcConfig(**{k: self.cfg[k] for k, _ in OrcConfig._fields_})
        self._keep = []
        mat_dt = np.uint16 if self.c.wdtype == BF16 else np.float32

        def mat(a):
            if a is None:
                return None
            a = np.ascontiguousarray(a)
            if a.dtype != mat_dt:
                raise TypeError(f"matrix dtype {a.dtype}, expected {mat_dt}")
            self._keep.append(a)
            return a.ctypes.data

        def vec(a):
            if a is None:
                return None
            a = _f32(a)
            self._keep.append(a)
            return a.ctypes.data

        def layer(d):
            kw = {}
            for key in _LAYER_KEYS:
                kw[key] = vec(d[key]) if key.endswith("norm") else mat(d[key])
            return OrcLayer(**kw)

        L = self.c.n_layers
        self._layers = (OrcLayer * L)(*[layer(d) for d in weights["layers"]])
        w = OrcWeights()
        w.tok_emb, w.final_norm, w.lm_head = mat(weights["tok_emb"]), vec(weights["final_norm"]), mat(weights["lm_head"])
        w.layers = C.cast(self._layers, C.POINTER(OrcLayer))
        w.draft_layer = layer(weights["draft_layer"])
        w.draft_fc_w, w.draft_fc_b = mat(weights["draft_fc_w"]), vec(weights.get("draft_fc_b"))
        w.ldlp_w_in, w.ldlp_b_in = mat(weights["ldlp_w_in"]), vec(weights["ldlp_b_in"])
        w.ldlp_w_res, w.ldlp_b_res = mat(weights.get("ldlp_w_res")), vec(weights.get("ldlp_b_res"))
        w.ldlp_w_out, w.ldlp_b_out = vec(weights["ldlp_w_out"]), vec(weights["ldlp_b_out"])
        self.w = w
        self.h = self.lib.orc_create(C.byref(self.c), C.byref(w))
        if not self.h:
            raise OracleError("orc_create rejected the configuration")

    def close(self):
        if getattr(self, "h", None):
            self.lib.orc_destroy(self.h)
            self.h = None

    __del__ = close

    def _chk(self, rc, what):
        if rc != 0:
            raise OracleError(f"{what} failed with code {rc}")

    def prefill(self, ids):
        ids = _i32(ids)
        self._chk(self.lib.orc_prefill(self.h, _ptr(ids, C.c_int32), len(ids)), "orc_prefill")

    def kv_import(self, layer, k, v):
        k, v = _f32(k), _f32(v)
        self._chk(self.lib.orc_kv_import(self.h, layer, _ptr(k, C.c_float), _ptr(v, C.c_float), k.shape[0]), "orc_kv_import")

    def set_state(self, kv_len, last_tok, pending, feat):
        feat = _f32(feat)
        self._chk(self.lib.orc_set_state(self.h, kv_len, last_tok, pending, _ptr(feat, C.c_float)), "orc_set_state")

    def ldlp(self):
        k, y = C.c_int(), C.c_float()
        self._chk(self.lib.orc_ldlp(self.h, C.byref(k), C.byref(y)), "orc_ldlp")
        return k.value, y.value

    def draft(self, k, override_ids=None, u_draft=None):
        out = np.zeros(self.c.k_max + 1, np.int32)
        ov, ud = _i32(override_ids), _f64(u_draft)
        self._chk(self.lib.orc_draft(self.h, k, _ptr(ov, C.c_int32), _ptr(ud, C.c_double), _ptr(out, C.c_int32)), "orc_draft")
        return out[:self.lib.orc_last_draft_len(self.h)]

    @property
    def draft_logprob(self):
        return self.lib.orc_draft_logprob(self.h)

    def verify(self, block_ids=None, n_rows=None):
        b = _i32(block_ids)
        n = len(b) if b is not None else n_rows
        self._chk(self.lib.orc_verify(self.h, _ptr(b, C.c_int32), n), "orc_verify")

    def accept(self, u=None):
        u = _f64(u)
        na, bonus = C.c_int(), C.c_int32()
        self._chk(self.lib.orc_accept(self.h, _ptr(u, C.c_double), C.byref(na), C.byref(bonus)), "orc_accept")
        return na.value, bonus.value

    def step(self, k_force=-1, override_ids=None, u_draft=None, u_accept=None):
        ov, ud, ua = _i32(override_ids), _f64(u_draft), _f64(u_accept)
        k, na = C.c_int(), C.c_int()
        toks = np.zeros(self.c.k_max + 1, np.int32)
        self._chk(self.lib.orc_step(self.h, k_force, _ptr(ov, C.c_int32), _ptr(ud, C.c_double), _ptr(ua, C.c_double),
                                    C.byref(k), C.byref(na), _ptr(toks, C.c_int32)), "orc_step")
        return k.value, na.value, toks[:na.value + 1].copy()

    def ar_greedy(self, n):
        out = np.zeros(n, np.int32)
        self._chk(self.lib.orc_ar_greedy(self.h, n, _ptr(out, C.c_int32)), "orc_ar_greedy")
        return out

    @property
    def kv_len(self):
        return self.lib.orc_kv_len(self.h)

    @property
    def pending(self):
        return self.lib.orc_pending(self.h)

    def logits(self, row):
        return np.ctypeslib.as_array(self.lib.orc_logits(self.h, row), (self.c.vocab,)).copy()

    def feature(self, row):
        return np.ctypeslib.as_array(self.lib.orc_feature(self.h, row), (self.c.d_model,)).copy()

    def draft_logits(self, i):
        return np.ctypeslib.as_array(self.lib.orc_draft_logits(self.h, i), (self.c.vocab,)).copy()

    def kv_row(self, layer, which, slot):
        n = self.c.n_kv_heads * self.c.head_dim
        return np.ctypeslib.as_array(self.lib.orc_kv_row(self.h, layer, which, slot), (n,)).copy()
