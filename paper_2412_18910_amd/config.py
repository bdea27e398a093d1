"""Model/step configurations (plain data, no arithmetic of the method)."""
from dataclasses import dataclass, asdict, replace

BF16, FP32 = 0, 1


@dataclass(frozen=True)
class Config:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-6
    dtype: int = BF16            # matrices + KV cache: BF16 or FP32
    k_max: int = 8               # upper clamp of the predicted draft length (Eq. 3)
    n_ctx_max: int = 4096        # KV capacity in tokens
    ldlp_in_mode: int = 0        # 0: [e ; f] (Sec. 3.2)   1: f only
    ldlp_hidden: int = 256
    ldlp_n_res: int = 0
    temperature: float = 0.0     # 0 => greedy
    ddd_enabled: int = 0         # AdaEAGLE-DDD exit rule (Sec. 3.4)
    ddd_threshold: float = -0.6  # log-probability threshold (Sec. 4.3.3)
    ldlp_cls: int = 0            # 1: LDLP classifies over 0..k_max instead of regressing (Sec. 4.3 ablation)

    def dict(self):
        return asdict(self)

    def with_(self, **kw):
        return replace(self, **kw)

    @property
    def d_kv(self):
        return self.n_kv_heads * self.head_dim


# The five workload shapes (random-init stand-ins for the paper's 7B-class models).
TINY = Config(2, 256, 4, 4, 64, 688, 4096, dtype=FP32, k_max=8, n_ctx_max=320, ldlp_hidden=64)
LLAMA_7B = Config(32, 4096, 32, 32, 128, 11008, 32000, k_max=8, n_ctx_max=2048 + 256 + 32, ldlp_hidden=256)
LLAMA_13B = Config(40, 5120, 40, 40, 128, 13824, 32000, k_max=10, n_ctx_max=4096 + 256 + 32, ldlp_hidden=256)
LLAMA_8B_GQA = Config(32, 4096, 32, 8, 128, 14336, 128256, rope_base=500000.0, rms_eps=1e-5, k_max=8,
                      n_ctx_max=8192 + 512 + 32, ldlp_hidden=256, temperature=1.0)

PRESETS = {"tiny": TINY, "7b": LLAMA_7B, "13b": LLAMA_13B, "8b-gqa": LLAMA_8B_GQA}
