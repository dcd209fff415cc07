"""Shapes of the benchmark windows (Llama-3 / Qwen-2.5 public dimensions).

A *layer window* is the run of consecutive decoder layers one device advances
per round (paper Sec. 3.1, Def. 1: window size w_m).  T is the number of tokens
advanced jointly (1 for plain decode, >1 for speculative verification, paper
App. A.12); n_past is n_kv, the number of tokens already in the KV cache
(paper App. A.3, memory-access latency).
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class ModelDims:
    e: int                # hidden size
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rope_theta: float
    rms_eps: float = 1e-5
    rope_mode: int = 0    # 0: pairs (i, i + D/2); 1: pairs (2i, 2i + 1)

    @property
    def qd(self):
        return self.n_q_heads * self.head_dim

    @property
    def kvd(self):
        return self.n_kv_heads * self.head_dim

    def q4k_bytes_per_layer(self):
        """b of App. A.3: bytes of the seven Q4_K matrices of one layer."""
        w = (self.qd * self.e + 2 * self.kvd * self.e + self.e * self.qd
             + 2 * self.ffn * self.e + self.e * self.ffn)
        return w // 256 * 144

    def kv_bytes_per_layer(self, n_kv):
        """2 (h_k e_k + h_v e_v) n_kv of App. A.3 (fp16 K and V)."""
        return 2 * (self.kvd + self.kvd) * n_kv


@dataclass(frozen=True)
class WindowConfig:
    name: str
    config_id: int
    dims: ModelDims
    n_layers: int
    T: int
    n_past: int
    vocab: int = 0        # > 0: final RMSNorm + lm_head after the window

    def with_(self, **kw):
        return replace(self, **kw)

    def bytes_per_step(self):
        """Algorithmic bytes of one window step: sum over layers of
        b + 2 (h_k e_k + h_v e_v) (n_past + T), plus b_o if there is an output layer."""
        d = self.dims
        per_layer = d.q4k_bytes_per_layer() + d.kv_bytes_per_layer(self.n_past + self.T)
        out = self.vocab * d.e // 256 * 144 if self.vocab else 0
        return self.n_layers * per_layer + out


_L8B = ModelDims(4096, 32, 8, 128, 14336, 5e5)
_Q14B = ModelDims(5120, 40, 8, 128, 13824, 1e6)
_Q32B = ModelDims(5120, 40, 8, 128, 27648, 1e6)
_L70B = ModelDims(8192, 64, 8, 128, 28672, 5e5)

CONFIGS = {
    "c0": WindowConfig("c0", 0, _L8B, 1, 1, 512),
    "c1": WindowConfig("c1", 1, _Q14B, 12, 1, 2048),
    "c2": WindowConfig("c2", 2, _Q32B, 16, 4, 4096),
    "c3": WindowConfig("c3", 3, _L70B, 20, 1, 4096),
    "c4k1": WindowConfig("c4k1", 4, _L70B, 80, 1, 8192, vocab=128256),
    "c4k8": WindowConfig("c4k8", 4, _L70B, 80, 8, 8192, vocab=128256),
}

# Small shapes for tests: same structure (GQA groups of 4 / 5 / 8, ragged tails), seconds on a CPU.
TINY = {
    "t0": WindowConfig("t0", 100, ModelDims(512, 4, 2, 64, 768, 1e4), 2, 1, 37),
    "t1": WindowConfig("t1", 101, ModelDims(768, 10, 2, 128, 1280, 1e6), 3, 4, 130),
    "t2": WindowConfig("t2", 102, ModelDims(1024, 8, 1, 128, 1536, 5e5, rope_mode=1), 2, 5, 63),
}
