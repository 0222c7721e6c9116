"""Workload descriptions: model shapes and decoding hyper-parameters.

The five named workloads are synthetic stand-ins for the shapes the paper decodes with
(LLaDA-8B and Dream-7B class models, generation length 256, few-shot prompts of a few
hundred to about a thousand tokens; Sec. 5.1 and App. E.3).  Only shapes are taken; the
weights are random (see gen.py).
"""
from dataclasses import dataclass, field, replace
from typing import List, Tuple


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    qkv_bias: bool = False
    w_std: float = 0.02
    lm_std: float = 0.0          # 0 -> 8/sqrt(d_model): logit std about 8 at every width

    @property
    def mask_id(self) -> int:
        return self.vocab - 1

    @property
    def lm_head_std(self) -> float:
        return self.lm_std if self.lm_std > 0 else 8.0 / (self.d_model ** 0.5)


@dataclass(frozen=True)
class DecodeParams:
    tau_dec: float = 0.9         # Eq. 1 threshold (>=)
    tau_merge: float = 0.5       # Alg. 2 merge threshold (>)
    tau_sync: int = 8            # Alg. 2 sync gap (>)
    refresh_interval: int = 8    # R: block forwards between full-sequence refreshes
    leader_rule: int = 0         # 0: most tokens decoded (Alg. 2); 1: highest mean confidence
    eos_id: int = -1             # end-of-sequence token of CheckEOS (Alg. 1); -1: no EOS handling


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelShape
    decode: DecodeParams
    gen_len: int
    block_sizes: Tuple[int, ...]
    prompt_lens: Tuple[int, ...]          # one entry per concurrent request
    seed: int = 0

    @property
    def n_requests(self) -> int:
        return len(self.prompt_lens)


TINY = ModelShape("tiny", 2, 256, 4, 4, 64, 688, 1024, lm_std=0.5)
LLADA = ModelShape("llada8b", 32, 4096, 32, 32, 128, 12288, 126464)
DREAM = ModelShape("dream7b", 28, 3584, 28, 4, 128, 18944, 152064, qkv_bias=True)

WORKLOAD_NAMES = ("tiny", "llada", "dream", "llada_x16", "llada_long")
# further settings run through the same path: the paper's main six-branch setting (App. E.3) and the
# single-branch special cases that stand for its baselines (one block size with a KV cache; no cache)
EXTRA_WORKLOAD_NAMES = ("llada_paper6", "llada_b32", "llada_vanilla")


def workload(name: str) -> Workload:
    """Return a named workload (prompt lengths of llada_x16 come from gen.py)."""
    if name == "tiny":
        return Workload("tiny", TINY, DecodeParams(refresh_interval=4, leader_rule=1), 64, (8, 16, 32), (64,))
    if name == "llada":
        return Workload("llada", LLADA, DecodeParams(refresh_interval=8), 256, (8, 16, 32, 64), (512,))
    if name == "dream":
        return Workload("dream", DREAM, DecodeParams(refresh_interval=8), 512, (16, 32, 64), (1024,))
    if name == "llada_x16":
        from .gen import gen_prompt_lengths
        lens = tuple(gen_prompt_lengths(0, 16, 256, 1024))
        return Workload("llada_x16", LLADA, DecodeParams(refresh_interval=8), 256, (8, 16, 32, 64), lens)
    if name == "llada_long":
        return Workload("llada_long", LLADA, DecodeParams(refresh_interval=16), 1024, (16, 32, 64, 128), (4096,))
    if name == "llada_paper6":      # six branches 4..128, tau_sync 8, R 32, tau_merge 0.5: 252 packed rows per step
        return Workload("llada_paper6", LLADA, DecodeParams(refresh_interval=32), 256, (4, 8, 16, 32, 64, 128), (512,))
    if name == "llada_b32":         # one branch, block 32, cached KV refreshed every 8 forwards
        return Workload("llada_b32", LLADA, DecodeParams(refresh_interval=8), 256, (32,), (512,))
    if name == "llada_vanilla":     # one block = the whole generation, refresh after every forward, one token per step
        return Workload("llada_vanilla", LLADA, DecodeParams(tau_dec=1.5, refresh_interval=1), 256, (256,), (512,))
    raise KeyError(name)


def scaled(model: ModelShape, **kw) -> ModelShape:
    """A copy of a model shape with some fields replaced (reduced-depth test variants)."""
    return replace(model, **kw)
