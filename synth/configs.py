"""Shapes of the synthetic draft/target pairs.

The pairs mirror the model pairs of the paper's Experimental Details section
(Vicuna-13B/160M, Vicuna-7B/68M, Llama-8B/1B) by shape only: weights are
seeded random-init, never trained checkpoints.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "bf16"  # "fp32" or "bf16": storage type of weights and KV cache; "q8": projection matrices and LM
                         # head as int8 with one fp32 scale per output row, everything else as for "bf16"

    def n_params(self) -> int:
        per_layer = (
            (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim * self.d_model
            + self.d_model * self.n_q_heads * self.head_dim
            + 3 * self.d_ffn * self.d_model
        )
        return self.n_layers * per_layer + self.vocab * self.d_model

    def weight_bytes(self) -> int:
        """Bytes streamed by one forward pass: every matrix once (embedding rows excluded)."""
        return self.n_params() * {"bf16": 2, "q8": 1}.get(self.dtype, 4)

    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_layers * self.n_kv_heads * self.head_dim * (4 if self.dtype == "fp32" else 2)


@dataclass(frozen=True)
class PairConfig:
    name: str
    target: ModelShape
    draft: ModelShape
    draft_kind: str          # "prefix": draft = first layers of target (+ its embedding/head/final norm);
                             # "projected_head": own weights, LM head = target head times a random projection;
                             # "independent": own weights, shared vocabulary only
    prompt_len: int
    n_generate: int
    gamma_max: int
    batch: int = 1


_T0 = ModelShape(4, 128, 4, 4, 32, 344, 512, 10000.0, 1e-5, "fp32")
_T1 = ModelShape(16, 2048, 32, 8, 64, 8192, 128256, 500000.0, 1e-5, "bf16")
_D1 = ModelShape(2, 768, 12, 12, 64, 3072, 128256, 500000.0, 1e-5, "bf16")
_T2 = ModelShape(32, 4096, 32, 32, 128, 11008, 32000, 10000.0, 1e-5, "bf16")
_D2 = ModelShape(12, 768, 12, 12, 64, 3072, 32000, 10000.0, 1e-5, "bf16")
_T3 = ModelShape(32, 4096, 32, 8, 128, 14336, 128256, 500000.0, 1e-5, "bf16")
_T4 = ModelShape(40, 5120, 40, 40, 128, 13824, 32000, 10000.0, 1e-5, "bf16")

_TS = ModelShape(3, 256, 8, 2, 32, 512, 1024, 500000.0, 1e-5, "bf16")
_DS = ModelShape(2, 128, 4, 4, 32, 256, 1024, 500000.0, 1e-5, "bf16")

_TH = ModelShape(2, 512, 4, 1, 128, 512, 1024, 10000.0, 1e-5, "bf16")
_DH = ModelShape(2, 128, 2, 2, 64, 256, 1024, 10000.0, 1e-5, "bf16")

PAIRS: Dict[str, PairConfig] = {
    # head sizes 128 (target, 4 query heads on 1 kv head) and 64 (draft)
    "small-bf16-hd128": PairConfig("small-bf16-hd128", _TH, _DH, "independent", 80, 64, 16),
    # small bf16 pair with grouped-query attention: exercises the 16-bit kernels at test speed
    "small-bf16": PairConfig("small-bf16", _TS, _DS, "independent", 48, 64, 16),
    # tiny fp32 pair; draft = first two target layers with the tied embedding / head
    "tiny": PairConfig("tiny", _T0, replace(_T0, n_layers=2), "prefix", 32, 64, 8),
    # 1B-shaped target with a 2-layer d=768 draft
    "1b": PairConfig("1b", _T1, _D1, "projected_head", 256, 256, 8),
    # 7B-shaped target with a 12-layer d=768 draft
    "7b": PairConfig("7b", _T2, _D2, "independent", 512, 256, 8),
    # 8B-shaped target with a 1B-shaped draft (headline)
    "8b": PairConfig("8b", _T3, _T1, "independent", 1024, 512, 16),
    # the headline shapes with 8-bit weights (the paper's largest pair runs quantised)
    "8b-q8": PairConfig("8b-q8", replace(_T3, dtype="q8"), replace(_T1, dtype="q8"), "independent", 1024, 512, 16),
    "small-q8": PairConfig("small-q8", replace(_TS, dtype="q8"), replace(_DS, dtype="q8"), "independent", 48, 64, 16),
    "small-q8-hd128": PairConfig("small-q8-hd128", replace(_TH, dtype="q8"), replace(_DH, dtype="q8"), "independent", 80, 64, 16),
    # 13B-shaped target, verify-only sweeps; the draft slot reuses the 160m-shaped model
    "13b": PairConfig("13b", _T4, _D2, "independent", 512, 64, 16),
}


def pair(name: str) -> PairConfig:
    return PAIRS[name]


def shrink(cfg: PairConfig, n_layers_t: int, n_layers_d: int) -> PairConfig:
    """Same widths, fewer layers: for parity runs the CPU oracle can finish."""
    return replace(
        cfg,
        name=f"{cfg.name}-L{n_layers_t}/{n_layers_d}",
        target=replace(cfg.target, n_layers=n_layers_t),
        draft=replace(cfg.draft, n_layers=n_layers_d),
    )
