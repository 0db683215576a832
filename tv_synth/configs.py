"""The five benchmark configurations (shapes only).

Model family follows the paper's evaluation setup (1-6 layer encoders, 4 heads,
embedding 128; sentence lengths up to 128 as in its dataset table); the larger
shapes extend it.  Values that a configuration leaves open (search steps,
vocabulary, class count) take the defaults documented next to each field.
"""
from dataclasses import dataclass, replace

ACT_RELU, ACT_TANH, ACT_GELU, ACT_LEAKY_RELU, ACT_SILU = 0, 1, 2, 3, 4
NORM_L1, NORM_L2, NORM_LINF = 1, 2, 0   # p of the perturbation ball; 0 encodes infinity


@dataclass(frozen=True)
class EncoderConfig:
    n_layers: int
    hidden: int        # D = embedding size E
    n_heads: int
    ffn: int
    activation: int    # ACT_*
    vocab: int = 1000
    max_len: int = 128
    n_classes: int = 2
    ln_eps: float = 1e-5
    act_alpha: float = 0.01   # slope of the leaky ReLU on x < 0 (read by that activation only)


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    enc: EncoderConfig
    seq_len: int
    n_perturbed: int
    p_norms: tuple      # which balls the configuration runs
    batch: int
    steps: int          # binary-search steps
    eps_lo: float = 0.0
    eps_hi: float = 1.0
    weight_std: float = 0.02


CONFIGS = {
    "c1": Workload("c1", 1, EncoderConfig(1, 64, 4, 128, ACT_RELU), 8, 1, (NORM_L2,), 4, 10),
    "c2": Workload("c2", 2, EncoderConfig(2, 128, 4, 256, ACT_RELU), 32, 1,
                   (NORM_L1, NORM_L2, NORM_LINF), 32, 10),
    "c3": Workload("c3", 3, EncoderConfig(3, 256, 8, 512, ACT_TANH), 32, 2, (NORM_LINF,), 64, 16),
    "c4": Workload("c4", 4, EncoderConfig(6, 512, 8, 2048, ACT_RELU), 64, 1, (NORM_L2,), 64, 10),
    "c5": Workload("c5", 5, EncoderConfig(12, 768, 12, 3072, ACT_GELU), 128, 2, (NORM_LINF,), 16, 10),
}


def get_workload(name: str) -> Workload:
    return CONFIGS[name]


def scaled(w: Workload, **kw) -> Workload:
    """A variant of a workload; encoder fields and workload fields may both be overridden."""
    enc_fields = {k: v for k, v in kw.items() if k in EncoderConfig.__dataclass_fields__}
    wl_fields = {k: v for k, v in kw.items() if k in Workload.__dataclass_fields__}
    unknown = set(kw) - set(enc_fields) - set(wl_fields)
    if unknown:
        raise KeyError(f"unknown fields {sorted(unknown)}")
    return replace(w, enc=replace(w.enc, **enc_fields), **wl_fields)
