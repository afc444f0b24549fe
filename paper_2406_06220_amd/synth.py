"""Seeded synthetic Transducer / TDT models and encoder outputs.

This module only draws random numbers and lays them out; it holds none of the
decoding method's arithmetic (no projections, no joint, no argmax), so that the
CPU oracle and the HIP path can both consume exactly the same arrays without
sharing any code of the method itself.

The shapes follow the paper's experimental setting (Sec. 4: 1024-token BPE
vocabularies, encoders with 8x / 4x subsampling, bfloat16) as named by the five
benchmark configurations; trained checkpoints and speech data are replaced by
Gaussian draws:

* encoder outputs   enc[b, t, :] ~ N(0, 1) for every frame, padding included
                    (padding must be ignored by any decoder);
* lengths           uniform integers in [len_lo, len_hi];
* weight matrices   N(0, 1/fan_in); embeddings N(0, 1) with the BOS/blank row
                    zeroed; LSTM, encoder- and predictor-projection biases 0;
* output bias       0 except the blank entry (a constant per configuration,
                    read from ``workload_bias.json``) and the TDT duration
                    entries (+1.5 on durations 1 and 2); the big blanks of a
                    multi-blank model get the blank's bias minus 0.1 per position;
* bf16 configs      ``enc`` and every weight matrix are rounded once, here, to
                    bfloat16-representable values (round to nearest even).

All matrices are stored ``[out_features, in_features]`` row-major.
"""
from __future__ import annotations

import json
import os
from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np

_BIAS_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "workload_bias.json")


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    dtype: str                 # "fp32" | "bf16"
    B: int
    T: int
    len_lo: int
    len_hi: int
    d_enc: int
    pred_kind: str             # "stateless" | "lstm"
    pred_layers: int           # LSTM layers, or stateless context size
    h_pred: int                # predictor output width (stateless: ctx * emb_dim)
    emb_dim: int
    h_joint: int
    vocab: int                 # V real labels; blank index == V
    durations: Tuple[int, ...]  # () for a plain Transducer
    max_symbols: int
    seed: int
    blank_target: float        # blank fraction the blank bias was tuned for
    default_blank_bias: float  # used until workload_bias.json has an entry
    # Multi-blank Transducer: the entries of `durations` are the frame increments of big-blank
    # symbols that sit in the label head behind the blank (outputs V+1 ...), not a duration head
    multi_blank: bool = False

    @property
    def n_dur(self) -> int:
        return len(self.durations)

    @property
    def n_out(self) -> int:
        return self.vocab + 1 + self.n_dur

    @property
    def blank(self) -> int:
        return self.vocab

    def with_batch(self, B: int, name: Optional[str] = None) -> "WorkloadConfig":
        return replace(self, B=B, name=name or f"{self.name}_b{B}")


CONFIGS: Dict[str, WorkloadConfig] = {}


def _register(cfg: WorkloadConfig) -> WorkloadConfig:
    CONFIGS[cfg.name] = cfg
    return cfg


CFG1 = _register(WorkloadConfig(
    name="cfg1_tiny_rnnt", dtype="fp32", B=4, T=50, len_lo=30, len_hi=50, d_enc=64,
    pred_kind="stateless", pred_layers=1, h_pred=64, emb_dim=64, h_joint=64, vocab=32,
    durations=(), max_symbols=5, seed=0, blank_target=0.70, default_blank_bias=2.0))
CFG2 = _register(WorkloadConfig(
    name="cfg2_rnnt_lstm", dtype="bf16", B=32, T=250, len_lo=125, len_hi=250, d_enc=512,
    pred_kind="lstm", pred_layers=1, h_pred=640, emb_dim=640, h_joint=640, vocab=1024,
    durations=(), max_symbols=10, seed=2, blank_target=0.80, default_blank_bias=3.0))
CFG3 = _register(WorkloadConfig(
    name="cfg3_tdt_lstm", dtype="bf16", B=32, T=250, len_lo=125, len_hi=250, d_enc=512,
    pred_kind="lstm", pred_layers=1, h_pred=640, emb_dim=640, h_joint=640, vocab=1024,
    durations=(0, 1, 2, 3, 4), max_symbols=10, seed=3, blank_target=0.80,
    default_blank_bias=3.0))
CFG4 = _register(WorkloadConfig(
    name="cfg4_rnnt_stateless", dtype="bf16", B=128, T=375, len_lo=190, len_hi=375, d_enc=512,
    pred_kind="stateless", pred_layers=2, h_pred=640, emb_dim=320, h_joint=640, vocab=1024,
    durations=(), max_symbols=10, seed=4, blank_target=0.80, default_blank_bias=3.0))
CFG5 = _register(WorkloadConfig(
    name="cfg5_large_tdt", dtype="bf16", B=256, T=1500, len_lo=750, len_hi=1500, d_enc=1024,
    pred_kind="lstm", pred_layers=2, h_pred=640, emb_dim=640, h_joint=1024, vocab=8192,
    durations=(0, 1, 2, 3, 4), max_symbols=10, seed=5, blank_target=0.75,
    default_blank_bias=3.5))
# The metric is also quoted at B=128: the models of configs 2 and 3, larger batch.
CFG2_B128 = _register(CFG2.with_batch(128))
CFG3_B128 = _register(CFG3.with_batch(128))

TDT_DURATION_BIAS = {1: 1.5, 2: 1.5}


# ----------------------------------------------------------------------------
# bfloat16 helpers (number format only)
# ----------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly representable in bfloat16."""
    return bf16_to_f32(bf16_bits(x)).reshape(np.shape(x))


# ----------------------------------------------------------------------------
# constants produced by the oracle-side calibration script
# ----------------------------------------------------------------------------
def _model_key(cfg: WorkloadConfig) -> str:
    # the B=128 variants reuse the weights (and the bias) of their base config
    for base in (CFG1, CFG2, CFG3, CFG4, CFG5):
        if replace(cfg, B=base.B, name=base.name) == base:
            return base.name
    return cfg.name


def blank_bias(cfg: WorkloadConfig) -> float:
    if os.path.exists(_BIAS_FILE):
        with open(_BIAS_FILE) as f:
            table = json.load(f)
        ent = table.get(_model_key(cfg))
        if ent is not None:
            return float(ent["blank_bias"])
    return cfg.default_blank_bias


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------
def generate_model(cfg: WorkloadConfig, blank_bias_override: Optional[float] = None
                   ) -> Dict[str, np.ndarray]:
    """Weights of one model as float32 arrays (bf16-representable for bf16 configs)."""
    rng = np.random.default_rng([cfg.seed, 0])
    q = round_to_bf16 if cfg.dtype == "bf16" else (lambda a: np.asarray(a, np.float32))

    def mat(n_out, n_in):
        return q((rng.standard_normal((n_out, n_in)) / np.sqrt(n_in)).astype(np.float32))

    V, H, Hp, E = cfg.vocab, cfg.h_joint, cfg.h_pred, cfg.emb_dim
    m: Dict[str, np.ndarray] = {}
    m["w_enc"] = mat(H, cfg.d_enc)
    m["b_enc"] = np.zeros(H, np.float32)
    if cfg.pred_kind == "lstm":
        emb = rng.standard_normal((V + 1, E)).astype(np.float32)
        emb[V] = 0.0
        m["emb"] = q(emb)
        in_dim = E
        for l in range(cfg.pred_layers):
            m[f"w_ih{l}"] = mat(4 * Hp, in_dim)
            m[f"w_hh{l}"] = mat(4 * Hp, Hp)
            m[f"b_lstm{l}"] = np.zeros(4 * Hp, np.float32)
            in_dim = Hp
    else:
        assert cfg.h_pred == cfg.pred_layers * E
        emb = rng.standard_normal((cfg.pred_layers, V + 1, E)).astype(np.float32)
        emb[:, V] = 0.0
        m["emb"] = q(emb)
    m["w_pred"] = mat(H, Hp)
    m["b_pred"] = np.zeros(H, np.float32)
    m["w_out"] = mat(cfg.n_out, H)
    b_out = np.zeros(cfg.n_out, np.float32)
    b_out[V] = blank_bias(cfg) if blank_bias_override is None else blank_bias_override
    for j, d in enumerate(cfg.durations):
        # (big blanks compete with the blank: its bias, the longer ones a little lower, which makes
        # every symbol of the head appear in the benchmark-sized and in the small test models)
        b_out[V + 1 + j] = b_out[V] - 0.1 * j if cfg.multi_blank else TDT_DURATION_BIAS.get(d, 0.0)
    m["b_out"] = b_out
    return m


def generate_inputs(cfg: WorkloadConfig) -> Tuple[np.ndarray, np.ndarray]:
    """(enc [B,T,d_enc] float32, enc_len [B] int32); padding frames hold noise too."""
    rng = np.random.default_rng([cfg.seed, 1, cfg.B])
    enc_len = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.B).astype(np.int32)
    enc = rng.standard_normal((cfg.B, cfg.T, cfg.d_enc), dtype=np.float32)
    if cfg.dtype == "bf16":
        enc = round_to_bf16(enc)
    return enc, enc_len


def small_config(name: str = "small", **kw) -> WorkloadConfig:
    """A reduced configuration for unit tests; every field can be overridden."""
    base = dict(name=name, dtype="fp32", B=3, T=12, len_lo=6, len_hi=12, d_enc=8,
                pred_kind="stateless", pred_layers=1, h_pred=8, emb_dim=8, h_joint=8, vocab=5,
                durations=(), max_symbols=3, seed=11, blank_target=0.5, default_blank_bias=1.0)
    base.update(kw)
    return WorkloadConfig(**base)
