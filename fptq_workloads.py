"""Seeded synthetic inputs for the W4A4 linear layer: shapes and value distributions of the
five benchmark configurations.  This module only draws inputs (activations, integer weights,
scales) and belongs to neither the HIP library's package nor the CPU checker: the tests and the
benchmark feed both from it, and neither of the two imports it.  The one statistic it computes,
the calibration constant s_a, is an input like the others (a float64 NumPy absmax over a separate
draw), not a step of the layer.

Activations are returned as bf16 bit patterns (uint16), weights as int8 in [-8, 7] (one value
per element, [N, K] = [out, in]), weight scales as float32 [N].  The static activation scale
s_a is a calibration constant: max |x~| / 7 over a separate 512-token draw of the same layer
(same outlier channels), where x~ is the tensor fed to the quantizer (row-scaled if the case
uses a row scale).
"""
import zlib
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

MODE_NONE, MODE_RMS, MODE_GIVEN = 0, 1, 2
EPS = 1e-5
CALIB_TOKENS = 512


@dataclass(frozen=True)
class LinearCase:
    config: str          # "c1" .. "c5"
    name: str            # layer name inside the config
    M: int
    N: int
    K: int
    dist: str            # "normal" | "student_t3"
    outlier_frac: float  # fraction of input channels scaled up (0 for none)
    outlier_count: int   # explicit count (overrides frac when > 0)
    outlier_mult: float
    mode: int            # row-scale mode fed to the quantizer
    seed: int
    self_calibrated: bool = False   # c1: s_a from the tensor itself
    eps: float = EPS

    @property
    def ops(self):
        return 2 * self.M * self.N * self.K

    @property
    def key(self):
        return f"{self.config}.{self.name}.M{self.M}"


def f32_to_bf16_bits(a):
    """Round float32 to bf16 (nearest even) and return the bit patterns as uint16.  Worked through in blocks of a
    million values so that the temporaries stay in cache (the big configurations convert hundreds of millions)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).reshape(-1)
    out = np.empty(u.shape[0], np.uint16)
    step = 1 << 20
    for i in range(0, u.shape[0], step):
        c = u[i:i + step]
        r = c >> np.uint32(16)
        r &= np.uint32(1)            # the bit that decides a tie
        r += np.uint32(0x7FFF)
        r += c
        r >>= np.uint32(16)
        out[i:i + step] = r
    return out.reshape(a.shape)


def bf16_bits_to_f32(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _n_outliers(case):
    if case.outlier_count > 0:
        return case.outlier_count
    return int(round(case.outlier_frac * case.K))


def _draw_x(rng, rows, case, channels):
    if case.dist == "normal":
        x = rng.standard_normal((rows, case.K), dtype=np.float32)
    elif case.dist == "student_t3":
        x = rng.standard_t(3.0, size=(rows, case.K)).astype(np.float32)
    else:
        raise ValueError(case.dist)
    if len(channels):
        x[:, channels] *= np.float32(case.outlier_mult)
    return f32_to_bf16_bits(x)


def _draw_given_scale(rng, rows):
    # per-token scale of a residual-like stream: log-normal spread around 1
    return np.exp(0.5 * rng.standard_normal(rows)).astype(np.float32)


def _quantizer_input_absmax(x_bits, mode, r, eps):
    x = bf16_bits_to_f32(x_bits).astype(np.float64)
    if mode == MODE_RMS:
        x = x / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + eps)
    elif mode == MODE_GIVEN:
        x = x * r.astype(np.float64)[:, None]
    return float(np.abs(x).max())


@dataclass
class LinearInputs:
    case: LinearCase
    x_bits: np.ndarray                 # uint16 [M, K]
    w_int: Optional[np.ndarray]        # int8 [N, K] (None when weights were not requested)
    s_w: Optional[np.ndarray]          # float32 [N]
    s_a: np.float32
    row_scale_in: Optional[np.ndarray] # float32 [M] for MODE_GIVEN
    channels: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))


def draw_weights(case, rng=None):
    if rng is None:   # the layer name enters the seed: gate and up share X but not W
        rng = np.random.default_rng([case.seed, zlib.crc32(case.name.encode())])
    w = rng.integers(-8, 8, size=(case.N, case.K), dtype=np.int8)
    s_w = rng.uniform(0.005, 0.02, size=case.N).astype(np.float32)
    return w, s_w


def draw(case: LinearCase, with_weights=True, M=None) -> LinearInputs:
    """All inputs of one linear-layer case.  M overrides the token count (e.g. a ragged test)."""
    rows = case.M if M is None else M
    rng = np.random.default_rng(case.seed)
    n_out = _n_outliers(case)
    channels = np.sort(rng.choice(case.K, n_out, replace=False)) if n_out else np.zeros(0, np.int64)
    x_bits = _draw_x(rng, rows, case, channels)
    r_in = _draw_given_scale(rng, rows) if case.mode == MODE_GIVEN else None
    if case.self_calibrated:
        amax = _quantizer_input_absmax(x_bits, case.mode, r_in, case.eps)
    else:
        crng = np.random.default_rng(case.seed + 1000)
        xc = _draw_x(crng, CALIB_TOKENS, case, channels)
        rc = _draw_given_scale(crng, CALIB_TOKENS) if case.mode == MODE_GIVEN else None
        amax = _quantizer_input_absmax(xc, case.mode, rc, case.eps)
    s_a = np.float32(amax / 7.0)
    w, s_w = draw_weights(case) if with_weights else (None, None)
    return LinearInputs(case, x_bits, w, s_w, s_a, r_in, channels)


def uniform_int4(rows, K, seed):
    """Uniform random int4 values as int8 [rows, K] (the dense-activation timing variant)."""
    return np.random.default_rng(seed).integers(-8, 8, size=(rows, K), dtype=np.int8)


def _case(config, name, M, N, K, dist, frac, mult, mode, seed, count=0, self_cal=False):
    return LinearCase(config, name, M, N, K, dist, frac, count, mult, mode, seed, self_cal)


def config_cases(config: str):
    """The linear layers of one benchmark configuration, in call order."""
    if config == "c1":   # tiny correctness case, literal absmax/7 over its own X
        return [_case("c1", "tiny_none", 128, 512, 512, "normal", 0, 20.0, MODE_NONE, 0, count=4, self_cal=True),
                _case("c1", "tiny_rms", 128, 512, 512, "normal", 0, 20.0, MODE_RMS, 0, count=4, self_cal=True)]
    if config == "c2":   # Llama-2-7B MLP, prefill 2048 tokens
        return [_case("c2", "gate", 2048, 11008, 4096, "normal", 0.01, 30.0, MODE_RMS, 1),
                _case("c2", "up", 2048, 11008, 4096, "normal", 0.01, 30.0, MODE_RMS, 1),
                _case("c2", "down", 2048, 4096, 11008, "normal", 0.01, 30.0, MODE_GIVEN, 11)]
    if config == "c3":   # Llama-3-8B decoder layer, prefill 4096 tokens, heavy-tailed activations
        return [_case("c3", "qkv", 4096, 6144, 4096, "student_t3", 0, 1.0, MODE_RMS, 2),
                _case("c3", "o", 4096, 4096, 4096, "student_t3", 0, 1.0, MODE_GIVEN, 12),
                _case("c3", "gate_up", 4096, 28672, 4096, "student_t3", 0, 1.0, MODE_RMS, 22),
                _case("c3", "down", 4096, 4096, 14336, "student_t3", 0, 1.0, MODE_GIVEN, 32)]
    if config == "c4":   # Llama-3-8B decode, 1 / 8 / 32 tokens
        out = []
        for M in (1, 8, 32):
            out += [_case("c4", "qkv", M, 6144, 4096, "normal", 0, 1.0, MODE_RMS, 3),
                    _case("c4", "o", M, 4096, 4096, "normal", 0, 1.0, MODE_GIVEN, 13),
                    _case("c4", "gate_up", M, 28672, 4096, "normal", 0, 1.0, MODE_RMS, 23),
                    _case("c4", "down", M, 4096, 14336, "normal", 0, 1.0, MODE_GIVEN, 33)]
        return out
    if config == "c5":   # Llama-3-70B layer, prefill 8192 tokens
        return [_case("c5", "qkv", 8192, 10240, 8192, "normal", 0.005, 50.0, MODE_RMS, 4),
                _case("c5", "o", 8192, 8192, 8192, "normal", 0.005, 50.0, MODE_GIVEN, 14),
                _case("c5", "gate_up", 8192, 57344, 8192, "normal", 0.005, 50.0, MODE_RMS, 24),
                _case("c5", "down", 8192, 8192, 28672, "normal", 0.005, 50.0, MODE_GIVEN, 34)]
    raise KeyError(config)


ALL_CONFIGS = ("c1", "c2", "c3", "c4", "c5")
