"""Seeded synthetic layer problems (inputs only; none of the pruning method's arithmetic).

The paper prunes BERT-base/large and GPT-2 layers with calibration activations taken from
SQuAD / GLUE / OpenWebText samples (Section 4 "Setup", Appendix H).  Those models and data are
not available here; these generators stand in for them with the same shapes (hidden 768/1024,
intermediate 3072/4096, 64-column heads, 128- or 1024-token sequences) and a plausible value
structure: post-GELU inputs for the second feed-forward matrix, per-channel-scaled Gaussians
for the attention output projection.

Every tensor is produced on the host in fp32 from a counter-based Philox stream, so the fp64
CPU oracle (which promotes the fp32 values) and the GPU library see bit-identical inputs.
seed = 1000*config + 10*layer + {0: X, 1: W, 2: channel scales}.
"""
from dataclasses import dataclass

import numpy as np
from scipy.special import erf


@dataclass(frozen=True)
class LayerSpec:
    name: str
    config: int
    layer: int
    d_row: int
    d_col: int
    group_size: int
    n_tok: int
    x_kind: str          # "normal" | "gelu" | "scaled_normal"
    w_std: float
    damp_rel: float = 0.01

    @property
    def n_groups(self):
        return self.d_col // self.group_size


def _rng(config, layer, which):
    return np.random.Generator(np.random.Philox(1000 * config + 10 * layer + which))


def gelu_exact(x32):
    """x * Phi(x) with the exact erf form, evaluated in fp64 and rounded to fp32."""
    x = x32.astype(np.float64)
    return (0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))).astype(np.float32)


def make_X(spec, chunk_rows=512):
    """Calibration inputs, shape (d_col, n_tok), fp32, feature-major (one row per input feature)."""
    rng = _rng(spec.config, spec.layer, 0)
    X = np.empty((spec.d_col, spec.n_tok), dtype=np.float32)
    scales = None
    if spec.x_kind == "scaled_normal":
        scales = np.exp(0.5 * _rng(spec.config, spec.layer, 2).standard_normal(spec.d_col)).astype(np.float32)
    for r0 in range(0, spec.d_col, chunk_rows):
        r1 = min(spec.d_col, r0 + chunk_rows)
        z = rng.standard_normal((r1 - r0, spec.n_tok), dtype=np.float32)
        if spec.x_kind == "gelu":
            z = gelu_exact(z)
        elif spec.x_kind == "scaled_normal":
            z = z * scales[r0:r1, None]
        elif spec.x_kind != "normal":
            raise ValueError(spec.x_kind)
        X[r0:r1] = z
    return X


def make_W(spec):
    """Layer weights, shape (d_row, d_col), fp32: N(0, w_std^2)."""
    rng = _rng(spec.config, spec.layer, 1)
    return (spec.w_std * rng.standard_normal((spec.d_row, spec.d_col), dtype=np.float32)).astype(np.float32)


def config(idx, layer=0, kind=None):
    """The benchmark configurations, numbered 1..5.

    1: toy FFN-out layer 256x1024, 2048 tokens N(0,1), single columns.
    2: BERT-base attention out-proj 768x768, 12 heads of 64 columns, 16384 tokens,
       N(0,1) times per-channel LogNormal(0, 0.5) scales.
    3: BERT-base FFN down-proj 768x3072, 16384 tokens GELU(N(0,1)), single columns.
    4: BERT-large FFN down-proj 1024x4096, 65536 tokens GELU(N(0,1)).
    5: GPT-2-small-shaped sweep, 12 layers of (kind="attn": 768x768 heads, N(0,1)) and
       (kind="ffn": 768x3072 columns, GELU(N(0,1))), 32768 tokens each.
    """
    if idx == 1:
        return LayerSpec("toy_ffn_256x1024", 1, 0, 256, 1024, 1, 2048, "normal", 1.0 / 32.0)
    if idx == 2:
        return LayerSpec("bert_base_attn_out_768x768_h64", 2, 0, 768, 768, 64, 16384, "scaled_normal", 0.02)
    if idx == 3:
        return LayerSpec("bert_base_ffn_down_768x3072", 3, 0, 768, 3072, 1, 16384, "gelu", 0.02)
    if idx == 4:
        return LayerSpec("bert_large_ffn_down_1024x4096", 4, 0, 1024, 4096, 1, 65536, "gelu", 0.02)
    if idx == 5:
        if kind == "attn":
            return LayerSpec("gpt2_small_attn_out_L%d" % layer, 5, 2 * layer, 768, 768, 64, 32768, "normal", 0.02)
        if kind == "ffn":
            return LayerSpec("gpt2_small_ffn_down_L%d" % layer, 5, 2 * layer + 1, 768, 3072, 1, 32768, "gelu", 0.02)
        raise ValueError("config 5 needs kind='attn' or 'ffn'")
    raise ValueError("unknown config %r" % (idx,))


def small(d_row, d_col, group_size, n_tok, x_kind="gelu", seed=0, w_std=0.05, damp_rel=0.01):
    """A free-form small problem for parity tests (config number 9, `seed` as the layer)."""
    return LayerSpec("small_%dx%d_g%d_n%d_%s_s%d" % (d_row, d_col, group_size, n_tok, x_kind, seed),
                     9, seed, d_row, d_col, group_size, n_tok, x_kind, w_std, damp_rel)
