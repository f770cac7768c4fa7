"""Seeded random-init weights for DSVT layers and the pooling module.

Matrices are Xavier-uniform U(+-sqrt(6/(fan_in+fan_out))), stored [out, in];
biases and LayerNorm shifts are U(+-0.1), LayerNorm gains 1+U(+-0.1), the
relative-position table N(0, 0.02^2), so that no term of a layer is silently
zero.  Matrix weights are rounded to bf16-representable values for dtype
'bf16'; vectors and the table stay fp32.
"""
import numpy as np
from .frames import _rng, round_bf16


def rel_table_size(win):
    L, W, H = win
    return (2 * L - 1) * (2 * W - 1) * (2 * H - 1)


def _xavier(rng, out_f, in_f, dtype):
    a = np.sqrt(6.0 / (in_f + out_f))
    w = rng.uniform(-a, a, (out_f, in_f)).astype(np.float32)
    return round_bf16(w) if dtype == "bf16" else w


def _vec(rng, n, centre=0.0):
    return (centre + rng.uniform(-0.1, 0.1, n)).astype(np.float32)


def make_layer_weights(seed, C, heads, hidden, win, dtype, rel_bias=True):
    rng = _rng(seed)
    w = dict(C=C, heads=heads, hidden=hidden, dtype=dtype, win=tuple(win), ln_eps=1e-5,
             w_qkv=_xavier(rng, 3 * C, C, dtype), b_qkv=_vec(rng, 3 * C),
             w_o=_xavier(rng, C, C, dtype), b_o=_vec(rng, C),
             w_1=_xavier(rng, hidden, C, dtype), b_1=_vec(rng, hidden),
             w_2=_xavier(rng, C, hidden, dtype), b_2=_vec(rng, C),
             ln1_g=_vec(rng, C, 1.0), ln1_b=_vec(rng, C), ln2_g=_vec(rng, C, 1.0), ln2_b=_vec(rng, C))
    table = (0.02 * rng.standard_normal((heads, rel_table_size(win)))).astype(np.float32)
    w["rel_bias"] = table if rel_bias else None
    return w


def make_pool_weights(seed, C, heads, dtype):
    rng = _rng(seed)
    return dict(C=C, heads=heads, dtype=dtype, ln_eps=1e-5,
                w_q=_xavier(rng, C, C, dtype), b_q=_vec(rng, C), w_k=_xavier(rng, C, C, dtype), b_k=_vec(rng, C),
                w_v=_xavier(rng, C, C, dtype), b_v=_vec(rng, C), w_o=_xavier(rng, C, C, dtype), b_o=_vec(rng, C),
                ln_g=_vec(rng, C, 1.0), ln_b=_vec(rng, C))


def make_vfe_weights(seed, C, f_in):
    """Per-point linear map of the voxel feature encoder: w [C, f_in] Xavier-uniform, b [C] U(+-0.1), float32."""
    rng = _rng(seed)
    return _xavier(rng, C, f_in, "f32"), _vec(rng, C)
