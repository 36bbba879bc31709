"""Seeded synthetic tensors and real-valued scales for the five workload shapes.

Only input generation lives here: int8 Q/K factors, their exact int32 products
(the attention scores), Swin relative-position biases, detection padding masks,
long-tailed int8 MLP activations and the per-layer real scales.  The paper's
ImageNet / COCO activations are not available, so these stand in for them with
the shapes and value distributions of the benchmark configurations.

Conventions: ``normal(0, s)`` takes ``s`` as the standard deviation and
``laplace(0, b)`` takes ``b`` as the scale; every tensor has its own
``numpy.random.SeedSequence`` child so that the order of generation is
irrelevant.
"""

from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import numpy as np

INT32_MIN = -(2 ** 31)

# name -> description.  A "unit" is one transformer layer (ViT/DeiT) or one
# stage (Swin): it owns one softmax tensor and one GELU tensor.
CONFIGS = {
    "deit_t": dict(
        index=0, batch=1, units=1, head_dim=64, qk_sigma=25.0, heavy_tail=None,
        heads=[3], tokens=[197], windows=[1], mlp_tokens=[197], mlp_width=[768],
        bias=False, mask=False, scales="pow2"),
    "vit_s": dict(
        index=1, batch=64, units=12, head_dim=64, qk_sigma=25.0, heavy_tail=None,
        heads=[6] * 12, tokens=[197] * 12, windows=[1] * 12,
        mlp_tokens=[197] * 12, mlp_width=[1536] * 12,
        bias=False, mask=False, scales="loguniform"),
    "vit_b": dict(
        index=2, batch=128, units=12, head_dim=64, qk_sigma=30.0, heavy_tail=(0.01, 8.0),
        heads=[12] * 12, tokens=[197] * 12, windows=[1] * 12,
        mlp_tokens=[197] * 12, mlp_width=[3072] * 12,
        bias=False, mask=False, scales="loguniform"),
    "swin_b": dict(
        index=3, batch=64, units=4, head_dim=32, qk_sigma=25.0, heavy_tail=None,
        heads=[4, 8, 16, 32], tokens=[49] * 4, windows=[64, 16, 4, 1],
        mlp_tokens=[3136, 784, 196, 49], mlp_width=[512, 1024, 2048, 4096],
        bias=True, mask=False, scales="loguniform"),
    "swin_s_det": dict(
        index=4, batch=2, units=1, head_dim=32, qk_sigma=25.0, heavy_tail=None,
        heads=[3], tokens=[49], windows=[1392],
        mlp_tokens=[66800], mlp_width=[384],
        bias=False, mask=True, scales="loguniform"),
}


def config_names():
    return list(CONFIGS.keys())


def _rng(seed: int, cfg_index: int, unit: int, tensor_id: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, cfg_index, unit, tensor_id]))


# --------------------------------------------------------------------------- tensors
def qk_pair(rng: np.random.Generator, lead: int, tokens: int, head_dim: int,
            sigma: float, heavy_tail=None):
    """Two int8 tensors [lead, tokens, head_dim]: round(N(0, sigma)) clipped to +-127.

    ``heavy_tail=(fraction, factor)`` multiplies that fraction of the entries by
    ``factor`` before rounding and clipping.
    """
    out = []
    for _ in range(2):
        x = rng.standard_normal((lead, tokens, head_dim), dtype=np.float32) * np.float32(sigma)
        if heavy_tail is not None:
            frac, factor = heavy_tail
            hit = rng.random((lead, tokens, head_dim), dtype=np.float32) < np.float32(frac)
            x = np.where(hit, x * np.float32(factor), x)
        out.append(np.clip(np.rint(x), -127, 127).astype(np.int8))
    return out[0], out[1]


def scores_from_qk(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """Exact int32 Q.K^T per leading index: [lead, tokens, tokens].

    float32 matmul is exact here: every partial sum is an integer below
    head_dim * 127^2 < 2^24.
    """
    assert q.shape[-1] * 127 * 127 < 2 ** 24
    s = np.matmul(q.astype(np.float32), np.swapaxes(k, -1, -2).astype(np.float32))
    return s.astype(np.int32)


def swin_bias(rng: np.random.Generator, heads: int, win_tokens: int) -> np.ndarray:
    """Additive int32 relative-position bias [heads * win_tokens, win_tokens] ~ round(N(0, 8))."""
    b = rng.standard_normal((heads * win_tokens, win_tokens)) * 8.0
    return np.rint(b).astype(np.int32)


def detection_key_mask(map_h: int = 200, map_w: int = 334, win: int = 7) -> np.ndarray:
    """Boolean [windows, win*win]: True where the key token of a window is padding.

    The token map is padded up to multiples of the window size (200x334 ->
    203x336, i.e. 29x48 = 1392 windows); padded tokens are the masked keys.
    """
    ph = -(-map_h // win) * win
    pw = -(-map_w // win) * win
    pad = np.zeros((ph, pw), dtype=bool)
    pad[map_h:, :] = True
    pad[:, map_w:] = True
    nh, nw = ph // win, pw // win
    return pad.reshape(nh, win, nw, win).transpose(0, 2, 1, 3).reshape(nh * nw, win * win)


def shifted_window_mask(map_h: int, map_w: int, win: int = 7, shift: int = 3) -> np.ndarray:
    """int32 [windows, win*win, win*win]: the additive attention mask of a shifted-window block.

    After the token map is rolled by `shift`, a window at the map's border holds tokens from up
    to four regions that were not neighbours before the roll; a query may only attend to keys of
    its own region.  Entry 0 where query and key share a region, INT32_MIN elsewhere.  Windows
    are numbered row-major over the map; a map of exactly one window has nothing to mask.
    """
    assert map_h % win == 0 and map_w % win == 0 and 0 < shift < win
    region = np.zeros((map_h, map_w), dtype=np.int64)
    edges_h = (0, map_h - win, map_h - shift, map_h)
    edges_w = (0, map_w - win, map_w - shift, map_w)
    rid = 0
    for a in range(3):
        for b in range(3):
            region[edges_h[a]:edges_h[a + 1], edges_w[b]:edges_w[b + 1]] = rid
            rid += 1
    nh, nw = map_h // win, map_w // win
    per_window = region.reshape(nh, win, nw, win).transpose(0, 2, 1, 3).reshape(nh * nw, win * win)
    same = per_window[:, :, None] == per_window[:, None, :]
    return np.where(same, 0, -(2 ** 31)).astype(np.int32)


# token map side of each Swin-B stage at 224 x 224 (stage 4 is a single window: no mask)
SWIN_B_MAP_SIDE = (56, 28, 14, 7)


_GELU_BLOCK_TOKENS = 2048


def _gelu_block(seed_seq, tokens: int, width: int, scale_row: np.ndarray) -> np.ndarray:
    rng = np.random.default_rng(seed_seq)
    n = tokens * width
    x = rng.standard_normal(n, dtype=np.float32)
    x *= np.float32(20.0)
    pick = np.flatnonzero(rng.random(n, dtype=np.float32) < np.float32(0.1))
    x[pick] = rng.laplace(0.0, 60.0, size=pick.size).astype(np.float32)
    x = x.reshape(tokens, width)
    x *= scale_row
    np.rint(x, out=x)
    np.clip(x, -127, 127, out=x)
    return x.astype(np.int8)


def gelu_input(rng: np.random.Generator, tokens: int, width: int) -> np.ndarray:
    """int8 [tokens, width]: 0.9*N(0,20) + 0.1*Laplace(0,60), 2% of channels x4, clipped to +-127.

    Drawn in blocks of 2048 tokens, each from its own child seed, so that the
    blocks can be filled by a few threads without changing the result.
    """
    from concurrent.futures import ThreadPoolExecutor

    n_out = max(1, int(round(0.02 * width)))
    chans = rng.choice(width, size=n_out, replace=False)
    scale_row = np.ones(width, dtype=np.float32)
    scale_row[chans] = 4.0
    n_blocks = -(-tokens // _GELU_BLOCK_TOKENS)
    seeds = rng.bit_generator.seed_seq.spawn(n_blocks)
    out = np.empty((tokens, width), dtype=np.int8)

    def fill(i):
        lo = i * _GELU_BLOCK_TOKENS
        hi = min(tokens, lo + _GELU_BLOCK_TOKENS)
        out[lo:hi] = _gelu_block(seeds[i], hi - lo, width, scale_row)

    with ThreadPoolExecutor(max_workers=8) as ex:
        list(ex.map(fill, range(n_blocks)))
    return out


# --------------------------------------------------------------------------- scales
def _gelu_real(x: float) -> float:
    return 0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0)))


def layer_scales(name: str, unit: int, seed: int = 0) -> dict:
    """Real-valued scales, zero-points and variant bits of one unit.

    ``pow2`` configs use fixed powers of two; the others draw the softmax input
    scale and the GELU input scale log-uniformly in [2^-10, 2^-4].  The GELU
    output quantizer covers [min GELU, GELU(127 * s_in)] with 256 levels.
    """
    cfg = CONFIGS[name]
    if cfg["scales"] == "pow2":
        return dict(s_delta=2.0 ** -7, s_in=2.0 ** -4, s_out=2.0 ** -5, zp_in=0, zp_out=0,
                    softmax_variant=1, gelu_variant=1)
    rng = _rng(seed, cfg["index"], unit, 9)
    s_delta = float(2.0 ** rng.uniform(-10.0, -4.0))
    s_in = float(2.0 ** rng.uniform(-10.0, -4.0))
    bits = rng.integers(0, 2, size=2)
    vals = [_gelu_real(s_in * q) for q in range(-128, 128)]
    gmin, gmax = min(vals), max(vals)
    s_out = (gmax - gmin) / 255.0
    zp_out = int(round(-128.0 - gmin / s_out))
    return dict(s_delta=s_delta, s_in=s_in, s_out=s_out, zp_in=0, zp_out=zp_out,
                softmax_variant=int(bits[0]), gelu_variant=int(bits[1]))


# --------------------------------------------------------------------------- cases
@dataclass
class SoftmaxCase:
    name: str
    unit: int
    scores: np.ndarray            # int32 [rows, cols]
    bias: Optional[np.ndarray]    # int32 [period_rows, cols] or None
    bias_period_rows: int
    s_delta: float
    variant: int


@dataclass
class GeluCase:
    name: str
    unit: int
    x: np.ndarray                 # int8 [tokens_total, width]
    s_in: float
    s_out: float
    zp_in: int
    zp_out: int
    variant: int


def softmax_qk(name: str, unit: int = 0, batch: Optional[int] = None, seed: int = 0):
    """The int8 Q, K factors of one unit, [batch*windows*heads, tokens, head_dim]."""
    cfg = CONFIGS[name]
    b = cfg["batch"] if batch is None else batch
    lead = b * cfg["windows"][unit] * cfg["heads"][unit]
    rng = _rng(seed, cfg["index"], unit, 1)
    return qk_pair(rng, lead, cfg["tokens"][unit], cfg["head_dim"], cfg["qk_sigma"],
                   cfg["heavy_tail"])


def softmax_bias(name: str, unit: int = 0, seed: int = 0):
    """(bias, bias_period_rows) of one unit, or (None, 0) for configs without a bias."""
    cfg = CONFIGS[name]
    if not cfg["bias"]:
        return None, 0
    heads, tokens = cfg["heads"][unit], cfg["tokens"][unit]
    return swin_bias(_rng(seed, cfg["index"], unit, 2), heads, tokens), heads * tokens


def softmax_case(name: str, unit: int = 0, batch: Optional[int] = None, seed: int = 0,
                 scores: Optional[np.ndarray] = None) -> SoftmaxCase:
    """Scores (and bias / mask where the config has them) of one unit.

    ``scores`` may carry an already formed product of ``softmax_qk`` (e.g. done
    on another device); masking is applied here either way.
    """
    cfg = CONFIGS[name]
    b = cfg["batch"] if batch is None else batch
    heads, tokens, windows = cfg["heads"][unit], cfg["tokens"][unit], cfg["windows"][unit]
    if scores is None:
        q, k = softmax_qk(name, unit, batch, seed)
        scores = scores_from_qk(q, k)
    scores = scores.reshape(b, windows, heads, tokens, tokens)
    if cfg["mask"]:
        km = detection_key_mask()                      # [windows, tokens]
        assert km.shape == (windows, tokens)
        scores = np.where(km[None, :, None, None, :], np.int32(INT32_MIN), scores)
    scores = np.ascontiguousarray(scores.reshape(-1, tokens), dtype=np.int32)
    bias, period = softmax_bias(name, unit, seed)
    sc = layer_scales(name, unit, seed)
    return SoftmaxCase(name, unit, scores, bias, period, sc["s_delta"], sc["softmax_variant"])


def gelu_case(name: str, unit: int = 0, batch: Optional[int] = None, seed: int = 0) -> GeluCase:
    cfg = CONFIGS[name]
    b = cfg["batch"] if batch is None else batch
    rng = _rng(seed, cfg["index"], unit, 3)
    x = gelu_input(rng, b * cfg["mlp_tokens"][unit], cfg["mlp_width"][unit])
    sc = layer_scales(name, unit, seed)
    return GeluCase(name, unit, x, sc["s_in"], sc["s_out"], sc["zp_in"], sc["zp_out"],
                    sc["gelu_variant"])
