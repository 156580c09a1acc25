"""Seeded synthetic inputs shaped like BLOOM block spans.

This module holds no arithmetic of the method: it only draws random tensors.
Both the CPU oracle's callers and the GPU library's callers take their inputs
from here, so the two sides always see identical bits.

The recipe (stand-in for BLOOM weights and real text, which are not available):
weights iid N(0, 0.02^2) fp32; biases N(0, 0.02^2) fp16; LayerNorm gain
N(1, 0.02^2) and bias N(0, 0.02^2) fp16; hidden states fp16 N(0,1) with a few
fixed feature dims (chosen once per config) carrying outliers whose sign is fixed
per dim and whose magnitude is redrawn per token from a uniform range.
"""
from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class SpanConfig:
    name: str
    n_blocks: int
    hidden: int
    n_heads: int
    batch: int          # sessions per call
    prompt: int         # prefill tokens per session
    decode: int         # decode steps after the prompt
    n_outlier_dims: int
    outlier_mag: tuple
    seed: int
    ln_outlier_gain: float = 1.0   # LayerNorm gain placed on the outlier dims
    prefixes: tuple = ()           # KV prefix lengths for decode-only workloads
    codec: bool = False            # hidden states cross the span boundary 8-bit quantized
    ffn: int = field(default=0)

    @property
    def F(self):
        return self.ffn or 4 * self.hidden

    @property
    def head_dim(self):
        return self.hidden // self.n_heads


# The five workloads named by the benchmark description, in its order.
CONFIGS = {
    # two equal outliers among 64 dims normalise to < 6 after a unit-gain LayerNorm,
    # so the tiny config puts gain 3 on its outlier dims to exercise the fp16 path
    "C1": SpanConfig("C1", 2, 64, 4, 1, 8, 4, 2, (20.0, 40.0), 0, ln_outlier_gain=3.0),
    "C2": SpanConfig("C2", 24, 1024, 16, 1, 128, 128, 1, (10.0, 60.0), 1),
    "C3": SpanConfig("C3", 30, 4096, 32, 8, 512, 256, 4, (10.0, 60.0), 2, codec=True),
    "C4": SpanConfig("C4", 12, 14336, 112, 1, 0, 1, 6, (20.0, 60.0), 3, prefixes=(128, 512, 2048)),
    "C5": SpanConfig("C5", 70, 14336, 112, 32, 512, 64, 6, (20.0, 60.0), 4, codec=True),
}

_TENSOR_IDS = {k: i for i, k in enumerate(
    ("w_qkv", "w_dense", "w_up", "w_down", "b_qkv", "b_dense", "b_up", "b_down",
     "ln1_g", "ln1_b", "ln2_g", "ln2_b"))}


def scaled(cfg, **kw):
    """A copy of cfg with some fields replaced (reduced depth or batch for tests)."""
    d = {f: getattr(cfg, f) for f in cfg.__dataclass_fields__}
    d.update(kw)
    return SpanConfig(**d)


def _rng(cfg, *key):
    return np.random.Generator(np.random.PCG64([cfg.seed, *key]))


def outlier_dims(cfg):
    """(dims, signs): the feature dims that carry outliers, fixed for the config."""
    r = _rng(cfg, 1000)
    dims = np.sort(r.choice(cfg.hidden, size=cfg.n_outlier_dims, replace=False))
    signs = r.choice(np.array([-1.0, 1.0]), size=cfg.n_outlier_dims)
    return dims, signs


def weight_shapes(cfg):
    H, F = cfg.hidden, cfg.F
    return {"w_qkv": (3 * H, H), "w_dense": (H, H), "w_up": (F, H), "w_down": (H, F)}


def block_params(cfg, block):
    """Host (numpy) parameters of one block: fp32 weights, fp16 biases / LayerNorm."""
    H = cfg.hidden
    p = {}
    for name, shape in weight_shapes(cfg).items():
        r = _rng(cfg, block, _TENSOR_IDS[name])
        p[name] = (r.standard_normal(shape, dtype=np.float32) * np.float32(0.02))
        bname = "b_" + name[2:]
        r = _rng(cfg, block, _TENSOR_IDS[bname])
        p[bname] = (r.standard_normal(shape[0]) * 0.02).astype(np.float16)
    dims, _ = outlier_dims(cfg)
    for ln in ("ln1", "ln2"):
        g = 1.0 + _rng(cfg, block, _TENSOR_IDS[ln + "_g"]).standard_normal(H) * 0.02
        g[dims] = cfg.ln_outlier_gain if cfg.ln_outlier_gain != 1.0 else g[dims]
        p[ln + "_g"] = g.astype(np.float16)
        p[ln + "_b"] = (_rng(cfg, block, _TENSOR_IDS[ln + "_b"]).standard_normal(H) * 0.02).astype(np.float16)
    return p


def hidden_states(cfg, call, B, T):
    """fp16 [B,T,H] input of the `call`-th server call (0 = prefill, 1.. = decode steps)."""
    r = _rng(cfg, 2000, call)
    x = r.standard_normal((B, T, cfg.hidden))
    dims, signs = outlier_dims(cfg)
    lo, hi = cfg.outlier_mag
    x[:, :, dims] = r.uniform(lo, hi, size=(B, T, len(dims))) * signs
    return x.astype(np.float16)


def kv_prefix(cfg, block, session, L, std=1.0):
    """fp16 [2, n_heads, L, head_dim] synthetic cache contents for decode-only workloads."""
    r = _rng(cfg, 3000, block, session)
    return (r.standard_normal((2, cfg.n_heads, L, cfg.head_dim), dtype=np.float32) * np.float32(std)).astype(np.float16)


def kv_prefix_device(cfg, block, session, L, std=1.0, device="cuda:0"):
    """Same recipe as kv_prefix, drawn on `device` with torch (different bits)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(((cfg.seed * 1000003 + block) * 4099 + session) * 64 + 63)
    kv = torch.empty((2, cfg.n_heads, L, cfg.head_dim), dtype=torch.float32, device=device)
    kv.normal_(0.0, std, generator=g)
    return kv.to(torch.float16)


# ---------------------------------------------------------------- device side
# Full-size weights (tens of GB) are drawn on the GPU with torch's seeded
# generator; whoever needs them on the host copies the rows it wants.

def block_params_device(cfg, block, device="cuda:0"):
    """Same recipe as block_params, drawn on `device` with torch (different bits)."""
    import torch
    H = cfg.hidden
    p = {}

    def gen(tid):
        g = torch.Generator(device=device)
        g.manual_seed((cfg.seed * 1000003 + block) * 64 + tid)
        return g

    for name, shape in weight_shapes(cfg).items():
        w = torch.empty(shape, dtype=torch.float32, device=device)
        w.normal_(0.0, 0.02, generator=gen(_TENSOR_IDS[name]))
        p[name] = w
        bname = "b_" + name[2:]
        b = torch.empty(shape[0], dtype=torch.float32, device=device)
        b.normal_(0.0, 0.02, generator=gen(_TENSOR_IDS[bname]))
        p[bname] = b.to(torch.float16)
    dims, _ = outlier_dims(cfg)
    for ln in ("ln1", "ln2"):
        g = torch.empty(H, dtype=torch.float32, device=device).normal_(1.0, 0.02, generator=gen(_TENSOR_IDS[ln + "_g"]))
        if cfg.ln_outlier_gain != 1.0:
            g[torch.as_tensor(dims, device=device)] = cfg.ln_outlier_gain
        p[ln + "_g"] = g.to(torch.float16)
        b = torch.empty(H, dtype=torch.float32, device=device).normal_(0.0, 0.02, generator=gen(_TENSOR_IDS[ln + "_b"]))
        p[ln + "_b"] = b.to(torch.float16)
    return p
