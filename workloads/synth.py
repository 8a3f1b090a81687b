"""Seeded synthetic inputs for the decode workloads.

Data preparation only: random draws and the weight-only int8 quantiser that
turns N(0, 0.02) weights into the int8 + per-output-channel bf16-scale format
the decode step consumes (Section 3.6 names the format; the recipe is symmetric
absmax, written below).  Nothing of the decode step's own arithmetic is here.
The HIP path and the CPU oracle are both fed from these generators; neither
imports the other.

Every tensor has its own generator stream keyed by (master seed, layer, kind),
so a single layer can be re-drawn without touching the rest.  Streams are
torch's: the same key gives the same bits on the same device type.
"""
from __future__ import annotations

import hashlib
from typing import Dict, Optional

import torch

from .configs import MASTER_SEED, Workload

_KINDS = ("w_in", "w_out", "gamma", "k_cache", "v_cache", "x", "positions", "w_vocab", "gamma_f", "embed",
          "uniforms")


def _stream(device, layer: int, kind: str, seed: int = MASTER_SEED) -> torch.Generator:
    assert kind in _KINDS, kind
    digest = hashlib.sha256(f"{seed}/{layer}/{kind}".encode()).digest()
    g = torch.Generator(device=device)
    g.manual_seed(int.from_bytes(digest[:7], "little"))
    return g


def quantize_per_channel(w: torch.Tensor):
    """Symmetric int8, one scale per output channel (= column of `w` [K, N]).

    scale[n] = bf16(max_k |w[k,n]| / 127); q = clamp(rne(w / scale), -127, 127).
    An all-zero column gets scale 1.  The scale is rounded to bf16 *before* the
    division so that q * scale is the dequantised value both sides use.
    """
    assert w.dim() == 2 and w.dtype == torch.float32
    absmax = w.abs().amax(dim=0)
    scale = (absmax / 127.0).to(torch.bfloat16)
    scale = torch.where(absmax == 0, torch.ones_like(scale), scale)
    # bf16 rounding can push a tiny absmax/127 to zero; keep the scale usable
    scale = torch.where(scale.float() == 0, torch.ones_like(scale), scale)
    q = torch.round(w / scale.float()).clamp_(-127, 127).to(torch.int8)
    return q, scale


def layer_weights(w: Workload, layer: int, device="cpu", sigma: float = 0.02,
                  seed: int = MASTER_SEED) -> Dict[str, torch.Tensor]:
    """One layer's canonical weights.

    w_in  [d_model, n_in]  int8, columns ordered q | k | v | gate | up
    s_in  [n_in]           bf16
    w_out [k_out, d_model] int8, rows ordered attention-out | FFN activation
    s_out [d_model]        bf16
    gamma [d_model]        bf16, 1 + N(0, 0.02) so a mis-indexed gain is visible

    A workload with weights == "bf16" gets the same draws rounded to bf16 instead
    of quantised: w_in, w_out bf16 and no scales.
    """
    d = w.d_model
    g = _stream(device, layer, "w_in", seed)
    w_in = torch.empty(d, w.n_in, dtype=torch.float32, device=device).normal_(0.0, sigma, generator=g)
    g = _stream(device, layer, "gamma", seed)
    gamma = (1.0 + torch.empty(d, dtype=torch.float32, device=device).normal_(0.0, 0.02, generator=g)
             ).to(torch.bfloat16)
    if w.weights == "bf16":
        w_in = w_in.to(torch.bfloat16)
        g = _stream(device, layer, "w_out", seed)
        w_out = torch.empty(w.k_out, d, dtype=torch.float32, device=device).normal_(0.0, sigma, generator=g)
        return {"w_in": w_in, "w_out": w_out.to(torch.bfloat16), "gamma": gamma}
    q_in, s_in = quantize_per_channel(w_in)
    del w_in
    g = _stream(device, layer, "w_out", seed)
    w_out = torch.empty(w.k_out, d, dtype=torch.float32, device=device).normal_(0.0, sigma, generator=g)
    q_out, s_out = quantize_per_channel(w_out)
    del w_out
    return {"w_in": q_in, "s_in": s_in, "w_out": q_out, "s_out": s_out, "gamma": gamma}


def hidden_state(w: Workload, device="cpu", batch: Optional[int] = None,
                 seed: int = MASTER_SEED) -> torch.Tensor:
    """x [B, d_model] bf16 ~ N(0, 1)."""
    b = w.batch if batch is None else batch
    g = _stream(device, 0, "x", seed)
    return torch.empty(b, w.d_model, dtype=torch.float32, device=device).normal_(generator=g).to(torch.bfloat16)


def kv_layer(w: Workload, layer: int, device="cpu", batch: Optional[int] = None,
             seed: int = MASTER_SEED):
    """Cached K and V of one layer, canonical [B, L_ctx, d_head] bf16 ~ N(0, 1)
    ([B, n_kv_heads, L_ctx, d_head] for a multihead workload).
    K is taken to be already rotated (the cache stores post-RoPE keys)."""
    b = w.batch if batch is None else batch
    shape = (b, w.l_ctx, w.d_head) if w.n_kv_heads == 1 else (b, w.n_kv_heads, w.l_ctx, w.d_head)
    out = []
    for kind in ("k_cache", "v_cache"):
        g = _stream(device, layer, kind, seed)
        t = torch.empty(*shape, dtype=torch.float32, device=device).normal_(generator=g)
        out.append(t.to(torch.bfloat16))
    return out[0], out[1]


def positions(w: Workload, device="cpu", batch: Optional[int] = None,
              seed: int = MASTER_SEED) -> torch.Tensor:
    """positions[b] = index of the token being decoded = tokens already cached."""
    b = w.batch if batch is None else batch
    if w.positions == "full":
        return torch.full((b,), w.l_ctx - 1, dtype=torch.int32, device=device)
    g = _stream("cpu", 0, "positions", seed)
    p = torch.randint(w.pos_lo, w.pos_hi, (b,), generator=g, dtype=torch.int32)
    return p.to(device)


def head_weights(w: Workload, vocab: int, device="cpu", sigma: float = 0.02,
                 seed: int = MASTER_SEED) -> Dict[str, torch.Tensor]:
    """Sampling head of the stack (stands in for PaLM's shared embedding matrix):

    w_vocab [d_model, vocab] int8 + s_vocab [vocab] bf16 (same quantiser as the layers),
    gamma_f [d_model] bf16 gain of the final LayerNorm, embed [vocab, d_model] bf16 ~ N(0, 1).
    """
    d = w.d_model
    g = _stream(device, -1, "w_vocab", seed)
    q, s = quantize_per_channel(torch.empty(d, vocab, dtype=torch.float32, device=device).normal_(0.0, sigma, generator=g))
    g = _stream(device, -1, "gamma_f", seed)
    gamma_f = (1.0 + torch.empty(d, dtype=torch.float32, device=device).normal_(0.0, 0.02, generator=g)
               ).to(torch.bfloat16)
    g = _stream(device, -1, "embed", seed)
    embed = torch.empty(vocab, d, dtype=torch.float32, device=device).normal_(generator=g).to(torch.bfloat16)
    return {"w_vocab": q, "s_vocab": s, "gamma_f": gamma_f, "embed": embed}


def uniforms(n_steps: int, batch: int, device="cpu", seed: int = MASTER_SEED) -> torch.Tensor:
    """The random numbers of the sampling loop, [n_steps, batch] fp32 in [0, 1): drawn here,
    passed to both sides as input."""
    g = _stream("cpu", -1, "uniforms", seed)
    return torch.rand(n_steps, batch, generator=g, dtype=torch.float32).to(device)
