"""Puts a synthetic workload on the device: packed weights, library-layout KV
cache, workspace.  Plumbing shared by the GPU tests, the smoke check and the
benchmark; all arithmetic of the step stays in the library."""
from __future__ import annotations

from typing import Callable, Optional

import torch

from workloads import synth
from . import binding


class DeviceStack:
    def __init__(self, workload, device="cuda", poison_unused: bool = False,
                 on_layer: Optional[Callable] = None, batch: Optional[int] = None,
                 positions: Optional[torch.Tensor] = None, x_in: Optional[torch.Tensor] = None):
        """`on_layer(l, weights, k, v)` sees each layer's canonical device tensors
        before they are released (e.g. to copy rows to the host for the oracle)."""
        w = self.w = workload
        self.device = device
        self.B = w.batch if batch is None else batch
        self.dec = binding.Decoder(w)
        self.desc = self.dec.desc
        self.layer_bytes = binding.packed_layer_bytes(self.desc)
        kvb = binding.kv_cache_bytes(self.desc, self.B, w.l_ctx)
        self.packed = torch.empty(w.n_layers * self.layer_bytes, dtype=torch.uint8, device=device)
        self.k_cache = torch.empty(kvb // 2, dtype=torch.bfloat16, device=device)
        self.v_cache = torch.empty(kvb // 2, dtype=torch.bfloat16, device=device)
        self.workspace = torch.empty(binding.workspace_bytes(self.desc, self.B, w.l_ctx),
                                     dtype=torch.uint8, device=device)
        self.positions = (synth.positions(w, device, batch=self.B) if positions is None
                          else positions.to(device=device, dtype=torch.int32).contiguous())
        self.x_in = synth.hidden_state(w, device, batch=self.B) if x_in is None else x_in.to(device)
        assert self.positions.shape == (self.B,) and self.x_in.shape == (self.B, w.d_model)
        self.x_out = torch.empty_like(self.x_in)
        live = (torch.arange(w.l_ctx, device=device)[None, :] <= self.positions[:, None].long())
        for l in range(w.n_layers):
            wts = synth.layer_weights(w, l, device)
            self.dec.pack_layer(wts, self.layer_view(l))
            k, v = synth.kv_layer(w, l, device, batch=self.B)
            if poison_unused:  # slots past the position must never be read
                lv = live[:, :, None] if k.dim() == 3 else live[:, None, :, None]
                k = torch.where(lv, k, torch.full_like(k, float("nan")))
                v = torch.where(lv, v, torch.full_like(v, float("inf")))
            self.dec.kv_import(k, self.k_cache, l, False)
            self.dec.kv_import(v, self.v_cache, l, True)
            if on_layer is not None:
                on_layer(l, wts, k, v)
            torch.cuda.synchronize()
            del wts, k, v

    def layer_view(self, l: int) -> torch.Tensor:
        return self.packed[l * self.layer_bytes:(l + 1) * self.layer_bytes]

    def step(self, stream=None) -> torch.Tensor:
        self.dec.decode_step(self.packed, self.k_cache, self.v_cache, self.x_in, self.positions,
                             self.w.l_ctx, self.x_out, self.workspace, stream)
        return self.x_out

    def export_kv(self, layer: int):
        G = self.w.n_kv_heads
        shape = (self.B, self.w.l_ctx, self.w.d_head) if G == 1 else (self.B, G, self.w.l_ctx, self.w.d_head)
        k = torch.empty(*shape, dtype=torch.bfloat16, device=self.device)
        v = torch.empty_like(k)
        self.dec.kv_export(self.k_cache, k, layer, False)
        self.dec.kv_export(self.v_cache, v, layer, True)
        return k, v


def k_cache_to_library(k: torch.Tensor) -> torch.Tensor:
    """Canonical [B, L_ctx, dh] -> library K layout, written with torch views
    from the layout stated in palmdecode.h (independent of the import kernel)."""
    B, L, dh = k.shape
    return k.view(B, L // 32, 32, dh // 16, 2, 8).permute(0, 1, 3, 4, 2, 5).contiguous().view(-1)


def v_cache_to_library(v: torch.Tensor) -> torch.Tensor:
    """Canonical [B, L_ctx, dh] -> library V layout (see palmdecode.h)."""
    B, L, dh = v.shape
    # t = 16*kk + 8*i + 4*g + j ; c = 32*db + cl  ->  [tb][db][kk][g][cl][4*i + j]
    return (v.view(B, L // 32, 2, 2, 2, 4, dh // 32, 32)
            .permute(0, 1, 6, 2, 4, 7, 3, 5).contiguous().view(-1))


class GenerateStack(DeviceStack):
    """DeviceStack plus the sampling head, the embedding table, the uniforms and the
    workspace of the generation loop."""

    def __init__(self, workload, vocab: int, n_steps: int, **kw):
        super().__init__(workload, **kw)
        w = workload
        self.vocab, self.n_steps = vocab, n_steps
        self.head = synth.head_weights(w, vocab, self.device)
        self.packed_head = torch.empty(binding.packed_head_bytes(self.desc, vocab), dtype=torch.uint8,
                                       device=self.device)
        self.dec.pack_head(self.head["w_vocab"], self.head["s_vocab"], self.head["gamma_f"], self.packed_head)
        self.embed = self.head["embed"]
        self.uniforms = synth.uniforms(n_steps, self.B, self.device)
        self.tokens = torch.full((n_steps, self.B), -1, dtype=torch.int32, device=self.device)
        self.gen_workspace = torch.empty(binding.generate_workspace_bytes(self.desc, vocab, self.B, w.l_ctx),
                                         dtype=torch.uint8, device=self.device)
        torch.cuda.synchronize()

    def generate(self, top_k: int, top_p: float, temperature: float, use_graph: bool, stream=None,
                 n_steps=None) -> torch.Tensor:
        """Runs the loop in place on x_in / positions / caches; returns tokens [n_steps, B]."""
        self.dec.generate(self.packed, self.packed_head, self.embed, self.k_cache, self.v_cache, self.x_in,
                          self.positions, self.w.l_ctx, self.vocab, self.n_steps if n_steps is None else n_steps,
                          top_k, top_p, temperature, self.uniforms, self.tokens, use_graph,
                          self.gen_workspace, stream)
        return self.tokens
