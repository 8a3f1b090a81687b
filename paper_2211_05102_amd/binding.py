"""Thin ctypes binding of libpalmdecode.so: argument marshalling only.

Every step of the decode path runs in the library's HIP kernels; torch is used
for device memory and streams.  There is no fallback: if the library is not
built, importing `lib()` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpalmdecode.so")

PD_OK = 0
PD_ERR_NULL, PD_ERR_ALIGN, PD_ERR_SHAPE, PD_ERR_RANGE = -1, -2, -3, -4
PD_ERR_WORKSPACE, PD_ERR_HIP, PD_ERR_POSITION, PD_ERR_STATE = -5, -6, -7, -8

EXPORTS = [
    "pd_status_string", "pd_last_error", "pd_packed_layer_bytes", "pd_kv_cache_bytes",
    "pd_workspace_bytes", "pd_create", "pd_destroy", "pd_set_option", "pd_pack_layer",
    "pd_pack_matrix", "pd_kv_import", "pd_kv_export", "pd_decode_step", "pd_decode_step_static", "pd_decode_layer",
    "pd_check_async", "pd_qgemm_workspace_bytes", "pd_qgemm_plan", "pd_qgemm", "pd_mqa_attend",
    "pd_graph_capture", "pd_graph_replay", "pd_graph_release", "pd_profile_read",
    "pd_packed_head_bytes", "pd_head_workspace_bytes", "pd_generate_workspace_bytes", "pd_pack_head",
    "pd_head_logits", "pd_sample", "pd_generate", "pd_prefill", "pd_pack_matrix_bf16", "pd_wgemm_bf16", "pd_ceiling_probe",
]

PD_FLAG_BF16_WEIGHTS = 1


class ModelDesc(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32),
                ("n_heads", ctypes.c_int32), ("d_head", ctypes.c_int32),
                ("d_ff", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("rope_base", ctypes.c_float), ("ln_eps", ctypes.c_float),
                ("flags", ctypes.c_int32)]


class PdError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"palmdecode error {code}: {text}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run __graft_entry__.build() "
                              "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        L.pd_status_string.restype = ctypes.c_char_p
        L.pd_last_error.restype = ctypes.c_char_p
        for name in EXPORTS[2:]:
            getattr(L, name).restype = ctypes.c_int32
        _lib = L
    return _lib


def _check(code: int) -> None:
    if code != PD_OK:
        raise PdError(code, lib().pd_last_error().decode() or lib().pd_status_string(code).decode())


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def make_desc(w) -> ModelDesc:
    """`w`: any object with the workload field names."""
    return ModelDesc(w.n_layers, w.d_model, w.n_heads, w.d_head, w.d_ff,
                     getattr(w, "n_kv_heads", 1), float(w.rope_base), float(w.ln_eps),
                     PD_FLAG_BF16_WEIGHTS if getattr(w, "weights", "int8") == "bf16" else 0)


def packed_layer_bytes(desc: ModelDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().pd_packed_layer_bytes(ctypes.byref(desc), ctypes.byref(n)))
    return n.value


def kv_cache_bytes(desc: ModelDesc, B: int, L_ctx: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().pd_kv_cache_bytes(ctypes.byref(desc), ctypes.c_int32(B), ctypes.c_int32(L_ctx), ctypes.byref(n)))
    return n.value


def workspace_bytes(desc: ModelDesc, B: int, L_ctx: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().pd_workspace_bytes(ctypes.byref(desc), ctypes.c_int32(B), ctypes.c_int32(L_ctx), ctypes.byref(n)))
    return n.value


def qgemm_workspace_bytes(B: int, K: int, N: int, workgroups: int = 0) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().pd_qgemm_workspace_bytes(ctypes.c_int32(B), ctypes.c_int32(K), ctypes.c_int32(N),
                                          ctypes.c_int32(workgroups), ctypes.byref(n)))
    return n.value


def qgemm_plan(B: int, K: int, N: int, workgroups: int = 0, c_split: int = 0, blk0: int = 1, blk1: int = 1):
    """Host only: (counts dict, range_begin list, first_slot list, slots_per_tile list)."""
    counts = (ctypes.c_int32 * 5)()
    args = [ctypes.c_int32(v) for v in (B, K, N, workgroups, c_split, blk0, blk1)]
    _check(lib().pd_qgemm_plan(*args, counts, None, None, None))
    G, T = counts[0], counts[1]
    rb = (ctypes.c_int64 * (G + 1))()
    fs = (ctypes.c_int32 * G)()
    spt = (ctypes.c_int32 * T)()
    _check(lib().pd_qgemm_plan(*args, counts, rb, fs, spt))
    names = ("workgroups", "tiles", "chunks_per_tile", "rows", "max_slots")
    return dict(zip(names, list(counts))), list(rb), list(fs), list(spt)


def packed_head_bytes(desc: ModelDesc, vocab: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().pd_packed_head_bytes(ctypes.byref(desc), ctypes.c_int32(vocab), ctypes.byref(n)))
    return n.value


def head_workspace_bytes(desc: ModelDesc, vocab: int, B: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().pd_head_workspace_bytes(ctypes.byref(desc), ctypes.c_int32(vocab), ctypes.c_int32(B), ctypes.byref(n)))
    return n.value


def generate_workspace_bytes(desc: ModelDesc, vocab: int, B: int, L_ctx: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().pd_generate_workspace_bytes(ctypes.byref(desc), ctypes.c_int32(vocab), ctypes.c_int32(B),
                                             ctypes.c_int32(L_ctx), ctypes.byref(n)))
    return n.value


def sample(logits: torch.Tensor, top_k: int, top_p: float, temperature: float, uniforms: torch.Tensor,
           tokens: torch.Tensor, stream=None) -> None:
    B, V = logits.shape
    assert logits.dtype == torch.float32 and logits.is_contiguous() and uniforms.dtype == torch.float32
    assert tokens.dtype == torch.int32 and tokens.numel() >= B and uniforms.numel() >= B
    _check(lib().pd_sample(_ptr(logits), ctypes.c_int32(B), ctypes.c_int32(V), ctypes.c_int32(top_k),
                           ctypes.c_float(top_p), ctypes.c_float(temperature), _ptr(uniforms), _ptr(tokens),
                           _stream(stream)))


def pack_matrix(w: torch.Tensor, packed: torch.Tensor, stream=None) -> None:
    K, N = w.shape
    assert w.dtype == torch.int8 and w.is_contiguous() and packed.numel() * packed.element_size() >= K * N
    _check(lib().pd_pack_matrix(_ptr(w), ctypes.c_int32(K), ctypes.c_int32(N), _ptr(packed), _stream(stream)))


def qgemm(packed_w: torch.Tensor, scale: torch.Tensor, a: torch.Tensor, N: int, out: torch.Tensor,
          workspace: torch.Tensor, workgroups: int = 0, stream=None) -> None:
    B, K = a.shape
    assert a.dtype == torch.bfloat16 and a.is_contiguous() and scale.dtype == torch.float32
    assert out.dtype == torch.float32 and out.shape == (B, N) and out.is_contiguous()
    _check(lib().pd_qgemm(_ptr(packed_w), _ptr(scale), _ptr(a), ctypes.c_int32(B), ctypes.c_int32(K),
                          ctypes.c_int32(N), _ptr(out), ctypes.c_int32(workgroups), _ptr(workspace),
                          ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))


def pack_matrix_bf16(w: torch.Tensor, packed: torch.Tensor, stream=None) -> None:
    K, N = w.shape
    assert w.dtype == torch.bfloat16 and w.is_contiguous() and packed.numel() * packed.element_size() >= 2 * K * N
    _check(lib().pd_pack_matrix_bf16(_ptr(w), ctypes.c_int32(K), ctypes.c_int32(N), _ptr(packed), _stream(stream)))


def wgemm_bf16(packed_w: torch.Tensor, a: torch.Tensor, N: int, out: torch.Tensor,
               workspace: torch.Tensor, workgroups: int = 0, stream=None) -> None:
    B, K = a.shape
    assert a.dtype == torch.bfloat16 and a.is_contiguous()
    assert out.dtype == torch.float32 and out.shape == (B, N) and out.is_contiguous()
    _check(lib().pd_wgemm_bf16(_ptr(packed_w), _ptr(a), ctypes.c_int32(B), ctypes.c_int32(K),
                               ctypes.c_int32(N), _ptr(out), ctypes.c_int32(workgroups), _ptr(workspace),
                               ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))


def ceiling_probe(buffer: torch.Tensor, mfma_per_unit: int, random_operands: int, sink: torch.Tensor,
                  stream=None) -> None:
    _check(lib().pd_ceiling_probe(_ptr(buffer), ctypes.c_size_t(buffer.numel() * buffer.element_size()),
                                  ctypes.c_int32(mfma_per_unit), ctypes.c_int32(int(random_operands)),
                                  _ptr(sink), _stream(stream)))


class Decoder:
    """Owns a pd_handle; methods mirror the C entry points one to one."""

    def __init__(self, workload):
        self.desc = make_desc(workload)
        self._h = ctypes.c_void_p(0)
        _check(lib().pd_create(ctypes.byref(self.desc), ctypes.byref(self._h)))

    def close(self) -> None:
        if self._h:
            lib().pd_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_option(self, name: str, value: int) -> None:
        _check(lib().pd_set_option(self._h, name.encode(), ctypes.c_int32(value)))

    def profile_read(self):
        """(summed milliseconds, launches) of the kernel class being timed."""
        ms, n = ctypes.c_double(0), ctypes.c_int32(0)
        _check(lib().pd_profile_read(self._h, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def pack_layer(self, wts: dict, packed_layer: torch.Tensor, stream=None) -> None:
        want = torch.bfloat16 if self.desc.flags & PD_FLAG_BF16_WEIGHTS else torch.int8
        assert wts["w_in"].dtype == want and wts["w_out"].dtype == want, "weight dtype does not match the handle"
        _check(lib().pd_pack_layer(self._h, _ptr(wts["w_in"]), _ptr(wts.get("s_in")), _ptr(wts["w_out"]),
                                   _ptr(wts.get("s_out")), _ptr(wts["gamma"]), _ptr(packed_layer),
                                   _stream(stream)))

    def kv_import(self, canonical: torch.Tensor, cache: torch.Tensor, layer: int, is_v: bool, stream=None) -> None:
        B, L_ctx = canonical.shape[0], canonical.shape[-2]  # [B, L, dh] or [B, G, L, dh]
        assert canonical.dtype == torch.bfloat16 and canonical.is_contiguous()
        _check(lib().pd_kv_import(self._h, _ptr(canonical), _ptr(cache), ctypes.c_int32(layer),
                                  ctypes.c_int32(B), ctypes.c_int32(L_ctx), ctypes.c_int32(int(is_v)),
                                  _stream(stream)))

    def kv_export(self, cache: torch.Tensor, canonical: torch.Tensor, layer: int, is_v: bool, stream=None) -> None:
        B, L_ctx = canonical.shape[0], canonical.shape[-2]  # [B, L, dh] or [B, G, L, dh]
        assert canonical.dtype == torch.bfloat16 and canonical.is_contiguous()
        _check(lib().pd_kv_export(self._h, _ptr(cache), _ptr(canonical), ctypes.c_int32(layer),
                                  ctypes.c_int32(B), ctypes.c_int32(L_ctx), ctypes.c_int32(int(is_v)),
                                  _stream(stream)))

    def _step_args(self, packed, k_cache, v_cache, x_in, positions, L_ctx, out, workspace, stream):
        B = x_in.shape[0]
        return (self._h, _ptr(packed), _ptr(k_cache), _ptr(v_cache), _ptr(x_in), _ptr(positions),
                ctypes.c_int32(B), ctypes.c_int32(L_ctx), _ptr(out), _ptr(workspace),
                ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))

    def decode_step(self, packed, k_cache, v_cache, x_in, positions, L_ctx, x_out, workspace, stream=None) -> None:
        _check(lib().pd_decode_step(*self._step_args(packed, k_cache, v_cache, x_in, positions, L_ctx,
                                                     x_out, workspace, stream)))

    def decode_step_static(self, packed, k_cache, v_cache, x_in, positions, L_ctx, x_out, stream=None) -> None:
        B = x_in.shape[0]
        _check(lib().pd_decode_step_static(self._h, _ptr(packed), _ptr(k_cache), _ptr(v_cache), _ptr(x_in),
                                           _ptr(positions), ctypes.c_int32(B), ctypes.c_int32(L_ctx),
                                           _ptr(x_out), _stream(stream)))

    def prefill(self, packed, k_cache, v_cache, x_in, seq_ids, positions, cache_rows, L_ctx, x_out, workspace,
                stream=None) -> None:
        n = x_in.shape[0]
        assert seq_ids.dtype == torch.int32 and positions.dtype == torch.int32
        _check(lib().pd_prefill(self._h, _ptr(packed), _ptr(k_cache), _ptr(v_cache), _ptr(x_in), _ptr(seq_ids),
                                _ptr(positions), ctypes.c_int32(n), ctypes.c_int32(cache_rows),
                                ctypes.c_int32(L_ctx), _ptr(x_out), _ptr(workspace),
                                ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))

    def decode_layer(self, layer, packed_layer, k_cache, v_cache, x_in, positions, L_ctx, y_out,
                     add_residual, workspace, stream=None) -> None:
        B = x_in.shape[0]
        _check(lib().pd_decode_layer(self._h, ctypes.c_int32(layer), _ptr(packed_layer), _ptr(k_cache),
                                     _ptr(v_cache), _ptr(x_in), _ptr(positions), ctypes.c_int32(B),
                                     ctypes.c_int32(L_ctx), _ptr(y_out), ctypes.c_int32(int(add_residual)),
                                     _ptr(workspace),
                                     ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                     _stream(stream)))

    def check_async(self, workspace, stream=None) -> None:
        _check(lib().pd_check_async(self._h, _ptr(workspace), _stream(stream)))

    def mqa_attend(self, layer, q, k_cache, v_cache, positions, L_ctx, o, workspace, stream=None) -> None:
        B = q.shape[0]
        assert q.dtype == torch.float32 and o.dtype == torch.float32 and q.is_contiguous()
        _check(lib().pd_mqa_attend(self._h, ctypes.c_int32(layer), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                   _ptr(positions), ctypes.c_int32(B), ctypes.c_int32(L_ctx), _ptr(o),
                                   _ptr(workspace),
                                   ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                   _stream(stream)))

    def pack_head(self, w_vocab, s_vocab, gamma_f, packed_head, stream=None) -> None:
        vocab = w_vocab.shape[1]
        _check(lib().pd_pack_head(self._h, _ptr(w_vocab), _ptr(s_vocab), _ptr(gamma_f), ctypes.c_int32(vocab),
                                  _ptr(packed_head), _stream(stream)))

    def head_logits(self, packed_head, vocab, x, logits, workspace, stream=None) -> None:
        B = x.shape[0]
        _check(lib().pd_head_logits(self._h, _ptr(packed_head), ctypes.c_int32(vocab), _ptr(x), ctypes.c_int32(B),
                                    _ptr(logits), _ptr(workspace),
                                    ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))

    def generate(self, packed, packed_head, embed, k_cache, v_cache, x, positions, L_ctx, vocab, n_steps,
                 top_k, top_p, temperature, uniforms, tokens_out, use_graph, workspace, stream=None) -> None:
        B = x.shape[0]
        _check(lib().pd_generate(self._h, _ptr(packed), _ptr(packed_head), _ptr(embed), _ptr(k_cache), _ptr(v_cache),
                                 _ptr(x), _ptr(positions), ctypes.c_int32(B), ctypes.c_int32(L_ctx),
                                 ctypes.c_int32(vocab), ctypes.c_int32(n_steps), ctypes.c_int32(top_k),
                                 ctypes.c_float(top_p), ctypes.c_float(temperature), _ptr(uniforms),
                                 _ptr(tokens_out), ctypes.c_int32(int(use_graph)), _ptr(workspace),
                                 ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))

    def graph_capture(self, packed, k_cache, v_cache, x_in, positions, L_ctx, x_out, workspace, stream) -> None:
        _check(lib().pd_graph_capture(*self._step_args(packed, k_cache, v_cache, x_in, positions, L_ctx,
                                                       x_out, workspace, stream)))

    def graph_replay(self, stream) -> None:
        _check(lib().pd_graph_replay(self._h, _stream(stream)))

    def graph_release(self) -> None:
        _check(lib().pd_graph_release(self._h))
