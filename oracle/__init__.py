"""ctypes face of the fp64 CPU oracle (palm_oracle.c).

TEST INFRASTRUCTURE: only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this.  It shares nothing with the HIP library and
never imports it.  Arrays are numpy; bf16 values travel as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "palm_oracle.c")
_LIB = os.path.join(_HERE, "libpalm_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP only spreads independent outputs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-march=native", "-fopenmp", "-fno-fast-math",
               "-ffp-contract=off", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Desc(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32),
                ("n_heads", ctypes.c_int32), ("d_head", ctypes.c_int32),
                ("d_ff", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("rope_base", ctypes.c_double), ("ln_eps", ctypes.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_bf16_to_f64.restype = ctypes.c_double
        _lib.orc_bf16_to_f64.argtypes = [ctypes.c_uint16]
        _lib.orc_f64_to_bf16.restype = ctypes.c_uint16
        _lib.orc_f64_to_bf16.argtypes = [ctypes.c_double]
        _lib.orc_num_threads.restype = ctypes.c_int
        _lib.orc_decode_layer.restype = ctypes.c_int
        _lib.orc_decode_layer_w16.restype = ctypes.c_int
        _lib.orc_sample_topk_topp.restype = ctypes.c_int
        _lib.orc_causal_layer.restype = ctypes.c_int
    return _lib


def _p(a: np.ndarray, dtype) -> ctypes.c_void_p:
    assert a.dtype == dtype, (a.dtype, dtype)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def make_desc(w) -> _Desc:
    """`w` is any object with the Workload field names."""
    return _Desc(w.n_layers, w.d_model, w.n_heads, w.d_head, w.d_ff,
                 getattr(w, "n_kv_heads", 1), float(w.rope_base), float(w.ln_eps))


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ------------------------------------------------------------------ pieces ---

def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Element by element through the C routine (small arrays; pins)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    f = lib().orc_bf16_to_f64
    return np.array([f(int(b)) for b in bits.ravel()], dtype=np.float64).reshape(bits.shape)


def f64_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    lib().orc_f64_to_bf16_n(_p(v, np.float64), _p(out, np.uint16), ctypes.c_int64(v.size))
    return out


def layernorm(x: np.ndarray, gamma_bits: np.ndarray, eps: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    h = np.empty_like(x)
    lib().orc_layernorm(_p(x, np.float64), _p(gamma_bits, np.uint16), ctypes.c_int32(x.shape[-1]),
                        ctypes.c_double(eps), _p(h, np.float64))
    return h


def qmatmul(a: np.ndarray, q8: np.ndarray, scale_bits: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    R, K = a.shape
    K2, N = q8.shape
    assert K == K2 and scale_bits.shape == (N,)
    out = np.empty((R, N), dtype=np.float64)
    lib().orc_qmatmul(_p(a, np.float64), _p(q8, np.int8), _p(scale_bits, np.uint16),
                      ctypes.c_int32(R), ctypes.c_int32(K), ctypes.c_int32(N), _p(out, np.float64))
    return out


def wmatmul_bf16(a: np.ndarray, w_bits: np.ndarray) -> np.ndarray:
    """a [R, K] fp64 times bf16 weights [K, N] (bit patterns), no scales."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    w = _bits(w_bits)
    R, K = a.shape
    assert w.shape[0] == K
    out = np.empty((R, w.shape[1]), dtype=np.float64)
    lib().orc_wmatmul_bf16(_p(a, np.float64), _p(w, np.uint16), ctypes.c_int32(R), ctypes.c_int32(K),
                           ctypes.c_int32(w.shape[1]), _p(out, np.float64))
    return out


def rope(y: np.ndarray, pos: int, base: float) -> np.ndarray:
    y = np.array(y, dtype=np.float64, copy=True)
    assert y.ndim == 1
    lib().orc_rope(_p(y, np.float64), ctypes.c_int32(y.shape[0]), ctypes.c_int32(pos),
                   ctypes.c_double(base))
    return y


def attend_mqa(q: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray, want_probs: bool = False):
    q = np.ascontiguousarray(q, dtype=np.float64)
    H, dh = q.shape
    T = k_bits.shape[0]
    assert k_bits.shape == (T, dh) and v_bits.shape == (T, dh)
    out = np.empty((H, dh), dtype=np.float64)
    probs = np.empty((H, T), dtype=np.float64) if want_probs else None
    lib().orc_attend_mqa(_p(q, np.float64), _p(k_bits, np.uint16), _p(v_bits, np.uint16),
                         ctypes.c_int32(H), ctypes.c_int32(dh), ctypes.c_int32(T),
                         _p(out, np.float64),
                         _p(probs, np.float64) if want_probs else ctypes.c_void_p(0))
    return (out, probs) if want_probs else out


def attend_mha(q: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.float64)
    H, dh = q.shape
    T = k_bits.shape[1]
    assert k_bits.shape == (H, T, dh) and v_bits.shape == (H, T, dh)
    out = np.empty((H, dh), dtype=np.float64)
    lib().orc_attend_mha(_p(q, np.float64), _p(k_bits, np.uint16), _p(v_bits, np.uint16),
                         ctypes.c_int32(H), ctypes.c_int32(dh), ctypes.c_int32(T),
                         _p(out, np.float64))
    return out


def swiglu(g: np.ndarray, u: np.ndarray) -> np.ndarray:
    g = np.ascontiguousarray(g, dtype=np.float64)
    u = np.ascontiguousarray(u, dtype=np.float64)
    a = np.empty_like(g)
    lib().orc_swiglu(_p(g, np.float64), _p(u, np.float64), ctypes.c_int32(g.shape[0]),
                     _p(a, np.float64))
    return a


def head_logits(x: np.ndarray, gamma_f_bits: np.ndarray, w_vocab: np.ndarray, s_vocab_bits: np.ndarray,
                eps: float) -> np.ndarray:
    """Final LayerNorm + vocabulary projection: x [R, d] fp64 -> logits [R, V] fp64."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    R, d = x.shape
    w = _i8(w_vocab)
    V = w.shape[1]
    assert w.shape == (d, V)
    out = np.empty((R, V), dtype=np.float64)
    gamma, scales = _bits(gamma_f_bits), _bits(s_vocab_bits)  # (kept alive across the call)
    assert gamma.shape == (d,) and scales.shape == (V,)
    lib().orc_head_logits(_p(x, np.float64), _p(gamma, np.uint16), _p(w, np.int8),
                          _p(scales, np.uint16), ctypes.c_int32(R), ctypes.c_int32(d),
                          ctypes.c_int32(V), ctypes.c_double(eps), _p(out, np.float64))
    return out


def sample_topk_topp(logits: np.ndarray, k: int, top_p: float, temperature: float, u: float):
    """One token from logits [V]: returns (token, kept entries, margin of the draw)."""
    logits = np.ascontiguousarray(logits, dtype=np.float64)
    assert logits.ndim == 1
    tok, kept, margin = ctypes.c_int32(-1), ctypes.c_int32(0), ctypes.c_double(0.0)
    rc = lib().orc_sample_topk_topp(_p(logits, np.float64), ctypes.c_int32(logits.shape[0]), ctypes.c_int32(k),
                                    ctypes.c_double(top_p), ctypes.c_double(temperature), ctypes.c_double(u),
                                    ctypes.byref(tok), ctypes.byref(kept), ctypes.byref(margin))
    if rc != 0:
        raise ValueError("oracle sample_topk_topp: bad argument")
    return tok.value, kept.value, margin.value


# ------------------------------------------------------------------ layers ---

def _bits(t) -> np.ndarray:
    """bf16 torch tensor or uint16 array -> uint16 bit array (C-contiguous)."""
    if isinstance(t, np.ndarray):
        return np.ascontiguousarray(t, dtype=np.uint16)
    import torch
    assert t.dtype == torch.bfloat16
    return np.ascontiguousarray(t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16))


def _i8(t) -> np.ndarray:
    if isinstance(t, np.ndarray):
        return np.ascontiguousarray(t, dtype=np.int8)
    return np.ascontiguousarray(t.detach().cpu().contiguous().numpy())


def decode_layer(desc: _Desc, weights: dict, kc: np.ndarray, vc: np.ndarray,
                 positions: Sequence[int], x: np.ndarray, l_ctx: int,
                 cache_row: Optional[Sequence[int]] = None, add_residual: bool = True) -> None:
    """One layer of one decode step, in place on `x` [R, d] fp64 and on the
    layer's cache `kc`, `vc` ([rows, L_ctx, d_head] uint16, canonical layout)."""
    R = x.shape[0]
    pos = np.ascontiguousarray(positions, dtype=np.int32)
    rows = np.arange(R, dtype=np.int32) if cache_row is None else np.ascontiguousarray(cache_row, dtype=np.int32)
    assert pos.shape == (R,) and rows.shape == (R,)
    G = desc.n_kv_heads
    tail = (l_ctx, desc.d_head) if G == 1 else (G, l_ctx, desc.d_head)
    assert kc.shape[1:] == tail and vc.shape == kc.shape, (kc.shape, tail)
    assert rows.max() < kc.shape[0]
    n_in = desc.n_heads * desc.d_head + 2 * G * desc.d_head + 2 * desc.d_ff
    k_out = desc.n_heads * desc.d_head + desc.d_ff
    gamma = _bits(weights["gamma"])
    if "s_in" not in weights:  # bf16 weights, no scales (Section 4.4 baseline)
        w_in, w_out = _bits(weights["w_in"]), _bits(weights["w_out"])
        assert w_in.shape == (desc.d_model, n_in) and w_out.shape == (k_out, desc.d_model)
        rc = lib().orc_decode_layer_w16(ctypes.byref(desc), _p(w_in, np.uint16), _p(w_out, np.uint16),
                                        _p(gamma, np.uint16), _p(kc, np.uint16), _p(vc, np.uint16),
                                        _p(rows, np.int32), _p(pos, np.int32), ctypes.c_int32(R),
                                        ctypes.c_int32(l_ctx), _p(x, np.float64),
                                        ctypes.c_int32(1 if add_residual else 0))
        if rc != 0:
            raise ValueError("oracle decode_layer (bf16 weights): bad argument")
        return
    w_in, w_out = _i8(weights["w_in"]), _i8(weights["w_out"])
    s_in, s_out = _bits(weights["s_in"]), _bits(weights["s_out"])
    assert w_in.shape == (desc.d_model, n_in) and w_out.shape == (k_out, desc.d_model)
    rc = lib().orc_decode_layer(ctypes.byref(desc), _p(w_in, np.int8), _p(s_in, np.uint16),
                                _p(w_out, np.int8), _p(s_out, np.uint16), _p(gamma, np.uint16),
                                _p(kc, np.uint16), _p(vc, np.uint16), _p(rows, np.int32),
                                _p(pos, np.int32), ctypes.c_int32(R), ctypes.c_int32(l_ctx),
                                _p(x, np.float64), ctypes.c_int32(1 if add_residual else 0))
    if rc != 0:
        raise ValueError("oracle decode_layer: bad argument")


def decode_step(desc: _Desc, layers, kcs, vcs, positions, x_bits: np.ndarray, l_ctx: int,
                cache_row=None):
    """Whole stack: `layers`, `kcs`, `vcs` are per-layer iterables (weights may be
    produced lazily, one layer at a time).  x_bits [R, d] bf16 bits in; returns
    (bf16 bits of the hidden state after the last layer, rounded once at the
    end; the same state in fp64 before that rounding)."""
    x = bf16_bits_to_f64_fast(x_bits)
    for wts, kc, vc in zip(layers, kcs, vcs):
        decode_layer(desc, wts, kc, vc, positions, x, l_ctx, cache_row)
    return f64_to_bf16_bits(x), x


def causal_layer(desc: _Desc, weights: dict, x: np.ndarray) -> None:
    """Prefill-style layer over T tokens of one sequence, in place on x [T, d]."""
    T = x.shape[0]
    w_in, w_out = _i8(weights["w_in"]), _i8(weights["w_out"])
    s_in, s_out, gamma = _bits(weights["s_in"]), _bits(weights["s_out"]), _bits(weights["gamma"])
    rc = lib().orc_causal_layer(ctypes.byref(desc), _p(w_in, np.int8), _p(s_in, np.uint16),
                                _p(w_out, np.int8), _p(s_out, np.uint16), _p(gamma, np.uint16),
                                ctypes.c_int32(T), _p(x, np.float64))
    if rc != 0:
        raise ValueError("oracle causal_layer: bad argument")


def bf16_bits_to_f64_fast(bits: np.ndarray) -> np.ndarray:
    """Bulk widening (exact): bf16 bits are the top half of an fp32."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
