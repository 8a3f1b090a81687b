"""Pins of the fp64 CPU oracle against things other than itself.

Each test is chosen so that a plausible slip in palm_oracle.c (dropped term,
wrong sign or index, transposed operand, wrong position, read past the live
slots) fails at least one of them.  No GPU, no HIP library.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from workloads import WORKLOADS, synth
from workloads.configs import Workload

RNG = np.random.default_rng(20221105)


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def rand_bf16(*shape, scale=1.0) -> np.ndarray:
    """bf16 bit patterns of N(0, scale) draws."""
    return bits_of((torch.from_numpy(RNG.standard_normal(shape)).float() * scale).to(torch.bfloat16))


def widen(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ------------------------------------------------------------------ bf16 ---

def test_bf16_rounding_matches_library_on_fp32_inputs():
    # torch rounds fp32 -> bf16 to nearest even; fp32 inputs are exact in fp64
    v = torch.from_numpy(RNG.standard_normal(20000).astype(np.float32)) * 37.0
    ties = torch.tensor([1.00390625, 1.01171875, -1.00390625, 255.5, 256.0 + 1.0, 3.0e38, 1e-40, 0.0])
    v = torch.cat([v, ties])
    want = bits_of(v.to(torch.bfloat16))
    got = oracle.f64_to_bf16_bits(v.double().numpy())
    assert np.array_equal(got, want)


def test_bf16_rounding_is_single_rounding():
    # just above a tie: rounding through fp32 first would land ON the tie and go down
    v = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert oracle.f64_to_bf16_bits(np.array([v]))[0] == 0x3F81
    assert oracle.f64_to_bf16_bits(np.array([-v]))[0] == 0xBF81


def test_bf16_widening_exact():
    bits = np.array([0x3F80, 0xC000, 0x0001, 0x7F7F, 0x0000, 0x8000], dtype=np.uint16)
    got = oracle.bf16_bits_to_f64(bits)
    assert np.array_equal(got, widen(bits))
    assert got[0] == 1.0 and got[1] == -2.0


# ------------------------------------------------- pieces vs library code ---

def test_layernorm_vs_numpy_moments():
    d = 200
    x = RNG.standard_normal(d) * 3.0 + 1.5
    gamma = rand_bf16(d) | 0  # arbitrary gains, including negative ones
    h = oracle.layernorm(x, gamma, 1e-6)
    g = widen(gamma)
    # invert the gain: the normalised vector has mean 0 and variance var/(var+eps)
    n = h / g
    assert abs(n.mean()) < 1e-12
    assert abs(n.var() - x.var() / (x.var() + 1e-6)) < 1e-12
    # library moments (np.mean / np.var are population moments)
    want = g * (x - np.mean(x)) / np.sqrt(np.var(x) + 1e-6)
    np.testing.assert_allclose(h, want, rtol=1e-12, atol=1e-13)


def test_layernorm_eps_is_inside_the_root():
    d = 64
    x = np.full(d, 2.5)  # zero variance: output must be exactly 0, not NaN
    h = oracle.layernorm(x, rand_bf16(d), 1e-6)
    assert np.array_equal(h, np.zeros(d))
    x = RNG.standard_normal(d) * 1e-4  # eps matters here
    g = np.full(d, 0x3F80, dtype=np.uint16)
    h = oracle.layernorm(x, g, 1e-6)
    assert abs(np.var(h) - np.var(x) / (np.var(x) + 1e-6)) < 1e-12


def test_qmatmul_vs_numpy_matmul():
    R, K, N = 3, 160, 700  # N spans more than one column block of the oracle and a ragged tail
    a = RNG.standard_normal((R, K))
    q8 = RNG.integers(-127, 128, size=(K, N), dtype=np.int8)
    s = rand_bf16(N, scale=1e-3)
    want = (a @ q8.astype(np.float64)) * widen(s)[None, :]
    got = oracle.qmatmul(a, q8, s)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_qmatmul_operand_orientation():
    # one-hot activation picks out ONE weight row; the scale belongs to the column
    K, N = 8, 5
    q8 = np.arange(K * N, dtype=np.int8).reshape(K, N)
    s = bits_of(torch.tensor([1.0, 2.0, 4.0, 8.0, 16.0]).to(torch.bfloat16))
    a = np.zeros((1, K))
    a[0, 3] = 1.0
    got = oracle.qmatmul(a, q8, s)[0]
    assert np.array_equal(got, q8[3].astype(np.float64) * np.array([1, 2, 4, 8, 16.0]))


def test_qmatmul_exact_integers():
    # integer activations, power-of-two scales: every partial sum is an integer
    # below 2^53, so the result is exact and must equal integer arithmetic
    R, K, N = 4, 4096, 96
    a = RNG.integers(-2, 3, size=(R, K)).astype(np.float64)
    q8 = RNG.integers(-127, 128, size=(K, N), dtype=np.int8)
    exps = RNG.integers(-8, 3, size=N)
    s = bits_of(torch.tensor(2.0 ** exps).to(torch.bfloat16))
    want = (a.astype(np.int64) @ q8.astype(np.int64)).astype(np.float64) * (2.0 ** exps)[None, :]
    assert np.array_equal(oracle.qmatmul(a, q8, s), want)


def test_swiglu_vs_scipy_expit():
    from scipy.special import expit
    g = RNG.standard_normal(300) * 4
    u = RNG.standard_normal(300)
    np.testing.assert_allclose(oracle.swiglu(g, u), g * expit(g) * u, rtol=1e-13, atol=1e-15)
    # closed forms: swish(0) = 0; swish(z) -> z for large z, -> 0 for very negative z
    assert oracle.swiglu(np.array([0.0]), np.array([3.0]))[0] == 0.0
    assert abs(oracle.swiglu(np.array([40.0]), np.array([1.0]))[0] - 40.0) < 1e-12
    assert abs(oracle.swiglu(np.array([-40.0]), np.array([1.0]))[0]) < 1e-12
    # the gate is the FIRST argument: swapping must change the result
    assert not np.allclose(oracle.swiglu(g, u), oracle.swiglu(u, g))


# ------------------------------------------------------------------ RoPE ---

def test_rope_position_zero_is_identity_and_norm_is_kept():
    y = RNG.standard_normal(64)
    assert np.array_equal(oracle.rope(y, 0, 10000.0), y)
    for p in (1, 17, 2047, 8191):
        r = oracle.rope(y, p, 10000.0)
        assert abs(np.linalg.norm(r) - np.linalg.norm(y)) < 1e-12
        assert not np.allclose(r, y)


def test_rope_closed_form_unit_vectors():
    dh, base, p = 16, 10000.0, 5
    half = dh // 2
    for i in (0, 3, half - 1):
        theta = base ** (-2.0 * i / dh)
        e = np.zeros(dh)
        e[i] = 1.0  # first element of pair i
        r = oracle.rope(e, p, base)
        want = np.zeros(dh)
        want[i], want[i + half] = math.cos(p * theta), math.sin(p * theta)
        np.testing.assert_allclose(r, want, atol=1e-15)
        e = np.zeros(dh)
        e[i + half] = 1.0  # second element of pair i
        r = oracle.rope(e, p, base)
        want = np.zeros(dh)
        want[i], want[i + half] = -math.sin(p * theta), math.cos(p * theta)
        np.testing.assert_allclose(r, want, atol=1e-15)
    # pair 0 turns by exactly `p` radians; the slowest pair by p * base^(-(dh-2)/dh)
    assert abs(oracle.rope(np.eye(dh)[0], 1, base)[0] - math.cos(1.0)) < 1e-15


def test_rope_scores_depend_on_relative_position_only():
    dh = 64
    q, k = RNG.standard_normal(dh), RNG.standard_normal(dh)
    base = 10000.0
    ref = oracle.rope(q, 40, base) @ oracle.rope(k, 33, base)
    for c in (1, 100, 4000):
        assert abs(oracle.rope(q, 40 + c, base) @ oracle.rope(k, 33 + c, base) - ref) < 1e-9
    assert abs(oracle.rope(q, 41, base) @ oracle.rope(k, 33, base) - ref) > 1e-6


# ------------------------------------------------------------- attention ---

def test_softmax_rows_sum_to_one_and_are_nonnegative():
    H, dh, T = 4, 64, 300
    q = RNG.standard_normal((H, dh)) * 3
    K, V = rand_bf16(T, dh), rand_bf16(T, dh)
    _, p = oracle.attend_mqa(q, K, V, want_probs=True)
    assert p.shape == (H, T)
    assert np.all(p >= 0)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-12)


def test_attention_vs_numpy_softmax():
    H, dh, T = 3, 32, 50
    q = RNG.standard_normal((H, dh))
    K, V = rand_bf16(T, dh), rand_bf16(T, dh)
    s = q @ widen(K).T / math.sqrt(dh)
    p = np.exp(s - s.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    out, probs = oracle.attend_mqa(q, K, V, want_probs=True)
    np.testing.assert_allclose(probs, p, atol=1e-14)
    np.testing.assert_allclose(out, p @ widen(V), atol=1e-13)


def test_multiquery_equals_multihead_with_replicated_kv():
    # Section 3.3: the single K/V head is shared by all query heads
    H, dh, T = 5, 64, 77
    q = RNG.standard_normal((H, dh))
    K, V = rand_bf16(T, dh), rand_bf16(T, dh)
    mqa = oracle.attend_mqa(q, K, V)
    mha = oracle.attend_mha(q, np.ascontiguousarray(np.broadcast_to(K, (H, T, dh))),
                            np.ascontiguousarray(np.broadcast_to(V, (H, T, dh))))
    np.testing.assert_allclose(mqa, mha, atol=1e-12)
    # and multihead really uses per-head K/V: perturbing head 2's keys moves only head 2
    K3 = np.ascontiguousarray(np.broadcast_to(K, (H, T, dh))).copy()
    K3[2] = rand_bf16(T, dh)
    mha2 = oracle.attend_mha(q, K3, np.ascontiguousarray(np.broadcast_to(V, (H, T, dh))))
    assert np.allclose(np.delete(mha2, 2, axis=0), np.delete(mha, 2, axis=0), atol=1e-12)
    assert not np.allclose(mha2[2], mha[2])


def test_single_slot_attention_returns_v_exactly():
    H, dh = 4, 64
    q = RNG.standard_normal((H, dh)) * 10
    K, V = rand_bf16(1, dh), rand_bf16(1, dh)
    out = oracle.attend_mqa(q, K, V)
    for j in range(H):
        assert np.array_equal(out[j], widen(V)[0])


def test_equal_keys_give_the_mean_of_v_and_a_dominant_key_selects_its_row():
    H, dh, T = 2, 32, 40
    q = RNG.standard_normal((H, dh))
    K = np.repeat(rand_bf16(1, dh), T, axis=0)
    V = rand_bf16(T, dh)
    out = oracle.attend_mqa(q, K, V)
    np.testing.assert_allclose(out, np.broadcast_to(widen(V).mean(axis=0), (H, dh)), atol=1e-13)
    # one key aligned with q_0 and large
    K = rand_bf16(T, dh, scale=0.01)
    big = bits_of(torch.from_numpy(q[0] * 50).to(torch.bfloat16))
    K[17] = big
    out = oracle.attend_mqa(q, K, V)
    np.testing.assert_allclose(out[0], widen(V)[17], atol=1e-9)


# ------------------------------------------------------- layer-level pins ---

TINY = Workload("pin", 2, 64, 2, 16, 128, 1, 16)


def tiny_layers(w=TINY, seed=7):
    return [synth.layer_weights(w, l, seed=seed) for l in range(w.n_layers)]


def empty_cache(w, rows, fill=0x7FC0):
    """NaN-poisoned cache: any read of a slot that was never written shows up."""
    return [np.full((rows, w.l_ctx, w.d_head), fill, dtype=np.uint16) for _ in range(w.n_layers)]


def test_decode_steps_equal_rows_of_a_causal_forward():
    # Section 2.2: decode continues the same forward pass prefill runs in parallel
    w, T = TINY, 9
    desc = oracle.make_desc(w)
    layers = tiny_layers()
    X = RNG.standard_normal((T, w.d_model))
    full = X.copy()
    for l in range(w.n_layers):
        oracle.causal_layer(desc, layers[l], full)
    kcs, vcs = empty_cache(w, 1), empty_cache(w, 1)
    for t in range(T):
        x = X[t:t + 1].copy()
        for l in range(w.n_layers):
            oracle.decode_layer(desc, layers[l], kcs[l], vcs[l], [t], x, w.l_ctx)
        assert np.all(np.isfinite(x))
        np.testing.assert_allclose(x[0], full[t], rtol=1e-10, atol=1e-11)
    # the steps wrote slots 0..T-1 and nothing else
    for l in range(w.n_layers):
        assert np.all(kcs[l][0, T:] == 0x7FC0) and np.all(vcs[l][0, T:] == 0x7FC0)
        assert not np.any(kcs[l][0, :T] == 0x7FC0)


def test_append_touches_exactly_one_slot_per_row():
    w = TINY.with_(n_layers=1)
    desc = oracle.make_desc(w)
    layer = tiny_layers(w)[0]
    rows, pos = 3, [4, 0, 15]
    kc = rand_bf16(rows, w.l_ctx, w.d_head)
    vc = rand_bf16(rows, w.l_ctx, w.d_head)
    k0, v0 = kc.copy(), vc.copy()
    x = RNG.standard_normal((rows, w.d_model))
    oracle.decode_layer(desc, layer, kc, vc, pos, x, w.l_ctx)
    changed_k = np.argwhere((kc != k0).any(axis=2))
    changed_v = np.argwhere((vc != v0).any(axis=2))
    want = np.array([[r, p] for r, p in enumerate(pos)])
    assert np.array_equal(changed_k, want) and np.array_equal(changed_v, want)


def test_slots_beyond_the_position_are_never_read():
    w = TINY.with_(n_layers=1)
    desc = oracle.make_desc(w)
    layer = tiny_layers(w)[0]
    kc, vc = rand_bf16(1, w.l_ctx, w.d_head), rand_bf16(1, w.l_ctx, w.d_head)
    x0 = RNG.standard_normal((1, w.d_model))
    a = x0.copy()
    oracle.decode_layer(desc, layer, kc.copy(), vc.copy(), [6], a, w.l_ctx)
    kc[:, 7:], vc[:, 7:] = 0x7FC0, 0x7F80  # NaN keys, +inf values past the position
    b = x0.copy()
    oracle.decode_layer(desc, layer, kc, vc, [6], b, w.l_ctx)
    assert np.array_equal(a, b) and np.all(np.isfinite(b))


def test_zero_output_projection_leaves_the_residual_untouched():
    w = TINY.with_(n_layers=1)
    desc = oracle.make_desc(w)
    layer = dict(tiny_layers(w)[0])
    layer["w_out"] = torch.zeros_like(layer["w_out"])
    x0 = RNG.standard_normal((2, w.d_model))
    x = x0.copy()
    kc, vc = rand_bf16(2, w.l_ctx, w.d_head), rand_bf16(2, w.l_ctx, w.d_head)
    oracle.decode_layer(desc, layer, kc, vc, [0, 3], x, w.l_ctx)
    assert np.array_equal(x, x0)


def _compose_layer_from_pieces(w, layer, kc, vc, pos, x_row, ffn=True, attn=True):
    """The block x + Attn(LN x) + FFN(LN x) (Section 3.4) assembled in the test
    from separately pinned pieces, with the column split written out here."""
    H, dh, F = w.n_heads, w.d_head, w.d_ff
    g = bits_of(layer["gamma"])
    h = oracle.layernorm(x_row, g, w.ln_eps)
    z = oracle.qmatmul(h[None, :], layer["w_in"].numpy(), bits_of(layer["s_in"]))[0]
    q = z[:H * dh].reshape(H, dh)
    k, v = z[H * dh:H * dh + dh], z[H * dh + dh:H * dh + 2 * dh]
    gate, up = z[H * dh + 2 * dh:H * dh + 2 * dh + F], z[H * dh + 2 * dh + F:]
    qr = np.stack([oracle.rope(q[j], pos, w.rope_base) for j in range(H)])
    K = kc[:pos + 1].copy()
    V = vc[:pos + 1].copy()
    K[pos] = oracle.f64_to_bf16_bits(oracle.rope(k, pos, w.rope_base))
    V[pos] = oracle.f64_to_bf16_bits(v)
    o = oracle.attend_mqa(qr, K, V).reshape(-1) if attn else np.zeros(H * dh)
    a = oracle.swiglu(gate, up) if ffn else np.zeros(F)
    y = oracle.qmatmul(np.concatenate([o, a])[None, :], layer["w_out"].numpy(), bits_of(layer["s_out"]))[0]
    return x_row + y


def test_layer_wiring_against_composition_of_pinned_pieces():
    w = TINY.with_(n_layers=1)
    desc = oracle.make_desc(w)
    layer = tiny_layers(w)[0]
    kc, vc = rand_bf16(1, w.l_ctx, w.d_head), rand_bf16(1, w.l_ctx, w.d_head)
    x0 = RNG.standard_normal((1, w.d_model))
    want = _compose_layer_from_pieces(w, layer, kc[0], vc[0], 5, x0[0])
    x = x0.copy()
    oracle.decode_layer(desc, layer, kc, vc, [5], x, w.l_ctx)
    np.testing.assert_allclose(x[0], want, rtol=1e-12, atol=1e-13)


def test_zero_gate_columns_remove_the_ffn_branch():
    w = TINY.with_(n_layers=1)
    desc = oracle.make_desc(w)
    layer = dict(tiny_layers(w)[0])
    H, dh, F = w.n_heads, w.d_head, w.d_ff
    w_in = layer["w_in"].clone()
    w_in[:, H * dh + 2 * dh:H * dh + 2 * dh + F] = 0  # gate columns
    layer["w_in"] = w_in
    kc, vc = rand_bf16(1, w.l_ctx, w.d_head), rand_bf16(1, w.l_ctx, w.d_head)
    x0 = RNG.standard_normal((1, w.d_model))
    want = _compose_layer_from_pieces(w, layer, kc[0], vc[0], 9, x0[0], ffn=False)
    x = x0.copy()
    oracle.decode_layer(desc, layer, kc, vc, [9], x, w.l_ctx)
    np.testing.assert_allclose(x[0], want, rtol=1e-12, atol=1e-13)
    # zeroing the UP columns instead must also kill the branch (a = swish(g) * 0)
    layer2 = dict(tiny_layers(w)[0])
    w_in = layer2["w_in"].clone()
    w_in[:, H * dh + 2 * dh + F:] = 0
    layer2["w_in"] = w_in
    x2 = x0.copy()
    oracle.decode_layer(desc, layer2, kc.copy(), vc.copy(), [9], x2, w.l_ctx)
    want2 = _compose_layer_from_pieces(w, layer2, kc[0], vc[0], 9, x0[0], ffn=False)
    np.testing.assert_allclose(x2[0], want2, rtol=1e-12, atol=1e-13)


def test_position_zero_attention_is_the_rounded_value_vector():
    # with P_b = 0 the only live slot is the one just appended: every head returns bf16(v)
    w = TINY.with_(n_layers=1)
    desc = oracle.make_desc(w)
    layer = dict(tiny_layers(w)[0])
    H, dh, F = w.n_heads, w.d_head, w.d_ff
    w_in = layer["w_in"].clone()
    w_in[:, H * dh + 2 * dh:] = 0  # no FFN
    layer["w_in"] = w_in
    kc, vc = empty_cache(w, 1)[0], empty_cache(w, 1)[0]
    x0 = RNG.standard_normal((1, w.d_model))
    x = x0.copy()
    oracle.decode_layer(desc, layer, kc, vc, [0], x, w.l_ctx, add_residual=False)
    v_bits = vc[0, 0]
    o = np.tile(widen(v_bits), H)
    want = oracle.qmatmul(np.concatenate([o, np.zeros(F)])[None, :], layer["w_out"].numpy(),
                          bits_of(layer["s_out"]))[0]
    np.testing.assert_allclose(x[0], want, rtol=1e-12, atol=1e-14)


def test_rows_are_independent_and_cache_rows_are_honoured():
    w = TINY.with_(n_layers=1)
    desc = oracle.make_desc(w)
    layer = tiny_layers(w)[0]
    kc, vc = rand_bf16(4, w.l_ctx, w.d_head), rand_bf16(4, w.l_ctx, w.d_head)
    X = RNG.standard_normal((4, w.d_model))
    pos = [3, 8, 0, 15]
    full = X.copy()
    oracle.decode_layer(desc, layer, kc.copy(), vc.copy(), pos, full, w.l_ctx)
    sub = X[[2, 1]].copy()  # a row subset against the same cache rows
    oracle.decode_layer(desc, layer, kc.copy(), vc.copy(), [pos[2], pos[1]], sub, w.l_ctx, cache_row=[2, 1])
    assert np.array_equal(sub, full[[2, 1]])


# ------------------------------------------------------------- quantiser ---

def test_quantiser_invariants():
    w = torch.from_numpy(RNG.standard_normal((300, 50)).astype(np.float32)) * 0.02
    w[:, 7] = 0.0
    q, s = synth.quantize_per_channel(w)
    assert q.dtype == torch.int8 and s.dtype == torch.bfloat16 and s.shape == (50,)
    assert int(q.min()) >= -127  # -128 is never produced
    nz = [c for c in range(50) if c != 7]
    assert all(int(q[:, c].abs().max()) == 127 for c in nz)
    assert float(s[7]) == 1.0 and int(q[:, 7].abs().max()) == 0
    err = (w - q.float() * s.float()).abs()
    # half a step, plus the slack bf16 rounding of the scale leaves at the clamp
    assert torch.all(err[:, nz] <= 0.5 * s.float()[nz] + 0.25 * s.float()[nz] + 1e-12)
    inner = q.abs() < 127
    assert torch.all(err[inner] <= (0.5 * s.float()[None, :].expand_as(err))[inner] * (1 + 1e-6))
    q2, s2 = synth.quantize_per_channel(q.float() * s.float())
    assert torch.equal(q2[:, nz], q[:, nz]) and torch.equal(s2[nz], s[nz])


def test_synthetic_streams_are_reproducible_and_independent():
    w = WORKLOADS["c1_tiny"]
    a, b = synth.layer_weights(w, 0), synth.layer_weights(w, 0)
    assert all(torch.equal(a[k], b[k]) for k in a)
    c = synth.layer_weights(w.with_(n_layers=2), 1)
    assert not torch.equal(a["w_in"], c["w_in"])
    assert abs(float(a["w_in"].float().std()) - 127 / 3.0) < 12  # absmax of ~256 normal draws ~ 3 sigma
    p = synth.positions(WORKLOADS["c5_62b_long"])
    assert p.shape == (256,) and int(p.min()) >= 4096 and int(p.max()) < 8192
    assert torch.equal(p, synth.positions(WORKLOADS["c5_62b_long"]))


# ------------------------------------------------- sampling head (Section 2.2) ---

def _np_sample(logits, k, top_p, temperature, u):
    """The same definition through numpy's library routines (stable argsort, cumsum,
    searchsorted): an independent route to the token."""
    order = np.argsort(-logits, kind="stable")[:k]          # largest first, ties by smaller index
    z = logits[order] / temperature
    p = np.exp(z - z.max())
    p /= p.sum()
    c = np.cumsum(p)
    n = int(np.searchsorted(c, top_p, side="left")) + 1       # shortest prefix with sum >= top_p
    n = min(n, k)
    c = np.cumsum(p[:n])
    i = int(np.searchsorted(c, u * c[-1], side="right"))     # first entry with running sum > target
    return int(order[min(i, n - 1)]), n


def test_sampler_vs_numpy_sort_and_cumsum():
    rng = np.random.default_rng(17)
    checked = 0
    for trial in range(300):
        V = int(rng.integers(1, 400))
        k = int(rng.integers(1, min(V, 64) + 1))
        top_p = float(rng.uniform(0.05, 1.0))
        T = float(rng.uniform(0.2, 2.0))
        u = float(rng.uniform(0, 1))
        logits = rng.standard_normal(V) * 3
        if trial % 5 == 0:
            logits = np.round(logits)  # many exact ties
        tok, kept, margin = oracle.sample_topk_topp(logits, k, top_p, T, u)
        want, n = _np_sample(logits, k, top_p, T, u)
        if margin > 1e-9:  # away from an interval boundary the two routes must agree exactly
            assert (tok, kept) == (want, n), (trial, V, k, top_p, T, u)
            checked += 1
    assert checked > 280


def test_sampler_degenerate_cases_are_argmax():
    rng = np.random.default_rng(3)
    logits = rng.standard_normal(1000)
    logits[[100, 700]] = logits.max() + 1.0  # tie for the maximum: the smaller index wins
    for u in (0.0, 0.3, 0.999999):
        assert oracle.sample_topk_topp(logits, 1, 1.0, 1.0, u)[0] == 100          # k = 1
        assert oracle.sample_topk_topp(logits, 50, 1e-9, 1.0, u)[:2] == (100, 1)  # top_p -> 0
    logits[700] -= 0.5
    for u in (0.0, 0.5, 0.99):
        assert oracle.sample_topk_topp(logits, 50, 1.0, 1e-3, u)[0] == 100        # temperature -> 0


def test_sampler_uniform_logits_invert_the_uniform_cdf():
    V = 37
    logits = np.full(V, 1.25)
    for u in np.linspace(0.0, 0.999, 101):
        tok, kept, _ = oracle.sample_topk_topp(logits, V, 1.0, 0.7, float(u))
        frac = u * V
        if abs(frac - round(frac)) > 1e-9:
            assert tok == int(math.floor(frac)) and kept == V


def test_sampler_two_tokens_closed_form_and_temperature():
    a, b = 0.3, 1.1
    for T in (0.5, 1.0, 2.0):
        p_b = 1.0 / (1.0 + math.exp((a - b) / T))  # larger logit comes first in the order
        for u in np.linspace(0.001, 0.999, 200):
            tok = oracle.sample_topk_topp(np.array([a, b]), 2, 1.0, T, float(u))[0]
            if abs(u - p_b) > 1e-9:
                assert tok == (1 if u < p_b else 0), (T, u)


def test_sampler_nucleus_keeps_the_shortest_prefix_and_renormalises():
    logits = np.log(np.array([0.2, 0.5, 0.3]))
    assert oracle.sample_topk_topp(logits, 3, 0.79, 1.0, 0.1)[1] == 2  # 0.5 + 0.3 reaches 0.79
    assert oracle.sample_topk_topp(logits, 3, 0.81, 1.0, 0.1)[1] == 3
    assert oracle.sample_topk_topp(logits, 3, 0.49, 1.0, 0.1)[1] == 1
    # inside the nucleus {0.5, 0.3} the draw uses the renormalised 0.625 / 0.375
    assert oracle.sample_topk_topp(logits, 3, 0.79, 1.0, 0.62)[0] == 1
    assert oracle.sample_topk_topp(logits, 3, 0.79, 1.0, 0.63)[0] == 2
    # top-k cuts before top-p
    assert oracle.sample_topk_topp(logits, 1, 1.0, 1.0, 0.99)[:2] == (1, 1)


def test_sampler_frequencies_follow_the_softmax():
    rng = np.random.default_rng(5)
    logits = rng.standard_normal(12)
    T, N = 0.8, 20000
    counts = np.zeros(12)
    for i in range(N):
        counts[oracle.sample_topk_topp(logits, 12, 1.0, T, (i + 0.5) / N)[0]] += 1
    p = np.exp(logits / T)
    p /= p.sum()
    assert np.max(np.abs(counts / N - p)) <= 1.5 / N * 12  # each interval end moves the count by at most one


def test_sampler_rejects_bad_arguments():
    for bad in ((0, 1.0, 1.0, 0.5), (4, 1.0, 1.0, 0.5), (1, 0.0, 1.0, 0.5), (1, 1.0, 0.0, 0.5), (1, 1.0, 1.0, 1.0)):
        with pytest.raises(ValueError):
            oracle.sample_topk_topp(np.zeros(3), *bad)


def test_head_logits_are_layernorm_then_projection():
    rng = np.random.default_rng(9)
    R, d, V = 3, 96, 50
    x = rng.standard_normal((R, d)) * 7 + 0.3
    gamma = torch.tensor(1 + 0.05 * rng.standard_normal(d)).to(torch.bfloat16)
    w = torch.tensor(rng.integers(-127, 128, (d, V)), dtype=torch.int8)
    s = torch.tensor(rng.uniform(1e-3, 2e-3, V)).to(torch.bfloat16)
    got = oracle.head_logits(x, gamma, w, s, 1e-6)
    g64, s64 = gamma.double().numpy(), s.double().numpy()
    mu = x.mean(axis=1, keepdims=True)
    h = g64 * (x - mu) / np.sqrt(((x - mu) ** 2).mean(axis=1, keepdims=True) + 1e-6)
    want = (h @ w.double().numpy()) * s64
    assert np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want))


# ------------------------------------------ multihead variant (Section 3.3, 4.2) ---

def _mha_inputs(seed=21):
    rng = np.random.default_rng(seed)
    H, dh, d, F, L, R = 3, 8, 32, 16, 12, 2
    mq = Workload("mq", 1, d, H, dh, F, R, L)
    mh = mq.with_(n_kv_heads=H)
    w_mq = synth.layer_weights(mq, 0, "cpu")
    # multihead weights whose K and V columns are the multiquery ones copied to every head
    q_cols = w_mq["w_in"][:, :H * dh]
    k_cols = w_mq["w_in"][:, H * dh:H * dh + dh]
    v_cols = w_mq["w_in"][:, H * dh + dh:H * dh + 2 * dh]
    ffn = w_mq["w_in"][:, H * dh + 2 * dh:]
    s = w_mq["s_in"]
    w_mh = dict(w_mq)
    w_mh["w_in"] = torch.cat([q_cols] + [k_cols] * H + [v_cols] * H + [ffn], dim=1).contiguous()
    w_mh["s_in"] = torch.cat([s[:H * dh]] + [s[H * dh:H * dh + dh]] * H + [s[H * dh + dh:H * dh + 2 * dh]] * H
                             + [s[H * dh + 2 * dh:]]).contiguous()
    kc = rng.integers(0x3c00, 0x4000, (R, L, dh)).astype(np.uint16)
    vc = rng.integers(0xbc00, 0xc000, (R, L, dh)).astype(np.uint16)
    x = rng.standard_normal((R, d))
    pos = np.array([5, 11], dtype=np.int32)
    return mq, mh, w_mq, w_mh, kc, vc, x, pos, H


def test_multihead_layer_with_replicated_kv_equals_multiquery_layer():
    mq, mh, w_mq, w_mh, kc, vc, x, pos, H = _mha_inputs()
    x1, k1, v1 = x.copy(), kc.copy(), vc.copy()
    oracle.decode_layer(oracle.make_desc(mq), w_mq, k1, v1, pos, x1, mq.l_ctx)
    x2 = x.copy()
    k2 = np.repeat(kc[:, None], H, axis=1).copy()  # [R, H, L, dh]: every head a copy of the shared one
    v2 = np.repeat(vc[:, None], H, axis=1).copy()
    oracle.decode_layer(oracle.make_desc(mh), w_mh, k2, v2, pos, x2, mh.l_ctx)
    assert np.max(np.abs(x1 - x2)) <= 1e-12 * np.max(np.abs(x1))
    for j in range(H):
        assert np.array_equal(k2[:, j], k1) and np.array_equal(v2[:, j], v1)  # same appended slot in every head


def test_multihead_heads_read_their_own_cache_only():
    _, mh, _, w_mh, kc, vc, x, pos, H = _mha_inputs(22)
    desc = oracle.make_desc(mh)
    # zero output rows for everything but the attention output of head 1: x' - x shows head 1 alone
    wts = dict(w_mh)
    w_out = torch.zeros_like(wts["w_out"])
    dh = mh.d_head
    w_out[dh:2 * dh] = wts["w_out"][dh:2 * dh]
    wts["w_out"] = w_out
    k2 = np.repeat(kc[:, None], H, axis=1).copy()
    v2 = np.repeat(vc[:, None], H, axis=1).copy()
    base = x.copy()
    oracle.decode_layer(desc, wts, k2.copy(), v2.copy(), pos, base, mh.l_ctx)
    for head, changes in ((0, False), (1, True), (2, False)):
        kk, vv = k2.copy(), v2.copy()
        vv[:, head, 2] ^= 0x0100  # perturb one cached value row of that head (a live slot for both rows)
        out = x.copy()
        oracle.decode_layer(desc, wts, kk, vv, pos, out, mh.l_ctx)
        assert (np.max(np.abs(out - base)) > 0) == changes, head


def test_multihead_byte_model_scales_kv_by_heads():
    from workloads import configs as C
    w = Workload("t", 4, 256, 8, 64, 512, 2, 128)
    assert C.kv_read_bytes(w.with_(n_kv_heads=8), [127, 63]) == 8 * C.kv_read_bytes(w, [127, 63])
    assert w.with_(n_kv_heads=8).n_in == w.n_in + 2 * 7 * 64


# ------------------------------------------------------ prefill (Section 2.2) ---

def test_token_rows_sharing_a_cache_row_are_a_causal_forward_pass():
    # the decode layer applied to T token rows of one sequence (all mapped to cache row 0, in
    # position order) is the prefill of those tokens: it must equal the separately written
    # causal [T x T] layer, token by token
    w = Workload("pf", 1, 64, 2, 16, 32, 1, 16)
    wts = synth.layer_weights(w, 0, "cpu")
    desc = oracle.make_desc(w)
    rng = np.random.default_rng(31)
    T = 11
    x = rng.standard_normal((T, w.d_model))
    a = x.copy()
    oracle.causal_layer(desc, wts, a)
    b = x.copy()
    kc = np.full((1, w.l_ctx, w.d_head), 0x7fc0, dtype=np.uint16)  # NaN everywhere: only appended slots may be read
    vc = kc.copy()
    oracle.decode_layer(desc, wts, kc, vc, np.arange(T, dtype=np.int32), b, w.l_ctx,
                        cache_row=np.zeros(T, dtype=np.int32))
    assert np.all(np.isfinite(b))
    assert np.max(np.abs(a - b)) <= 1e-12 * np.max(np.abs(a))


# ------------------------------------------- bf16 weights (Section 4.4 baseline) ---

def test_wmatmul_bf16_vs_numpy_matmul_and_orientation():
    a = RNG.standard_normal((5, 96))
    w = rand_bf16(96, 40, scale=0.05)
    got = oracle.wmatmul_bf16(a, w)
    want = a @ widen(w)
    assert np.max(np.abs(got - want)) <= 1e-13 * np.max(np.abs(want))
    # a one-hot row of `a` picks a row of w, never a column
    e = np.zeros((1, 96)); e[0, 17] = 1.0
    assert np.array_equal(oracle.wmatmul_bf16(e, w)[0], widen(w)[17])


def test_bf16_weight_layer_equals_int8_layer_when_the_weights_coincide():
    # int8 values times a power-of-two scale are exact in bf16 (|q| <= 127 fits the 8-bit
    # significand): the layer with bf16 weights q * 2^-e must equal the int8 layer with scales
    # 2^-e, whatever the wiring between the two projections is
    w = Workload("w16", 1, 128, 2, 64, 256, 3, 64)
    wts = synth.layer_weights(w, 0, "cpu")
    e_in = torch.from_numpy(RNG.integers(6, 10, w.n_in)).float()
    e_out = torch.from_numpy(RNG.integers(6, 10, w.d_model)).float()
    wts["s_in"] = torch.pow(2.0, -e_in).to(torch.bfloat16)
    wts["s_out"] = torch.pow(2.0, -e_out).to(torch.bfloat16)
    w16 = {"w_in": (wts["w_in"].float() * wts["s_in"].float()).to(torch.bfloat16),
           "w_out": (wts["w_out"].float() * wts["s_out"].float()).to(torch.bfloat16),
           "gamma": wts["gamma"]}
    assert torch.equal(w16["w_in"].float(), wts["w_in"].float() * wts["s_in"].float())  # exact
    desc = oracle.make_desc(w)
    kc, vc = (bits_of(t) for t in synth.kv_layer(w, 0, "cpu"))
    pos = np.array([5, 63, 0], dtype=np.int32)
    x = RNG.standard_normal((3, w.d_model))
    xa, ka, va = x.copy(), kc.copy(), vc.copy()
    oracle.decode_layer(desc, wts, ka, va, pos, xa, w.l_ctx)
    xb, kb, vb = x.copy(), kc.copy(), vc.copy()
    oracle.decode_layer(desc, w16, kb, vb, pos, xb, w.l_ctx)
    assert np.max(np.abs(xa - xb)) <= 1e-12 * np.max(np.abs(xa))
    assert np.array_equal(ka, kb) and np.array_equal(va, vb)


def test_bf16_weight_workload_streams_and_byte_model():
    from workloads import configs as C
    w8 = Workload("t", 2, 128, 2, 64, 256, 2, 64)
    w16 = w8.with_(weights="bf16")
    a, b = synth.layer_weights(w16, 1, "cpu"), synth.layer_weights(w16, 1, "cpu")
    assert set(a) == {"w_in", "w_out", "gamma"} and a["w_in"].dtype == torch.bfloat16
    assert torch.equal(a["w_in"], b["w_in"]) and torch.equal(a["gamma"], synth.layer_weights(w8, 1, "cpu")["gamma"])
    assert C.weight_bytes(w16) == 2 * C.weight_bytes(w8)
