"""GPU parity of prefill / incremental prefill (Section 2.2, Section 3.5): many tokens per
sequence in one call, causal attention through the cache, against the fp64 oracle applied
to the same token rows in position order."""
import numpy as np
import pytest
import torch

import oracle
from workloads import synth
from workloads.configs import Workload

pytestmark = pytest.mark.gpu
MAX_SCALED, REL_L2 = 2e-2, 5e-3


@pytest.fixture(scope="module")
def pd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_05102_amd as m
    m.lib()
    return m


def bits_np(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def widen(b):
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


@pytest.mark.parametrize("case", [
    # (layers, d, H, G, dh, F, cache rows, L_ctx, tokens already cached per sequence, new tokens per sequence)
    (2, 256, 4, 1, 64, 512, 3, 128, [0, 0, 0], [40, 7, 1]),          # whole prefill, ragged lengths
    (2, 384, 6, 1, 128, 384, 2, 352, [17, 64], [300, 150]),          # incremental, several 256-row chunks
    (1, 512, 4, 4, 128, 256, 2, 96, [5, 0], [33, 64]),               # multihead K/V
    (2, 256, 4, 1, 64, 384, 2, 320, [3, 0], [290, 40], "bf16"),      # bf16 weights, two chunks
])
def test_prefill_vs_oracle(pd, case):
    from paper_2211_05102_amd import binding
    L_, d, H, G, dh, F, S, L, cached, new = case[:10]
    w = Workload("prefill", L_, d, H, dh, F, S, L, n_kv_heads=G, weights=case[10] if len(case) > 10 else "int8")
    dec = pd.Decoder(w)
    desc_o = oracle.make_desc(w)
    # token rows, interleaved round-robin over the sequences, each sequence in position order
    rows = []
    for i in range(max(new)):
        for s in range(S):
            if i < new[s]:
                rows.append((s, cached[s] + i))
    seq = np.array([r[0] for r in rows], dtype=np.int32)
    pos = np.array([r[1] for r in rows], dtype=np.int32)
    N = len(rows)
    g = torch.Generator(device="cuda").manual_seed(7)
    x = torch.randn(N, d, generator=g, device="cuda").to(torch.bfloat16)

    layer_bytes = binding.packed_layer_bytes(dec.desc)
    packed = torch.empty(L_ * layer_bytes, dtype=torch.uint8, device="cuda")
    kvb = binding.kv_cache_bytes(dec.desc, S, L)
    kc = torch.empty(kvb // 2, dtype=torch.bfloat16, device="cuda")
    vc = torch.empty_like(kc)
    live = torch.arange(L, device="cuda")[None, :] < torch.tensor(cached, device="cuda")[:, None]
    lv = live[:, :, None] if G == 1 else live[:, None, :, None]
    x64 = oracle.bf16_bits_to_f64_fast(bits_np(x))
    k_after, k_before = [], []
    for l in range(L_):
        wts = synth.layer_weights(w, l, "cuda")
        dec.pack_layer(wts, packed[l * layer_bytes:(l + 1) * layer_bytes])
        k, v = synth.kv_layer(w, l, "cuda")
        k = torch.where(lv, k, torch.full_like(k, float("nan")))  # nothing beyond the cached prefix may be read
        v = torch.where(lv, v, torch.full_like(v, float("inf")))
        dec.kv_import(k, kc, l, False)
        dec.kv_import(v, vc, l, True)
        kb, vb = bits_np(k), bits_np(v)
        k_before.append((kb.copy(), vb.copy()))
        oracle.decode_layer(desc_o, {n: t.cpu() for n, t in wts.items()}, kb, vb, pos, x64, L, cache_row=seq)
        k_after.append((kb, vb))
    ws = torch.empty(binding.workspace_bytes(dec.desc, min(N, 256), L), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    out = torch.full((N, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dec.prefill(packed, kc, vc, x, torch.from_numpy(seq).cuda(), torch.from_numpy(pos).cuda(), S, L, out, ws)
    dec.check_async(ws)
    got = widen(bits_np(out))
    want = widen(oracle.f64_to_bf16_bits(x64))
    assert np.all(np.isfinite(got))
    scaled = float(np.max(np.abs(got - want) / np.maximum(1.0, np.abs(want))))
    rel = float(np.linalg.norm(got - want) / np.linalg.norm(want))
    print(f"[prefill] {case}: {N} token rows, scaled-max {scaled:.3e} rel-L2 {rel:.3e}", flush=True)
    assert scaled <= MAX_SCALED and rel <= REL_L2
    # cache: exactly the slots [cached, cached + new) of every sequence (and K/V head) changed,
    # and they hold the oracle's values to a bf16 step
    t = np.arange(L)[None, :]
    want_changed = (t >= np.array(cached)[:, None]) & (t < (np.array(cached) + np.array(new))[:, None])
    shape = (S, L, dh) if G == 1 else (S, G, L, dh)
    for l in range(L_):
        kg = torch.empty(*shape, dtype=torch.bfloat16, device="cuda")
        vg = torch.empty_like(kg)
        dec.kv_export(kc, kg, l, False)
        dec.kv_export(vc, vg, l, True)
        for got_c, (before, after) in ((bits_np(kg), (k_before[l][0], k_after[l][0])),
                                        (bits_np(vg), (k_before[l][1], k_after[l][1]))):
            changed = (got_c != before).any(axis=-1)
            wc = want_changed if G == 1 else np.broadcast_to(want_changed[:, None, :], changed.shape)
            assert np.array_equal(changed, wc), l
            a, b = widen(got_c[changed]), widen(after[changed])
            assert np.max(np.abs(a - b) / np.maximum(1.0, np.abs(b))) <= MAX_SCALED


def test_prefill_flags_bad_sequence_ids(pd):
    from paper_2211_05102_amd import binding
    w = Workload("pfbad", 1, 256, 4, 64, 256, 2, 64)
    dec = pd.Decoder(w)
    packed = torch.empty(binding.packed_layer_bytes(dec.desc), dtype=torch.uint8, device="cuda")
    dec.pack_layer(synth.layer_weights(w, 0, "cuda"), packed)
    kc = torch.zeros(binding.kv_cache_bytes(dec.desc, 2, 64) // 2, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    k0 = kc.clone()
    x = torch.randn(3, 256, device="cuda").to(torch.bfloat16)
    ws = torch.empty(binding.workspace_bytes(dec.desc, 3, 64), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(x)
    seq = torch.tensor([0, 2, 1], dtype=torch.int32, device="cuda")  # 2 is not a cache row
    dec.prefill(packed, kc, vc, x, seq, torch.zeros(3, dtype=torch.int32, device="cuda"), 2, 64, out, ws)
    with pytest.raises(pd.PdError) as e:
        dec.check_async(ws)
    assert e.value.code == binding.PD_ERR_POSITION
    assert not torch.equal(kc.view(torch.int16), k0.view(torch.int16))  # rows 0 and 1 did append


def test_prefill_62b_shaped_first_tokens_and_decode_consistency(pd):
    # prefill at the size the benchmark times: 256-row chunks through the 62B-shaped stack, attention
    # lengths up to 2048.  Here the sequence continues a cached prefix of 1024 seeded tokens with 1024
    # new ones (incremental prefill, Section 3.5): the oracle follows the first four new tokens.  (The
    # very first tokens of a sequence prefilled from nothing attend to one to four slots; over 64
    # layers of these synthetic weights the fp64 definition itself, re-run with 2^-24 noise, moves
    # their outputs by 0.2 scaled-max, so they cannot carry an elementwise comparison.)  The last
    # token is checked against the decode step of the same token on a cache prefilled up to it
    # (Section 2.2: both phases compute the same function), and the slots it appends against each other.
    import gc
    from workloads import WORKLOADS
    from paper_2211_05102_amd import binding, harness
    gc.collect()
    torch.cuda.empty_cache()
    base = WORKLOADS["c3_62b"]
    P0 = base.l_ctx // 2
    N = base.l_ctx - P0
    w = base.with_(batch=1, name="c3_62b[prefill]")
    desc_o = oracle.make_desc(w)
    g = torch.Generator(device="cuda").manual_seed(11)
    x = torch.randn(N, w.d_model, generator=g, device="cuda").to(torch.bfloat16)
    first = 4
    x64 = oracle.bf16_bits_to_f64_fast(bits_np(x[:first]))
    pos4 = np.arange(P0, P0 + first, dtype=np.int32)

    def follow(l, wts, k, v):  # k, v: the seeded prefix, NaN / Inf from slot P0 on
        oracle.decode_layer(desc_o, {n: t.cpu() for n, t in wts.items()}, bits_np(k), bits_np(v), pos4, x64, w.l_ctx,
                            cache_row=np.zeros(first, dtype=np.int32))
        if l % 16 == 15:
            print(f"[prefill 62b] oracle through layer {l + 1}/{w.n_layers}", flush=True)

    st = harness.DeviceStack(w, poison_unused=True, on_layer=follow,
                             positions=torch.full((1,), P0 - 1, dtype=torch.int32), x_in=x[:1].clone())
    ws = torch.empty(binding.workspace_bytes(st.desc, 256, w.l_ctx), dtype=torch.uint8, device="cuda")
    seq = torch.zeros(N, dtype=torch.int32, device="cuda")
    pos = torch.arange(P0, P0 + N, dtype=torch.int32, device="cuda")
    out = torch.full((N, w.d_model), float("nan"), dtype=torch.bfloat16, device="cuda")
    k_start, v_start = st.k_cache.clone(), st.v_cache.clone()
    st.dec.prefill(st.packed, st.k_cache, st.v_cache, x, seq, pos, 1, w.l_ctx, out, ws)
    st.dec.check_async(ws)
    got = widen(bits_np(out))
    assert np.all(np.isfinite(got))

    def errors(a, b):
        return (float(np.max(np.abs(a - b) / np.maximum(1.0, np.abs(b)))),
                float(np.linalg.norm(a - b) / np.linalg.norm(b)))

    scaled, rel = errors(got[:first], widen(oracle.f64_to_bf16_bits(x64)))
    print(f"[prefill 62b] first {first} new tokens against the oracle: scaled-max {scaled:.3e} rel-L2 {rel:.3e}",
          flush=True)
    assert scaled <= MAX_SCALED and rel <= REL_L2
    k_full, v_full = st.export_kv(0), st.export_kv(w.n_layers - 1)
    # the same last token as a decode step after prefilling the tokens before it
    st.k_cache.copy_(k_start)
    st.v_cache.copy_(v_start)
    out2 = torch.empty(N - 1, w.d_model, dtype=torch.bfloat16, device="cuda")
    st.dec.prefill(st.packed, st.k_cache, st.v_cache, x[:N - 1].contiguous(), seq[:N - 1].contiguous(),
                   pos[:N - 1].contiguous(), 1, w.l_ctx, out2, ws)
    assert torch.equal(out2[:N - 256].view(torch.int16), out[:N - 256].view(torch.int16))  # whole chunks: same bits
    st.x_in.copy_(x[N - 1:N])
    st.positions.fill_(P0 + N - 1)
    last = st.step()
    st.dec.check_async(st.workspace)
    scaled, rel = errors(widen(bits_np(last)), got[N - 1:N])
    print(f"[prefill 62b] last token: decode step against its prefill row: scaled-max {scaled:.3e} rel-L2 {rel:.3e}",
          flush=True)
    assert scaled <= MAX_SCALED and rel <= REL_L2
    T = P0 + N - 1
    for (ka, va), layer in ((k_full, 0), (v_full, w.n_layers - 1)):
        kb, vb = st.export_kv(layer)
        for a, b in ((ka, kb), (va, vb)):
            assert torch.equal(a[:, :P0].view(torch.int16), b[:, :P0].view(torch.int16))  # the prefix is untouched
            da, db = widen(bits_np(a[:, P0:T + 1])), widen(bits_np(b[:, P0:T + 1]))
            assert np.all(np.isfinite(da)) and np.all(np.isfinite(db))
            assert np.max(np.abs(da - db) / np.maximum(1.0, np.abs(db))) <= MAX_SCALED
    del st
    gc.collect()
    torch.cuda.empty_cache()
