"""GPU parity of the generation loop (Section 2.2) and its sampling head against the
fp64 oracle.  Integer work -- which entries make the top k, the order of equal
logits, the token drawn from identical logits -- is compared bit for bit; where a
floating-point sum decides the token, the comparison is made where the oracle's own
margin shows the decision is not a rounding coin toss."""
import numpy as np
import pytest
import torch

import oracle
from workloads import synth
from workloads.configs import Workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_05102_amd as m
    m.lib()
    return m


def bits_np(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def decision_margins(logits, k, top_p, T, u, eps=1e-5):
    """Oracle-side conditioning of one draw, through numpy.  Returns
      gap  : k-th minus (k+1)-th logit (how firmly the top-k set is decided);
      safe : True if the token does not depend on how the nucleus cut and the running sums
             round: the target u * c_n stays more than `eps` (plus the probability mass whose
             membership in the nucleus is within `eps` of the threshold) away from both ends
             of the chosen entry's interval, and the chosen entry lies inside the nucleus
             under either reading of the cut."""
    order = np.argsort(-logits, kind="stable")
    gap = np.inf if k >= logits.shape[0] else logits[order[k - 1]] - logits[order[k]]
    z = logits[order[:k]] / T
    p = np.exp(z - z.max())
    p /= p.sum()
    c = np.cumsum(p)
    n_lo = min(int(np.searchsorted(c, top_p - eps, side="left")) + 1, k)   # shortest plausible nucleus
    n_hi = min(int(np.searchsorted(c, top_p + eps, side="left")) + 1, k)   # longest plausible nucleus
    amb = c[n_hi - 1] - c[n_lo - 1]
    n = min(int(np.searchsorted(c, top_p, side="left")) + 1, k)
    edges = np.concatenate([[0.0], c[:n]]) / c[n - 1]
    pick = min(int(np.searchsorted(c[:n], u * c[n - 1], side="right")), n - 1)
    draw = float(np.min(np.abs(edges - u)))
    return gap, bool(draw > eps + 2 * amb and pick < n_lo)


@pytest.mark.parametrize("V,k,top_p,T", [
    (1000, 1, 1.0, 1.0), (1000, 40, 0.9, 0.8), (32000, 64, 0.95, 1.3), (256000, 40, 0.9, 1.0), (77, 64, 1.0, 0.5),
    (5000, 7, 0.3, 1.0),
])
def test_sampler_matches_oracle_on_the_same_logits(pd, V, k, top_p, T):
    from paper_2211_05102_amd import binding
    B = 24
    g = torch.Generator().manual_seed(V + k)
    logits = (torch.randn(B, V, generator=g) * 2.5).float()
    logits[1] = torch.round(logits[1])              # thousands of exact ties, also at the k-th place
    logits[2] = 0.25                                # every entry equal: pure index order
    logits[3, :] = -3.0
    logits[3, [5, V - 1, V // 2]] = 4.0             # three-way tie for the maximum
    u = torch.rand(B, generator=g).float()
    u[0] = 0.0
    tok = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    binding.sample(logits.cuda(), k, top_p, T, u.cuda(), tok)
    torch.cuda.synchronize()
    got = tok.cpu().numpy()
    checked = 0
    for b in range(B):
        lg = logits[b].double().numpy()
        want, kept, margin = oracle.sample_topk_topp(lg, k, top_p, T, float(u[b]))
        gap, safe = decision_margins(lg, k, top_p, T, float(u[b]))
        topk = set(np.argsort(-lg, kind="stable")[:k].tolist())
        assert int(got[b]) in topk, (b, got[b])     # selection and tie order are exact integer work
        if safe:                                    # the fp32 sums decide the same way as the fp64 ones
            assert int(got[b]) == want, (b, got[b], want, kept, margin)
            checked += 1
    assert checked >= B - 3
    # bit-reproducible
    tok2 = torch.empty_like(tok)
    binding.sample(logits.cuda(), k, top_p, T, u.cuda(), tok2)
    torch.cuda.synchronize()
    assert torch.equal(tok, tok2)


def test_sampler_all_equal_logits_inverts_the_uniform_cdf(pd):
    from paper_2211_05102_amd import binding
    V, k = 4096, 64
    B = 50
    u = (torch.arange(B).float() + 0.37) / B
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    binding.sample(torch.full((B, V), 1.5, device="cuda"), k, 1.0, 0.9, u.cuda(), tok)
    torch.cuda.synchronize()
    # the k smallest indices are kept, each with mass 1/k: token = floor(u * k)
    assert tok.cpu().tolist() == [int(np.floor(float(x) * k)) for x in u]


def test_head_logits_vs_oracle(pd):
    from paper_2211_05102_amd import binding
    w = Workload("head", 1, 512, 4, 128, 512, 9, 64)
    V = 1504
    dec = pd.Decoder(w)
    hw = synth.head_weights(w, V, "cuda")
    packed = torch.empty(binding.packed_head_bytes(dec.desc, V), dtype=torch.uint8, device="cuda")
    dec.pack_head(hw["w_vocab"], hw["s_vocab"], hw["gamma_f"], packed)
    x = (synth.hidden_state(w, "cuda").float() * 20 + 0.5).to(torch.bfloat16)
    logits = torch.full((w.batch, V), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(binding.head_workspace_bytes(dec.desc, V, w.batch), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    dec.head_logits(packed, V, x, logits, ws)
    torch.cuda.synchronize()
    want = oracle.head_logits(oracle.bf16_bits_to_f64_fast(bits_np(x)), hw["gamma_f"], hw["w_vocab"],
                              hw["s_vocab"], w.ln_eps)
    got = logits.cpu().double().numpy()
    assert np.all(np.isfinite(got))
    assert np.max(np.abs(got - want)) <= 2e-6 * np.max(np.abs(want))


def oracle_generate(w, st, top_k, top_p, T, n_steps, layers_cpu, kcs, vcs):
    """The loop of Section 2.2 on the oracle: returns tokens [n_steps, B] and, per draw, whether
    its decisions are well away from rounding (gap of the top-k set, nucleus cut, draw)."""
    desc = oracle.make_desc(w)
    B = st.B
    x_bits = bits_np(st.x_in)
    pos = st.positions.cpu().numpy().copy()
    u = st.uniforms.cpu().numpy()
    embed_bits = bits_np(st.embed)
    tokens = np.zeros((n_steps, B), dtype=np.int64)
    robust = np.zeros((n_steps, B), dtype=bool)
    for i in range(n_steps):
        hidden_bits, _ = oracle.decode_step(desc, layers_cpu, kcs, vcs, pos, x_bits, w.l_ctx)
        logits = oracle.head_logits(oracle.bf16_bits_to_f64_fast(hidden_bits), st.head["gamma_f"],
                                    st.head["w_vocab"], st.head["s_vocab"], w.ln_eps)
        for b in range(B):
            tokens[i, b], _, _ = oracle.sample_topk_topp(logits[b], top_k, top_p, T, float(u[i, b]))
            gap, safe = decision_margins(logits[b], top_k, top_p, T, float(u[i, b]), eps=1e-3)
            robust[i, b] = gap > 1e-3 and safe
        x_bits = embed_bits[tokens[i]]
        pos = pos + 1
    return tokens, robust, x_bits, pos


@pytest.mark.parametrize("top_k,top_p,T,weights", [(1, 1.0, 1.0, "int8"), (16, 0.9, 0.7, "int8"),
                                                   (8, 0.95, 1.0, "bf16")])
def test_generate_loop_vs_oracle(pd, top_k, top_p, T, weights):
    from paper_2211_05102_amd import harness
    n_steps, V = 8, 1024
    w = Workload("gen", 2, 256, 4, 64, 512, 5, 96, positions="ragged", pos_lo=0, pos_hi=96 - n_steps,
                 weights=weights)
    layers_cpu, kcs, vcs = [], [], []
    st = harness.GenerateStack(w, V, n_steps, on_layer=lambda l, wts, k, v: (
        layers_cpu.append({n: t.cpu() for n, t in wts.items()}), kcs.append(bits_np(k)), vcs.append(bits_np(v))))
    x0, p0 = st.x_in.clone(), st.positions.clone()
    k0, v0 = st.k_cache.clone(), st.v_cache.clone()
    want, robust, x_last, pos_last = oracle_generate(w, st, top_k, top_p, T, n_steps, layers_cpu, kcs, vcs)

    results = []
    for use_graph in (False, True):
        st.x_in.copy_(x0); st.positions.copy_(p0); st.k_cache.copy_(k0); st.v_cache.copy_(v0)
        st.tokens.fill_(-1)
        st.gen_workspace.fill_(0xFF)
        stream = torch.cuda.Stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            st.generate(top_k, top_p, T, use_graph, stream)
        stream.synchronize()
        st.dec.check_async(st.gen_workspace, stream)
        results.append((st.tokens.cpu().numpy().copy(), bits_np(st.x_in), st.positions.cpu().numpy().copy(),
                        st.k_cache.clone(), st.v_cache.clone()))
    (tok_e, x_e, p_e, kc_e, vc_e), (tok_g, x_g, p_g, kc_g, vc_g) = results
    # graph replay of the step == eager launches, bit for bit
    assert np.array_equal(tok_e, tok_g) and np.array_equal(x_e, x_g) and np.array_equal(p_e, p_g)
    assert torch.equal(kc_e.view(torch.int16), kc_g.view(torch.int16))
    assert torch.equal(vc_e.view(torch.int16), vc_g.view(torch.int16))
    assert np.array_equal(p_e, pos_last)
    # tokens: a row is followed while the two sides agree; a well-conditioned draw must agree
    compared = 0
    for b in range(w.batch):
        for i in range(n_steps):
            if robust[i, b]:
                assert tok_e[i, b] == want[i, b], (i, b, tok_e[i, b], want[i, b])
            if tok_e[i, b] != want[i, b]:
                break  # a coin-toss decision went the other way: the sequences differ from here on
            compared += 1
    print(f"[generate] top_k {top_k} top_p {top_p} T {T}: {compared} of {n_steps * w.batch} draws compared and equal, "
          f"{int(robust.sum())} well-conditioned", flush=True)
    assert compared >= 0.8 * n_steps * w.batch
    # exactly the slots P_b .. P_b + n_steps - 1 of every row and layer were appended
    t = torch.arange(w.l_ctx, device="cuda")[None, :]
    p = p0.long()[:, None]
    want_changed = (t >= p) & (t < p + n_steps)
    for l in range(w.n_layers):
        ka, va = st.export_kv(l)
        k_orig, v_orig = synth.kv_layer(w, l, "cuda")
        for got, ref in ((ka, k_orig), (va, v_orig)):
            changed = (got.view(torch.int16) != ref.view(torch.int16)).any(dim=2)
            assert torch.equal(changed, want_changed), l
    # the state handed back is the embedding of the last token drawn
    assert np.array_equal(x_e, bits_np(st.embed)[tok_e[-1]])


def test_generate_rejects_bad_sampling_arguments(pd):
    from paper_2211_05102_amd import harness, binding
    w = Workload("genbad", 1, 256, 4, 64, 256, 2, 64, positions="ragged", pos_lo=0, pos_hi=32)
    st = harness.GenerateStack(w, 256, 2)
    for k, p, T in ((0, 0.9, 1.0), (65, 0.9, 1.0), (8, 0.0, 1.0), (8, 1.5, 1.0), (8, 0.9, 0.0)):
        with pytest.raises(pd.PdError) as e:
            st.generate(k, p, T, False)
        assert e.value.code == binding.PD_ERR_RANGE


def test_generate_62b_shaped_first_tokens_sampled_rows(pd):
    # the generation loop in the configuration the benchmark times (62B-shaped stack, batch 64,
    # 256,000-entry vocabulary, top-k 40 / top-p 0.9, graph replay), two steps that fill the cache;
    # the oracle follows three sequences through the first step (stack, head, draw)
    import gc
    from workloads import WORKLOADS
    from paper_2211_05102_amd import harness
    gc.collect()
    torch.cuda.empty_cache()
    n_steps, V, top_k, top_p, T = 2, 256000, 40, 0.9, 1.0
    base = WORKLOADS["c3_62b"]
    start = base.l_ctx - n_steps
    w = base.with_(positions="ragged", pos_lo=start, pos_hi=start + 1)
    rows = [0, 63, 17]
    desc = oracle.make_desc(w)
    x_in = synth.hidden_state(w, "cuda")
    x64 = oracle.bf16_bits_to_f64_fast(bits_np(x_in)[rows])
    pos = np.full(len(rows), start, dtype=np.int32)

    def follow(l, wts, k, v):
        oracle.decode_layer(desc, {n: t.cpu() for n, t in wts.items()}, bits_np(k[rows]), bits_np(v[rows]), pos, x64,
                            w.l_ctx)
        if l % 16 == 15:
            print(f"[generate 62b] oracle through layer {l + 1}/{w.n_layers}", flush=True)

    st = harness.GenerateStack(w, V, n_steps, on_layer=follow, x_in=x_in)
    hidden = oracle.bf16_bits_to_f64_fast(oracle.f64_to_bf16_bits(x64))  # the stack hands bf16 to the head
    logits = oracle.head_logits(hidden, st.head["gamma_f"], st.head["w_vocab"], st.head["s_vocab"], w.ln_eps)
    u = st.uniforms.cpu().numpy()
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        st.generate(top_k, top_p, T, True, stream)
    stream.synchronize()
    st.dec.check_async(st.gen_workspace, stream)
    tok = st.tokens.cpu().numpy()
    assert tok.shape == (n_steps, w.batch) and tok.min() >= 0 and tok.max() < V
    compared = 0
    for i, b in enumerate(rows):
        want, _, _ = oracle.sample_topk_topp(logits[i], top_k, top_p, T, float(u[0, b]))
        gap, safe = decision_margins(logits[i], top_k, top_p, T, float(u[0, b]), eps=1e-3)
        print(f"[generate 62b] row {b}: gpu {tok[0, b]} oracle {want} gap {gap:.2e} safe {safe}", flush=True)
        if gap > 1e-3 and safe:
            assert tok[0, b] == want, (b, tok[0, b], want)
            compared += 1
    assert compared >= 1
    # state handed back: every position advanced by two, the input is the embedding of the last token
    assert torch.equal(st.positions.cpu(), torch.full((w.batch,), start + n_steps, dtype=torch.int32))
    assert np.array_equal(bits_np(st.x_in), bits_np(st.embed[torch.from_numpy(tok[-1]).long().cuda()]))
    # exactly the last two slots of every row were appended (first, middle and last layer)
    t = torch.arange(w.l_ctx, device="cuda")[None, :]
    want_changed = (t >= start).expand(w.batch, -1)
    for l in (0, 31, 63):
        ka, va = st.export_kv(l)
        k0, v0 = synth.kv_layer(w, l, "cuda")
        for got, ref in ((ka, k0), (va, v0)):
            changed = (got.view(torch.int16) != ref.view(torch.int16)).any(dim=2)
            assert torch.equal(changed, want_changed), l
    del st
    gc.collect()
    torch.cuda.empty_cache()
