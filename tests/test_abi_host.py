"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, sizes follow the documented formulas, and argument errors are
caught before anything is enqueued (no GPU needed, no compute call made)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2211_05102_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2211_05102_amd import build
        os.environ.setdefault("PD_QUIET", "1")
        build.build()
    b.lib()
    return b


def header_symbols():
    text = open(os.path.join(ROOT, "include", "palmdecode.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pd_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(binding):
    syms = header_symbols()
    assert len(syms) >= 20
    L = binding.lib()
    for s in syms:
        assert hasattr(L, s), s
    assert sorted(binding.EXPORTS) == syms


def test_sizes(binding):
    from workloads import WORKLOADS
    from workloads import configs as C
    from workloads import VARIANTS
    for w in list(WORKLOADS.values()) + [VARIANTS["c3_62b_bf16w"]]:
        d = binding.make_desc(w)
        assert binding.kv_cache_bytes(d, w.batch, w.l_ctx) * 2 == C.kv_alloc_bytes(w)
        pl = binding.packed_layer_bytes(d)
        raw = C.weight_bytes_per_layer(w) + 4 * (w.n_in + 2 * w.d_model)
        assert raw <= pl <= raw + 5 * 256 and pl % 256 == 0
        assert binding.workspace_bytes(d, w.batch, w.l_ctx) % 256 == 0


def test_bad_descriptions_are_rejected(binding):
    from workloads import WORKLOADS
    w = WORKLOADS["c1_tiny"]
    for bad in (w.with_(d_model=200), w.with_(d_head=96), w.with_(n_heads=33), w.with_(n_kv_heads=3),
                w.with_(d_ff=1000), w.with_(n_layers=0), w.with_(d_ff=1056)):
        with pytest.raises(binding.PdError) as e:
            binding.Decoder(bad)
        assert e.value.code == binding.PD_ERR_SHAPE
    with pytest.raises(binding.PdError):
        binding.kv_cache_bytes(binding.make_desc(w), 1, 100)  # L_ctx not a multiple of 32
    d = binding.make_desc(w)
    d.flags = 2  # not a defined flag
    with pytest.raises(binding.PdError) as e:
        binding.packed_layer_bytes(d)
    assert e.value.code == binding.PD_ERR_SHAPE
    # a matrix of 4 GiB or more: fine as int8 (2^31 bytes), refused as bf16 (2^32 bytes)
    big = w.with_(d_model=32768, n_heads=28, d_head=256, d_ff=28672)  # n_in = 7168 + 512 + 57344 = 65024; 32768*65024 < 2^31
    assert binding.packed_layer_bytes(binding.make_desc(big)) > 0
    big16 = big.with_(weights="bf16", d_ff=30208)  # n_in = 68096: 32768 * 68096 * 2 >= 2^32
    with pytest.raises(binding.PdError) as e:
        binding.packed_layer_bytes(binding.make_desc(big16))
    assert e.value.code == binding.PD_ERR_SHAPE
    with pytest.raises(binding.PdError):
        binding.workspace_bytes(binding.make_desc(w), 0, 128)


def test_argument_errors_come_before_any_launch(binding):
    from workloads import WORKLOADS
    w = WORKLOADS["c1_tiny"]
    dec = binding.Decoder(w)
    L = binding.lib()
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(0x1000)      # aligned, never dereferenced on these paths
    odd = ctypes.c_void_p(0x1008)       # not 256-aligned
    i32 = ctypes.c_int32
    big = ctypes.c_size_t(1 << 30)
    rc = L.pd_decode_step(dec._h, null, fake, fake, fake, fake, i32(1), i32(128), fake, fake, big, null)
    assert rc == binding.PD_ERR_NULL
    rc = L.pd_decode_step(dec._h, odd, fake, fake, fake, fake, i32(1), i32(128), fake, fake, big, null)
    assert rc == binding.PD_ERR_ALIGN
    rc = L.pd_decode_step(dec._h, fake, fake, fake, fake, fake, i32(0), i32(128), fake, fake, big, null)
    assert rc == binding.PD_ERR_SHAPE
    rc = L.pd_decode_step(dec._h, fake, fake, fake, fake, fake, i32(1), i32(100), fake, fake, big, null)
    assert rc == binding.PD_ERR_SHAPE
    rc = L.pd_decode_step(dec._h, fake, fake, fake, fake, fake, i32(1), i32(128), fake, fake, ctypes.c_size_t(16), null)
    assert rc == binding.PD_ERR_WORKSPACE
    assert b"workspace" in L.pd_last_error()
    rc = L.pd_decode_layer(dec._h, i32(5), fake, fake, fake, fake, fake, i32(1), i32(128), fake, i32(1), fake, big, null)
    assert rc == binding.PD_ERR_RANGE
    rc = L.pd_graph_replay(dec._h, null)
    assert rc == binding.PD_ERR_STATE
    with pytest.raises(binding.PdError):
        dec.set_option("no_such_option", 1)
    with pytest.raises(binding.PdError):
        dec.set_option("gemm_workgroups_in", 5000)   # at most 4096
    dec.set_option("gemm_workgroups_in", 2)
    dec.set_option("gemm_workgroups_in", 0)
    assert L.pd_status_string(i32(-7)).decode().startswith("position")
    dec.close()
    # the bf16-weight entries and the ceiling probe
    sz = ctypes.c_size_t
    assert L.pd_pack_matrix_bf16(null, i32(128), i32(32), fake, null) == binding.PD_ERR_NULL
    assert L.pd_pack_matrix_bf16(fake, i32(100), i32(32), fake, null) == binding.PD_ERR_SHAPE
    assert L.pd_pack_matrix_bf16(fake, i32(65536), i32(32768), fake, null) == binding.PD_ERR_SHAPE  # 4 GiB as bf16
    assert L.pd_pack_matrix_bf16(fake, i32(128), i32(32), odd, null) == binding.PD_ERR_ALIGN
    assert L.pd_wgemm_bf16(fake, null, i32(1), i32(128), i32(32), fake, i32(0), fake, big, null) == binding.PD_ERR_NULL
    assert L.pd_wgemm_bf16(fake, fake, i32(300), i32(128), i32(32), fake, i32(0), fake, big, null) == binding.PD_ERR_SHAPE
    assert L.pd_wgemm_bf16(fake, fake, i32(1), i32(128), i32(32), fake, i32(0), fake, sz(16), null) == binding.PD_ERR_WORKSPACE
    assert L.pd_ceiling_probe(null, sz(8388608), i32(48), i32(1), fake, null) == binding.PD_ERR_NULL
    assert L.pd_ceiling_probe(fake, sz(1000), i32(48), i32(1), fake, null) == binding.PD_ERR_SHAPE
    assert L.pd_ceiling_probe(fake, sz(8388608), i32(47), i32(1), fake, null) == binding.PD_ERR_RANGE
    assert L.pd_ceiling_probe(fake, sz(8388608), i32(48), i32(3), fake, null) == binding.PD_ERR_RANGE
    # a handle for bf16 weights takes no scale vectors; one for int8 weights needs them
    dec16 = binding.Decoder(w.with_(weights="bf16"))
    assert L.pd_pack_layer(dec16._h, fake, null, fake, null, fake, odd, null) == binding.PD_ERR_ALIGN  # past the NULL check
    dec8 = binding.Decoder(w)
    assert L.pd_pack_layer(dec8._h, fake, null, fake, null, fake, fake, null) == binding.PD_ERR_NULL
    dec16.close(); dec8.close()


# ---- host logic: the deterministic work split of the projections ----------------

@pytest.mark.parametrize("B,K,N,wg,c_split,blk0,blk1", [
    (64, 8192, 74240, 0, 0, 1, 64),        # 62B-shaped input projection (one scale block per row)
    (64, 40960, 8192, 0, 64, 16, 16),      # 62B-shaped output projection
    (32, 18432, 20480, 0, 0, 1, 144),      # 540B-shard input projection
    (256, 8192, 74240, 64, 0, 1, 64),      # four row groups
    (8, 1280, 256, 3, 0, 1, 1), (1, 128, 32, 1, 0, 1, 1), (33, 512, 96, 2, 0, 1, 1),
    (64, 4096, 544, 0, 0, 1, 1), (5, 384, 1000 // 32 * 32, 7, 1, 1, 2), (64, 40960, 256, 16, 64, 16, 16),
    (130, 384, 320, 4096, 0, 1, 1),
])
def test_projection_work_split_covers_every_unit_once(binding, B, K, N, wg, c_split, blk0, blk1):
    counts, begin, first_slot, slots = binding.qgemm_plan(B, K, N, wg, c_split, blk0, blk1)
    G, T, C = counts["workgroups"], counts["tiles"], counts["chunks_per_tile"]
    U = T * C
    assert C == K // 128 and T == -(-N // 256) and 1 <= G <= max(1, min(wg or 256, U))
    if wg == 0 and B <= 64 and U >= 4096:
        assert G >= 224  # the automatic count gives up at most one eighth of the compute units
    assert counts["rows"] % 32 == 0 and counts["rows"] >= B and counts["rows"] - B < 64
    # ranges: contiguous, ordered, cover [0, U) exactly once, balanced to within the alignment
    assert begin[0] == 0 and begin[G] == U and all(begin[g] <= begin[g + 1] for g in range(G))
    sizes = [begin[g + 1] - begin[g] for g in range(G)]
    assert max(sizes) - min(sizes) <= 8
    # slots: brute force over the ranges -- a tile has one slot per range that holds one of its
    # units, numbered in range order; first_slot[g] is range g's number in the tile it starts in
    per_tile = [0] * T
    for g in range(G):
        if begin[g] == begin[g + 1]:
            continue
        t_first, t_last = begin[g] // C, (begin[g + 1] - 1) // C
        assert first_slot[g] == per_tile[t_first], (g, first_slot[g], per_tile[t_first])
        for t in range(t_first, t_last + 1):
            per_tile[t] += 1
    assert per_tile == slots and max(slots) == counts["max_slots"] and min(slots) >= 1


def test_projection_work_split_rejects_bad_arguments(binding):
    L = binding.lib()
    import ctypes
    counts = (ctypes.c_int32 * 5)()
    i32 = ctypes.c_int32
    assert L.pd_qgemm_plan(i32(8), i32(100), i32(32), i32(0), i32(0), i32(1), i32(1), counts, None, None, None) == binding.PD_ERR_SHAPE
    assert L.pd_qgemm_plan(i32(8), i32(128), i32(32), i32(5000), i32(0), i32(1), i32(1), counts, None, None, None) == binding.PD_ERR_RANGE
    assert L.pd_qgemm_plan(i32(8), i32(128), i32(32), i32(0), i32(2), i32(1), i32(1), counts, None, None, None) == binding.PD_ERR_RANGE
    assert L.pd_qgemm_plan(i32(8), i32(128), i32(32), i32(0), i32(0), i32(1), i32(1), None, None, None, None) == binding.PD_ERR_NULL


def test_automatic_split_of_the_62b_projections_is_even(binding):
    # the kernel is bandwidth-bound: its time follows the longest range, so the automatic
    # workgroup count prefers an even split to using every compute unit
    counts, begin, _, _ = binding.qgemm_plan(64, 8192, 74240, 0, 0, 1, 64)
    sizes = {begin[g + 1] - begin[g] for g in range(counts["workgroups"])}
    assert counts["workgroups"] == 232 and sizes == {80}
    counts, begin, _, _ = binding.qgemm_plan(64, 40960, 8192, 0, 64, 16, 16)
    sizes = {begin[g + 1] - begin[g] for g in range(counts["workgroups"])}
    assert counts["workgroups"] == 256 and sizes == {40}
