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
    for w in WORKLOADS.values():
        d = binding.make_desc(w)
        assert binding.kv_cache_bytes(d, w.batch, w.l_ctx) * 2 == C.kv_alloc_bytes(w)
        pl = binding.packed_layer_bytes(d)
        raw = C.weight_bytes_per_layer(w) + 4 * (w.n_in + 2 * w.d_model)
        assert raw <= pl <= raw + 5 * 256 and pl % 256 == 0
        assert binding.workspace_bytes(d, w.batch, w.l_ctx) % 256 == 0


def test_bad_descriptions_are_rejected(binding):
    from workloads import WORKLOADS
    w = WORKLOADS["c1_tiny"]
    for bad in (w.with_(d_model=200), w.with_(d_head=96), w.with_(n_heads=33), w.with_(n_kv_heads=4),
                w.with_(d_ff=1000), w.with_(n_layers=0), w.with_(d_ff=1056)):
        with pytest.raises(binding.PdError) as e:
            binding.Decoder(bad)
        assert e.value.code == binding.PD_ERR_SHAPE
    with pytest.raises(binding.PdError):
        binding.kv_cache_bytes(binding.make_desc(w), 1, 100)  # L_ctx not a multiple of 32
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
