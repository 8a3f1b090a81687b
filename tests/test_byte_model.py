"""Closed-form pins of the byte/flop accounting the roofline report uses,
against the figures the paper prints (tests/golden) and the sizes the workload
definitions quote."""
import os

import pytest

from workloads import WORKLOADS
from workloads import configs as C

GIB = 1 << 30


def _rows(path):
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_table1_max_context(golden_dir):
    hbm = 64 * 32 * GIB  # 64 chips x 32 GiB (Section 4)
    for name, d_head, copies, at128, at512 in _rows(os.path.join(golden_dir, "table1_max_context.txt")):
        for batch, printed in ((128, float(at128)), (512, float(at512))):
            got = C.max_context_tokens(hbm, 0.30, 118, int(copies), int(d_head), batch)
            assert abs(got - printed) / printed < 0.02, (name, batch, got, printed)


def test_text_figures(golden_dir):
    vals = {k: float(v) for k, v in _rows(os.path.join(golden_dir, "text_figures.txt"))}
    kv = C.kv_bytes_per_token(118, 48, 128) * 512 * 2048
    assert abs(kv - vals["kv_total_bytes_mha_540b_b512_l2048"]) / kv < 0.03
    mfu = 2 * 540e9 * 64 / (28.5e-3 * 64 * 275e12)
    assert abs(mfu - vals["mfu_540b_b64_64chips"]) < 0.005


def test_workload_sizes_match_the_quoted_ones():
    c3, c4, c5, c2, c1 = (WORKLOADS[k] for k in ("c3_62b", "c4_540b_shard8", "c5_62b_long", "c2_8b", "c1_tiny"))
    assert c3.n_in == 74240 and c3.k_out == 40960
    assert c1.n_in == 2432 and c1.k_out == 1280
    assert abs(C.weight_bytes(c3) / 1e9 - 60.398) < 0.01      # "~62 GB int8 weights"
    assert abs(C.weight_bytes(c4) / 1e9 - 67.929) < 0.01      # "~67 GB"
    assert abs(C.kv_alloc_bytes(c3) / 1e9 - 8.590) < 0.01     # "~8.6 GB"
    assert abs(C.kv_alloc_bytes(c5) / 1e9 - 137.4) < 0.1      # "~137 GB"
    full = lambda w: [w.l_ctx - 1] * w.batch
    assert abs(C.algorithmic_bytes(c2, full(c2)) / 1e9 - 8.120) < 0.001
    assert abs(C.algorithmic_bytes(c3, full(c3)) / 1e9 - 68.988) < 0.001
    assert abs(C.algorithmic_bytes(c4, full(c4)) / 1e9 - 75.848) < 0.001
    assert C.kv_read_bytes(c3, full(c3)) == C.kv_alloc_bytes(c3)


def test_flops_are_two_per_parameter_per_token():
    c3 = WORKLOADS["c3_62b"]
    pos = [c3.l_ctx - 1] * c3.batch
    proj = 2 * C.weight_bytes(c3) * c3.batch
    attn = C.algorithmic_flops(c3, pos) - proj
    assert abs(proj / 1e12 - 7.73) < 0.01
    assert attn == 4 * c3.n_layers * c3.n_heads * c3.d_head * c3.batch * c3.l_ctx
