"""The entry point that allocates nothing (pd_decode_step_static) against
pd_decode_step: same kernels, so the hidden state and the caches must agree bit
for bit; two calls in a row on the library's static scratch, the second with a
smaller input; a shape beyond the scratch limit is refused before any launch."""
import pytest
import torch

from workloads.configs import Workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_05102_amd as m
    m.lib()
    return m


def _pair(harness, w):
    """Two identical device stacks of workload `w`."""
    return harness.DeviceStack(w), harness.DeviceStack(w)


def test_static_scratch_step_matches_workspace_step(pd):
    from paper_2211_05102_amd import harness, binding
    big = Workload("noalloc_a", 3, 1024, 8, 128, 2048, 48, 256, positions="ragged", pos_lo=0, pos_hi=256)
    small = Workload("noalloc_b", 2, 384, 4, 64, 384, 5, 96, positions="ragged", pos_lo=0, pos_hi=96)
    for w in (big, small):  # second call: smaller input, scratch still holds the first call's data
        ref, sta = _pair(harness, w)
        want = ref.step().clone()
        ref.dec.check_async(ref.workspace)
        sta.workspace.fill_(0xFF)  # not used by the static entry point
        sta.dec.decode_step_static(sta.packed, sta.k_cache, sta.v_cache, sta.x_in, sta.positions,
                                   w.l_ctx, sta.x_out)
        sta.dec.check_async(None)
        torch.cuda.synchronize()
        assert torch.equal(sta.x_out.view(torch.int16), want.view(torch.int16)), w.name
        assert torch.equal(sta.k_cache.view(torch.int16), ref.k_cache.view(torch.int16)), w.name
        assert torch.equal(sta.v_cache.view(torch.int16), ref.v_cache.view(torch.int16)), w.name
        assert int((sta.workspace != 0xFF).sum()) == 0  # the caller's buffer was not touched


def test_static_scratch_limit_is_enforced(pd):
    from paper_2211_05102_amd import binding
    from workloads import WORKLOADS
    w = WORKLOADS["c3_62b"]  # needs about 100 MiB of scratch
    dec = binding.Decoder(w)
    fake = torch.empty(4096, dtype=torch.uint8, device="cuda")
    x = torch.empty(w.batch, w.d_model, dtype=torch.bfloat16, device="cuda")
    pos = torch.zeros(w.batch, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.PdError) as e:
        dec.decode_step_static(fake, fake, fake, x, pos, w.l_ctx, x)
    assert e.value.code == binding.PD_ERR_WORKSPACE and "64" in str(e.value) or "67108864" in str(e.value)
