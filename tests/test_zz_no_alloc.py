"""The entry point that allocates nothing (sat_loss_grad_static, for callers that cannot
call hipMalloc or carry a workspace) against sat_loss_grad with a workspace: same kernels,
so gradients and loss must agree bit for bit, and both must meet the oracle's bound. Two calls
in a row, the second on a smaller input (the static array keeps the first call's contents)."""
import sys

import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc

pytestmark = pytest.mark.gpu
RTOL = 1e-5


def _say(msg):
    print("[no_alloc] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def env():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs the GPU")
    import paper_2308_13466_amd as sat
    sat.lib()
    from tests import gpu_util as gu
    return sat, gu, torch


def _one_call(sat, gu, torch, n, C, seed, bf16=False):
    rng = np.random.default_rng(seed)
    HL = (3.0 * rng.standard_normal((n, C))).astype(np.float32)
    y = rng.integers(0, C, size=n).astype(np.int32)
    ld = gu.ld_for(C, 8)
    dt = sat.BF16 if bf16 else sat.F32
    if bf16:
        bits = syn.bf16_bits_from_f32(HL)
        HL = syn.f32_from_bf16_bits(bits)
        HL_d = gu.to_dev_bits(bits, ld)
        mk = lambda: torch.full((n, ld), 0x4040, dtype=torch.int16, device=gu.DEV)
    else:
        HL_d = gu.to_dev(HL, ld)
        mk = lambda: gu.dev_empty(n, ld, fill=-3.0)
    y_d = gu.to_dev(y)
    # existing entry point, caller's workspace
    g_ws, loss_ws = mk(), torch.zeros(1, dtype=torch.float32, device=gu.DEV)
    wsb = sat.loss_workspace_bytes(n)
    ws = gu.workspace(wsb)
    sat.loss_grad(HL_d, ld, n, C, y_d, g_ws, ld, loss=loss_ws, dtype=dt, workspace=ws,
                  workspace_bytes=wsb, stream=gu.stream_ptr())
    # the entry point that allocates nothing: outputs are allocated BEFORE the call
    g_st, loss_st = mk(), torch.zeros(1, dtype=torch.float32, device=gu.DEV)
    gu.sync()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    sat.loss_grad_static(HL_d, ld, n, C, y_d, g_st, ld, loss=loss_st, dtype=dt,
                         stream=gu.stream_ptr())
    gu.sync()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    assert torch.equal(g_st, g_ws), "gradients differ from sat_loss_grad's"
    assert loss_st.item() == loss_ws.item(), "loss differs from sat_loss_grad's"
    loss, g = orc.loss_and_grad(HL, y)
    if bf16:
        got = syn.f32_from_bf16_bits(gu.bits_to_host(g_st, C))
        gu.assert_close(got, g, 2e-2, "dH^(L) bf16")
    else:
        gu.assert_close(gu.to_host(g_st, C), g, RTOL, "dH^(L)")
        assert torch.all(g_st[:, C:] == -3.0)
    assert abs(float(loss_st.item()) - loss) <= 2 * RTOL * abs(loss)


def test_static_scratch_loss_grad_two_calls_second_smaller(env):
    sat, gu, torch = env
    _say("call 1: n=50000 C=47")
    _one_call(sat, gu, torch, 50000, 47, seed=1)
    _say("call 2: n=777 C=47 (smaller: stale partial sums of call 1 lie behind its own)")
    _one_call(sat, gu, torch, 777, 47, seed=2)
    _say("call 3: n=3001 C=172 bf16")
    _one_call(sat, gu, torch, 3001, 172, seed=3, bf16=True)
    _say("call 4: n=1 C=2")
    _one_call(sat, gu, torch, 1, 2, seed=4)


def test_static_scratch_rejects_sizes_beyond_its_maximum(env):
    sat, gu, torch = env
    mx = sat.loss_grad_static_max_rows()
    assert mx == 262144 * 128
    t = torch.zeros(64, dtype=torch.float32, device=gu.DEV)
    yi = torch.zeros(64, dtype=torch.int32, device=gu.DEV)
    with pytest.raises(sat.SatError) as e:      # rejected on the host, nothing is enqueued
        sat.loss_grad_static(t, 8, mx + 1, 8, yi, t, 8, loss=t, stream=gu.stream_ptr())
    assert e.value.status == -2
    gu.sync()
    # no loss requested: no scratch needed, same result as the workspace call
    _say("no loss output")
    rng = np.random.default_rng(9)
    HL = rng.standard_normal((300, 40)).astype(np.float32)
    y = rng.integers(0, 40, size=300).astype(np.int32)
    g1, g2 = gu.dev_empty(300, 40), gu.dev_empty(300, 40)
    sat.loss_grad(gu.to_dev(HL), 40, 300, 40, gu.to_dev(y), g1, 40, stream=gu.stream_ptr())
    sat.loss_grad_static(gu.to_dev(HL), 40, 300, 40, gu.to_dev(y), g2, 40, stream=gu.stream_ptr())
    gu.sync()
    assert torch.equal(g1, g2)
