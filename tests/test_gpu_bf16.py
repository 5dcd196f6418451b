"""GPU parity of the bf16 storage mode (features, activations and history in
bfloat16, sums in fp32): the oracle sees exactly the bf16 values the GPU sees
(widened to fp64) and results are held to 2e-2; copies are bit-exact."""
import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc

pytestmark = pytest.mark.gpu
RTOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    import paper_2308_13466_amd as sat
    sat.lib()
    from tests import gpu_util as gu
    return sat, gu, torch


def _say(msg):
    print("[case] " + msg, flush=True)


def _bf16(a):
    """(bit patterns, the exact fp32 values they stand for)"""
    bits = syn.bf16_bits_from_f32(a)
    return bits, syn.f32_from_bf16_bits(bits)


@pytest.mark.parametrize("d,ld_t,ld_o", [(1, 1, 1), (3, 5, 3), (8, 8, 16), (128, 128, 128),
                                         (100, 104, 128), (256, 256, 264), (13, 17, 15)])
def test_bf16_gather_push_bit_exact(env, d, ld_t, ld_o):
    sat, gu, torch = env
    _say("bf16 gather/push d=%d ld_t=%d ld_o=%d" % (d, ld_t, ld_o))
    rng = np.random.default_rng(d)
    n_rows, n = 3000, 2222
    table = rng.integers(0, 65536, size=(n_rows, ld_t)).astype(np.uint16)
    ids = rng.integers(0, n_rows, size=n).astype(np.int32)
    t_d, i_d = gu.to_dev_bits(table), gu.to_dev(ids)
    out = torch.full((n, ld_o), 77, dtype=torch.int16, device=gu.DEV)
    sat.history_gather(t_d, n_rows, ld_t, i_d, n, d, out, ld_o, dtype=sat.BF16, stream=gu.stream_ptr())
    gu.sync()
    got = gu.bits_to_host(out)
    assert np.array_equal(got[:, :d], orc.history_gather(table, ids)[:, :d])
    assert np.all(got[:, d:] == 77)
    pid = rng.permutation(n_rows)[:n].astype(np.int32)
    H = rng.integers(0, 65536, size=(n, ld_o)).astype(np.uint16)
    ref = orc.history_push(table.copy(), pid, H[:, :d])
    sat.history_push(t_d, n_rows, ld_t, gu.to_dev(pid), n, d, gu.to_dev_bits(H), ld_o,
                     dtype=sat.BF16, stream=gu.stream_ptr())
    gu.sync()
    assert np.array_equal(gu.bits_to_host(t_d), ref)


def _graph(kind):
    from tests.test_gpu_parity import _graph as g
    return g(kind)


@pytest.mark.parametrize("kind,d", [("tiny", 64), ("tiny", 8), ("powerlaw", 128), ("powerlaw", 256),
                                    ("hub", 256), ("hub", 128), ("powerlaw", 100), ("tiny", 1),
                                    ("onepart", 600), ("tiny", 2056)])
def test_bf16_spmm_parity(env, kind, d):
    sat, gu, torch = env
    _say("bf16 spmm %s d=%d" % (kind, d))
    g = _graph(kind)
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    n_l, n_h = v["n_local"], v["n_halo"]
    rng = np.random.default_rng(d)
    hb_bits, hb = _bf16(rng.standard_normal((n_l + n_h, d)).astype(np.float32))
    g_bits, gv = _bf16(rng.standard_normal((n_l, d)).astype(np.float32))
    ld = gu.ld_for(d, 8)
    pv = gu.upload_view(v)
    agg = torch.full((n_l, ld), 77, dtype=torch.int16, device=gu.DEV)
    sat.spmm_fwd(pv, gu.to_dev_bits(hb_bits, ld), ld, d, agg, ld, dtype=sat.BF16, stream=gu.stream_ptr())
    dl = torch.full((n_l, ld), 77, dtype=torch.int16, device=gu.DEV)
    dh = torch.full((max(n_h, 1), ld), 77, dtype=torch.int16, device=gu.DEV)
    sat.spmm_bwd(pv, gu.to_dev_bits(g_bits, ld), ld, d, dl, ld, dh if n_h else None, ld,
                 dtype=sat.BF16, stream=gu.stream_ptr())
    gu.sync()
    got = syn.f32_from_bf16_bits(gu.bits_to_host(agg, d))
    gu.assert_close(got, orc.spmm_fwd(v, hb), RTOL_BF16, "bf16 spmm_fwd")
    assert np.all(gu.bits_to_host(agg)[:, d:] == 77)
    # the result is the fp32 sum rounded once: it must sit within one bf16 step of the oracle
    ref = orc.spmm_fwd(v, hb)
    rms = np.sqrt(np.mean(ref * ref))
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * rms)
    rl, rh = orc.spmm_bwd(v, gv, want_halo=True)
    gu.assert_close(syn.f32_from_bf16_bits(gu.bits_to_host(dl, d)), rl, RTOL_BF16, "bf16 spmm_bwd")
    if n_h:
        gu.assert_close(syn.f32_from_bf16_bits(gu.bits_to_host(dh, d))[:n_h], rh, RTOL_BF16,
                        "bf16 spmm_bwd halo")
