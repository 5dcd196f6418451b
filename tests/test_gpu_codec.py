"""GPU parity of the compression codec of stored embeddings (decimal rounding +
Encoded Polyline character coding): row offsets and code bytes bit for bit
against the oracle, decoded values bit for bit (one correctly rounded division on
both sides), the lossy error bound, gather-by-id decoding and the bf16 storage
mode."""
import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    import paper_2308_13466_amd as sat
    sat.lib()
    from tests import gpu_util as gu
    return sat, gu, torch


def _compress(sat, gu, torch, H_dev, ld, n, d, prec, dtype):
    wsb = sat.history_compress_workspace_bytes(n)
    ws = torch.zeros(max(wsb // 8, 1) + 1, dtype=torch.int64, device=gu.DEV)
    row_off = torch.full((n + 1,), -1, dtype=torch.int64, device=gu.DEV)
    sat.history_compress_plan(H_dev, ld, n, d, prec, row_off, dtype=dtype, workspace=ws,
                              workspace_bytes=wsb, stream=gu.stream_ptr())
    gu.sync()
    total = int(row_off[-1].item())
    codes = torch.full((total + 16,), 7, dtype=torch.uint8, device=gu.DEV)   # 16 guard bytes
    sat.history_compress_encode(H_dev, ld, n, d, prec, row_off, codes, total, dtype=dtype,
                                stream=gu.stream_ptr())
    gu.sync()
    return row_off, codes, total


@pytest.mark.parametrize("n,d,ld,prec", [(3000, 256, 256, 2), (5000, 100, 104, 1), (777, 37, 40, 4),
                                         (2049, 1, 4, 3), (4100, 602, 608, 2), (1, 64, 64, 0),
                                         (1501, 370, 376, 2)])   # rows around 512 bytes: both decoder paths
def test_codec_fp32_bit_exact(env, n, d, ld, prec):
    sat, gu, torch = env
    print("[case] codec fp32 n=%d d=%d precision=%d" % (n, d, prec), flush=True)
    rng = np.random.default_rng(n + d)
    H = (np.maximum(rng.standard_normal((n, d)), 0) * 2.0).astype(np.float32)   # relu-shaped
    H[rng.integers(0, n, 20), rng.integers(0, d, 20)] = -rng.random(20).astype(np.float32) * 300.0
    H_dev = gu.to_dev(H, ld)
    row_off, codes, total = _compress(sat, gu, torch, H_dev, ld, n, d, prec, 0)
    ref_codes, ref_off = orc.polyline_encode_rows(H, prec)
    assert np.array_equal(row_off.cpu().numpy(), ref_off)
    got = codes.cpu().numpy()
    assert np.array_equal(got[:total], ref_codes) and np.all(got[total:] == 7)
    # decode: every row, then a gather with repeats and bad ids
    out = gu.dev_empty(n, ld, fill=-9.0)
    sat.history_decompress(codes, row_off, n, None, n, d, prec, out, ld, stream=gu.stream_ptr())
    ids = rng.integers(0, n, size=min(n, 500)).astype(np.int32)
    if ids.size > 2:
        ids[0], ids[1] = -1, n
    out2 = gu.dev_empty(ids.size, ld, fill=-9.0)
    sat.history_decompress(codes, row_off, n, gu.to_dev(ids), ids.size, d, prec, out2, ld,
                           stream=gu.stream_ptr())
    gu.sync()
    back = orc.polyline_decode_rows(ref_codes, ref_off, np.arange(n), d, prec)
    got = out.cpu().numpy()
    assert np.array_equal(got[:, :d].view(np.uint32), back.view(np.uint32))
    assert np.all(got[:, d:] == -9.0)
    assert np.abs(back.astype(np.float64) - H).max() <= 0.5 * 10.0 ** -prec * (1 + 1e-5) + 3e-5
    got2 = out2.cpu().numpy()
    ok = (ids >= 0) & (ids < n)
    assert np.array_equal(got2[ok][:, :d], back[ids[ok]]) and np.all(got2[~ok] == -9.0)
    print("[case] ratio %.2fx against fp32" % (4.0 * n * d / max(total, 1)), flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_codec_out_of_range_nan_and_inf(env, dtype):
    """Values whose quantised magnitude would pass 2^30 saturate there (7-byte codes), +-inf
    with them, NaN and -0.0 code as 0: offsets, code bytes and decoded values bit for bit
    against the oracle, rows mixing such values with ordinary ones (every encoder path)."""
    sat, gu, torch = env
    print("[case] codec edge values %s" % dtype, flush=True)
    rng = np.random.default_rng(17)
    n, d, ld = 530, 72, 72
    H = (rng.standard_normal((n, d)) * 2.0).astype(np.float32)
    edge = [1e30, -1e30, np.inf, -np.inf, np.nan, -0.0, 3.4e38, -3.4e38, 1073741824.0, -1073741824.0,
            1.0737418e7, -1.0737418e7, 1.07374e7, 5e9, -5e9]
    where = rng.integers(0, n * d, size=600)
    H.reshape(-1)[where] = np.array([edge[i % len(edge)] for i in range(600)], dtype=np.float32)
    H[7, :] = np.inf                      # a row of 7-byte codes only: the longest row a width can give
    H[8, :] = np.nan
    bf16 = dtype == "bf16"
    if bf16:
        bits = syn.bf16_bits_from_f32(H)
        H = syn.f32_from_bf16_bits(bits)
        H_dev = gu.to_dev_bits(bits, ld)
    else:
        H_dev = gu.to_dev(H, ld)
    for prec in (0, 2):
        row_off, codes, total = _compress(sat, gu, torch, H_dev, ld, n, d, prec, 1 if bf16 else 0)
        ref_codes, ref_off = orc.polyline_encode_rows(H, prec)
        assert np.array_equal(row_off.cpu().numpy(), ref_off)
        assert ref_off[8] - ref_off[7] == 7 * d and ref_off[9] - ref_off[8] == d
        got = codes.cpu().numpy()
        assert np.array_equal(got[:total], ref_codes) and np.all(got[total:] == 7)
        back = orc.polyline_decode_rows(ref_codes, ref_off, np.arange(n), d, prec)
        if bf16:
            out = torch.zeros((n, ld), dtype=torch.int16, device=gu.DEV)
            sat.history_decompress(codes, row_off, n, None, n, d, prec, out, ld, dtype=1,
                                   stream=gu.stream_ptr())
            gu.sync()
            assert np.array_equal(gu.bits_to_host(out, d), syn.bf16_bits_from_f32(back))
        else:
            out = gu.dev_empty(n, ld, fill=-9.0)
            sat.history_decompress(codes, row_off, n, None, n, d, prec, out, ld, stream=gu.stream_ptr())
            gu.sync()
            assert np.array_equal(out.cpu().numpy()[:, :d].view(np.uint32), back.view(np.uint32))
        assert np.isfinite(back).all() and np.abs(back).max() == np.float32(2.0 ** 30) / np.float32(10.0 ** prec)


@pytest.mark.parametrize("case", ["unaligned_codes", "wide_rows", "unaligned_rows"])
def test_codec_encoder_paths_give_the_same_bytes(env, case):
    """The encoder assembles rows in LDS and writes 16-byte pieces when the code array is 16-byte
    aligned and a row has at most 2338 values, and writes byte by byte otherwise; rows whose start
    is not 16-byte aligned are read value by value. Every path must give the oracle's bytes."""
    sat, gu, torch = env
    print("[case] codec encoder path: " + case, flush=True)
    rng = np.random.default_rng(31)
    n, d, ld, prec = (300, 2400, 2400, 2) if case == "wide_rows" else (1500, 130, 131 if case == "unaligned_rows" else 136, 2)
    H = (np.maximum(rng.standard_normal((n, d)), 0) * 2.0).astype(np.float32)
    H[rng.integers(0, n, 20), rng.integers(0, d, 20)] = -rng.random(20).astype(np.float32) * 3000.0
    H_dev = gu.to_dev(H, ld)
    wsb = sat.history_compress_workspace_bytes(n)
    ws = torch.zeros(max(wsb // 8, 1) + 1, dtype=torch.int64, device=gu.DEV)
    row_off = torch.full((n + 1,), -1, dtype=torch.int64, device=gu.DEV)
    sat.history_compress_plan(H_dev, ld, n, d, prec, row_off, workspace=ws, workspace_bytes=wsb,
                              stream=gu.stream_ptr())
    gu.sync()
    total = int(row_off[-1].item())
    ref_codes, ref_off = orc.polyline_encode_rows(H, prec)
    assert np.array_equal(row_off.cpu().numpy(), ref_off) and total == ref_codes.size
    buf = torch.full((total + 64,), 7, dtype=torch.uint8, device=gu.DEV)
    shift = 5 if case == "unaligned_codes" else 16
    codes = buf[shift:shift + total + 16]
    assert (codes.data_ptr() % 16 == 0) == (case != "unaligned_codes")
    sat.history_compress_encode(H_dev, ld, n, d, prec, row_off, codes, total, stream=gu.stream_ptr())
    gu.sync()
    got = buf.cpu().numpy()
    assert np.array_equal(got[shift:shift + total], ref_codes)
    assert np.all(got[:shift] == 7) and np.all(got[shift + total:] == 7)     # nothing outside [0, total)


def test_codec_bf16_storage(env):
    sat, gu, torch = env
    from paper_2308_13466_amd import binding as B
    print("[case] codec bf16", flush=True)
    rng = np.random.default_rng(8)
    n, d, ld, prec = 4000, 256, 256, 2
    Hb = syn.bf16_bits_from_f32(np.maximum(rng.standard_normal((n, d)), 0).astype(np.float32))
    H = syn.f32_from_bf16_bits(Hb)
    H_dev = gu.to_dev_bits(Hb, ld)
    row_off, codes, total = _compress(sat, gu, torch, H_dev, ld, n, d, prec, B.BF16)
    ref_codes, ref_off = orc.polyline_encode_rows(H, prec)
    assert np.array_equal(row_off.cpu().numpy(), ref_off)
    assert np.array_equal(codes.cpu().numpy()[:total], ref_codes)
    out = gu.to_dev_bits(np.zeros((n, d), np.uint16), ld)
    sat.history_decompress(codes, row_off, n, None, n, d, prec, out, ld, dtype=B.BF16,
                           stream=gu.stream_ptr())
    gu.sync()
    back = orc.round_bf16(orc.polyline_decode_rows(ref_codes, ref_off, np.arange(n), d, prec))
    assert np.array_equal(syn.f32_from_bf16_bits(gu.bits_to_host(out, d)), back.astype(np.float32))


def test_codec_large_table_offsets(env):
    """More rows than one scan workgroup covers twice over (three scan levels)."""
    sat, gu, torch = env
    print("[case] codec offsets, 5M rows", flush=True)
    n, d, prec = 5_000_000, 4, 1
    rng = np.random.default_rng(3)
    H = (rng.standard_normal((n, d)) * 5).astype(np.float32)
    H_dev = gu.to_dev(H)
    row_off, codes, total = _compress(sat, gu, torch, H_dev, d, n, d, prec, 0)
    q = orc.polyline_quantise(H, prec)
    u = (q << 1) ^ (q >> 63)
    bits = np.where(u > 0, np.floor(np.log2(np.maximum(u, 1))).astype(np.int64) + 1, 1)
    sizes = ((bits + 4) // 5).sum(axis=1)
    ref_off = np.zeros(n + 1, np.int64)
    np.cumsum(sizes, out=ref_off[1:])
    assert np.array_equal(row_off.cpu().numpy(), ref_off)
    rows = rng.integers(0, n, size=2000)
    sub_codes, sub_off = orc.polyline_encode_rows(H[rows], prec)
    got = codes.cpu().numpy()
    for j, r in enumerate(rows[:200]):
        assert np.array_equal(got[ref_off[r]:ref_off[r + 1]], sub_codes[sub_off[j]:sub_off[j + 1]])


def test_codec_argument_checks(env):
    sat, gu, torch = env
    H = gu.dev_empty(8, 8)
    ro = torch.zeros(9, dtype=torch.int64, device=gu.DEV)
    with pytest.raises(sat.SatError):
        sat.history_compress_plan(H, 8, 8, 8, 12, ro, workspace=ro, workspace_bytes=72)   # precision
    with pytest.raises(sat.SatError) as e:
        sat.history_compress_plan(H, 8, 8, 8, 2, ro, workspace=None, workspace_bytes=0)
    assert e.value.status == -4
