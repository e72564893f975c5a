"""GPU tests of the on-disk cache of transformed weights (Section 3.1.2): what is read back is
bit for bit what the weight transformation wrote, for every kind; files that do not match
the request are refused; reading the raw weights and transforming gives the same bytes as
reading the cache."""
import numpy as np
import pytest

from nnv_workloads import ConvLayer, layer_tensors

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2206_07446_amd as nnv
    assert torch.cuda.is_available(), "GPU tests need the HIP device"
    nnv.load()
    return nnv, torch


def transformed(nnv, torch, layer, kind, half, seed=3):
    dev = torch.device("cuda:0")
    desc = nnv.make_desc(layer, nnv.F16 if half else nnv.F32)
    w = torch.from_numpy(layer_tensors(layer, seed)[0]).to(dev)
    wt = torch.empty(nnv.nnv_transformed_bytes(desc, kind), dtype=torch.uint8, device=dev)
    nnv.nnv_transform_weights(desc, kind, w, wt)
    torch.cuda.synchronize()
    return desc, w, wt


CONV = ConvLayer("c3", 37, 14, 14, 20, 3, 3, 1, 1)
DW = ConvLayer("dw", 48, 14, 14, 48, 3, 3, 1, 1, 48)
CASES = [(CONV, 0, False), (CONV, 1, False), (CONV, 1, True), (CONV, 2, False), (CONV, 2, True), (CONV, 3, False),
         (CONV, 3, True), (CONV, 5, False), (DW, 4, False), (DW, 4, True)]


@pytest.mark.parametrize("layer,kind,half", CASES, ids=[f"{l.name}-k{k}-{'f16' if h else 'f32'}" for l, k, h in CASES])
def test_round_trip_is_bit_exact(env, tmp_path, layer, kind, half):
    nnv, torch = env
    desc, _, wt = transformed(nnv, torch, layer, kind, half)
    path = str(tmp_path / "w.nnvc")
    nnv.nnv_cache_write(path, desc, kind, wt)
    back = torch.full_like(wt, 0xA5)
    io = nnv.nnv_cache_read(path, desc, kind, back, verify=True)
    assert torch.equal(back, wt)
    assert io.bytes == wt.numel() and io.total_ms >= io.file_ms > 0 and io.direct_io in (0, 1)


def test_many_pieces_through_the_staging_ring(env, tmp_path):
    """37.7 MB of F(4x4) weights: five 8 MiB pieces alternate between the two pinned buffers."""
    nnv, torch = env
    layer = ConvLayer("l4", 512, 7, 7, 512, 3, 3, 1, 1)
    desc, _, wt = transformed(nnv, torch, layer, nnv.WINO_F4, False)
    assert wt.numel() > 4 * (8 << 20)
    path = str(tmp_path / "big.nnvc")
    nnv.nnv_cache_write(path, desc, nnv.WINO_F4, wt)
    for verify in (False, True):
        back = torch.zeros_like(wt)
        nnv.nnv_cache_read(path, desc, nnv.WINO_F4, back, verify=verify)
        assert torch.equal(back, wt)


def test_mismatching_file_is_refused_and_leaves_the_buffer_alone(env, tmp_path):
    nnv, torch = env
    desc, _, wt = transformed(nnv, torch, CONV, nnv.WINO_F4, False)
    path = str(tmp_path / "w.nnvc")
    nnv.nnv_cache_write(path, desc, nnv.WINO_F4, wt)
    other = nnv.make_desc(ConvLayer("o", 37, 14, 14, 24, 3, 3, 1, 1))
    for d, kind in ((desc, nnv.WINO_F2), (desc, nnv.WINO_F6), (other, nnv.WINO_F4), (nnv.make_desc(CONV, nnv.F16), nnv.WINO_F4)):
        back = torch.full((nnv.nnv_transformed_bytes(d, kind),), 0x5A, dtype=torch.uint8, device=wt.device)
        with pytest.raises(nnv.NnvError) as e:
            nnv.nnv_cache_read(path, d, kind, back)
        assert e.value.status == -9
        assert bool((back == 0x5A).all())
    # spatial size, stride and padding do not change the weights: such a descriptor may share the file
    same_w = nnv.make_desc(ConvLayer("s", 37, 28, 28, 20, 3, 3, 1, 1))
    back = torch.zeros_like(wt)
    nnv.nnv_cache_read(path, same_w, nnv.WINO_F4, back)
    assert torch.equal(back, wt)


def test_checksum_catches_a_flipped_payload_byte(env, tmp_path):
    nnv, torch = env
    desc, _, wt = transformed(nnv, torch, CONV, nnv.IM2COL_GEMM, False)
    path = str(tmp_path / "w.nnvc")
    nnv.nnv_cache_write(path, desc, nnv.IM2COL_GEMM, wt)
    raw = bytearray(open(path, "rb").read())
    assert len(raw) == 4096 + wt.numel()
    raw[4096 + 1234] ^= 0x10
    open(path, "wb").write(bytes(raw))
    back = torch.zeros_like(wt)
    nnv.nnv_cache_read(path, desc, nnv.IM2COL_GEMM, back, verify=False)      # unchecked read passes
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_cache_read(path, desc, nnv.IM2COL_GEMM, back, verify=True)
    assert e.value.status == -9
    # truncated payload
    open(path, "wb").write(bytes(raw[:4096 + 100]))
    with pytest.raises(nnv.NnvError) as e:
        nnv.nnv_cache_read(path, desc, nnv.IM2COL_GEMM, back)
    assert e.value.status == -9


def test_read_raw_then_transform_equals_read_cache(env, tmp_path):
    """The two cold-start alternatives of Table 2 end with the same bytes in device memory."""
    nnv, torch = env
    for kind in (nnv.IM2COL_GEMM, nnv.WINO_F2, nnv.WINO_F4, nnv.WINO_F6):
        desc, w, wt = transformed(nnv, torch, CONV, kind, False)
        raw_path, tx_path = str(tmp_path / "raw.nnvc"), str(tmp_path / "tx.nnvc")
        nnv.nnv_cache_write(raw_path, desc, nnv.DIRECT, w)
        nnv.nnv_cache_write(tx_path, desc, kind, wt)
        w2 = torch.zeros_like(w)
        nnv.nnv_cache_read(raw_path, desc, nnv.DIRECT, w2)
        assert torch.equal(w2, w)
        a = torch.zeros_like(wt)
        nnv.nnv_transform_weights(desc, kind, w2, a)
        b = torch.zeros_like(wt)
        nnv.nnv_cache_read(tx_path, desc, kind, b)
        torch.cuda.synchronize()
        assert torch.equal(a, b)


def test_file_payload_is_the_oracle_layout(env, tmp_path):
    """The payload on disk is the documented layout: the oracle's packing of the same weights."""
    from oracle import layouts as OL
    nnv, torch = env
    desc, w, wt = transformed(nnv, torch, CONV, nnv.IM2COL_GEMM, False)
    path = str(tmp_path / "w.nnvc")
    nnv.nnv_cache_write(path, desc, nnv.IM2COL_GEMM, wt)
    payload = np.frombuffer(open(path, "rb").read()[4096:], dtype=np.float32)
    exp = OL.pack_gemm(w.cpu().numpy(), False)
    assert np.array_equal(payload.view(np.uint32), exp.view(np.uint32))
