"""GPU parity of the wire form of a message (dgs_encode / dgs_decode) against the oracle's
byte-by-byte statement of it: byte-exact both ways.  The layout is this library's own (the
paper asks only for coordinate format), so the parity is to that statement, not to the paper."""
import numpy as np
import pytest

from paper_1910_10929_amd import dgs, synth
from harness import Worker, to_dev, to_host_u32

pytestmark = pytest.mark.gpu


def random_message(oracle, off, rho, rng):
    kj, K = oracle.nnz(off, rho)
    idx = np.concatenate([np.sort(rng.choice(int(off[j + 1] - off[j]), int(kj[j]), replace=False)) + int(off[j])
                          for j in range(len(off) - 1)]).astype(np.uint32)
    val = rng.integers(0, 1 << 32, K, dtype=np.uint64).astype(np.uint32).view(np.float32)   # any bit pattern
    return idx, val


def check_both_ways(oracle, ctx, off, rho, idx, val):
    import torch
    K = idx.size
    want = oracle.encode(off, rho, idx, val)
    assert ctx.wire_bytes(rho) == want.size == oracle.wire_bytes(off, rho)
    wire = torch.full((want.size,), 0xA5, dtype=torch.uint8, device=ctx.device)    # every byte must be written
    ctx.encode(rho, to_dev(idx, ctx.device), to_dev(val, ctx.device), wire)
    torch.cuda.synchronize()
    got = wire.cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.nonzero(got != want)[0]
        raise AssertionError(f"{bad.size} wire bytes differ, first at {bad[0]} of {want.size} (values end at {4 * K})")
    di = torch.zeros(K, dtype=torch.int32, device=ctx.device)
    dv = torch.zeros(K, dtype=torch.float32, device=ctx.device)
    ctx.decode(rho, to_dev(want, ctx.device), di, dv)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u32(di), idx)
    assert np.array_equal(dv.cpu().numpy().view(np.uint32), val.view(np.uint32))


SIZES = [1, 2, 3, 31, 32, 33, 255, 256, 257, 1000, 4096, 65_536, 65_537, 100_003, 1 << 20, 5, 3_000_000]


@pytest.mark.parametrize("rho", [1e-6, 1e-3, 0.01, 0.3, 1.0])
def test_wire_form_ragged_layout(oracle, rho):
    off = synth.offsets_from_sizes(SIZES)
    rng = np.random.default_rng(90)
    ctx = dgs.Context(off, W=0)
    ctx.set_option(dgs.OPT_VALIDATE, 1)
    for _ in range(2):
        idx, val = random_message(oracle, off, rho, rng)
        check_both_ways(oracle, ctx, off, rho, idx, val)
    ctx.close()


def check_both_ways16(oracle, ctx, off, rho, idx, val):
    """The same with bfloat16 values: wire bytes against the oracle's, decoded values against the
    oracle's decoding (the rounded values widened again, bit for bit)."""
    import torch
    K = idx.size
    want = oracle.encode16(off, rho, idx, val)
    assert ctx.wire_bytes(rho) == want.size == oracle.wire_bytes16(off, rho)
    wire = torch.full((want.size,), 0xA5, dtype=torch.uint8, device=ctx.device)
    ctx.encode(rho, to_dev(idx, ctx.device), to_dev(val, ctx.device), wire)
    torch.cuda.synchronize()
    got = wire.cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.nonzero(got != want)[0]
        raise AssertionError(f"{bad.size} wire bytes differ, first at {bad[0]} of {want.size} (values end at {2 * K})")
    wi, wv = oracle.decode16(off, rho, want)
    di = torch.zeros(K, dtype=torch.int32, device=ctx.device)
    dv = torch.zeros(K, dtype=torch.float32, device=ctx.device)
    ctx.decode(rho, to_dev(want, ctx.device), di, dv)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u32(di), idx) and np.array_equal(wi, idx)
    assert np.array_equal(dv.cpu().numpy().view(np.uint32), wv.view(np.uint32))


@pytest.mark.parametrize("rho", [1e-6, 1e-3, 0.01, 0.3, 1.0])
def test_wire_form_with_bfloat16_values(oracle, rho):
    """DGS_OPT_WIRE_VALUE_BITS = 16: any bit pattern as a value (NaNs, infinities, subnormals,
    halfway cases planted), odd and even K, and back to 32 bits on the same context."""
    off = synth.offsets_from_sizes(SIZES)
    rng = np.random.default_rng(91)
    ctx = dgs.Context(off, W=0)
    ctx.set_option(dgs.OPT_WIRE_VALUE_BITS, 16)
    for _ in range(2):
        idx, val = random_message(oracle, off, rho, rng)
        planted = np.array([0x3F808000, 0x3F818000, 0x00018000, 0x7F7FFFFF, 0x7F800001, 0xFF7FFFFF, 0x007F8000],
                           np.uint32)
        m = min(planted.size, val.size)
        val.view(np.uint32)[:m] = planted[:m]
        check_both_ways16(oracle, ctx, off, rho, idx, val)
    ctx.set_option(dgs.OPT_WIRE_VALUE_BITS, 32)
    idx, val = random_message(oracle, off, rho, rng)
    check_both_ways(oracle, ctx, off, rho, idx, val)
    with pytest.raises(dgs.DgsError):
        ctx.set_option(dgs.OPT_WIRE_VALUE_BITS, 8)
    ctx.close()


def test_wire_form_of_a_worker_message_resnet50_shapes(oracle):
    """25,557,032 parameters, density 1e-3: the message dgs_worker_step returns, encoded on the
    device, decoded, pushed; bytes against the oracle's encoding of the oracle's message."""
    import torch
    off = synth.layout_resnet50()
    n = int(off[-1])
    scales = synth.tensor_scales(len(off) - 1, 91)
    rng = np.random.default_rng(92)
    g = synth.gaussian_grads(off, scales, rng)
    s_ref = np.zeros(n, np.float32)
    wi, wv = oracle.worker_step(g, s_ref, off, 1.0, np.float32(0.9), 1e-3)
    want = oracle.encode(off, 1e-3, wi, wv)
    ctx = dgs.Context(off, W=0)
    w = Worker(ctx, density_max=1e-3)
    w.step(g, 1.0, 0.9, 1e-3)
    wire = torch.zeros(ctx.wire_bytes(1e-3), dtype=torch.uint8, device=ctx.device)
    ctx.encode(1e-3, w.idx, w.val, wire)
    di = torch.zeros_like(w.idx)
    dv = torch.zeros_like(w.val)
    ctx.decode(1e-3, wire, di, dv)
    torch.cuda.synchronize()
    assert np.array_equal(wire.cpu().numpy(), want)
    assert want.size == 4 * 25_670 + 4 * sum((int(k) * max(1, (int(nj) - 1).bit_length()) + 31) // 32
                                              for k, nj in zip(oracle.nnz(off, 1e-3)[0], np.diff(off)))
    assert np.array_equal(to_host_u32(di), wi) and np.array_equal(dv.cpu().numpy().view(np.uint32), wv.view(np.uint32))
    ctx.close()


def test_wire_form_ten_million_entries(oracle):
    """1e9 parameters in 64 tensors at density 1e-2 (K = 1e7, 24-bit indices): round trip on the
    device, and the oracle's bytes for three sampled tensors' blocks plus all the values."""
    import torch
    off = synth.layout_equal(1_000_000_000, 64)
    rho = 1e-2
    nj, kj = 15_625_000, 156_250
    rng = np.random.default_rng(93)
    base = rng.choice(nj, kj, replace=False).astype(np.uint64)
    local = [np.sort((base + 7 * j) % nj).astype(np.uint32) for j in range(64)]   # distinct per tensor
    idx = np.concatenate([(local[j].astype(np.uint64) + j * nj).astype(np.uint32) for j in range(64)])
    val = rng.standard_normal(idx.size).astype(np.float32)
    ctx = dgs.Context(off, W=0)
    K = ctx.nnz(rho)
    assert K == idx.size == 10_000_000
    nbytes = ctx.wire_bytes(rho)
    assert nbytes == 4 * K + 64 * 4 * ((kj * 24 + 31) // 32)
    wire = torch.zeros(nbytes, dtype=torch.uint8, device=ctx.device)
    d_idx, d_val = to_dev(idx, ctx.device), to_dev(val, ctx.device)
    ctx.encode(rho, d_idx, d_val, wire)
    di = torch.zeros_like(d_idx)
    dv = torch.zeros_like(d_val)
    ctx.decode(rho, wire, di, dv)
    torch.cuda.synchronize()
    assert torch.equal(di, d_idx) and torch.equal(dv.view(torch.int32), d_val.view(torch.int32))
    got = wire.cpu().numpy()
    assert np.array_equal(got[:4 * K], val.view(np.uint8))
    one = synth.layout_flat(nj)
    words = (kj * 24 + 31) // 32
    for j in (0, 37, 63):
        sl = slice(j * kj, (j + 1) * kj)
        ref = oracle.encode(one, rho, local[j], val[sl])
        block = got[4 * K + 4 * words * j: 4 * K + 4 * words * (j + 1)]
        assert np.array_equal(block, ref[4 * kj:]), f"index block of tensor {j}"
    ctx.close()
    del wire, d_idx, d_val, di, dv
    torch.cuda.empty_cache()


def test_wire_form_argument_errors_and_validation(oracle):
    import torch
    off = synth.offsets_from_sizes([100, 50])
    ctx = dgs.Context(off, W=0)
    L = dgs.lib()
    h = ctx._h
    rho = 0.02
    K = ctx.nnz(rho)                                  # 2 + 1
    idx = to_dev(np.array([5, 99, 120], np.uint32), ctx.device)
    val = torch.ones(K, device=ctx.device)
    wire = torch.zeros(ctx.wire_bytes(rho), dtype=torch.uint8, device=ctx.device)
    assert L.dgs_encode(h, 0.0, idx.data_ptr(), val.data_ptr(), wire.data_ptr()) == dgs.DGS_EINVAL
    assert L.dgs_encode(h, rho, None, val.data_ptr(), wire.data_ptr()) == dgs.DGS_EINVAL
    assert L.dgs_encode(h, rho, idx.data_ptr(), val.data_ptr(), wire.data_ptr() + 1) == dgs.DGS_EINVAL
    assert L.dgs_decode(h, rho, None, idx.data_ptr(), val.data_ptr()) == dgs.DGS_EINVAL
    assert L.dgs_wire_bytes(h, 1.5, None) == dgs.DGS_EINVAL
    ctx.set_option(dgs.OPT_VALIDATE, 1)
    bad = to_dev(np.array([5, 99, 20], np.uint32), ctx.device)          # third entry is not in tensor 1
    assert L.dgs_encode(h, rho, bad.data_ptr(), val.data_ptr(), wire.data_ptr()) == dgs.DGS_EINVAL
    assert L.dgs_encode(h, rho, idx.data_ptr(), val.data_ptr(), wire.data_ptr()) == dgs.DGS_OK
    torch.cuda.synchronize()
    w = wire.cpu().numpy().copy()
    assert np.array_equal(w, oracle.encode(off, rho, np.array([5, 99, 120], np.uint32), np.ones(3, np.float32)))
    w[4 * K] = 0x7F                                                      # local index 127 >= 100
    di = torch.zeros(K, dtype=torch.int32, device=ctx.device)
    assert L.dgs_decode(h, rho, to_dev(w, ctx.device).data_ptr(), di.data_ptr(), val.data_ptr()) == dgs.DGS_EINVAL
    assert L.dgs_decode(h, rho, wire.data_ptr(), di.data_ptr(), val.data_ptr()) == dgs.DGS_OK
    ctx.close()
