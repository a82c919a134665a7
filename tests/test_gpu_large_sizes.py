"""GPU parity at sizes whose element indices do not fit 32 bits: tensors of more than 2^32
elements through the Q node, the random stream and the update.  The tensors live on the GPU only
(tens of GB); the oracle computes sampled elements one by one -- the head, the ragged tail, both
sides of index 2^32 and random positions."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

TWO32 = 1 << 32


@pytest.fixture(scope="module")
def mp8():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1905_12334_amd as m
    m.lib()
    return m


def sample_indices(n, seed):
    rng = np.random.default_rng(seed)
    parts = [np.arange(0, 2048), np.arange(n - 2048, n), np.arange(TWO32 - 1024, min(TWO32 + 1024, n)),
             rng.integers(0, n, 20000)]
    return np.unique(np.concatenate(parts).astype(np.int64))


def take(t, idx):
    import torch
    return t.reshape(-1)[torch.from_numpy(idx).cuda()].cpu().numpy()


def oracle_sr_codes(x, idx, seed, offset):
    """Element by element: the code of x[i] with the random halfword of stream position idx[i]."""
    return np.array([oracle.e5m2_encode(float(v), oracle.SR, oracle.sr_bits(seed, offset, int(i)))
                     for v, i in zip(x, idx)], dtype=np.uint8)


def test_quantize_flat_beyond_2_32_elements(mp8):
    import torch
    n = TWO32 + 3 * 4096 + 3            # three elements in the ragged tail
    x = torch.empty((1, n), dtype=torch.float32, device="cuda").normal_()
    x.mul_(torch.empty((1, n), dtype=torch.float32, device="cuda").uniform_(0.0, 8.0).exp2_())
    idx = sample_indices(n, 1)
    xs = take(x, idx)
    d = torch.full((n + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    seed, offset = 0x5EED_0000_1234, 9
    mp8.quantize_e5m2(x, d[:n], round=mp8.SR, seed=seed, offset=offset)
    torch.cuda.synchronize()
    assert bool((d[n:] == 0xAA).all()), "write past the end of dst"
    assert np.array_equal(take(d[:n], idx), oracle_sr_codes(xs, idx, seed, offset))
    # the variant that gathers statistics (other block shape, grid-stride loop): same codes everywhere
    d2 = torch.empty(n, dtype=torch.uint8, device="cuda")
    st = mp8.new_stats()
    mp8.quantize_e5m2(x, d2, round=mp8.SR, seed=seed, offset=offset, stats=st)
    torch.cuda.synchronize()
    assert bool(torch.equal(d2, d[:n]))
    # round to nearest even, against the oracle's array routine on the sampled values
    mp8.quantize_e5m2(x, d[:n], round=mp8.RNE)
    torch.cuda.synchronize()
    assert np.array_equal(take(d[:n], idx), oracle.quantize_e5m2(xs.reshape(1, -1))[0].reshape(-1))


def test_quantize_with_transposed_copy_beyond_2_32_elements(mp8):
    import torch
    rows, cols = 65536 + 4, 65536 + 8   # ragged against the 128 x 128 tiles
    n = rows * cols
    assert n > TWO32
    x = torch.empty((rows, cols), dtype=torch.float32, device="cuda").normal_()
    idx = sample_indices(n, 2)
    xs = take(x, idx)
    d = torch.full((n + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    dt = torch.full((n + 64,), 0xAA, dtype=torch.uint8, device="cuda")
    seed, offset = 77, 3
    mp8.quantize_e5m2(x, d[:n].view(rows, cols), dt[:n].view(cols, rows), round=mp8.SR, seed=seed, offset=offset)
    torch.cuda.synchronize()
    assert bool((d[n:] == 0xAA).all()) and bool((dt[n:] == 0xAA).all()), "write past the end"
    want = oracle_sr_codes(xs, idx, seed, offset)
    assert np.array_equal(take(d[:n], idx), want)
    r, c = idx // cols, idx % cols
    assert np.array_equal(take(dt[:n], c * rows + r), want)
    del x
    assert bool(torch.equal(dt[:n].view(cols, rows).t(), d[:n].view(rows, cols))), "copies differ somewhere"


def test_random_stream_beyond_2_32_elements(mp8):
    import torch
    n = TWO32 + 1000
    out = torch.empty(n, dtype=torch.int16, device="cuda")
    seed, offset = 0xABCDEF, 1 << 40
    mp8.sr_bits(out, seed, offset)
    torch.cuda.synchronize()
    idx = sample_indices(n, 3)
    got = take(out, idx).view(np.uint16)
    assert got.tolist() == [oracle.sr_bits(seed, offset, int(i)) for i in idx]


def test_update_beyond_2_32_elements(mp8):
    import torch
    n = TWO32 + 8 * 777 + 5             # five elements in the ragged tail
    w = torch.empty(n, dtype=torch.float16, device="cuda").normal_(0, 0.05)
    g = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 256)
    g = torch.where((g & 0x7C) == 0x7C, g & 0xBF, g)          # finite codes only
    idx = sample_indices(n, 4)
    ws, gs = take(w.view(torch.int16), idx).view(np.uint16), take(g, idx)
    mp8.sgd_update_fp16_sr(w.view(torch.int16), g, 0.02, 1.0 / 1024, round=mp8.RNE)
    torch.cuda.synchronize()
    want, _ = oracle.sgd_update_fp16(ws, gs, 0.02, 1.0 / 1024, mode=oracle.RNE)
    assert np.array_equal(take(w.view(torch.int16), idx).view(np.uint16), want)
