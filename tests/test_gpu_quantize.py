"""GPU parity: aiq_quantize_weights against the oracle, bit for bit (codes, scales, dequantized values)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

BITS = (32, 16, 8, 6, 4, 2)
# (cout, k): dense 3x3 rows of the ResNet stages, the stem, depthwise, MobileNetV2 1x1 and classifier
# rows, plus ragged sizes around the 64-lane and 4-channels-per-block tiling
SHAPES = [(16, 27), (16, 144), (32, 288), (64, 576), (96, 9), (10, 64), (10, 1280), (160, 960),
          (1, 1), (3, 63), (5, 65), (7, 129), (130, 200),
          # row-in-registers path: one 16-byte element per lane exactly, one over, its largest row, one beyond it
          (9, 256), (6, 260), (5, 1284), (3, 2564), (5, 5120), (2, 5124), (3, 8192)]


@pytest.fixture(scope="module")
def aiq():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2512_14090_amd as m
    m.load_library()
    return m


def _w(cout, k, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    w = (rng.standard_normal((cout, k)) * np.sqrt(2.0 / k)).astype(np.float32)
    g = rng.uniform(0.7, 1.3, cout).astype(np.float32)
    return (w * g[:, None]).astype(np.float32)


@pytest.mark.parametrize("bits", BITS)
def test_bit_exact_against_oracle(aiq, bits):
    import torch
    import oracle
    for i, (cout, k) in enumerate(SHAPES):
        w = _w(cout, k, 1000 + i)
        if cout > 2:
            w[1] = 0.0  # all-zero channel
        print(f"quantize bits={bits} cout={cout} k={k}", flush=True)
        w_dq, s, q = aiq.quantize_weights(torch.from_numpy(w).cuda(), bits, want_codes=True)
        torch.cuda.synchronize()
        r_dq, r_s, r_q = oracle.quantize_weights(w, bits)
        assert s.cpu().numpy().tobytes() == r_s.tobytes(), (bits, cout, k)
        assert w_dq.cpu().numpy().tobytes() == r_dq.tobytes(), (bits, cout, k)
        if bits != 32:
            np.testing.assert_array_equal(q.cpu().numpy(), r_q)


def test_half_way_quotients_and_extremes(aiq):
    """Rows built so that many quotients are exact .5 ties, plus huge and tiny magnitudes."""
    import torch
    import oracle
    rows = []
    for scale in (1.0, 2.0 ** -20, 2.0 ** 30, 3.0e-38, 1.0e36):
        r = np.arange(-127, 128, dtype=np.float32) * np.float32(0.5) * np.float32(scale)
        rows.append(np.concatenate([r, [np.float32(63.5 * scale)]]).astype(np.float32))
    w = np.stack(rows)
    for bits in (16, 8, 6, 4, 2):
        w_dq, s, q = aiq.quantize_weights(torch.from_numpy(w).cuda(), bits)
        torch.cuda.synchronize()
        r_dq, r_s, r_q = oracle.quantize_weights(w, bits)
        assert s.cpu().numpy().tobytes() == r_s.tobytes(), bits
        np.testing.assert_array_equal(q.cpu().numpy(), r_q)
        assert w_dq.cpu().numpy().tobytes() == r_dq.tobytes(), bits


def test_stress_shape_sample(aiq):
    """The bandwidth-stress shape (8192 x 4608): a sample of rows is compared one by one."""
    import torch
    import oracle
    rng = np.random.Generator(np.random.PCG64(77))
    w = (rng.standard_normal((8192, 4608)) * 0.02).astype(np.float32)
    wd = torch.from_numpy(w).cuda()
    for bits in (8, 4):
        w_dq, s, q = aiq.quantize_weights(wd, bits, want_codes=False)
        torch.cuda.synchronize()
        rows = rng.choice(8192, 64, replace=False)
        r_dq, r_s, _ = oracle.quantize_weights(w[rows], bits)
        assert s.cpu().numpy()[rows].tobytes() == r_s.tobytes()
        assert w_dq[torch.from_numpy(rows).cuda()].cpu().numpy().tobytes() == r_dq.tobytes()
        # invariant at full size: every element is an integer multiple of its row scale within [-qmax, qmax]
        qmax = 2 ** (bits - 1) - 1
        ratio = (w_dq / s[:, None]).round().abs().max().item()
        assert ratio == qmax


@pytest.mark.parametrize("bits", BITS)
def test_per_tensor_bit_exact_against_oracle(aiq, bits):
    """One scale per matrix: codes, the (replicated) scale and the dequantized values, bit for bit."""
    import torch
    import oracle
    for i, (cout, k) in enumerate(SHAPES):
        w = _w(cout, k, 2000 + i)
        print(f"per-tensor quantize bits={bits} cout={cout} k={k}", flush=True)
        w_dq, s, q = aiq.quantize_weights(torch.from_numpy(w).cuda(), bits, want_codes=True, per_tensor=True)
        torch.cuda.synchronize()
        r_dq, r_s, r_q = oracle.quantize_weights(w, bits, per_tensor=True)
        assert s.cpu().numpy().tobytes() == r_s.tobytes(), (bits, cout, k)
        assert w_dq.cpu().numpy().tobytes() == r_dq.tobytes(), (bits, cout, k)
        if bits != 32:
            np.testing.assert_array_equal(q.cpu().numpy(), r_q)
    # all-zero matrix: scale 1, codes 0
    z = torch.zeros((3, 8), dtype=torch.float32, device="cuda")
    w_dq, s, q = aiq.quantize_weights(z, 8, per_tensor=True)
    torch.cuda.synchronize()
    assert s.cpu().tolist() == [1.0] * 3 and not w_dq.any().item()


def test_unaligned_rows_take_the_scalar_path(aiq):
    """A weight matrix that starts 4 bytes into an allocation (rows not 16-byte aligned)."""
    import torch
    import oracle
    w = _w(12, 288, 5)
    buf = torch.zeros(12 * 288 + 1, dtype=torch.float32, device="cuda")
    buf[1:] = torch.from_numpy(w).reshape(-1).cuda()
    wv = buf[1:].view(12, 288)
    assert wv.data_ptr() % 16 == 4
    for bits in (8, 2):
        w_dq, s, q = aiq.quantize_weights(wv, bits)
        torch.cuda.synchronize()
        r_dq, r_s, r_q = oracle.quantize_weights(w, bits)
        assert s.cpu().numpy().tobytes() == r_s.tobytes()
        assert w_dq.cpu().numpy().tobytes() == r_dq.tobytes()
        np.testing.assert_array_equal(q.cpu().numpy(), r_q)


def test_empty_and_errors(aiq):
    import torch
    w = torch.zeros((0, 5), dtype=torch.float32, device="cuda")
    aiq.quantize_weights(w, 8)
    w = torch.zeros((4, 0), dtype=torch.float32, device="cuda")
    _, s, _ = aiq.quantize_weights(w, 8)
    torch.cuda.synchronize()
    assert s.cpu().tolist() == [1.0] * 4
    w = torch.ones((2, 2), dtype=torch.float32, device="cuda")
    for bad in (0, 3, 5, 7, 12, 33):
        with pytest.raises(aiq.AiqError) as e:
            aiq.quantize_weights(w, bad)
        assert e.value.code == 2
