"""GPU parity of the layer's input quantisation (Section 5.3, first step) against the CPU oracle."""
import numpy as np
import pytest

from paper_2209_06979_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(2, 64, 16), (8, 4096, 64), (3, 1001), (5,), (1, 2)])
def test_absmax_and_int8_codes_equal_the_oracle(shape):
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    x = wl.normal_fp32(shape, 6000 + len(shape))
    xd = torch.from_numpy(x).cuda()
    m = float(mc.absmax(xd).cpu()[0])
    assert m == float(np.max(np.abs(x)))
    want, s = oracle.quantize_per_tensor(x, 8)
    assert np.float32(np.float64(m) / 127.0) == s
    got = mc.quantize(xd, float(s), 8).cpu().numpy()
    assert got.dtype == np.int8 and np.array_equal(got, want)


@pytest.mark.parametrize("shape", [(2, 64, 16), (8, 4096, 64), (3, 1002), (1, 2)])
def test_int4_codes_and_packing_equal_the_oracle(shape):
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    x = wl.normal_fp32(shape, 6100 + len(shape))
    q, s = oracle.quantize_per_tensor(x, 4)
    packed = oracle.pack_int4(q)
    got = mc.quantize(torch.from_numpy(x).cuda(), float(s), 4).cpu().numpy()
    assert got.dtype == np.uint8 and got.shape == packed.shape and np.array_equal(got, packed)
    assert np.array_equal(oracle.unpack_int4(got).astype(np.int8), q)


def test_rounding_boundaries_and_clamping():
    """Values placed on and next to the rounding boundaries of the fp64 definition, and far outside the range."""
    import torch
    import oracle
    from paper_2209_06979_amd import binding as mc
    s = np.float32(0.0371)
    k = np.arange(-130, 131, dtype=np.float64)
    exact = ((k + 0.5) * np.float64(s)).astype(np.float32)           # nearest fp32 to each boundary
    x = np.concatenate([exact, np.nextafter(exact, np.float32(np.inf)), np.nextafter(exact, np.float32(-np.inf)),
                        np.array([1e9, -1e9, 0.0, -0.0, 127.49 * s, 127.51 * s], np.float32)]).astype(np.float32)
    x = np.concatenate([x, np.zeros((-len(x)) % 2, np.float32)])
    for bits, qmax in ((8, 127), (4, 7)):
        want = np.clip(np.rint(x.astype(np.float64) / np.float64(s)), -qmax, qmax).astype(np.int8)
        got = mc.quantize(torch.from_numpy(x).cuda(), float(s), bits).cpu().numpy()
        if bits == 4:
            got = oracle.unpack_int4(got).astype(np.int8)
        assert np.array_equal(got, want), bits


def test_argument_checks():
    import torch
    from paper_2209_06979_amd import binding as mc
    x = torch.zeros(16, dtype=torch.float32, device="cuda")
    for scale, bits in ((0.0, 8), (float("inf"), 8), (1.0, 16)):
        with pytest.raises(mc.MagicubeError):
            mc.quantize(x, scale, bits)
    with pytest.raises(mc.MagicubeError):
        mc.quantize(x[:15].clone(), 1.0, 4, out=torch.zeros(8, dtype=torch.uint8, device="cuda"))
