"""GPU parity, part 1: the random direction and the perturb / update / staging streams must
reproduce the oracle bit for bit (integer and rounding work: no tolerance)."""
import numpy as np
import pytest
import torch

import paper_2507_03211_amd as zo_amd
import zo_inputs as zi
from oracle import zo_oracle as zo
from gpu_util import DEV, to_dev, to_host

pytestmark = pytest.mark.gpu


def _z_gpu(n, seed, tid, first=0):
    out = torch.empty(max(n, 1), dtype=torch.float32, device=DEV)
    zo_amd.zo_kernel_z(out, n, seed, tid, first)
    torch.cuda.synchronize()
    return out[:n].cpu().numpy()


@pytest.mark.parametrize("seed,tid,first,n", [(42, 0, 0, 1 << 20), (42, 1, 0, 4099), (0, 33, 3, 1001), (2**63 + 11, 7, 2**34 + 1, 777),
                                              (9, 2, 5, 1), (9, 2, 0, 0)])
def test_z_bits_exact(seed, tid, first, n):
    got = _z_gpu(n, seed, tid, first)
    want = zo.z_values(seed, tid, first, n)
    assert got.tobytes() == want.tobytes()


def _pairs_gpu(words):
    dev_words = torch.from_numpy(words.view(np.int32)).to(DEV)
    out = torch.empty(words.size, dtype=torch.float32, device=DEV)
    zo_amd.zo_kernel_normal_pairs(dev_words, out, words.size // 2)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_normal_transform_bits_exact_over_all_radii_and_angle_edges():
    # every one of the 2^23 radius codes once (the cosine's sign bit alternating), with pseudo-random angles; then the
    # angle's edge cases: zero, the quarter turns, both signs, integers that the conversion to fp32 rounds (ties too)
    rng = np.random.Generator(np.random.PCG64(5))
    ra = (np.arange(1 << 23, dtype=np.uint64) << 9).astype(np.uint32) | ((np.arange(1 << 23, dtype=np.uint32) & np.uint32(1)) << np.uint32(8))
    rb = rng.integers(0, 2**32, size=ra.size, dtype=np.uint64).astype(np.uint32)
    edge = [0, 1, 2, 0x7F, 0x80, 0x81, 0x01000000, 0x01000001, 0x01000002, 0x01000003, 0x3FFFFFFF, 0x40000000, 0x40000020, 0x40000040,
            0x40000060, 0x7FFFFF80, 0x7FFFFFBF, 0x7FFFFFC0, 0x7FFFFFFF]
    eb = np.array(edge + [(-v) & 0xFFFFFFFF for v in edge] + [0x80000000, 0x80000001, 0xC0000000], dtype=np.uint32)
    ea = rng.integers(0, 2**32, size=eb.size, dtype=np.uint64).astype(np.uint32)
    words = np.empty(2 * (ra.size + eb.size), dtype=np.uint32)
    words[0::2] = np.concatenate([ra, ea])
    words[1::2] = np.concatenate([rb, eb])
    want = zo.normal_pairs(words)
    got = _pairs_gpu(words)
    assert got.tobytes() == want.tobytes(), np.flatnonzero(got.view(np.uint32) != want.view(np.uint32))[:10]


def test_normal_transform_bits_exact_over_all_angle_codes():
    # all 2^26 values of the angle word's top 26 bits (rb = i << 6: every fp32 the conversion can give from them, both
    # signs) in one launch, the radius code walking through its range beside them
    i = np.arange(1 << 26, dtype=np.uint64)
    words = np.empty(2 << 26, dtype=np.uint32)
    words[0::2] = ((i * 2654435761) & 0xFFFFFFFF).astype(np.uint32)
    words[1::2] = (i << 6).astype(np.uint32)
    want = zo.normal_pairs(words)
    got = _pairs_gpu(words)
    assert got.tobytes() == want.tobytes(), np.flatnonzero(got.view(np.uint32) != want.view(np.uint32))[:10]


def _theta_sample(rng, n, dtype):
    x = (0.02 * rng.standard_normal(n)).astype(np.float32)
    x[:8] = [0.0, -0.0, 1e-40, -1e-40, 6e-8, 65504.0, -65504.0, 3.0e38]   # zeros, subnormals, near the type maxima
    if dtype == zi.FP16:
        x[7] = 60000.0
    return zi.round_to_storage(x, dtype)


@pytest.mark.parametrize("dtype", [zi.FP32, zi.BF16, zi.FP16])
@pytest.mark.parametrize("n", [1, 7, 8, 4096, 4097, 8192, 8193, 3 * 8192 + 13, 1 << 20])
def test_axpy_bits_exact(dtype, n):
    rng = np.random.Generator(np.random.PCG64(n))
    theta = _theta_sample(rng, max(n, 8), dtype)[:n]
    for scale in (1e-3, -2e-3, -3.17e-6, 0.0):
        src = to_dev(theta, dtype)
        dst = torch.empty_like(src)
        zo_amd.zo_kernel_axpy_z(src, dst, dtype, n, 42, 5, scale)
        got = to_host(dst, dtype)
        want = zo.axpy_z(theta, dtype, 42, 5, scale)
        assert got.tobytes() == want.tobytes(), (dtype, n, scale)
        if scale == 0.0:      # unchanged, except that 0*z + (-0) is +0 under IEEE rules
            t32 = zo.widen(theta, dtype)
            keep = ~((t32 == 0) & np.signbit(t32))
            assert got[keep].tobytes() == theta[keep].tobytes()
    # in place, scalar read from device memory (the form the update inside zo_step uses)
    src = to_dev(theta, dtype)
    dev_scale = torch.tensor([-1.25e-4], dtype=torch.float32, device=DEV)
    zo_amd.zo_kernel_axpy_z(src, src, dtype, n, 43, 6, 123.0, dev_scale)
    assert to_host(src, dtype).tobytes() == zo.axpy_z(theta, dtype, 43, 6, np.float32(-1.25e-4)).tobytes()


@pytest.mark.parametrize("dtype", [zi.FP32, zi.BF16, zi.FP16])
@pytest.mark.parametrize("rows,cols,transpose", [(64, 64, True), (100, 72, True), (1, 8, True), (200, 264, True), (130, 8, True),
                                                 (1, 4099, False), (37, 100, False), (300, 768, False)])
def test_stage_pm_bits_exact(dtype, rows, cols, transpose):
    rng = np.random.Generator(np.random.PCG64(rows * 1000 + cols))
    theta = zi.round_to_storage((0.02 * rng.standard_normal((rows, cols))).astype(np.float32), dtype)
    src = to_dev(theta, dtype)
    wp, wm = torch.zeros_like(src).reshape(-1), torch.zeros_like(src).reshape(-1)
    eps = 1e-3
    zo_amd.zo_kernel_stage_pm(src, wp, wm, dtype, rows, cols, transpose, 77, 9, eps)
    want_p = zo.axpy_z(theta, dtype, 77, 9, eps)
    want_m = zo.axpy_z(theta, dtype, 77, 9, -np.float32(eps))
    if transpose:
        want_p, want_m = np.ascontiguousarray(want_p.T), np.ascontiguousarray(want_m.T)
    assert to_host(wp, dtype).tobytes() == want_p.tobytes()
    assert to_host(wm, dtype).tobytes() == want_m.tobytes()


def test_same_seed_same_z_across_kernels_and_chunkings():
    # the z an in-place pass uses, the z a staging pass uses and the bare z kernel agree for any split
    n = 10000
    theta = np.zeros(n, dtype=np.float32)
    src = to_dev(theta, zi.FP32)
    out = torch.empty_like(src)
    zo_amd.zo_kernel_axpy_z(src, out, zi.FP32, n, 1234, 3, 1.0)     # 0 + 1*z = z
    z_axpy = to_host(out, zi.FP32)
    wp, wm = torch.empty_like(src), torch.empty_like(src)
    zo_amd.zo_kernel_stage_pm(src, wp, wm, zi.FP32, 100, 100, 0, 1234, 3, 1.0)
    pieces = np.concatenate([_z_gpu(b - a, 1234, 3, a) for a, b in [(0, 3), (3, 4096), (4096, 9999), (9999, 10000)]])
    assert z_axpy.tobytes() == pieces.tobytes() == to_host(wp, zi.FP32).tobytes()
    assert (-to_host(wm, zi.FP32)).tobytes() == z_axpy.tobytes()
    assert z_axpy.tobytes() == zo.z_values(1234, 3, 0, n).tobytes()
