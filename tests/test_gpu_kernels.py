"""GPU parity of single kernels through the C ABI: the bf16 MFMA GEMM against a float64 matmul of
the same bf16 values (several tile shapes, ragged tails), and the plain f32 GEMM."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def _rand_bf16(shape, seed, std=1.0):
    a = np.empty(int(np.prod(shape)), dtype=np.uint16)
    synth.weights.fill_normal(a, seed, 77, std=std)
    return a.reshape(shape)


# row counts that land on every accumulator height of the MFMA kernel (32 ... 256 rows, with ragged
# last 16-row tiles), column counts off the 256 grid, K of one slab; (50, 30, 64) has a column count
# that is not a multiple of 4 and takes the plain kernel
@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (2304, 512, 256), (300, 1000, 128), (1, 256, 4096),
                                   (129, 384, 192), (577, 256, 1024), (64, 32000, 256),
                                   (17, 260, 128), (33, 256, 128), (95, 256, 192), (161, 516, 128),
                                   (224, 256, 128), (255, 256, 128), (257, 256, 128), (513, 772, 256),
                                   (700, 256, 128), (4608, 256, 64), (50, 30, 64)])
def test_gemm_bf16_mfma(M, N, K):
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev
    A = _rand_bf16((M, K), 1)
    W = _rand_bf16((N, K), 2, std=0.05)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    P.spec_gemm(dev(A), dev(W), C, M, N, K, P.SPEC_BF16)
    torch.cuda.synchronize()
    ref = synth.bf16_bits_to_f32(A).astype(np.float64) @ synth.bf16_bits_to_f32(W).astype(np.float64).T
    got = C.cpu().numpy()
    assert np.isfinite(got).all()
    scale = np.sqrt(K) * 0.05
    assert np.abs(got - ref).max() < 2e-5 * scale * 10, np.abs(got - ref).max()
    # and the plain kernel agrees too
    C2 = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    P.spec_gemm(dev(A), dev(W), C2, M, N, K, P.SPEC_BF16, P.SPEC_FLAG_SIMPLE_KERNELS)
    torch.cuda.synchronize()
    assert np.abs(C2.cpu().numpy() - ref).max() < 2e-5 * scale * 10


@pytest.mark.parametrize("tile_cols", [128, 256])
@pytest.mark.parametrize("tile_rows", [32, 64, 96, 128, 160, 192, 224, 256])
def test_gemm_bf16_mfma_every_tile_variant(tile_rows, tile_cols):
    """Every accumulator height of the MFMA kernel at both tile widths (the launcher's own choice visits
    only some of the combinations at any given shape): two full row tiles and a ragged third, a column
    count off the tile grid, K long enough for the steady-state loop and its tail."""
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev
    M, N, K = 2 * tile_rows + 17, 3 * tile_cols // 2 + 20, 1152
    A = _rand_bf16((M, K), 3)
    W = _rand_bf16((N, K), 4, std=0.05)
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    P.spec_debug_gemm(dev(A), dev(W), C, M, N, K, tile_rows, tile_cols)
    torch.cuda.synchronize()
    ref = synth.bf16_bits_to_f32(A).astype(np.float64) @ synth.bf16_bits_to_f32(W).astype(np.float64).T
    got = C.cpu().numpy()
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() < 2e-4 * np.sqrt(K) * 0.05, np.abs(got - ref).max()


def test_gemm_f32_plain():
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev
    rng = np.random.default_rng(0)
    M, N, K = 70, 130, 100
    A = rng.standard_normal((M, K)).astype(np.float32)
    W = rng.standard_normal((N, K)).astype(np.float32)
    C = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    P.spec_gemm(dev(A), dev(W), C, M, N, K, P.SPEC_F32)
    torch.cuda.synchronize()
    assert np.abs(C.cpu().numpy() - A.astype(np.float64) @ W.astype(np.float64).T).max() < 1e-4
