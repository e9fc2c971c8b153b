"""GPU parity of the bf16 MFMA GEMM building block against numpy float64 matmul on the same
bf16-rounded inputs: both operand orientations, both tile configurations, ragged M/N, split-k."""
import numpy as np
import pytest
import torch

import synth_inputs as SI
from parity_util import rel_err, to_np

pytestmark = pytest.mark.gpu


def _rand(shape, seed):
    return SI.round_to_bf16(np.random.default_rng(seed).standard_normal(shape)).astype(np.float64)


@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (256, 256, 128), (200, 136, 192), (520, 776, 256),
                                   (4096, 2304, 768), (8, 8, 64), (1000, 72, 64)])
def test_gemm_k_contiguous(M, N, K):
    import paper_2203_17189_amd as P
    a, b = _rand((M, K), 1), _rand((N, K), 2)
    c = P.t5_gemm_bf16(torch.from_numpy(a).cuda().bfloat16(), torch.from_numpy(b).cuda().bfloat16(), True, True)
    torch.cuda.synchronize()
    e = rel_err(to_np(c), a @ b.T)
    assert e[0] < 2e-5, e


@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (256, 512, 4096), (768, 2048, 16384), (136, 200, 192),
                                   (8, 16, 64), (776, 520, 1024)])
def test_gemm_m_contiguous(M, N, K):
    import paper_2203_17189_amd as P
    a, b = _rand((K, M), 3), _rand((K, N), 4)
    c = P.t5_gemm_bf16(torch.from_numpy(a).cuda().bfloat16(), torch.from_numpy(b).cuda().bfloat16(), False, False)
    torch.cuda.synchronize()
    e = rel_err(to_np(c), a.T @ b)
    assert e[0] < 2e-5, e
