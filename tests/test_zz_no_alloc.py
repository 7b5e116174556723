"""The entry point that allocates nothing (bitlinear_a8_sparse_static) against bitlinear_a8_sparse:
same outputs and accumulators bit for bit, two calls in a row on the library's static scratch, the
second with a smaller input, for the dense and the row-skipping decode kernels."""
import numpy as np
import pytest
import torch

from paper_2411_04965_amd import binding as B
from paper_2411_04965_amd import synth as S

pytestmark = pytest.mark.gpu
EPS = 1e-5


def _dev(x, dtype=torch.bfloat16):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda().to(dtype).contiguous()


@pytest.mark.parametrize("layout", [B.BL_W_GEMM, B.BL_W_KMAJOR])
def test_static_scratch_matches_workspace_form(layout):
    print("no-alloc entry point, layout %d" % layout, flush=True)
    N, K = 4096, 11008
    W = torch.from_numpy(S.latent_weights(N, K, S.seed_for(2, 77))).cuda()
    p, a = B.pack_ternary(W, EPS, layout)
    del W
    # the larger call first, then a smaller one on the same scratch
    for M in ((8, 3) if layout == B.BL_W_KMAJOR else (32, 8, 1)):
        X = _dev(S.glu_like(M, K, S.seed_for(2, 78 + M)))
        Y_ref, acc_ref = B.bitlinear_a8_sparse(X, K // 2, p, a, N, EPS, layout, torch.bfloat16, True)
        Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        acc = torch.full((M, N), -1, dtype=torch.int32, device="cuda")
        B.bitlinear_a8_sparse_static(X, K // 2, p, a, N, Y, EPS, layout, acc)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc_ref), "accumulators differ at M=%d" % M
        assert torch.equal(Y, Y_ref), "outputs differ at M=%d" % M


def test_static_scratch_limits():
    L = B.lib()
    # 65 tokens, or a workspace beyond the static buffer: refused before anything is enqueued
    assert L.bitlinear_a8_sparse_static(16, B.BL_BF16, 65, 4096, 2048, 16, 0, 16, 4096, EPS, 16, B.BL_BF16, None, None) == -7
    assert L.bitlinear_a8_sparse_static(16, B.BL_BF16, 8, 4096, 2048, 16, B.BL_W_KMAJOR, 16, 1 << 17, EPS, 16,
                                        B.BL_BF16, None, None) == -7
    assert L.bl_status_string(-7).decode().startswith("request needs more scratch")
