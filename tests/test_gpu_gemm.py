"""The bf16 projection GEMM against the definition C = A W^T + bias evaluated in fp64 (numpy) on
the same bf16-valued operands.  The kernel accumulates in fp32 and rounds once to bf16, so an
element may differ by one bf16 rounding (2^-8 relative with a safety factor) plus an fp32
accumulation error far below that."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import memosight_oracle as O

pytestmark = pytest.mark.gpu

CASES = [
    # M, N, K, output widths, split_k, bias
    (1, 128, 32, [128], 1, False),
    (7, 256, 64, [128, 128], 1, True),
    (257, 256, 128, [256], 2, True),              # second row tile holds a single row
    (448, 512, 3584, [512], 1, True),             # K / V projection of a 64 x 7 token step
    (448, 4608, 3584, [3584, 512, 512], 1, True),  # fused Q / K / V projection into three tensors
    (448, 3584, 18944, [3584], 4, False),         # MLP down projection, K split four ways
    (300, 1024, 2048, [128, 512, 256, 128], 8, True),
]


@pytest.mark.parametrize("m,n,k,widths,split,with_bias", CASES)
def test_gemm_matches_fp64_definition(m, n, k, widths, split, with_bias):
    from paper_2604_14889_amd import binding as M
    from paper_2604_14889_amd import session as S
    rng = W.make_rng(900, m, n, k)
    a = W.normal_bf16_bits(rng, (m, k), 1.0)
    w = W.normal_bf16_bits(rng, (n, k), k ** -0.5)
    b = W.normal_bf16_bits(rng, (n,), 0.5) if with_bias else None
    f64 = lambda x: O.bf16_bits_to_f32(x).astype(np.float64)
    ref = f64(a) @ f64(w).T + (f64(b) if with_bias else 0.0)
    outs = [torch.full((m, wd), float("nan"), dtype=torch.bfloat16, device="cuda") for wd in widths]
    ws = None
    if split > 1:
        need = M.ms_gemm_workspace_bytes(m, n, split)
        assert need == split * m * n * 4
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    M.ms_gemm_bf16(S.to_device(a, M.MS_BF16), S.to_device(w, M.MS_BF16), None if b is None else S.to_device(b, M.MS_BF16),
                   outs, split, ws)
    torch.cuda.synchronize()
    got = np.concatenate([o.float().cpu().numpy() for o in outs], axis=1).astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    bound = 2.0 ** -8 * np.abs(ref) + 1e-5 * np.abs(ref).max()
    assert (err <= bound).all(), f"max excess {np.max(err - bound):.3e} at {np.unravel_index(np.argmax(err - bound), err.shape)}"


def test_gemm_rejects_what_it_is_not_built_for():
    from paper_2604_14889_amd import binding as M
    a = torch.zeros(4, 64, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(192, 64, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(4, 192, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.MsError) as e:
        M.ms_gemm_bf16(a, w, None, [out])                       # 192 is not a multiple of 128
    assert e.value.code == M.MS_ERR_UNSUPPORTED
    w = torch.zeros(256, 64, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(4, 256, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(M.MsError) as e:
        M.ms_gemm_bf16(a, w, None, [out], split_k=2)            # no workspace
    assert e.value.code == M.MS_ERR_WORKSPACE
    with pytest.raises(M.MsError) as e:
        M.ms_gemm_bf16(a, w, None, [out], split_k=4)            # 64 is not a multiple of 32 x 4
    assert e.value.code == M.MS_ERR_UNSUPPORTED
    with pytest.raises(M.MsError) as e:
        M.ms_gemm_bf16(a, w, None, [out[:, :64].contiguous(), torch.zeros(4, 192, dtype=torch.bfloat16, device="cuda")])
    assert e.value.code == M.MS_ERR_INVALID                     # boundary at column 64
