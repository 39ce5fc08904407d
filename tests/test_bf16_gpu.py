"""The float path with bf16 operands in the per-position GEMM (WINO_BF16), through the C ABI,
against the oracle's definition of it (transforms in the pinned fp32 arithmetic, U and V
rounded to bf16, exact channel sums).  A speed variant: its error against the direct convolution is
reported and bounded loosely, not held to the float mode's 1e-4."""
import numpy as np
import pytest

from helpers import make_case, max_rel, run_gpu
from paper_2002_10711_amd.workloads import Layer

pytestmark = pytest.mark.gpu

# GPU against the oracle's bf16 pipeline: both round the same fp32 transform results (the
# pinned chains), so the operands agree bit for bit; what differs is the order of the fp32
# channel sums on the matrix cores and the output transform in fp32 instead of fp64.
TOL = 2e-5

CASES = [
    Layer("b_f2", 3, 20, 24, 9, 11, m=2, dtype="bf16", relu_input=False, seed=301),
    Layer("b_f4", 2, 70, 33, 13, 10, m=4, dtype="bf16", seed=302),
    Layer("b_f4_pad0", 2, 16, 16, 10, 12, m=4, pad=0, dtype="bf16", seed=303),
    Layer("b_f4_c64_k64_16px", 4, 64, 64, 16, 16, m=4, dtype="bf16", seed=304),
    Layer("b_f2_c200_k130", 2, 200, 130, 12, 14, m=2, dtype="bf16", seed=305),    # three k blocks, ragged channels
    Layer("b_f4_c256_k256_8px", 8, 256, 256, 8, 8, m=4, dtype="bf16", seed=306),
    Layer("b_f2_1x1out", 1, 3, 2, 3, 3, m=2, pad=0, dtype="bf16", seed=307),
    Layer("b_f4_32px", 2, 64, 64, 32, 32, m=4, dtype="bf16", seed=308),
]


@pytest.mark.parametrize("layer", CASES, ids=lambda l: l.name)
def test_bf16_against_the_oracle(oracle, layer):
    case = make_case(oracle, layer)
    out = run_gpu(case, taps=False)
    ref = oracle.winograd_bf16(case["X"], case["g"], case["BT"], case["G"], case["AT"], layer.pad)
    assert out["Y"].shape == ref.shape
    err = max_rel(out["Y"], ref)
    assert err <= TOL, err
    # against the convolution itself: bf16 operands cost two to three digits (more for
    # F4, whose transforms amplify: the paper's Table 1 in miniature)
    direct = oracle.conv2d_direct_f64(case["X"], case["g"], 1, layer.pad)
    e_direct = max_rel(out["Y"], direct)
    print("%s: vs bf16 oracle %.2e, vs direct convolution %.2e" % (layer.name, err, e_direct))
    assert 1e-5 < e_direct < 0.2
