"""tq_quantize_dequantize against the oracle (client step of Alg. 1, then the server's look-up
of the level) and against the library's own compress -> decode round trip: bit for bit."""
import numpy as np
import pytest
import torch

from oracle import binding as O
from paper_2402_01798_amd import binding as B
from gpu_common import oracle_params, small_gradient

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("grid", [B.GRID_UNIFORM, B.GRID_NONUNIFORM, B.GRID_BISCALED])
@pytest.mark.parametrize("d,bucket", [(1, 0), (13, 0), (2048, 0), (61_706, 0), (3 * 2048 + 5, 2048 + 128), (40_001, 4096)])
def test_values_match_oracle_and_round_trip(bits, grid, d, bucket):
    g_dev, g_np = small_gradient("cfg1", 2, d)
    P = oracle_params(g_np, bits, grid, bucket_elems=bucket)
    params_dev = B.params_from_numpy(P)
    out = torch.full((d,), 7.0, dtype=torch.float32, device="cuda")
    B.tq_quantize_dequantize(g_dev, params_dev, out, bits, 0xABCDEF0123, 5, 9, bucket)
    want = O.quantize_dequantize(g_np, P, 0xABCDEF0123, 5, 9, bucket_elems=bucket)
    assert (out.cpu().numpy() == want).all()
    # the library's own round trip gives the same values
    pay = B.alloc_payload(d, bits)
    B.tq_compress(g_dev, params_dev, pay, bits, 0xABCDEF0123, 5, 9, bucket)
    rt = torch.empty(d, dtype=torch.float32, device="cuda")
    B.tq_decompress_aggregate([pay], [params_dev], rt, bits, bucket)
    assert torch.equal(rt, out)
    # accumulate adds a second worker's values in binary32
    B.tq_quantize_dequantize(g_dev, params_dev, out, bits, 0xABCDEF0123, 6, 9, bucket, accumulate=True)
    want2 = want + O.quantize_dequantize(g_np, P, 0xABCDEF0123, 6, 9, bucket_elems=bucket)
    assert (out.cpu().numpy() == want2).all()


def test_bf16_and_special_values():
    d = 5000
    g = torch.randn(d).mul_(1e-3).to(torch.bfloat16)
    g[[0, 7, 4999]] = torch.tensor([float("nan"), float("inf"), float("-inf")], dtype=torch.bfloat16)
    g_np = g.view(torch.uint16).numpy()
    P = oracle_params(g_np, 3, B.GRID_NONUNIFORM)
    out = torch.empty(d, dtype=torch.float32, device="cuda")
    B.tq_quantize_dequantize(g.cuda(), B.params_from_numpy(P), out, 3, 1, 0, 0)
    want = O.quantize_dequantize(g_np, P, 1, 0, 0)
    got = out.cpu().numpy()
    assert (got == want).all()
    a = float(P["alpha"][0])
    assert got[7] == np.float32(a) and got[4999] == np.float32(-a)          # +-Inf -> +-alpha
