"""The no-allocation column sum (partials in the library's static device array) against the workspace entry point:
two calls in a row, the second on a smaller input, each bit-identical to mlm_colsum and within the parity bound of
the oracle's plain column sum; sizes beyond the static array are refused before any launch."""
import numpy as np
import pytest
import torch

from helpers import TOL, check
from paper_1909_08053_amd import binding as B
from paper_1909_08053_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_colsum_noalloc_matches_workspace_entry_point(dtype):
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    code = B.MLM_BF16 if dtype == "bf16" else B.MLM_F32
    errs = []
    # first a large ragged problem (many chunks, fills much of the static array), then a smaller one: stale partials
    # of the first call must not leak into the second
    for (b, s, H) in ((3, 701, 1024), (2, 37, 264)):
        T = b * s
        dims = B.make_dims(b, s, H, 1, 4 * H, 8, 1, 0, code)
        rng = np.random.default_rng(T + H)
        dy = rng.standard_normal((T, H)).astype(np.float32) + 0.25
        if dtype == "bf16":
            dy = synth.round_to_bf16(dy)
        d_dy = torch.from_numpy(dy).to(DEV).to(dt).contiguous()
        ws = torch.empty(B.mlm_workspace_bytes(dims, B.WS_COLSUM), device=DEV, dtype=torch.uint8)
        want = torch.empty(H, device=DEV, dtype=dt)
        got = torch.full((H,), 7.0, device=DEV, dtype=dt)
        B.mlm_colsum(dims, d_dy, want, ws)
        B.mlm_colsum_noalloc(dims, d_dy, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"T={T} H={H}: differs from mlm_colsum"
        check(f"colsum_noalloc T={T} H={H}", got.float().cpu().numpy().astype(np.float64),
              dy.astype(np.float64).sum(0), TOL[dtype], errs)


def test_colsum_noalloc_refuses_sizes_beyond_the_static_array():
    # ceil(T / 64) * H = 256 * 4104 floats > 2^20: refused on the host, nothing launched
    dims = B.make_dims(16, 1024, 4104, 1, 4 * 4104, 8, 1, 0, B.MLM_BF16)
    x = torch.zeros(8, device=DEV, dtype=torch.bfloat16)
    with pytest.raises(B.MlmError) as ei:
        B.mlm_colsum_noalloc(dims, x, x)
    assert ei.value.code == -4
