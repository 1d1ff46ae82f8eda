"""mecefo_block_bwd_skip_noalloc (the entry point for callers that cannot allocate or bring a workspace)
against mecefo_block_bwd_skip: the same kernels on the library's static device scratch instead of a caller's
workspace, so the results must be identical; two calls in a row, the second on a smaller input (the scratch
keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2510_16415_amd import binding as B
from gpu_util import Layer, host
from test_gpu_parity import make_case, oracle_block
from gpu_util import TOL, assert_close

EPS = 1e-6


def _both(seed, b, d, f, r, dtype):
    c = make_case(seed, b, d, f, r, dtype)
    lay = Layer(b, d, f, dtype, c["Wg"], c["Wu"], c["Wd"], c["gamma"], c["Pg"], c["Pu"], c["Pd"], EPS)
    ref = lay.block_bwd_skip(c["H"], c["dOut"])                     # existing entry point, caller's workspace
    for t in (lay.dWg, lay.dWu, lay.dWd, lay.dgamma):
        t.fill_(float("nan"))
    Hd, dOd = lay.act(c["H"]), lay.act(c["dOut"])
    dX = torch.full_like(dOd, float("nan"))
    B.mecefo_block_bwd_skip_noalloc(lay.desc, Hd, dOd, lay.gamma, lay.Wg, lay.Wu, lay.Wd, *lay.projs(), lay.side,
                                    dX, lay.dgamma, lay.dWg, lay.dWu, lay.dWd, 0)
    torch.cuda.synchronize()
    got = lay.results(dX)
    for k in ref:
        assert np.array_equal(got[k], ref[k]), (k, (b, d, f, r, dtype))
    assert_close(got, oracle_block(c), TOL[dtype], label=f"noalloc {(b, d, f, r, dtype)}: ")


@pytest.mark.gpu
def test_noalloc_entry_point_two_calls_in_a_row_second_one_smaller():
    _both(901, 700, 520, 1365, 264, "bf16")     # ragged against every tile edge, about 12 MiB of scratch
    _both(902, 130, 64, 104, 8, "bf16")         # smaller input right behind it, on the same scratch
    _both(903, 77, 48, 100, 12, "f32")          # and the fp32 path


@pytest.mark.gpu
def test_noalloc_entry_point_rejects_shapes_beyond_its_scratch():
    d = B.make_desc(8192, 4096, 11008, B.BF16)                       # the 7B-shaped layer: 0.75 GiB of workspace
    assert B.mecefo_workspace_bytes(d, 1024, 1024, 1024) > B.NOALLOC_SCRATCH_BYTES
    fake = torch.empty(16, dtype=torch.bfloat16, device="cuda")
    P = B.Proj(fake.data_ptr(), 1024, 1024)
    with pytest.raises(B.MecefoError) as e:
        B.mecefo_block_bwd_skip_noalloc(d, fake, fake, fake, fake, fake, fake, P, P, P, B.SIDE_INPUT, fake, None, fake,
                                        fake, fake, 0)
    assert e.value.status == B.ERR_WORKSPACE_TOO_SMALL and "static buffer" in str(e.value)
