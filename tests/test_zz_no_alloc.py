"""The entry point that allocates nothing (gla_decode_noalloc) against the
ordinary entry points: same kernels, partial results in the library's own fixed
buffer instead of a caller workspace.  Results must be bit-identical, also on a
second, smaller call that finds the first call's leftovers in the buffer."""
import numpy as np
import pytest
import torch

import paper_2505_21487_amd as gla
from paper_2505_21487_amd.harness import DeviceProblem
from workloads import config, make_problem

pytestmark = pytest.mark.gpu


def both_ways(p, **kw):
    dp = DeviceProblem(p, poison_unused=True)
    is_gta = p.kind == "gta"
    res = []
    for noalloc in (False, True):
        out = torch.full((p.B, p.T, p.h_q, p.d_v), float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full((p.B, p.T, p.h_q), float("nan"), dtype=torch.float32, device="cuda")
        prm = gla.make_params(*dp.args()[:6], p.scale, out=out, lse=lse, workspace=None, causal=bool(p.causal),
                              impl=gla.GLA_IMPL_TUNED, **kw)
        if noalloc:
            gla.gla_decode_noalloc(prm, is_gta)      # workspace fields stay null: they are ignored
        else:
            need = gla.gla_decode_workspace_size(prm, is_gta)
            ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")
            prm.workspace, prm.workspace_bytes = ws.data_ptr(), ws.numel()
            gla.decode_prepared(prm, is_gta)
        torch.cuda.synchronize()
        res.append((out.float().cpu().numpy(), lse.cpu().numpy()))
    (o0, l0), (o1, l1) = res
    assert not np.isnan(o1).any()
    assert np.array_equal(o0, o1) and np.array_equal(l0, l1)


def test_noalloc_matches_the_workspace_entry_points_twice_in_a_row():
    # first a batch whose units span several chunks each (partials and the merge kernel in use) ...
    both_ways(config(1, batch=8, max_len=4096))
    # ... then a smaller and differently shaped one on the same buffer
    both_ways(make_problem("noalloc_small", seq_lens=[700, 0, 65, 3], T=2, h_q=128, h_c=2, d_v=256, seed=610,
                           num_pages=512, poison_tail=True))
    both_ways(make_problem("noalloc_gta", kind="gta", seq_lens=[1500, 33], T=1, h_q=32, h_c=4, d_v=128, seed=611,
                           num_pages=512, poison_tail=True))


def test_noalloc_rejects_what_does_not_fit():
    p = config(1, batch=12)
    dp = DeviceProblem(p)
    out = torch.empty(p.B, p.T, p.h_q, p.d_v, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(p.B, p.T, p.h_q, dtype=torch.float32, device="cuda")
    prm = gla.make_params(*dp.args()[:6], p.scale, out=out, lse=lse, workspace=None, impl=gla.GLA_IMPL_TUNED,
                          num_splits=128)
    assert gla.gla_decode_workspace_size(prm) > gla.GLA_DECODE_NOALLOC_SCRATCH_BYTES
    with pytest.raises(gla.GlaError) as e:
        gla.gla_decode_noalloc(prm)
    assert e.value.status == gla.GLA_ERR_WORKSPACE_TOO_SMALL
