"""lcn_variant_bwd_static (the entry point for callers that cannot allocate: its scratch is a device array inside
the library) against lcn_variant_bwd with a caller's workspace, through the C ABI: two calls in a row, the second
on a smaller map, for every flag combination; the results must be the same bit for bit (same kernels), which is
well inside the 1e-4 bar."""
import numpy as np
import pytest
import torch

import paper_1502_03409_amd as lc
import workloads as wl
from conftest import rel_fro

pytestmark = pytest.mark.gpu


def _run_both(shape, ks, flags, seed):
    x = torch.from_numpy(wl.feature_maps(*shape, seed=seed, signed=False)).cuda()
    dy = torch.from_numpy(wl.feature_maps(*shape, seed=seed + 1)).cuda()
    stat = shape if flags & lc.LCN_PER_CHANNEL else shape[:3]
    y = torch.empty(shape, device="cuda")
    mu, rstd = torch.empty(stat, device="cuda"), torch.empty(stat, device="cuda")
    lc.lcn_variant_fwd(x, y, mu, rstd, ks, wl.LCN_SIGMA, wl.LCN_EPS, flags)
    nws = lc.lcn_variant_workspace_bytes(shape, flags)
    ws = torch.full((nws // 4,), float("nan"), device="cuda") if nws else None
    ref = torch.full(shape, float("nan"), device="cuda")
    lc.lcn_variant_bwd(x, mu, rstd, dy, ref, ks, wl.LCN_SIGMA, flags, ws)
    got = torch.full(shape, float("nan"), device="cuda")
    lc.lcn_variant_bwd_static(x, mu, rstd, dy, got, ks, wl.LCN_SIGMA, flags)
    torch.cuda.synchronize()
    return got.cpu().numpy(), ref.cpu().numpy()


@pytest.mark.parametrize("flags", range(8))
def test_static_scratch_entry_point_matches_the_workspace_one(flags):
    print(f"case lcn_variant_bwd_static flags {flags}", flush=True)
    # two calls in a row on the same GPU's array: a larger map first, then a smaller one that reuses its start
    for shape, ks, seed in (((6, 44, 44, 32), 5, 3), ((2, 9, 10, 3), 5, 7), ((3, 20, 37, 32), 7, 11)):
        got, ref = _run_both(shape, ks, flags, seed)
        assert np.all(np.isfinite(got))
        assert rel_fro(got, ref) <= 1e-4
        np.testing.assert_array_equal(got, ref)


def test_static_scratch_entry_point_refuses_maps_beyond_its_array():
    shape = (40, 64, 64, 64)     # per-channel two-stage scratch: 40 MiB > LCN_STATIC_SCRATCH_BYTES
    flags = lc.LCN_PER_CHANNEL | lc.LCN_TWO_STAGE
    assert lc.lcn_variant_workspace_bytes(shape, flags) > lc.LCN_STATIC_SCRATCH_BYTES
    z = torch.zeros(shape, device="cuda")
    with pytest.raises(lc.LcError) as e:
        lc.lcn_variant_bwd_static(z, z.clone(), z.clone(), z.clone(), z.clone(), 5, 1.0, flags)
    assert e.value.code == lc.LC_EWORKSPACE and "static" in str(e.value)
    # the one-stage forms need no scratch and are never refused for size
    lc.lcn_variant_bwd_static(z, z.clone(), z.clone() + 1, z.clone(), z.clone(), 5, 1.0, lc.LCN_PER_CHANNEL)
    torch.cuda.synchronize()
