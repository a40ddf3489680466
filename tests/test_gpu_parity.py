"""GPU parity: every entry point of the C ABI against the fp64 oracle, element by element, on the same
seeded inputs.  Bar (fp32): relative Frobenius error <= 1e-4 per output tensor."""
import numpy as np
import pytest
import torch

import oracle
import paper_1502_03409_amd as lc
import workloads as wl
from conftest import rel_fro

pytestmark = pytest.mark.gpu
TOL = 1e-4


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def forward_workspace(G):
    """The optional workspace of lc_forward (layers with few fields), NaN-filled, or None."""
    nbytes = lc.workspace_bytes(G, lc.LC_OP_FORWARD)
    if nbytes == 0:
        return None
    return torch.full((nbytes // 4,), float("nan"), device="cuda").view(torch.uint8)


def run_forward(g, x, w, bias=None, alpha=1.0, use_ws=True):
    G = lc.geom(*g.as_tuple())
    y = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda")
    ws = forward_workspace(G) if use_ws else None
    lc.lc_forward(G, dev(x), dev(w), None if bias is None else dev(bias), alpha, y, lc.LC_F32, ws)
    return host(y)


def run_backward_data(g, dy, w):
    G = lc.geom(*g.as_tuple())
    dx = torch.full((g.B, g.H, g.W, g.C), float("nan"), device="cuda")
    lc.lc_backward_data(G, dev(dy), dev(w), dx)
    return host(dx)


def run_backward_weights(g, x, dy, beta=0.0, prev=None):
    G = lc.geom(*g.as_tuple())
    dw = torch.full((g.LH, g.LW, g.K, g.F), float("nan"), device="cuda") if prev is None else dev(prev)
    lc.lc_backward_weights(G, dev(x), dev(dy), beta, dw)
    return host(dw)


SMALL = {
    "cfg1": (wl.CONFIG_GEOM["cfg1"], "gaussian"),
    "cfg2": (wl.CONFIG_GEOM["cfg2"], "pink"),
    # ragged everything: batch, filters and patch rows off the tile sizes, floor geometry
    "ragged_a": (wl.LCGeom(B=5, H=23, W=26, C=2, R=5, S=3, F=10), "gaussian"),
    "ragged_b": (wl.LCGeom(B=37, H=19, W=33, C=3, R=7, S=2, F=40), "pink"),
    "ragged_c": (wl.LCGeom(B=70, H=14, W=15, C=5, R=4, S=4, F=19), "gaussian"),   # stride = field, no overlap
    "gaps": (wl.LCGeom(B=9, H=17, W=20, C=1, R=3, S=5, F=7), "gaussian"),         # stride > field
    "one_loc": (wl.LCGeom(B=20, H=6, W=6, C=4, R=6, S=1, F=33), "gaussian"),      # single location = plain GEMM
    "wide_c": (wl.LCGeom(B=33, H=12, W=12, C=32, R=4, S=2, F=48), "halfnormal"),
    "many_f": (wl.LCGeom(B=16, H=10, W=10, C=3, R=4, S=2, F=200), "gaussian"),
    "s5_stage2": (wl.LCGeom(B=24, H=15, W=15, C=16, R=6, S=2, F=32), "halfnormal"),
    # shapes that take the pipelined kernels, with every kind of raggedness they allow
    "fast_b65": (wl.LCGeom(B=65, H=28, W=44, C=4, R=8, S=4, F=32), "gaussian"),     # batch tile + 1 image
    "fast_b130": (wl.LCGeom(B=130, H=24, W=30, C=3, R=8, S=4, F=16), "pink"),       # two batch tiles, F=16
    "fast_floor": (wl.LCGeom(B=72, H=27, W=31, C=4, R=6, S=2, F=64), "halfnormal"), # floor geometry, F=64
    "fast_f128": (wl.LCGeom(B=80, H=14, W=18, C=8, R=4, S=2, F=128), "halfnormal"), # filters split over waves
    "fast_lw1": (wl.LCGeom(B=96, H=20, W=8, C=4, R=8, S=4, F=32), "gaussian"),      # one field per row
    "wide_f16": (wl.LCGeom(B=100, H=132, W=136, C=3, R=8, S=4, F=16), "pink"),      # eight fields per workgroup, ragged strip
    "bd_ap8": (wl.LCGeom(B=80, H=40, W=44, C=3, R=16, S=2, F=16), "pink"),           # 64 fields per cell, eight cells per workgroup
    "wide_f256": (wl.LCGeom(B=150, H=10, W=12, C=16, R=4, S=2, F=256), "halfnormal"),  # workgroup-tiled forward, ragged batch tile
    "wide_bd_c64": (wl.LCGeom(B=80, H=11, W=13, C=64, R=4, S=2, F=64), "halfnormal"),  # workgroup-tiled backward data, uncovered edge
    "bd_ap4_n48": (wl.LCGeom(B=72, H=28, W=32, C=3, R=16, S=4, F=32), "pink"),       # 4x4 covering fields, 48-value cells
    "bd_ap3_n48": (wl.LCGeom(B=72, H=20, W=24, C=3, R=12, S=4, F=16), "pink"),       # 3x3 covering fields
    "bd_ap4_wide": (wl.LCGeom(B=72, H=24, W=262, C=3, R=16, S=4, F=16), "pink"),     # 66 cells per row: eight cells per workgroup, ragged last strip
    "bd_ap5_n72": (wl.LCGeom(B=72, H=28, W=15, C=8, R=15, S=3, F=80), "halfnormal"),  # 5x5 covering fields, 72-value cells: two cells per workgroup
    "bd_ap8_n24": (wl.LCGeom(B=88, H=25, W=24, C=6, R=16, S=2, F=48), "halfnormal"),  # 8x8 covering fields, 24-value cells
    "dense_small": (wl.LCGeom(B=80, H=24, W=24, C=8, R=24, S=1, F=128), "halfnormal"),  # one field: contraction cut into slices
    "dense_k16": (wl.LCGeom(B=72, H=12, W=12, C=4, R=12, S=1, F=128), "halfnormal"),    # one field, 16-value chunks
    "wide_k16": (wl.LCGeom(B=72, H=14, W=16, C=4, R=4, S=2, F=128), "halfnormal"),      # 16-value chunks, many fields
    "single_img": (wl.LCGeom(B=1, H=9, W=9, C=2, R=3, S=3, F=5), "gaussian"),
    # workgroup-tiled kernels: batches that 64-image tiles pad least (the other cases take 96 or 128)
    "wide_b320": (wl.LCGeom(B=320, H=8, W=10, C=32, R=4, S=2, F=128), "halfnormal"),
    # 32 filters under 5x5 covering fields: the backward-data kernel whose chunks hold whole 128-byte lines
    "bd_line_edge": (wl.LCGeom(B=70, H=28, W=36, C=3, R=20, S=4, F=32), "pink"),        # fewer field rows than cover a cell: edge rows only
    "bd_line_in": (wl.LCGeom(B=100, H=44, W=50, C=2, R=20, S=4, F=32), "gaussian"),     # interior and edge rows, ragged batch tile and strip
    "bd_line_c1": (wl.LCGeom(B=64, H=40, W=30, C=1, R=10, S=2, F=32), "gaussian"),      # 4-value cells: one partly used tile
    "bd_line_f64": (wl.LCGeom(B=72, H=32, W=28, C=3, R=20, S=4, F=64), "pink"),         # two blocks of 32 filters per field row
    "bd_line4_f96": (wl.LCGeom(B=66, H=32, W=40, C=3, R=16, S=4, F=96), "pink"),        # 4x4 covering fields, three blocks of 32 filters
    # weight gradient: last block of patch elements with fewer live groups of tiles than the others (skipped, not
    # padded): K = 180 in blocks of 4 groups of 32, K = 36 and K = 400 in blocks of 2 groups of 64
    "bw_groups_va2": (wl.LCGeom(B=16, H=20, W=22, C=5, R=6, S=2, F=32), "pink"),
    "bw_groups_f16": (wl.LCGeom(B=32, H=15, W=17, C=4, R=3, S=2, F=16), "gaussian"),
    "bw_groups_k400": (wl.LCGeom(B=48, H=22, W=26, C=4, R=10, S=2, F=32), "halfnormal"),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_lc_primitives_match_oracle(name):
    g, kind = SMALL[name]
    print(f"case {name} geom {g}", flush=True)
    x, w, dy, bias = wl.lc_inputs(g, kind, seed=0, with_bias=True)
    t = g.as_tuple()
    y = run_forward(g, x, w, bias, 0.75)
    assert rel_fro(y, oracle.lc_forward(t, x, w, bias, 0.75)) <= TOL
    y0 = run_forward(g, x, w, use_ws=False)          # without the optional workspace
    assert rel_fro(y0, oracle.lc_forward(t, x, w)) <= TOL
    dx = run_backward_data(g, dy, w)
    ref_dx = oracle.lc_backward_data(t, dy, w)
    assert rel_fro(dx, ref_dx) <= TOL
    assert np.all(dx[ref_dx == 0.0] == 0.0)          # uncovered pixels are written as exact zeros
    dw = run_backward_weights(g, x, dy)
    ref_dw = oracle.lc_backward_weights(t, x, dy)
    assert rel_fro(dw, ref_dw) <= TOL
    prev = np.random.default_rng(5).standard_normal(ref_dw.shape).astype(np.float32)
    dw1 = run_backward_weights(g, x, dy, 1.0, prev)
    assert rel_fro(dw1, ref_dw + prev) <= TOL


# Shapes at the size where the launchers change their plan: at least 512 workgroups of the largest tile.  Whole
# tensors against the oracle, outputs pre-filled with NaN.
LARGE = {
    "cfg3": (wl.CONFIG_GEOM["cfg3"], "pink"),
    "cfg4": (wl.CONFIG_GEOM["cfg4"], "halfnormal"),
    # the grid of cfg3 with ragged batches: the forward pass runs as a main launch of 64-image tiles plus a
    # remainder launch of 32-image tiles, both with addresses clamped into x beyond the batch
    "cfg3_b72": (wl.CONFIG_GEOM["cfg3"].with_batch(72), "pink"),
    "cfg3_b127": (wl.CONFIG_GEOM["cfg3"].with_batch(127), "pink"),
    # 96 filters (three blocks of 32), patch rows of 60 values from 10 x 10 x 6 fields, batch 130 (three 64-image
    # tiles, the last nearly empty): the forward kernel that loads x straight into LDS, with its remainder launch
    "direct_f96": (wl.LCGeom(B=130, H=60, W=60, C=6, R=10, S=2, F=96), "halfnormal"),
    # the first layer's field (16 x 16 x 3, stride 4) with 256 filters on a 23 x 23 grid (odd: the last strip of
    # two fields is half empty; large enough for two rounds of workgroups, below which the layer keeps the
    # register-staged kernel) and batch 70 (a 64-image tile and a ragged one): the same kernel on blocks of 128
    "direct_f256": (wl.LCGeom(B=70, H=104, W=104, C=3, R=16, S=4, F=256), "pink"),
    # 16 filters per field, eight fields per workgroup: rings of 8, 6 and 5 k-steps, and 48 filters (three blocks)
    "eight_u8": (wl.LCGeom(B=100, H=102, W=102, C=4, R=8, S=2, F=16), "halfnormal"),
    "eight_u6": (wl.LCGeom(B=100, H=100, W=100, C=3, R=8, S=2, F=16), "pink"),
    "eight_u5": (wl.LCGeom(B=100, H=104, W=104, C=2, R=10, S=2, F=16), "pink"),
    "eight_f48": (wl.LCGeom(B=72, H=102, W=102, C=4, R=8, S=2, F=48), "halfnormal"),
    # filter counts that are no multiple of 16 on the same grids: the masked kernels
    "eight_f24": (wl.LCGeom(B=100, H=102, W=102, C=4, R=8, S=2, F=24), "halfnormal"),
    "eight_f40": (wl.LCGeom(B=100, H=100, W=100, C=3, R=8, S=2, F=40), "pink"),
}


@pytest.mark.parametrize("name", list(LARGE))
def test_lc_primitives_large_whole_tensor(name):
    """Every output of the three layer primitives against the oracle at the sizes the benchmark times
    (Sec. 3.1 geometry; Eq. 1's W x, W^T h and the weight gradient)."""
    g, kind = LARGE[name]
    print(f"case large {name} geom {g}", flush=True)
    x, w, dy = wl.lc_inputs(g, kind, seed=0)
    t = g.as_tuple()
    G = lc.geom(*t)
    xd, wd, dyd = dev(x), dev(w), dev(dy)
    y = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda")
    dx = torch.full((g.B, g.H, g.W, g.C), float("nan"), device="cuda")
    dw = torch.full((g.LH, g.LW, g.K, g.F), float("nan"), device="cuda")
    lc.lc_forward(G, xd, wd, None, 1.0, y, lc.LC_F32, forward_workspace(G))
    lc.lc_backward_data(G, dyd, wd, dx)
    lc.lc_backward_weights(G, xd, dyd, 0.0, dw)
    yh, dxh, dwh = host(y), host(dx), host(dw)
    del xd, wd, dyd, y, dx, dw
    e = rel_fro(yh, oracle.lc_forward(t, x, w))
    print(f"  lc_forward rel err {e:.2e}", flush=True)
    assert e <= TOL
    ref = oracle.lc_backward_data(t, dy, w)
    e = rel_fro(dxh, ref)
    print(f"  lc_backward_data rel err {e:.2e}", flush=True)
    assert e <= TOL
    assert np.all(dxh[ref == 0.0] == 0.0)
    del ref
    e = rel_fro(dwh, oracle.lc_backward_weights(t, x, dy))
    print(f"  lc_backward_weights rel err {e:.2e}", flush=True)
    assert e <= TOL


@pytest.mark.parametrize("name", ["paper_layer1", "paper_layer3"])
def test_lc_primitives_full_size_sampled(name):
    """The paper's first layer and its dense last layer (a single field covering its whole input) at the sizes
    the architecture section states (Sec. 3.1): 6.1 GB and 1.5 GB of weights, too large for the whole-tensor
    oracle.  A sample of outputs against the oracle's single-output evaluators, plus the adjoint identities on
    the GPU results."""
    g, kind = (wl.PAPER_LAYER1, "pink") if name == "paper_layer1" else (wl.PAPER_LAYER3, "halfnormal")
    print(f"case {name} geom {g}", flush=True)
    x, w, dy = wl.lc_inputs_blocked(g, kind, seed=0)
    t = g.as_tuple()
    G = lc.geom(*t)
    xd, wd, dyd = dev(x), dev(w), dev(dy)
    y = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda")
    dx = torch.full((g.B, g.H, g.W, g.C), float("nan"), device="cuda")
    dw = torch.full((g.LH, g.LW, g.K, g.F), float("nan"), device="cuda")
    lc.lc_forward(G, xd, wd, None, 1.0, y, lc.LC_F32, forward_workspace(G))
    lc.lc_backward_data(G, dyd, wd, dx)
    lc.lc_backward_weights(G, xd, dyd, 0.0, dw)
    # no output was left unwritten
    assert not torch.isnan(y).any() and not torch.isnan(dx).any() and not torch.isnan(dw).any()
    # adjoint identities, evaluated in fp64 on the device results
    lhs = torch.dot(y.double().flatten(), dyd.double().flatten()).item()
    rhs = torch.dot(xd.double().flatten(), dx.double().flatten()).item()
    rhw = torch.dot(wd.double().flatten(), dw.double().flatten()).item()
    scale = (y.double().norm() * dyd.double().norm()).item()
    assert abs(lhs - rhs) <= 1e-5 * scale and abs(lhs - rhw) <= 1e-5 * scale
    yh, dxh, dwh = host(y), host(dx), host(dw)
    r = np.random.default_rng(11)
    n = 160
    gy, ry, gx, rx, gw, rw = ([] for _ in range(6))
    corners_l = [(0, 0), (g.LH - 1, g.LW - 1), (0, g.LW - 1), (g.LH - 1, 0)]
    for s in range(n):
        b = int(r.integers(g.B)) if s >= 4 else (0 if s % 2 else g.B - 1)
        i, j = (int(r.integers(g.LH)), int(r.integers(g.LW))) if s >= 4 else corners_l[s]
        f, k = int(r.integers(g.F)), int(r.integers(g.K))
        row, col, c = int(r.integers(g.H)), int(r.integers(g.W)), int(r.integers(g.C))
        if s < 4:
            row, col = [(0, 0), (g.H - 1, g.W - 1), (0, g.W - 1), (g.H - 1, 0)][s]
        gy.append(yh[b, i, j, f]); ry.append(oracle.lc_forward_at(t, x, w, None, 1.0, b, i, j, f))
        gx.append(dxh[b, row, col, c]); rx.append(oracle.lc_backward_data_at(t, dy, w, b, row, col, c))
        gw.append(dwh[i, j, k, f]); rw.append(oracle.lc_backward_weights_at(t, x, dy, i, j, k, f))
    assert rel_fro(gy, ry) <= TOL
    assert rel_fro(gx, rx) <= TOL
    assert rel_fro(gw, rw) <= TOL


BF16_CASES = {
    "small": (wl.LCGeom(B=32, H=12, W=14, C=8, R=4, S=2, F=64), "halfnormal"),
    "two_fblocks": (wl.LCGeom(B=48, H=10, W=10, C=16, R=6, S=2, F=128), "halfnormal"),
    "cfg4_quarter": (wl.LCGeom(B=144, H=20, W=22, C=32, R=8, S=2, F=128), "halfnormal"),
    "cfg2": (wl.CONFIG_GEOM["cfg2"], "pink"),                                          # workload cfg2 with bf16 operands
    "tiled_b80": (wl.LCGeom(B=80, H=12, W=14, C=16, R=4, S=2, F=128), "halfnormal"),   # 128-image tiles, ragged
    "tiled_bd_c64": (wl.LCGeom(B=80, H=11, W=13, C=64, R=4, S=2, F=64), "halfnormal"),  # two cell blocks, uncovered edge
    "tiled_f256": (wl.LCGeom(B=272, H=10, W=10, C=16, R=4, S=2, F=256), "halfnormal"), # two filter blocks, two batch tiles
    # shapes outside the bf16 MFMA kernels: the fp32 pipelined kernels reading bf16 storage
    "storage_cfg3_like": (wl.LCGeom(B=72, H=44, W=48, C=3, R=20, S=4, F=32), "pink"),       # 60-value patch rows, 5x5 covering fields
    "storage_cfg5s1_like": (wl.LCGeom(B=132, H=30, W=36, C=3, R=16, S=2, F=16), "pink"),    # 16 filters: eight-wave workgroups
    "storage_f48": (wl.LCGeom(B=72, H=28, W=32, C=3, R=16, S=4, F=48), "pink"),             # one filter tile per wave
    "storage_c16": (wl.LCGeom(B=40, H=15, W=17, C=16, R=6, S=2, F=32), "halfnormal"),       # uncovered last column
    # forward through the strip-sharing bf16 kernel: partial 16-value blocks, 64 / 16 filters, patch rows cut in two
    "strip_f64": (wl.LCGeom(B=48, H=24, W=28, C=3, R=20, S=4, F=64), "pink"),
    "strip_f16": (wl.LCGeom(B=36, H=12, W=14, C=2, R=6, S=2, F=16), "pink"),
    "strip_sub": (wl.LCGeom(B=40, H=14, W=16, C=16, R=10, S=2, F=32), "halfnormal"),
    # batches in steps of 16 images: the weight gradient through the bf16 kernel with in-register transposes
    "rows_cfg3_like": (wl.LCGeom(B=80, H=44, W=48, C=3, R=20, S=4, F=32), "pink"),          # one step in flight
    "rows_f16": (wl.LCGeom(B=144, H=30, W=36, C=3, R=16, S=2, F=16), "pink"),
    "rows_f64": (wl.LCGeom(B=64, H=24, W=28, C=3, R=20, S=4, F=64), "pink"),                # two steps in flight
    "rows_f48": (wl.LCGeom(B=64, H=28, W=32, C=3, R=16, S=4, F=48), "pink"),                # three filter blocks
    "wstrip_rc96": (wl.LCGeom(B=48, H=15, W=17, C=16, R=6, S=2, F=32), "halfnormal"),       # weight gradient through LDS: two 64-value blocks per patch row, uncovered column
    "wstrip_b112": (wl.LCGeom(B=112, H=26, W=32, C=3, R=20, S=4, F=16), "pink"),            # batch short of the 128 staged rows, one filter tile
    "bd_ap5_n72": (wl.LCGeom(B=72, H=28, W=15, C=8, R=15, S=3, F=80), "halfnormal"),        # backward data: two cells per workgroup
    "bd_ap8_n24": (wl.LCGeom(B=88, H=25, W=24, C=6, R=16, S=2, F=48), "halfnormal"),
    # wide layers on batches of 129 to 256 images: the 256-image tiles of the workgroup-tiled kernels
    "pair_odd_row": (wl.LCGeom(B=144, H=12, W=12, C=32, R=4, S=2, F=128), "halfnormal"),     # five fields per row, 144 of 256 image rows in use
    "pair_two_chunks": (wl.LCGeom(B=208, H=20, W=20, C=32, R=8, S=4, F=128), "halfnormal"),  # fields two chunks apart
    "pair_c64_f256": (wl.LCGeom(B=160, H=9, W=9, C=64, R=3, S=1, F=256), "halfnormal"),      # two filter blocks, seven fields per row
    # shapes outside every aligned set: the masked kernels on bf16 storage
    "cfg1": (wl.CONFIG_GEOM["cfg1"], "gaussian"),
    "masked_ragged_a": (wl.LCGeom(B=5, H=23, W=26, C=2, R=5, S=3, F=10), "gaussian"),
    "masked_ragged_b": (wl.LCGeom(B=37, H=19, W=33, C=3, R=7, S=2, F=40), "pink"),
    "masked_gaps": (wl.LCGeom(B=9, H=17, W=20, C=1, R=3, S=5, F=7), "gaussian"),
    "masked_one_loc": (wl.LCGeom(B=20, H=6, W=6, C=4, R=6, S=1, F=33), "gaussian"),
    "masked_f200": (wl.LCGeom(B=16, H=10, W=10, C=3, R=4, S=2, F=200), "gaussian"),
    "masked_single_img": (wl.LCGeom(B=1, H=9, W=9, C=2, R=3, S=3, F=5), "gaussian"),
    # the three stages of workload cfg5 at full size
    "cfg5_s1": (wl.CONFIG_GEOM["cfg5_s1"], "pink"),
    "cfg5_s2": (wl.CONFIG_GEOM["cfg5_s2"], "halfnormal"),
    "cfg5_s3": (wl.CONFIG_GEOM["cfg5_s3"], "halfnormal"),
}


@pytest.mark.parametrize("name", list(BF16_CASES))
def test_lc_primitives_bf16_match_oracle(name):
    """bf16 operands, fp32 accumulation: the oracle takes the unrounded fp32 inputs; bar 2e-2."""
    g, kind = BF16_CASES[name]
    print(f"case bf16 {name} geom {g}", flush=True)
    x, w, dy, bias = wl.lc_inputs(g, kind, seed=0, with_bias=True)
    t = g.as_tuple()
    G = lc.geom(*t)
    bf = lambda a: torch.from_numpy(wl.to_bf16_round(a).view(np.int16)).cuda().view(torch.bfloat16)
    xd, wd, dyd = bf(x), bf(w), bf(dy)
    y = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda")
    dx = torch.full((g.B, g.H, g.W, g.C), float("nan"), device="cuda")
    dw = torch.full((g.LH, g.LW, g.K, g.F), float("nan"), device="cuda")
    lc.lc_forward(G, xd, wd, dev(bias), 0.75, y, lc.LC_BF16)
    lc.lc_backward_data(G, dyd, wd, dx, lc.LC_BF16)
    lc.lc_backward_weights(G, xd, dyd, 0.0, dw, lc.LC_BF16)
    assert rel_fro(host(y), oracle.lc_forward(t, x, w, bias, 0.75)) <= 2e-2
    assert rel_fro(host(dx), oracle.lc_backward_data(t, dy, w)) <= 2e-2
    ref_dw = oracle.lc_backward_weights(t, x, dy)
    assert rel_fro(host(dw), ref_dw) <= 2e-2
    # against the oracle fed with the same rounded operands the remaining error is fp32 accumulation only
    rnd = lambda a: (wl.to_bf16_round(a).astype(np.uint32) << 16).view(np.float32)
    assert rel_fro(host(y), oracle.lc_forward(t, rnd(x), rnd(w), bias, 0.75)) <= 1e-4
    assert rel_fro(host(dx), oracle.lc_backward_data(t, rnd(dy), rnd(w))) <= 1e-4
    assert rel_fro(host(dw), oracle.lc_backward_weights(t, rnd(x), rnd(dy))) <= 1e-4
    prev = np.random.default_rng(5).standard_normal(ref_dw.shape).astype(np.float32)
    dw1 = dev(prev)
    lc.lc_backward_weights(G, xd, dyd, 1.0, dw1, lc.LC_BF16)
    assert rel_fro(host(dw1), ref_dw + prev) <= 2e-2


@pytest.mark.parametrize("cfg", ["cfg4", "cfg3"])
def test_bf16_full_size_sampled(cfg):
    """Workloads cfg4 (bf16 MFMA kernels) and cfg3 (bf16 storage through the fp32 kernels) with bf16 operands at
    full size: sampled outputs against the oracle's single-output evaluators on the unrounded fp32 inputs (bar
    2e-2), and the adjoint identities on the device results."""
    g = wl.CONFIG_GEOM[cfg]
    print(f"case {cfg} bf16 geom {g}", flush=True)
    x, w, dy = wl.lc_inputs(g, wl.CONFIG_IMAGE_KIND[cfg], seed=0)
    t = g.as_tuple()
    G = lc.geom(*t)
    bf = lambda a: torch.from_numpy(wl.to_bf16_round(a).view(np.int16)).cuda().view(torch.bfloat16)
    xd, wd, dyd = bf(x), bf(w), bf(dy)
    y = torch.empty((g.B, g.LH, g.LW, g.F), device="cuda")
    dx = torch.empty((g.B, g.H, g.W, g.C), device="cuda")
    dw = torch.empty((g.LH, g.LW, g.K, g.F), device="cuda")
    lc.lc_forward(G, xd, wd, None, 1.0, y, lc.LC_BF16)
    lc.lc_backward_data(G, dyd, wd, dx, lc.LC_BF16)
    lc.lc_backward_weights(G, xd, dyd, 0.0, dw, lc.LC_BF16)
    lhs = torch.dot(y.double().flatten(), dyd.double().flatten()).item()
    rhs = torch.dot(xd.double().flatten(), dx.double().flatten()).item()
    rhw = torch.dot(wd.double().flatten(), dw.double().flatten()).item()
    scale = (y.double().norm() * dyd.double().norm()).item()
    assert abs(lhs - rhs) <= 1e-5 * scale and abs(lhs - rhw) <= 1e-5 * scale
    yh, dxh, dwh = host(y), host(dx), host(dw)
    r = np.random.default_rng(12)
    gy, ry, gx, rx, gw, rw = ([] for _ in range(6))
    for s in range(120):
        b, i, j = int(r.integers(g.B)), int(r.integers(g.LH)), int(r.integers(g.LW))
        f, k = int(r.integers(g.F)), int(r.integers(g.K))
        row, col, c = int(r.integers(g.H)), int(r.integers(g.W)), int(r.integers(g.C))
        gy.append(yh[b, i, j, f]); ry.append(oracle.lc_forward_at(t, x, w, None, 1.0, b, i, j, f))
        gx.append(dxh[b, row, col, c]); rx.append(oracle.lc_backward_data_at(t, dy, w, b, row, col, c))
        gw.append(dwh[i, j, k, f]); rw.append(oracle.lc_backward_weights_at(t, x, dy, i, j, k, f))
    assert rel_fro(gy, ry) <= 2e-2
    assert rel_fro(gx, rx) <= 2e-2
    assert rel_fro(gw, rw) <= 2e-2


def test_bf16_forward_small_batch_tile():
    """32-image tiles of the strip-sharing bf16 forward kernel (the backward passes need more than 32 images)."""
    g = wl.LCGeom(B=24, H=16, W=20, C=4, R=8, S=2, F=32)
    print(f"case bf16 strip small batch geom {g}", flush=True)
    x, w, _, bias = wl.lc_inputs(g, "pink", seed=3, with_bias=True)
    t = g.as_tuple()
    bf = lambda a: torch.from_numpy(wl.to_bf16_round(a).view(np.int16)).cuda().view(torch.bfloat16)
    rnd = lambda a: (wl.to_bf16_round(a).astype(np.uint32) << 16).view(np.float32)
    y = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda")
    lc.lc_forward(lc.geom(*t), bf(x), bf(w), dev(bias), 1.25, y, lc.LC_BF16)
    assert rel_fro(host(y), oracle.lc_forward(t, rnd(x), rnd(w), bias, 1.25)) <= 1e-4


def test_bf16_takes_every_shape():
    """No geometry is refused for its operand type: a shape outside the bf16 matrix-instruction kernels (here C = 3,
    F = 10, batch 8) runs the masked kernels on bf16 storage."""
    g = wl.LCGeom(B=8, H=9, W=9, C=3, R=3, S=2, F=10)
    x, w, dy = wl.lc_inputs(g, "gaussian", seed=4)
    t = g.as_tuple()
    G = lc.geom(*t)
    bf = lambda a: torch.from_numpy(wl.to_bf16_round(a).view(np.int16)).cuda().view(torch.bfloat16)
    rnd = lambda a: (wl.to_bf16_round(a).astype(np.uint32) << 16).view(np.float32)
    y = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda")
    dx = torch.full((g.B, g.H, g.W, g.C), float("nan"), device="cuda")
    dw = torch.full((g.LH, g.LW, g.K, g.F), float("nan"), device="cuda")
    lc.lc_forward(G, bf(x), bf(w), None, 1.0, y, lc.LC_BF16)
    lc.lc_backward_data(G, bf(dy), bf(w), dx, lc.LC_BF16)
    lc.lc_backward_weights(G, bf(x), bf(dy), 0.0, dw, lc.LC_BF16)
    assert rel_fro(host(y), oracle.lc_forward(t, rnd(x), rnd(w))) <= TOL
    assert rel_fro(host(dx), oracle.lc_backward_data(t, rnd(dy), rnd(w))) <= TOL
    assert rel_fro(host(dw), oracle.lc_backward_weights(t, rnd(x), rnd(dy))) <= TOL


def test_forward_determinism_and_empty_tail():
    g = wl.LCGeom(B=17, H=21, W=21, C=3, R=6, S=3, F=24)
    x, w, dy = wl.lc_inputs(g, "gaussian", seed=2)
    a, b = run_forward(g, x, w), run_forward(g, x, w)
    np.testing.assert_array_equal(a, b)
    a, b = run_backward_data(g, dy, w), run_backward_data(g, dy, w)
    np.testing.assert_array_equal(a, b)
    a, b = run_backward_weights(g, x, dy), run_backward_weights(g, x, dy)
    np.testing.assert_array_equal(a, b)


POOL_SHAPES = [((3, 9, 11, 5), 3, 1), ((2, 12, 12, 32), 3, 1), ((2, 10, 9, 8), 2, 2), ((1, 7, 7, 3), 3, 2),
               ((4, 46, 46, 32), 3, 1), ((2, 19, 35, 16), 5, 1), ((1, 3, 3, 4), 3, 1), ((2, 9, 9, 8), 1, 1),
               ((1, 8, 8, 600), 3, 1), ((2, 57, 57, 16), 3, 1),
               ((128, 46, 46, 32), 3, 1)]    # the last one: cfg3's pooling call at full size


@pytest.mark.parametrize("shape,ks,st", POOL_SHAPES)
def test_l2pool_matches_oracle(shape, ks, st):
    print(f"case pool {shape} {ks} {st}", flush=True)
    x = wl.feature_maps(*shape, seed=1)
    eps = wl.POOL_EPS
    ref = oracle.l2pool_fwd(x, ks, st, eps)
    xd = dev(x)
    y = torch.full(ref.shape, float("nan"), device="cuda")
    lc.l2pool_fwd(xd, y, ks, st, eps)
    assert rel_fro(host(y), ref) <= TOL
    dy = wl.feature_maps(*ref.shape, seed=2)
    dx = torch.full(shape, float("nan"), device="cuda")
    lc.l2pool_bwd(xd, y, dev(dy), dx, ks, st)
    assert rel_fro(host(dx), oracle.l2pool_bwd(x, ref, dy, ks, st)) <= TOL


LCN_SHAPES = [((2, 9, 10, 3), 5), ((3, 20, 37, 32), 5), ((2, 16, 16, 8), 3), ((1, 3, 2, 5), 5), ((2, 33, 17, 6), 7),
              ((1, 5, 40, 130), 5), ((4, 44, 44, 32), 5),
              ((2, 45, 44, 32), 5),      # two bands of whole rows, the second one row short
              ((2, 50, 20, 64), 7),      # 16 lanes per pixel, 7x7 window
              ((3, 21, 30, 4), 5),       # one lane per pixel
              ((2, 30, 150, 32), 5),     # rows too long for a band of eight: the tile kernels
              ((128, 44, 44, 32), 5)]   # last: cfg3 at full size


@pytest.mark.parametrize("shape,ks", LCN_SHAPES)
def test_lcn_matches_oracle(shape, ks):
    print(f"case lcn {shape} {ks}", flush=True)
    x = wl.feature_maps(*shape, seed=3, signed=False)
    ref_y, ref_mu, ref_rstd = oracle.lcn_fwd(x, ks, wl.LCN_SIGMA, wl.LCN_EPS)
    xd = dev(x)
    y = torch.full(shape, float("nan"), device="cuda")
    mu = torch.full(shape[:3], float("nan"), device="cuda")
    rstd = torch.full(shape[:3], float("nan"), device="cuda")
    lc.lcn_fwd(xd, y, mu, rstd, ks, wl.LCN_SIGMA, wl.LCN_EPS)
    assert rel_fro(host(mu), ref_mu) <= TOL
    assert rel_fro(host(rstd), ref_rstd) <= TOL
    assert rel_fro(host(y), ref_y) <= TOL
    dy = wl.feature_maps(*shape, seed=4)
    dx = torch.full(shape, float("nan"), device="cuda")
    # backward from the oracle's saved statistics, so that only lcn_bwd itself is under test
    lc.lcn_bwd(xd, dev(ref_mu.astype(np.float32)), dev(ref_rstd.astype(np.float32)), dev(dy), dx, ks, wl.LCN_SIGMA)
    assert rel_fro(host(dx), oracle.lcn_bwd(x, ref_mu, ref_rstd, dy, ks, wl.LCN_SIGMA)) <= TOL


# l2pool_lcn_fwd: (input shape, pooling window, pooling stride, LCN window)
POOL_LCN_SHAPES = [((4, 46, 46, 32), 3, 1, 5),      # cfg3's maps: two bands of 22 rows, 13 rows per lane
                   ((3, 57, 57, 16), 3, 1, 5),      # cfg5 stage 1: four lanes per pixel, four segments
                   ((5, 25, 25, 32), 3, 1, 5),      # cfg5 stage 2
                   ((130, 9, 9, 32), 3, 1, 5),      # cfg5 stage 3: one band per image, most lanes idle
                   ((2, 31, 40, 8), 3, 1, 3),       # two lanes per pixel, 3x3 LCN window
                   ((2, 20, 13, 64), 3, 1, 7),      # sixteen lanes per pixel (two columns per wave), 7x7 window
                   ((1, 3, 3, 16), 3, 1, 5),        # one pooled pixel
                   ((2, 4, 90, 32), 3, 1, 5),       # a row of 88 pooled pixels: 15 waves per segment
                   ((2, 70, 30, 32), 3, 1, 5),      # tall maps: more bands than the chip needs, so that a lane's rows fit
                   ((70, 132, 137, 8), 3, 1, 7),    # wide maps, 7x7 window: more bands still, so that the band's maps fit LDS
                   ((2, 12, 120, 32), 3, 1, 5),     # rows too long for one workgroup: the two kernels one after the other
                   ((2, 17, 19, 5), 3, 1, 5),       # channels no multiple of four: the two kernels
                   ((2, 21, 21, 16), 2, 2, 5),      # another pooling window: the two kernels
                   ((128, 46, 46, 32), 3, 1, 5)]    # last: cfg3 at full size


@pytest.mark.parametrize("shape,pk,ps,lk", POOL_LCN_SHAPES)
def test_l2pool_lcn_fwd_matches_oracle(shape, pk, ps, lk):
    """The fused call against the oracle's pooling followed by the oracle's LCN (the order Sec. 3.1's layers chain
    them), every output: p, y, mu, rstd."""
    print(f"case pool+lcn {shape} {pk} {ps} {lk}", flush=True)
    x = wl.feature_maps(*shape, seed=5)
    ref_p = oracle.l2pool_fwd(x, pk, ps, wl.POOL_EPS)
    ref_y, ref_mu, ref_rstd = oracle.lcn_fwd(ref_p, lk, wl.LCN_SIGMA, wl.LCN_EPS)
    p = torch.full(ref_p.shape, float("nan"), device="cuda")
    y = torch.full(ref_p.shape, float("nan"), device="cuda")
    mu = torch.full(ref_p.shape[:3], float("nan"), device="cuda")
    rstd = torch.full(ref_p.shape[:3], float("nan"), device="cuda")
    lc.l2pool_lcn_fwd(dev(x), p, y, mu, rstd, pk, ps, wl.POOL_EPS, lk, wl.LCN_SIGMA, wl.LCN_EPS)
    for nm, got, ref in (("p", p, ref_p), ("mu", mu, ref_mu), ("rstd", rstd, ref_rstd), ("y", y, ref_y)):
        e = rel_fro(host(got), ref)
        print(f"  {nm} rel err {e:.2e}", flush=True)
        assert e <= TOL


@pytest.mark.parametrize("shape,pk,ps,lk", POOL_LCN_SHAPES)
def test_lcn_l2pool_bwd_matches_oracle(shape, pk, ps, lk):
    """The fused gradient call against the oracle's LCN gradient followed by its pooling gradient, fed the oracle's
    saved p, mu and rstd so that only the gradient is under test."""
    print(f"case lcn+pool bwd {shape} {pk} {ps} {lk}", flush=True)
    x = wl.feature_maps(*shape, seed=6)
    ref_p = oracle.l2pool_fwd(x, pk, ps, wl.POOL_EPS)
    _, ref_mu, ref_rstd = oracle.lcn_fwd(ref_p, lk, wl.LCN_SIGMA, wl.LCN_EPS)
    dn = wl.feature_maps(*ref_p.shape, seed=7)
    ref_dp = oracle.lcn_bwd(ref_p, ref_mu, ref_rstd, dn, lk, wl.LCN_SIGMA)
    ref_dx = oracle.l2pool_bwd(x, ref_p, ref_dp, pk, ps)
    f32 = lambda a: dev(np.asarray(a, dtype=np.float32))
    scratch = torch.full(ref_p.shape, float("nan"), device="cuda")
    dx = torch.full(shape, float("nan"), device="cuda")
    lc.lcn_l2pool_bwd(dev(x), f32(ref_p), f32(ref_mu), f32(ref_rstd), dev(dn), scratch, dx, pk, ps, lk, wl.LCN_SIGMA)
    e = rel_fro(host(dx), ref_dx)
    print(f"  dx rel err {e:.2e}", flush=True)
    assert e <= TOL


def _pool_lcn_sweep_shapes(n, seed):
    """Seeded random maps for the fused pooling + LCN calls: channel counts inside and outside the one-kernel set,
    map sizes from one pooled pixel to rows that need all sixteen waves, small and large batches."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        C_ = int(rng.choice([8, 16, 32, 64, 4, 12]))
        H, W = int(rng.integers(3, 70)), int(rng.integers(3, 70))
        B = int(rng.choice([1, 2, 3, 7, 33, 130, 300]))
        while B * H * W * C_ > 6_000_000:       # keeps the oracle's part of a case under a second
            B = max(1, B // 2)
        out.append(((B, H, W, C_), int(rng.choice([3, 5, 7]))))
    return out


@pytest.mark.parametrize("idx", range(16))
def test_pool_lcn_calls_sweep(idx):
    shape, lk = _pool_lcn_sweep_shapes(16, seed=23)[idx]
    print(f"case pool+lcn sweep {shape} lcn window {lk}", flush=True)
    x = wl.feature_maps(*shape, seed=100 + idx)
    ref_p = oracle.l2pool_fwd(x, 3, 1, wl.POOL_EPS)
    ref_y, ref_mu, ref_rstd = oracle.lcn_fwd(ref_p, lk, wl.LCN_SIGMA, wl.LCN_EPS)
    p = torch.full(ref_p.shape, float("nan"), device="cuda")
    y = torch.full(ref_p.shape, float("nan"), device="cuda")
    mu = torch.full(ref_p.shape[:3], float("nan"), device="cuda")
    rstd = torch.full(ref_p.shape[:3], float("nan"), device="cuda")
    xd = dev(x)
    lc.l2pool_lcn_fwd(xd, p, y, mu, rstd, 3, 1, wl.POOL_EPS, lk, wl.LCN_SIGMA, wl.LCN_EPS)
    for nm, got, ref in (("p", p, ref_p), ("mu", mu, ref_mu), ("rstd", rstd, ref_rstd), ("y", y, ref_y)):
        assert rel_fro(host(got), ref) <= TOL, nm
    # the gradient call on the kernel's own p, mu, rstd (which the checks above hold to the oracle's)
    dn = wl.feature_maps(*ref_p.shape, seed=200 + idx)
    ref_dx = oracle.l2pool_bwd(x, ref_p, oracle.lcn_bwd(ref_p, ref_mu, ref_rstd, dn, lk, wl.LCN_SIGMA), 3, 1)
    scratch = torch.full(ref_p.shape, float("nan"), device="cuda")
    dx = torch.full(shape, float("nan"), device="cuda")
    lc.lcn_l2pool_bwd(xd, p, mu, rstd, dev(dn), scratch, dx, 3, 1, lk, wl.LCN_SIGMA)
    assert rel_fro(host(dx), ref_dx) <= TOL


LCN_VARIANT_SHAPES = [((2, 9, 10, 3), 5), ((3, 20, 37, 32), 5), ((1, 3, 2, 5), 5), ((2, 33, 17, 6), 7),
                      ((1, 5, 40, 130), 3), ((2, 35, 18, 12), 15), ((8, 44, 44, 32), 5)]


@pytest.mark.parametrize("flags", range(8))
@pytest.mark.parametrize("shape,ks", LCN_VARIANT_SHAPES)
def test_lcn_variants_match_oracle(shape, ks, flags):
    """flags: 1 per-channel statistics, 2 zero-padded borders, 4 two stages (Sec. 3.1 leaves LCN undefined)."""
    print(f"case lcn variant {shape} {ks} flags {flags}", flush=True)
    x = wl.feature_maps(*shape, seed=3, signed=False)
    ref_y, ref_mu, ref_rstd = oracle.lcn_var_fwd(x, ks, wl.LCN_SIGMA, wl.LCN_EPS, flags)
    stat = shape if flags & lc.LCN_PER_CHANNEL else shape[:3]
    xd = dev(x)
    y = torch.full(shape, float("nan"), device="cuda")
    mu = torch.full(stat, float("nan"), device="cuda")
    rstd = torch.full(stat, float("nan"), device="cuda")
    lc.lcn_variant_fwd(xd, y, mu, rstd, ks, wl.LCN_SIGMA, wl.LCN_EPS, flags)
    assert rel_fro(host(mu), ref_mu) <= TOL
    assert rel_fro(host(rstd), ref_rstd) <= TOL
    assert rel_fro(host(y), ref_y) <= TOL
    dy = wl.feature_maps(*shape, seed=4)
    dx = torch.full(shape, float("nan"), device="cuda")
    nws = lc.lcn_variant_workspace_bytes(shape, flags)
    assert (nws > 0) == bool(flags & lc.LCN_TWO_STAGE)
    ws = torch.full((nws // 4,), float("nan"), device="cuda") if nws else None
    # backward from the oracle's saved statistics, so that only the gradient kernels are under test
    lc.lcn_variant_bwd(xd, dev(ref_mu.astype(np.float32)), dev(ref_rstd.astype(np.float32)), dev(dy), dx, ks,
                       wl.LCN_SIGMA, flags, ws)
    assert rel_fro(host(dx), oracle.lcn_var_bwd(x, ref_mu, ref_rstd, dy, ks, wl.LCN_SIGMA, flags)) <= TOL


def run_sae(g, x, w, b, alpha, lam, eps_s, lr, flags, with_h=True):
    G = lc.geom(*g.as_tuple())
    wd, bd = dev(w), dev(b)
    ad = torch.tensor([alpha], device="cuda", dtype=torch.float32)
    cost = torch.full((1,), float("nan"), device="cuda")
    h = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda") if with_h else None
    ws = torch.empty(lc.workspace_bytes(G, lc.LC_OP_SAE_STEP), dtype=torch.uint8, device="cuda")
    lc.sae_step(G, dev(x), wd, bd, ad, lam, eps_s, lr, flags, h, cost, ws)
    return host(cost)[0], host(wd), host(bd), host(ad)[0], (host(h) if with_h else None)


def update_bar(new, ref_update, projected=False):
    """Bar for an update `new - old` formed from fp32 values.  The stated bar is 1e-4.  A stored fp32 value is off
    by at most 2^-24 of its size (one rounding to nearest), so the difference to the old value carries an error
    of up to c 2^-24 ||new|| whatever the kernel does; where the step is so small that this floor comes near the
    bar, the bar is the floor plus half the stated one.  c = 1 for the plain update (one rounding of w - lr dW);
    c = 3 with the row projection (the product with the inverse norm rounds once more, and the inverse norm's own
    fp32 error moves a whole filter)."""
    c = 3.0 if projected else 1.0
    floor = c * 2.0 ** -24 * np.linalg.norm(np.asarray(new, dtype=np.float64).ravel()) / np.linalg.norm(
        np.asarray(ref_update, dtype=np.float64).ravel())
    return max(TOL, 0.5 * TOL + floor), floor


def check_sae_results(tag, got, ref, old, alpha, flags):
    """got / ref = (J, w', b', alpha', h) of the GPU and of the oracle; old = (w, b)."""
    J, w2, b2, a2, h = got
    Jo, wo, bo, ao, ho = ref
    w, b = old
    e = abs(J - Jo) / abs(Jo)
    print(f"  {tag} cost rel err {e:.2e}", flush=True)
    assert e <= TOL
    if h is not None:
        e = rel_fro(h, ho)
        print(f"  {tag} h rel err {e:.2e}", flush=True)
        assert e <= TOL
    # compare the updates, not the updated values, so a small step cannot hide an error
    for nm, new, refnew, base in (("dW", w2, wo, w), ("db", b2, bo, b)):
        ref_update = refnew - base
        bar, floor = update_bar(new, ref_update, projected=bool(flags & 1) and nm == "dW")
        e = rel_fro(new.astype(np.float64) - base, ref_update)
        print(f"  {tag} {nm} rel err {e:.2e} (bar {bar:.2e}, fp32 rounding floor of the stored values {floor:.2e})",
              flush=True)
        assert e <= bar, nm
    if flags & 2:
        bar = max(TOL, 0.5 * TOL + 2.0 ** -24 * abs(a2) / abs(ao - alpha))
        e = abs((a2 - alpha) - (ao - alpha)) / abs(ao - alpha)
        print(f"  {tag} dalpha rel err {e:.2e} (bar {bar:.2e})", flush=True)
        assert e <= bar
    else:
        assert a2 == np.float32(alpha)
    if flags & 1:
        norms = np.linalg.norm(w2.astype(np.float64), axis=2)
        np.testing.assert_allclose(norms[norms > 0], 1.0, rtol=1e-5)


SAE_CASES = {
    "cfg1": (wl.CONFIG_GEOM["cfg1"], "gaussian"),
    "floor": (wl.LCGeom(B=12, H=23, W=23, C=4, R=6, S=2, F=8), "halfnormal"),
    "ragged": (wl.LCGeom(B=7, H=14, W=17, C=3, R=5, S=3, F=10), "gaussian"),
    "stage_like": (wl.LCGeom(B=32, H=32, W=32, C=3, R=16, S=2, F=16), "pink"),
    # the first stage of the three-stage workload on a small image: 16 filters, patch rows of 48, a batch of 128 (the
    # forward and weight-gradient kernels that stage strips of eight fields straight into LDS, both gradient terms)
    "stage_b128": (wl.LCGeom(B=128, H=36, W=40, C=3, R=16, S=2, F=16), "pink"),
    "wide": (wl.LCGeom(B=80, H=12, W=14, C=8, R=4, S=2, F=128), "halfnormal"),       # the workgroup-tiled forward inside the step
    "cells128": (wl.LCGeom(B=72, H=10, W=12, C=32, R=4, S=2, F=32), "halfnormal"),   # the workgroup-tiled backward data inside the step
    # one field covering its whole input: the dense last layer of Sec. 3.1 scaled down (forward cut into slices)
    "one_field": (wl.LCGeom(B=80, H=24, W=24, C=8, R=24, S=1, F=128), "halfnormal"),
    "one_field_ragged": (wl.LCGeom(B=20, H=7, W=7, C=3, R=7, S=1, F=10), "gaussian"),
}


@pytest.mark.parametrize("name", list(SAE_CASES))
@pytest.mark.parametrize("flags", [0, 1, 2, 3])
def test_sae_step_matches_oracle(name, flags):
    g, kind = SAE_CASES[name]
    print(f"case sae {name} flags {flags}", flush=True)
    x, w, _ = wl.lc_inputs(g, kind, seed=1)
    b = (0.05 * np.random.default_rng(3).standard_normal((g.H, g.W, g.C))).astype(np.float32)
    # lambda as the paper gives it: 0.1 for the locally connected layers, 0.01 for the dense last one (next to Eq. 1)
    lam = wl.SAE_LAMBDA_DENSE if g.L == 1 else wl.SAE_LAMBDA
    alpha, eps_s, lr = 0.9, wl.SAE_EPS, 1e-2
    got = run_sae(g, x, w, b, alpha, lam, eps_s, lr, flags)
    ref = oracle.sae_step(g.as_tuple(), x, w, b, alpha, lam, eps_s, lr, flags)
    check_sae_results(f"{name}/{flags}", got, ref, (w, b), alpha, flags)


def test_sae_step_projection_leaves_a_zero_filter_alone():
    """A filter that is all zeros has zero response and zero gradient, and Eq. 1's unit-norm constraint has nothing
    to rescale: it must come out as zeros (not NaN), like the oracle's."""
    g, kind = SAE_CASES["stage_like"]
    x, w, _ = wl.lc_inputs(g, kind, seed=1)
    w = w.copy()
    w[2, 3, :, 5] = 0.0
    b = np.zeros((g.H, g.W, g.C), dtype=np.float32)
    got = run_sae(g, x, w, b, 1.0, wl.SAE_LAMBDA, wl.SAE_EPS, 1e-2, 1)
    ref = oracle.sae_step(g.as_tuple(), x, w, b, 1.0, wl.SAE_LAMBDA, wl.SAE_EPS, 1e-2, 1)
    assert np.all(np.isfinite(got[1])) and np.all(got[1][2, 3, :, 5] == 0.0)
    check_sae_results("zero filter", got, ref, (w, b), 1.0, 1)


def test_sae_step_paper_dense_layer_full_size():
    """One RICA step (Eq. 1, lambda = 0.01, row projection and learned alpha) on the dense last layer at the size
    Sec. 3.1 states: 62 x 62 x 24 responses -> 4096 units, mini-batch 192.  The oracle is the one-field form of
    the same step written with fp64 matrix products; every output is compared."""
    g = wl.PAPER_LAYER3
    print(f"case sae paper_layer3 geom {g}", flush=True)
    x, w, _ = wl.lc_inputs_blocked(g, "halfnormal", seed=0)
    b = (0.05 * np.random.default_rng(3).standard_normal((g.H, g.W, g.C))).astype(np.float32)
    alpha, lam, eps_s, lr, flags = 0.9, wl.SAE_LAMBDA_DENSE, wl.SAE_EPS, 3e-4, 3
    got = run_sae(g, x, w, b, alpha, lam, eps_s, lr, flags)
    ref = oracle.sae_step_one_field(g.as_tuple(), x, w, b, alpha, lam, eps_s, lr, flags)
    check_sae_results("paper_layer3", got, ref, (w, b), alpha, flags)


def test_sae_step_without_h_out_and_descent():
    g, kind = SAE_CASES["cfg1"]
    x, w, _ = wl.lc_inputs(g, kind, seed=1)
    b = np.zeros((g.H, g.W, g.C), dtype=np.float32)
    costs = []
    for _ in range(5):
        J, w, b, _, h = run_sae(g, x, w, b, 1.0, wl.SAE_LAMBDA, wl.SAE_EPS, 1e-2, 0, with_h=False)
        assert h is None
        costs.append(J)
    assert all(c1 < c0 for c0, c1 in zip(costs, costs[1:])), costs


def test_sae_step_is_bitwise_reproducible():
    """The cost, the alpha step and the bias update are summed by whichever workgroup of the sparsity pass finishes
    last, from partial sums the others have written: the same step from the same state must give the same bits every
    time (a sum that missed a partial, or took a stale one, would not).  Shape of cfg5's second stage: the pass runs
    as 157 workgroups plus those of the bias update."""
    g = wl.CONFIG_GEOM["cfg5_s2"]
    x, w, _ = wl.lc_inputs(g, "halfnormal", seed=2)
    G = lc.geom(*g.as_tuple())
    xd, w0 = dev(x), dev(w)
    b0 = dev((0.01 * np.random.default_rng(4).standard_normal((g.H, g.W, g.C))).astype(np.float32))
    ws = torch.empty(lc.workspace_bytes(G, lc.LC_OP_SAE_STEP), dtype=torch.uint8, device="cuda")
    first = None
    for it in range(40):
        wd, bd = w0.clone(), b0.clone()
        ad, cost = torch.full((1,), 0.9, device="cuda"), torch.full((1,), float("nan"), device="cuda")
        ws.fill_(it & 0xff)       # whatever the workspace held before must not matter
        lc.sae_step(G, xd, wd, bd, ad, wl.SAE_LAMBDA, wl.SAE_EPS, 1e-5, 3, None, cost, ws)
        now = (host(cost).tobytes(), host(ad).tobytes(), host(bd).tobytes(), host(wd)[::7, ::5].tobytes())
        if first is None:
            first = now
            assert np.isfinite(host(cost)[0])
        assert now == first, f"call {it} differs from call 0"


@pytest.mark.parametrize("flags", [0, 3])
def test_cfg5_three_stage_step_full_size(flags):
    """Workload cfg5 at full size, in the launch configuration the benchmark times: every stage takes one
    SGD step (Eq. 1) and hands l2pool -> LCN of its features to the next.  The oracle runs its own chain
    from the same images and initial weights; each stage's cost, features and updates are compared."""
    x_ref = wl.pink_images(np.random.default_rng(0), 128, 128, 128, 3)
    x_gpu = dev(x_ref)
    alpha, lam, eps_s = 0.9, wl.SAE_LAMBDA, wl.SAE_EPS
    for si, key in enumerate(("cfg5_s1", "cfg5_s2", "cfg5_s3")):
        g = wl.CONFIG_GEOM[key]
        t = g.as_tuple()
        print(f"case cfg5 stage {si + 1} flags {flags} geom {g}", flush=True)
        assert tuple(x_gpu.shape) == (g.B, g.H, g.W, g.C)
        rw = np.random.default_rng(100 + si)
        w = (rw.standard_normal((g.LH, g.LW, g.K, g.F)) / np.sqrt(g.K)).astype(np.float32)
        b = (0.05 * rw.standard_normal((g.H, g.W, g.C))).astype(np.float32)
        lr = 10.0 * wl.SAE_LR        # a step large enough for the update to stand clear of fp32 rounding of w
        G = lc.geom(*t)
        wd, bd = dev(w), dev(b)
        ad = torch.tensor([alpha], device="cuda", dtype=torch.float32)
        cost = torch.full((1,), float("nan"), device="cuda")
        h = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda")
        ws = torch.empty(lc.workspace_bytes(G, lc.LC_OP_SAE_STEP), dtype=torch.uint8, device="cuda")
        lc.sae_step(G, x_gpu, wd, bd, ad, lam, eps_s, lr, flags, h, cost, ws)
        ref = oracle.sae_step(t, x_ref, w, b, alpha, lam, eps_s, lr, flags)
        ho = ref[4]
        check_sae_results(f"cfg5 stage {si + 1}/{flags}", (host(cost)[0], host(wd), host(bd), host(ad)[0], host(h)), ref,
                          (w, b), alpha, flags)
        # next stage's input, each side from its own features
        p = torch.empty((g.B, g.LH - 2, g.LW - 2, g.F), device="cuda")
        n = torch.empty_like(p)
        mu = torch.empty(p.shape[:3], device="cuda")
        rstd = torch.empty_like(mu)
        lc.l2pool_fwd(h, p, wl.POOL_KSIZE, wl.POOL_STRIDE, wl.POOL_EPS)
        lc.lcn_fwd(p, n, mu, rstd, wl.LCN_KSIZE, wl.LCN_SIGMA, wl.LCN_EPS)
        n_ref = oracle.lcn_fwd(oracle.l2pool_fwd(ho, wl.POOL_KSIZE, wl.POOL_STRIDE, wl.POOL_EPS),
                               wl.LCN_KSIZE, wl.LCN_SIGMA, wl.LCN_EPS)[0]
        assert rel_fro(host(n), n_ref) <= TOL
        x_gpu, x_ref = n, n_ref.astype(np.float32)


def _sweep_geometries(n, seed):
    """Seeded random layer geometries: half of them aligned (C a multiple of 4, F of 16, R of S), so that
    the pipelined kernels and their tile rules are exercised as well as the generic ones."""
    r = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        aligned = len(out) % 2 == 0
        S = int(r.integers(1, 5))
        R = S * int(r.integers(1, 6)) if aligned else int(r.integers(1, 9))
        C = int(r.choice([4, 8, 16])) if aligned else int(r.integers(1, 7))
        F = int(r.choice([16, 32, 48, 64, 128])) if aligned else int(r.integers(1, 41))
        B = int(r.choice([17, 33, 64, 65, 96, 129, 140])) if aligned else int(r.integers(1, 70))
        H, W = R + int(r.integers(0, 14)), R + int(r.integers(0, 22))
        g = wl.LCGeom(B=B, H=H, W=W, C=C, R=R, S=S, F=F)
        if g.flop_per_pass > 3e8 or g.params > 4e6:
            continue
        out.append(g)
    return out


@pytest.mark.parametrize("idx", range(28))
def test_lc_primitives_geometry_sweep(idx):
    g = _sweep_geometries(28, seed=2024)[idx]
    print(f"case sweep {idx} geom {g}", flush=True)
    x, w, dy, bias = wl.lc_inputs(g, "gaussian", seed=idx, with_bias=True)
    t = g.as_tuple()
    assert rel_fro(run_forward(g, x, w, bias, 1.25), oracle.lc_forward(t, x, w, bias, 1.25)) <= TOL
    dx = run_backward_data(g, dy, w)
    ref_dx = oracle.lc_backward_data(t, dy, w)
    assert rel_fro(dx, ref_dx) <= TOL
    assert np.all(dx[ref_dx == 0.0] == 0.0)
    assert rel_fro(run_backward_weights(g, x, dy), oracle.lc_backward_weights(t, x, dy)) <= TOL


def _bf16_sweep_geometries(n, seed):
    """Seeded random geometries inside the aligned set the bf16 kernels cover."""
    r = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        S = int(r.choice([1, 2, 4]))
        R = S * int(r.integers(1, 5))
        C = int(r.choice([4, 8, 16, 32, 64]))
        F = int(r.choice([64, 128, 256]))
        B = 16 * int(r.integers(1, 18))
        H, W = R + int(r.integers(0, 12)), R + 4 * int(r.integers(0, 6))
        g = wl.LCGeom(B=B, H=H, W=W, C=C, R=R, S=S, F=F)
        if (R * C) % 16 or (S * C) % 4 or (W * C) % 4 or g.flop_per_pass > 1e9 or g.params > 8e6:
            continue
        out.append(g)
    return out


@pytest.mark.parametrize("idx", range(14))
def test_lc_primitives_bf16_geometry_sweep(idx):
    """bf16 operands against the oracle fed the same rounded values: what is left is fp32 accumulation."""
    g = _bf16_sweep_geometries(14, seed=77)[idx]
    print(f"case bf16 sweep {idx} geom {g}", flush=True)
    x, w, dy = wl.lc_inputs(g, "halfnormal", seed=idx)
    t = g.as_tuple()
    G = lc.geom(*t)
    bf = lambda a: torch.from_numpy(wl.to_bf16_round(a).view(np.int16)).cuda().view(torch.bfloat16)
    rnd = lambda a: (wl.to_bf16_round(a).astype(np.uint32) << 16).view(np.float32)
    y = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda")
    dx = torch.full((g.B, g.H, g.W, g.C), float("nan"), device="cuda")
    dw = torch.full((g.LH, g.LW, g.K, g.F), float("nan"), device="cuda")
    lc.lc_forward(G, bf(x), bf(w), None, 1.0, y, lc.LC_BF16)
    lc.lc_backward_data(G, bf(dy), bf(w), dx, lc.LC_BF16)
    lc.lc_backward_weights(G, bf(x), bf(dy), 0.0, dw, lc.LC_BF16)
    assert rel_fro(host(y), oracle.lc_forward(t, rnd(x), rnd(w))) <= TOL
    assert rel_fro(host(dx), oracle.lc_backward_data(t, rnd(dy), rnd(w))) <= TOL
    assert rel_fro(host(dw), oracle.lc_backward_weights(t, rnd(x), rnd(dy))) <= TOL


def _bf16_narrow_geometries(n, seed):
    """Seeded random geometries of the narrow layers: patch rows in whole 4-value vectors only, filters in blocks
    of 16, any batch that is a multiple of 4 above 32."""
    r = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        S = int(r.choice([1, 2, 4]))
        R = S * int(r.choice([2, 3, 4, 5, 8]))
        C = int(r.choice([1, 2, 3, 4, 6, 8, 12]))
        F = 16 * int(r.integers(1, 6))
        B = 4 * int(r.integers(9, 40))
        H, W = R + int(r.integers(0, 14)), R + int(r.integers(0, 14))
        g = wl.LCGeom(B=B, H=H, W=W, C=C, R=R, S=S, F=F)
        if R > 24 or (S * C) % 4 or S * C > 60 or (W * C) % 4 or g.K < 64 or g.flop_per_pass > 1e9 or g.params > 8e6:
            continue
        out.append(g)
    return out


@pytest.mark.parametrize("idx", range(14))
def test_lc_primitives_bf16_narrow_sweep(idx):
    """The bf16 kernels of the narrow layers against the oracle fed the same rounded values."""
    g = _bf16_narrow_geometries(14, seed=91)[idx]
    print(f"case bf16 narrow sweep {idx} geom {g}", flush=True)
    x, w, dy = wl.lc_inputs(g, "pink", seed=idx)
    t = g.as_tuple()
    G = lc.geom(*t)
    bf = lambda a: torch.from_numpy(wl.to_bf16_round(a).view(np.int16)).cuda().view(torch.bfloat16)
    rnd = lambda a: (wl.to_bf16_round(a).astype(np.uint32) << 16).view(np.float32)
    y = torch.full((g.B, g.LH, g.LW, g.F), float("nan"), device="cuda")
    dx = torch.full((g.B, g.H, g.W, g.C), float("nan"), device="cuda")
    dw = torch.full((g.LH, g.LW, g.K, g.F), float("nan"), device="cuda")
    lc.lc_forward(G, bf(x), bf(w), None, 1.0, y, lc.LC_BF16)
    lc.lc_backward_data(G, bf(dy), bf(w), dx, lc.LC_BF16)
    lc.lc_backward_weights(G, bf(x), bf(dy), 0.0, dw, lc.LC_BF16)
    assert rel_fro(host(y), oracle.lc_forward(t, rnd(x), rnd(w))) <= TOL
    assert rel_fro(host(dx), oracle.lc_backward_data(t, rnd(dy), rnd(w))) <= TOL
    assert rel_fro(host(dw), oracle.lc_backward_weights(t, rnd(x), rnd(dy))) <= TOL
