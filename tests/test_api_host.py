"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares,
derives geometry, and rejects bad arguments before anything is launched."""
import ctypes as C
import os
import re

import pytest

import paper_1502_03409_amd as lc
from paper_1502_03409_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a 16-byte aligned non-null "pointer"; validation fails before it could be used


def header_functions():
    names = set()
    for header in ("lc.h", "lc_plan.h"):
        src = open(os.path.join(ROOT, "include", header)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(?:int|size_t|const char \*)\s*\*?\s*(\w+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = lc.lib()
    names = header_functions()
    assert set(names) == set(B.EXPORTS), names
    for n in names:
        assert hasattr(L, n), n


def test_geometry_derivation_and_limits():
    assert lc.geom_derive(lc.geom(192, 300, 300, 3, 16, 4, 384)) == (72, 72, 768)   # Sec. 3.1 first layer
    assert lc.geom_derive(lc.geom(128, 55, 55, 16, 6, 2, 32)) == (25, 25, 576)      # floor geometry
    for bad in [(0, 8, 8, 1, 2, 1, 1), (1, 8, 8, 1, 9, 1, 1), (1, 8, 8, 1, 2, 0, 1), (1, 8, 8, 0, 2, 1, 1),
                (1, 8, 8, 1, 2, 1, 0), (1, 8, 4, 1, 5, 1, 1), (-3, 8, 8, 1, 2, 1, 1)]:
        with pytest.raises(lc.LcError) as e:
            lc.geom_derive(lc.geom(*bad))
        assert e.value.code == B.LC_EINVAL
    assert lc.lib().lc_geom_derive(None, None, None, None) == B.LC_EINVAL


def test_workspace_query():
    g = lc.geom(8, 32, 32, 3, 8, 4, 16)
    assert lc.workspace_bytes(g, B.LC_OP_FORWARD) == 0
    assert lc.workspace_bytes(g, B.LC_OP_BACKWARD_DATA) == 0
    assert lc.workspace_bytes(g, B.LC_OP_BACKWARD_WEIGHTS) == 0
    n = lc.workspace_bytes(g, B.LC_OP_SAE_STEP)
    assert n >= 4 * (2 * 8 * 49 * 16 + 8 * 32 * 32 * 3)
    assert lc.workspace_bytes(lc.geom(0, 1, 1, 1, 1, 1, 1), B.LC_OP_SAE_STEP) == 0
    assert lc.workspace_bytes(g, B.LC_OP_SAE_STEP, 7) == 0
    # lc_forward's optional workspace: only layers with very few fields ask for one (the dense last layer of
    # Sec. 3.1 is a single field: up to 16 slices of a [B, L, F] fp32 result)
    dense = lc.geom(192, 62, 62, 24, 62, 1, 4096)
    n = lc.workspace_bytes(dense, B.LC_OP_FORWARD)
    assert n > 0 and n % (4 * 192 * 4096) == 0 and n // (4 * 192 * 4096) <= 16
    assert lc.workspace_bytes(dense, B.LC_OP_FORWARD, B.LC_BF16) == 0
    assert lc.workspace_bytes(lc.geom(128, 200, 200, 3, 20, 4, 32), B.LC_OP_FORWARD) == 0


def test_argument_validation_happens_before_any_launch():
    L = lc.lib()
    g = lc.geom(8, 32, 32, 3, 8, 4, 16)
    gp = C.byref(g)
    bad = lc.geom(8, 4, 32, 3, 8, 4, 16)
    assert L.lc_forward(C.byref(bad), FAKE, FAKE, None, 1.0, FAKE, 0, None, 0, None) == B.LC_EINVAL
    assert L.lc_forward(gp, None, FAKE, None, 1.0, FAKE, 0, None, 0, None) == B.LC_ENULL
    assert L.lc_forward(gp, FAKE, FAKE, None, 1.0, None, 0, None, 0, None) == B.LC_ENULL
    assert L.lc_forward(gp, FAKE + 4, FAKE, None, 1.0, FAKE, 0, None, 0, None) == B.LC_EALIGN
    assert L.lc_forward(gp, FAKE, FAKE, FAKE + 8, 1.0, FAKE, 0, None, 0, None) == B.LC_EALIGN
    assert L.lc_forward(gp, FAKE, FAKE, None, 1.0, FAKE, 5, None, 0, None) == B.LC_EINVAL
    assert L.lc_forward(gp, FAKE, FAKE, None, 1.0, FAKE, 0, FAKE + 4, 64, None) == B.LC_EALIGN   # workspace
    assert L.lc_backward_data(gp, FAKE, None, FAKE, 0, None, 0, None) == B.LC_ENULL
    assert L.lc_backward_data(gp, FAKE, FAKE, FAKE + 2, 0, None, 0, None) == B.LC_EALIGN
    assert L.lc_backward_weights(gp, FAKE, FAKE, 0.5, FAKE, 0, None, 0, None) == B.LC_EINVAL
    assert L.lc_backward_weights(gp, FAKE, FAKE, 1.0, None, 0, None, 0, None) == B.LC_ENULL
    assert L.l2pool_fwd(FAKE, FAKE, 1, 8, 8, 4, 9, 1, 0.0, None) == B.LC_EINVAL
    assert L.l2pool_fwd(FAKE, FAKE, 1, 8, 8, 4, 3, 0, 0.0, None) == B.LC_EINVAL
    assert L.l2pool_fwd(FAKE, FAKE, 1, 8, 8, 4, 3, 1, -1.0, None) == B.LC_EINVAL
    assert L.l2pool_fwd(None, FAKE, 1, 8, 8, 4, 3, 1, 0.0, None) == B.LC_ENULL
    assert L.l2pool_bwd(FAKE, FAKE, FAKE, FAKE + 1, 1, 8, 8, 4, 3, 1, None) == B.LC_EALIGN
    assert L.lcn_fwd(FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 4, 1.0, 1e-4, None) == B.LC_EINVAL     # even window
    assert L.lcn_fwd(FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 17, 1.0, 1e-4, None) == B.LC_EINVAL    # too large
    assert L.lcn_fwd(FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 5, 0.0, 1e-4, None) == B.LC_EINVAL     # sigma
    assert L.lcn_fwd(FAKE, FAKE, None, FAKE, 1, 8, 8, 4, 5, 1.0, 1e-4, None) == B.LC_ENULL
    assert L.lcn_bwd(FAKE, FAKE, FAKE, FAKE, None, 1, 8, 8, 4, 5, 1.0, None) == B.LC_ENULL
    # the fused pooling + LCN call checks both halves' arguments
    assert L.lcn_l2pool_bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 3, 0, 5, 1.0, None) == B.LC_EINVAL
    assert L.lcn_l2pool_bwd(FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 1, 8, 8, 4, 3, 1, 5, 1.0, None) == B.LC_ENULL
    assert L.lcn_l2pool_bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 3, 1, 5, 1.0, None) == B.LC_EINVAL  # scratch is dy
    assert L.l2pool_lcn_fwd(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 9, 1, 0.0, 5, 1.0, 1e-4, None) == B.LC_EINVAL
    assert L.l2pool_lcn_fwd(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 3, 1, 0.0, 4, 1.0, 1e-4, None) == B.LC_EINVAL
    assert L.l2pool_lcn_fwd(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 3, 1, 0.0, 5, 0.0, 1e-4, None) == B.LC_EINVAL
    assert L.l2pool_lcn_fwd(FAKE, None, FAKE, FAKE, FAKE, 1, 8, 8, 4, 3, 1, 0.0, 5, 1.0, 1e-4, None) == B.LC_ENULL
    assert L.l2pool_lcn_fwd(FAKE, FAKE, FAKE, FAKE + 4, FAKE, 1, 8, 8, 4, 3, 1, 0.0, 5, 1.0, 1e-4, None) == B.LC_EALIGN
    # LCN variants: unknown flag bits, the two-stage gradient without its scratch, aliased output
    assert L.lcn_variant_fwd(FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 5, 1.0, 1e-4, 8, None) == B.LC_EINVAL
    assert L.lcn_variant_fwd(FAKE, FAKE, FAKE, None, 1, 8, 8, 4, 5, 1.0, 1e-4, 7, None) == B.LC_ENULL
    assert L.lcn_variant_bwd(FAKE, FAKE, FAKE, FAKE, FAKE + 16, 1, 8, 8, 4, 5, 1.0, 4, None, 0, None) == B.LC_EWORKSPACE
    assert L.lcn_variant_bwd(FAKE, FAKE, FAKE, FAKE, FAKE + 16, 1, 8, 8, 4, 5, 1.0, 4, FAKE, 255, None) == B.LC_EWORKSPACE
    assert L.lcn_variant_bwd(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 5, 1.0, 1, None, 0, None) == B.LC_EINVAL
    assert L.lcn_variant_workspace_bytes(1, 8, 8, 4, 4) == 8 * 8 * 4
    assert L.lcn_variant_workspace_bytes(1, 8, 8, 4, 5) == 8 * 8 * 4 * 4
    assert L.lcn_variant_workspace_bytes(1, 8, 8, 4, 3) == 0
    need = lc.workspace_bytes(g, B.LC_OP_SAE_STEP)
    args = (gp, FAKE, FAKE, FAKE, FAKE, 0.1, 1e-6, 1e-3, 0, None, FAKE)
    assert L.sae_step(*args, None, 0, None) == B.LC_EWORKSPACE
    assert L.sae_step(*args, FAKE, need - 1, None) == B.LC_EWORKSPACE
    assert L.sae_step(gp, FAKE, FAKE, FAKE, FAKE, 0.1, 1e-6, 1e-3, 8, None, FAKE, FAKE, need, None) == B.LC_EINVAL
    assert L.sae_step(gp, FAKE, FAKE, FAKE, FAKE, -0.1, 1e-6, 1e-3, 0, None, FAKE, FAKE, need, None) == B.LC_EINVAL
    assert L.sae_step(gp, FAKE, FAKE, None, FAKE, 0.1, 1e-6, 1e-3, 0, None, FAKE, FAKE, need, None) == B.LC_ENULL
    assert L.lc_last_error() == b""


def test_binding_rejects_cpu_tensors():
    import torch
    g = lc.geom(2, 8, 8, 1, 3, 1, 4)
    x = torch.zeros(2, 8, 8, 1)
    w = torch.zeros(6, 6, 9, 4)
    y = torch.zeros(2, 6, 6, 4)
    with pytest.raises(ValueError):
        lc.lc_forward(g, x, w, None, 1.0, y)


def test_static_scratch_entry_point_checks_on_the_host():
    """lcn_variant_bwd_static: the checks of lcn_variant_bwd, and a map whose scratch exceeds the library's static
    array is refused before anything touches the GPU, with a message that says why."""
    L = lc.lib()
    assert L.lcn_variant_bwd_static(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 4, 5, 1.0, 1, None) == B.LC_EINVAL
    assert L.lcn_variant_bwd_static(FAKE, FAKE, None, FAKE, FAKE + 16, 1, 8, 8, 4, 5, 1.0, 4, None) == B.LC_ENULL
    assert L.lcn_variant_bwd_static(FAKE, FAKE, FAKE, FAKE, FAKE + 16, 1, 8, 8, 4, 5, 1.0, 9, None) == B.LC_EINVAL
    assert L.lcn_variant_workspace_bytes(40, 64, 64, 64, 5) > B.LCN_STATIC_SCRATCH_BYTES
    assert L.lcn_variant_bwd_static(FAKE, FAKE, FAKE, FAKE, FAKE + 16, 40, 64, 64, 64, 5, 1.0, 5, None) == B.LC_EWORKSPACE
    assert b"static" in L.lc_last_error()
