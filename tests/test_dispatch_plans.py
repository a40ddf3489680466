"""Launch plans of the three layer primitives, checked on the host (no GPU): lc_plan_query runs the launchers'
own planning and host checks; this file walks many seeded geometries through it and re-derives, independently of
the C++ checks, what a plan has to satisfy: LDS within the kernel's budget, staging registers that hold a chunk,
every tile of the problem covered exactly once by the grid (the kernels' block-index arithmetic is replayed here),
and clamped staging addresses inside the tensor.  Geometry follows Sec. 3.1 (fields of size R at stride S)."""
import numpy as np
import pytest

import paper_1502_03409_amd as lc
import workloads as wl
from paper_1502_03409_amd import binding as B

OPS = (B.LC_OP_FORWARD, B.LC_OP_BACKWARD_DATA, B.LC_OP_BACKWARD_WEIGHTS)
LDS_PER_CU = 160 * 1024


def cdiv(a, b):
    return -(-a // b)


def remap_xcd(wg, n_wg, xcds=8):
    """Work index of hardware workgroup `wg`: each of the 8 XCDs walks a contiguous range (as the kernels do)."""
    per = cdiv(n_wg, xcds)
    full = n_wg - (per - 1) * xcds
    xcd, slot = wg % xcds, wg // xcds
    start = xcd * per if xcd < full else full * per + (xcd - full) * (per - 1)
    return start + slot


def test_remap_is_a_permutation():
    for n in (1, 7, 8, 9, 63, 64, 65, 552, 1300):
        assert sorted(remap_xcd(w, n) for w in range(n)) == list(range(n))


def sample_geometries(n, seed):
    """Seeded layer geometries of every kind the launchers distinguish: aligned and ragged, few and many fields,
    narrow and wide filter banks, tiny and large batches."""
    r = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        kind = len(out) % 5
        if kind == 0:      # anything goes
            S, R, C = int(r.integers(1, 7)), int(r.integers(1, 13)), int(r.integers(1, 9))
            F, Bn = int(r.integers(1, 70)), int(r.integers(1, 150))
        elif kind == 1:    # aligned narrow layers (the pipelined kernels)
            S = int(r.choice([1, 2, 3, 4]))
            R = S * int(r.choice([1, 2, 3, 4, 5, 6, 8]))
            C = int(r.choice([1, 2, 3, 4, 6, 8, 12, 16]))
            F, Bn = 16 * int(r.integers(1, 9)), int(r.choice([17, 33, 48, 64, 65, 72, 96, 100, 127, 128, 130, 192, 256]))
        elif kind == 2:    # wide layers (the workgroup-tiled kernels)
            S = int(r.choice([1, 2, 4]))
            R = S * int(r.integers(1, 5))
            C = int(r.choice([8, 16, 32, 64]))
            F, Bn = 128 * int(r.integers(1, 4)), int(r.choice([65, 80, 96, 128, 150, 192, 256, 320]))
        elif kind == 3:    # large grids of small fields: enough workgroups for the tiered and eight-wave plans
            S = int(r.choice([2, 4]))
            R = S * int(r.choice([2, 4, 5]))
            C = int(r.choice([1, 2, 3, 4]))
            F, Bn = int(r.choice([16, 24, 32, 40, 48])), int(r.choice([65, 72, 100, 127, 128]))
        else:              # one or very few fields (the dense last layer is the one-field case)
            S, C = 1, int(r.choice([3, 4, 8, 24]))
            R = int(r.integers(4, 40))
            F, Bn = int(r.choice([10, 64, 128, 256, 1024])), int(r.choice([20, 80, 192]))
        if kind == 3:
            H, W = R + S * int(r.integers(20, 60)), R + S * int(r.integers(20, 60)) + int(r.integers(0, 3))
        elif kind == 4:
            H, W = R + int(r.integers(0, 2)), R + int(r.integers(0, 2))
        else:
            H, W = R + int(r.integers(0, 30)), R + int(r.integers(0, 40))
        g = wl.LCGeom(B=Bn, H=H, W=W, C=C, R=R, S=S, F=F)
        if g.params > 3e8 or g.B * g.H * g.W * g.C > 2 ** 30:
            continue
        out.append(g)
    return out


NAMED = dict(wl.CONFIG_GEOM, paper_layer1=wl.PAPER_LAYER1, paper_layer3=wl.PAPER_LAYER3,
             cfg3_b72=wl.CONFIG_GEOM["cfg3"].with_batch(72), cfg3_b127=wl.CONFIG_GEOM["cfg3"].with_batch(127))


# ------------------------------------------------------------------------------------------ per-family replays
def covered_forward_fast(g, plans):
    """(strip, batch tile, filter block) -> count over all launches, replaying the kernel's index arithmetic."""
    seen = {}
    for p in plans:
        MT, NT, NLOC, UNR, NW = p["tparam"][:5]
        first, count, nbt, strips = p["arg"][4:8]
        gx, gy, _ = p["grid"]
        assert gx == count * nbt
        for bx in range(gx):
            t_id = remap_xcd(bx, gx)
            work, bt = first + t_id // nbt, t_id % nbt
            for by in range(gy):
                for wave in range(NW):
                    wl_, wf = wave % NLOC, wave // NLOC
                    i, j = work // strips, (work % strips) * NLOC + wl_
                    if j >= g.LW:
                        continue
                    f0 = (by * (NW // NLOC) + wf) * NT * 16
                    for mt in range(MT):
                        for nt in range(NT):
                            key = (i, j, bt * MT + mt, f0 // 16 + nt)
                            seen[key] = seen.get(key, 0) + 1
    return seen


def check_forward_fast(g, plans):
    total = 0
    for p in plans:
        MT, NT, NLOC, UNR, NW, ES, SPC, NRT, SLOTS = p["tparam"][:9]
        CQ, sq4, RS, NR, first, count, nbt, strips = p["arg"][:8]
        BT, NTHR, SC, WC = 16 * MT, 64 * NW, g.S * g.C, g.W * g.C
        assert p["block"] == NTHR
        # LDS: budget of the launcher (three four-wave workgroups, or two eight-wave ones, per compute unit)
        assert p["lds_bytes"] <= (78 if NW == 8 else 52) * 1024 and p["lds_bytes"] == BT * RS * 4
        # staging slots x threads hold one chunk of dwordx4
        assert SLOTS * NTHR >= BT * NR * sq4
        assert 4 * sq4 >= CQ + (NLOC - 1) * SC and RS >= NR * 4 * sq4 + 2
        assert (g.R * g.C) % CQ == 0 and CQ % (4 * UNR) == 0 and g.R % NR == 0
        assert p["grid"][1] * (NW // NLOC) * NT * 16 == g.F
        total += count
        if SPC > 0:
            # every staging slot loads from a clamped address: the largest one must end inside x
            img = g.H * WC
            for work in (first, first + count - 1):
                i, j0 = work // strips, (work % strips) * NLOC
                col0 = j0 * SC
                lim0 = WC - col0
                assert lim0 >= 4
                for b0 in {0, (nbt - 1) * BT}:
                    for kh in (0, g.R - NRT):
                        row = b0 * img + (i * g.S + kh) * WC + col0
                        so_max = min(BT - 1, g.B - 1 - b0) * img + (NR - 1) * WC + min(4 * sq4 - 4, max(lim0 - 4, 0))
                        assert row + so_max + 4 <= g.B * img
                        assert row >= 0
    strips = plans[0]["arg"][7]
    assert total == strips * g.LH
    # the launches take consecutive ranges of strips
    nxt = 0
    for p in plans:
        assert p["arg"][4] == nxt
        nxt += p["arg"][5]


def check_forward_direct(g, plans):
    """The forward kernel that loads x straight into LDS: same work split as lc_forward_fast."""
    total = 0
    for p in plans:
        MT, NT, NLOC, U, NW, ES, SPC, NRT, NSLOT, NBUF = p["tparam"][:10]
        RC, sq4, RS, NR, first, count, nbt, strips = p["arg"][:8]
        BT, NTHR, SC, WC, NS = 16 * MT, 64 * NW, g.S * g.C, g.W * g.C, SPC * NRT
        assert p["block"] == NTHR and ES == 4 and NBUF in (1, 2)
        assert RC == g.R * g.C == 4 * SPC and NR == NRT and g.R % NRT == 0
        assert WC % 4 == 0 and (NLOC * SC) % 4 == 0 and SC % 2 == 0
        assert 4 * sq4 >= RC + (NLOC - 1) * SC and RS % 4 == 0 and RS // 4 >= NRT * sq4 and (RS // 4) % 2 == 1
        assert NSLOT * NTHR >= BT * (RS // 4) and p["lds_bytes"] == NBUF * NSLOT * NTHR * 16 <= LDS_PER_CU
        assert NS % U == 0 and U - 1 + NSLOT <= 63 and NS <= 63      # loads in flight the kernel's waits count
        assert p["grid"][1] * (NW // NLOC) * NT * 16 == g.F
        assert g.B * g.H * WC * 4 < 2 ** 32
        total += count
        # every lane loads from an address clamped into x: the largest one ends inside x
        img = g.H * WC
        for work in (first, first + count - 1):
            i, j0 = work // strips, (work % strips) * NLOC
            col0 = j0 * SC
            assert WC - col0 >= 4
            for b0 in {0, (nbt - 1) * BT}:
                for kh in (0, g.R - NRT):
                    row = b0 * img + (i * g.S + kh) * WC + col0
                    off_max = min(BT - 1, g.B - 1 - b0) * img + (NRT - 1) * WC + min(4 * sq4 - 4, WC - col0 - 4)
                    assert 0 <= row and row + off_max + 4 <= g.B * img
    assert total == plans[0]["arg"][7] * g.LH
    nxt = 0
    for p in plans:
        assert p["arg"][4] == nxt
        nxt += p["arg"][5]


def covered_backward_data_fast(g, p):
    MT, NT, NCELL, AP, NW = p["tparam"][:5]
    strips, RS, nbt = p["arg"][:3]
    gx, gy, _ = p["grid"]
    r_lo = AP - 1
    n_in = g.LH - r_lo if g.LH > r_lo else 0
    per_row = strips * nbt
    n_first = n_in * per_row
    seen = {}
    for bx in range(gx):
        if bx < n_first:
            t_id = remap_xcd(bx, n_first)
            ri = r_lo + t_id // per_row
        elif n_in > 0:
            t_id = bx - n_first
            rb = t_id // per_row
            ri = rb if rb < r_lo else g.LH + (rb - r_lo)
        else:
            t_id = remap_xcd(bx, gx)
            ri = t_id // per_row
        wi0 = ((t_id // nbt) % strips) * NCELL
        bt = t_id % nbt
        key = (ri, wi0, bt)
        seen[key] = seen.get(key, 0) + 1
    return seen


def check_backward_data_fast(g, p):
    # KIND 0: pipelined kernel staging through registers (bf16 storage); 1: whole-line chunks; 2: dy straight into LDS
    MT, NT, NCELL, AP, NW, ES, KIND = p["tparam"][:7]
    strips, RS, nbt = p["arg"][:3]
    BT, JW, FCH = 16 * MT, NCELL + AP - 1, 32 if KIND == 1 else 16
    CH, CW, NCV = cdiv(g.H, g.S), cdiv(g.W, g.S), g.S * g.S * g.C
    assert g.R % g.S == 0 and AP == g.R // g.S and g.F % FCH == 0
    assert RS >= JW * FCH
    if KIND == 0:      # two halves of a buffer plus one dump vector of four elements per lane
        assert p["lds_bytes"] == 2 * (BT * RS + 64 * NW * 4) * ES
    elif KIND == 1:    # one buffer
        assert p["lds_bytes"] == BT * RS * ES
    else:              # two buffers of whole 16-byte-per-lane loads; a row is JW*4 vectors and a pad vector
        RV = JW * 4 + 1
        nslot = cdiv(BT * RV, 64 * NW)
        assert ES == 4 and RS == RV * 4 and RV <= 64 and p["lds_bytes"] == 2 * nslot * 64 * NW * 16
        assert AP * NT - NT + nslot <= 63 and AP * NT <= 63      # loads in flight the kernel's waits count
    assert KIND == 1 or BT * g.LH * g.LW * g.F * ES < 2 ** 32     # 32-bit byte offsets of the staging slots
    assert p["lds_bytes"] <= LDS_PER_CU
    assert p["grid"][0] == strips * CH * nbt and strips == cdiv(CW, NCELL) and nbt == cdiv(g.B, BT)
    assert p["grid"][1] == cdiv(NCV, (NW // NCELL) * NT * 16)


FAMILY_LDS_BUDGET = {   # bytes per workgroup the launchers aim at (several workgroups per compute unit)
    "lc_forward_generic": LDS_PER_CU, "lc_bwd_data_generic": LDS_PER_CU, "lc_forward_wide": 80 * 1024,
    "lc_bwd_data_wide": 80 * 1024, "lc_forward_bf16_strip": 48 * 1024, "lc_bwd_weights_bf16_strip": 48 * 1024,
    "lc_forward_bf16_tiled": 80 * 1024, "lc_bwd_data_bf16_tiled": 80 * 1024, "lc_bwd_weights_bf16_tiled": LDS_PER_CU,
}


def check_plans(g, op, dtype, plans, replay):
    assert len(plans) >= 1
    for p in plans:
        assert p["lds_bytes"] <= FAMILY_LDS_BUDGET.get(p["kernel"], LDS_PER_CU), p
        assert 64 <= p["block"] <= 1024 and p["block"] % 64 == 0
        assert all(d >= 1 for d in p["grid"]) and p["grid"][1] <= 65535 and p["grid"][2] <= 65535
    fams = {p["kernel"] for p in plans}
    if fams == {"lc_forward_fast"} or fams == {"lc_forward_direct"}:
        (check_forward_fast if fams == {"lc_forward_fast"} else check_forward_direct)(g, plans)
        if replay:
            seen = covered_forward_fast(g, plans)
            MT = plans[0]["tparam"][0]
            want = {(i, j, bt, ft) for i in range(g.LH) for j in range(g.LW)
                    for bt in range(cdiv(g.B, 16)) for ft in range(g.F // 16)}
            got = {k for k in seen if k[2] < cdiv(g.B, 16)}
            assert got == want and all(seen[k] == 1 for k in got), (g, MT)
    elif fams <= {"lc_bwd_data_fast", "lc_bwd_data_line", "lc_bwd_data_direct"}:
        assert len(plans) == 1
        check_backward_data_fast(g, plans[0])
        if replay:
            p = plans[0]
            NCELL, strips, nbt = p["tparam"][2], p["arg"][0], p["arg"][2]
            seen = covered_backward_data_fast(g, p)
            want = {(ri, ws * NCELL, bt) for ri in range(cdiv(g.H, g.S)) for ws in range(strips) for bt in range(nbt)}
            assert set(seen) == want and all(v == 1 for v in seen.values()), g
    elif fams == {"lc_bwd_weights_strip"}:
        # strips of NLOC fields (one per wave), the whole batch per chunk, x staged straight into LDS
        p = plans[0]
        MTR, NB, NSLOT, RV, NLOC = p["tparam"][:5]
        strips, sq4 = p["arg"][:2]
        SC, WC, NTHR = g.S * g.C, g.W * g.C, 64 * p["tparam"][4]
        assert NLOC in (8, 16) and p["block"] == NTHR and g.B == 4 * NB and NB % 16 == 0
        assert g.R * g.C == 16 * MTR and g.F % 16 == 0
        assert list(p["grid"][:2]) == [cdiv(g.LW, NLOC) * g.LH, g.F // 16] and strips == cdiv(g.LW, NLOC)
        assert WC % 4 == 0 and (NLOC * SC) % 4 == 0 and g.R * g.C + (NLOC - 1) * SC <= 4 * sq4 and sq4 <= RV
        assert (4 * RV) % 64 in (16, 48)                       # an LDS read's 16 floats x 4 rows: 64 banks
        assert NSLOT * NTHR >= g.B * RV and p["lds_bytes"] == 2 * NSLOT * NTHR * 16 <= LDS_PER_CU
        assert (4 * (NB // 2 - 1) * 4 * RV + 16 * (MTR - 1)) * 4 < 65536 and NSLOT <= NB // 4 and 4 * MTR + NSLOT <= 63
        assert g.B * g.H * WC * 4 < 2 ** 32 and g.K * g.F * 4 < 2 ** 31 and WC - (strips - 1) * NLOC * SC >= 4
        # largest clamped offset ends inside x
        img = g.H * WC
        row = (g.LH - 1) * g.S + g.R - 1
        last = (strips - 1) * NLOC * SC
        assert (g.B - 1) * img + row * WC + last + min(4 * sq4 - 4, WC - last - 4) + 4 <= g.B * img
    elif fams == {"lc_bwd_weights_fast"} or fams == {"lc_bwd_weights_generic"} or fams == {"lc_bwd_weights_bf16_rows"}:
        p = plans[0]
        kblocks, ntasks = p["arg"][:2]
        assert ntasks == g.L * kblocks and p["grid"][0] == cdiv(ntasks, 4)
        rows = {"lc_bwd_weights_fast": p["tparam"][0] * p["tparam"][1] * 16,
                "lc_bwd_weights_generic": p["tparam"][0] * 16,
                "lc_bwd_weights_bf16_rows": p["tparam"][0] * 64}[p["kernel"]]
        ntile = p["tparam"][2] if p["kernel"] == "lc_bwd_weights_fast" else p["tparam"][1]
        assert kblocks * rows >= g.K > (kblocks - 1) * rows
        assert p["grid"][1] * ntile * 16 >= g.F > (p["grid"][1] - 1) * ntile * 16


# ------------------------------------------------------------------------------------------------------ tests
@pytest.mark.parametrize("name", list(NAMED))
def test_named_workloads_plan_and_cover(name):
    g = NAMED[name]
    G = lc.geom(*g.as_tuple())
    small = g.L * cdiv(g.B, 16) * cdiv(g.F, 16) <= 3_000_000
    for op in OPS:
        for dtype in (B.LC_F32, B.LC_BF16):
            check_plans(g, op, dtype, lc.plan_query(G, op, dtype), replay=small)
    plans = lc.plan_query(G, B.LC_OP_SAE_STEP)
    names = [p["kernel"] for p in plans]
    assert "sae_sparsity" in names and names[-2:] == ["sae_row_norm", "sae_rescale"]


def test_headline_workload_takes_the_tiered_forward_plan():
    """cfg3's forward pass: the kernel that loads x straight into LDS, 512 strips as 64-image tiles (two whole rounds
    of 2 x 256 workgroups), the last 40 strips as 32-image tiles, together every strip once; weight ring as deep as
    a patch row."""
    g = wl.CONFIG_GEOM["cfg3"]
    plans = lc.plan_query(lc.geom(*g.as_tuple()), B.LC_OP_FORWARD)
    assert [p["kernel"] for p in plans] == ["lc_forward_direct", "lc_forward_direct"]
    assert plans[0]["tparam"][:10] == [4, 2, 4, 15, 4, 4, 15, 1, 7, 2] and plans[0]["arg"][4:7] == [0, 512, 2]
    assert plans[1]["tparam"][:10] == [2, 2, 4, 15, 4, 4, 15, 1, 4, 2] and plans[1]["arg"][4:7] == [512, 40, 4]
    # bf16 storage keeps the kernels that stage through registers
    plans = lc.plan_query(lc.geom(*g.as_tuple()), B.LC_OP_FORWARD, B.LC_BF16)
    assert all(p["kernel"] != "lc_forward_direct" for p in plans)


def test_filter_counts_off_the_tile_size_never_take_a_tiled_plan():
    """Layers with at least 512 workgroups of work and F not a multiple of 16 (Sec. 3.1 allows any F): the
    pipelined kernels' grids count F in whole tiles, so these must go to the masked kernel."""
    for F in (20, 24, 40, 17, 63):
        for base in (wl.LCGeom(B=128, H=128, W=128, C=3, R=16, S=2, F=F), wl.LCGeom(B=100, H=102, W=102, C=4, R=8, S=2, F=F)):
            plans = lc.plan_query(lc.geom(*base.as_tuple()), B.LC_OP_FORWARD)
            assert [p["kernel"] for p in plans] == ["lc_forward_generic"], (base, plans)
            p = plans[0]
            NLOC, NT = p["tparam"][2], p["tparam"][1]
            assert p["grid"][1] * (4 // NLOC) * NT * 16 >= F


def test_eight_wave_forward_variants_are_reachable():
    """The shapes the GPU parity suite uses for the eight-wave forward kernel do take it, with rings of 8, 6 and 5."""
    want = {(8, 1, 8, 8, 8): wl.LCGeom(B=100, H=102, W=102, C=4, R=8, S=2, F=16),
            (8, 1, 8, 6, 8): wl.LCGeom(B=100, H=100, W=100, C=3, R=8, S=2, F=16),
            (8, 1, 8, 5, 8): wl.LCGeom(B=100, H=104, W=104, C=2, R=10, S=2, F=16)}
    for tp, g in want.items():
        plans = lc.plan_query(lc.geom(*g.as_tuple()), B.LC_OP_FORWARD)
        assert len(plans) == 1 and tuple(plans[0]["tparam"][:5]) == tp and plans[0]["tparam"][6] == 0, plans
    g = wl.LCGeom(B=72, H=102, W=102, C=4, R=8, S=2, F=48)
    plans = lc.plan_query(lc.geom(*g.as_tuple()), B.LC_OP_FORWARD)
    assert tuple(plans[0]["tparam"][:5]) == (8, 1, 8, 8, 8) and plans[0]["grid"][1] == 3


@pytest.mark.parametrize("chunk", range(8))
def test_seeded_geometries_plan_within_their_invariants(chunk):
    """10 400 seeded geometries x three primitives x two operand types: every plan passes the library's host
    checks (lc_plan_query would return LC_EINTERNAL otherwise) and the independent ones above; the grid
    arithmetic is replayed block by block for the smaller ones."""
    geoms = sample_geometries(1300, seed=1000 + chunk)
    families = set()
    for n, g in enumerate(geoms):
        G = lc.geom(*g.as_tuple())
        for op in OPS:
            for dtype in (B.LC_F32, B.LC_BF16):
                try:
                    plans = lc.plan_query(G, op, dtype)
                except lc.LcError as e:
                    # the only refusal left: a ragged layer whose patch row does not fit the LDS of the masked kernel
                    assert e.code == B.LC_EUNSUPPORTED and op == B.LC_OP_FORWARD and g.R * g.C > 2000, (g, op, dtype, e)
                    continue
                replay = n % 8 == 0 and g.L * cdiv(g.B, 16) * cdiv(g.F, 16) <= 400_000
                check_plans(g, op, dtype, plans, replay)
                families.update(p["kernel"] for p in plans)
    # the sampler reaches every family of the fp32 path and the bf16 ones
    assert {"lc_forward_fast", "lc_forward_generic", "lc_forward_wide", "lc_bwd_data_fast", "lc_bwd_data_generic",
            "lc_bwd_data_wide", "lc_bwd_weights_fast", "lc_bwd_weights_generic"} <= families, families


def test_bf16_is_never_refused_on_shape_alone():
    """Any geometry the fp32 path takes, the bf16 path takes too (shapes outside the bf16 matrix-instruction kernels
    run the masked kernels on bf16 storage)."""
    for g in (wl.CONFIG_GEOM["cfg1"], wl.LCGeom(B=8, H=9, W=9, C=3, R=3, S=2, F=10), wl.LCGeom(B=5, H=23, W=26, C=2, R=5, S=3, F=10),
              wl.LCGeom(B=1, H=9, W=9, C=2, R=3, S=3, F=5), wl.LCGeom(B=70, H=14, W=15, C=5, R=4, S=4, F=19)):
        G = lc.geom(*g.as_tuple())
        for op in OPS:
            assert len(lc.plan_query(G, op, B.LC_BF16)) >= 1


# ------------------------------------------------------------------------- addresses of the hand-scheduled kernels
def _x_strip_offsets_inside(g, BT, NRT, NSLOT, NTHR, RV, sq4, NLOC, strips, nbt, works):
    """Element offsets into x of every lane's 16-byte load of the kernels that stage strips of fields straight into
    LDS (forward: NRT patch rows per chunk and batch tiles; weight gradient: one row, the whole batch)."""
    SC, WC = g.S * g.C, g.W * g.C
    img = g.H * WC
    tid = np.arange(NTHR)
    for work in works:
        i, j0 = work // strips, (work % strips) * NLOC
        col0 = j0 * SC
        lim = WC - col0 - 4
        for bt in range(nbt):
            b0 = bt * BT
            for q in range(NSLOT):
                P = q * NTHR + tid
                b, v = P // RV, P % RV
                r, vv = v // sq4, v % sq4
                data = (b < BT) & (r < NRT)
                goff = np.where(data, np.minimum(b, g.B - 1 - b0) * img + r * WC + np.minimum(4 * vv, max(lim, 0)), 0)
                for kh in (0, g.R - NRT):
                    a = b0 * img + (i * g.S + kh) * WC + col0 + goff
                    assert a.min() >= 0 and a.max() + 4 <= g.B * img, (g, work, bt, q, kh)


@pytest.mark.parametrize("name", ["cfg5_s1", "cfg5_s2", "cfg5_s3", "cfg2", "cfg3", "stage_small"])
def test_hand_scheduled_kernels_stay_inside_their_tensors(name):
    """The kernels with inline-assembly loads compute their addresses from offsets worked out once per workgroup;
    this replays that arithmetic for every workgroup of the launch plan and checks each address against its tensor."""
    g = wl.LCGeom(B=128, H=36, W=40, C=3, R=16, S=2, F=16) if name == "stage_small" else wl.CONFIG_GEOM[name]
    G = lc.geom(*g.as_tuple())
    SC, WC, RC = g.S * g.C, g.W * g.C, g.R * g.C
    seen = set()
    for op in OPS:
        for p in lc.plan_query(G, op):
            seen.add(p["kernel"])
            if p["kernel"] == "lc_forward_direct":
                MT, NT, NLOC, U, NW, _, SPC, NRT, NSLOT, NBUF = p["tparam"][:10]
                _, sq4, RS, _, first, count, nbt, strips = p["arg"][:8]
                _x_strip_offsets_inside(g, 16 * MT, NRT, NSLOT, 64 * NW, RS // 4, sq4, NLOC, strips, nbt,
                                        range(first, first + count))
                # rows of w[l] a chunk's k-steps contract: groups of 16 (lane kk takes rows 4kk..4kk+3) and a tail group
                rows = [kh * RC + r * RC + (16 * (s_ // 4) + (s_ & 3) + 12 if s_ // 4 < SPC // 4
                                           else 16 * (SPC // 4) + (s_ - 4 * (SPC // 4)) + 3 * (SPC % 4))
                        for kh in range(0, g.R, NRT) for r in range(NRT) for s_ in range(SPC)]
                assert max(rows) < g.K
            elif p["kernel"] == "lc_bwd_weights_strip":
                MTR, NB, NSLOT, RV, NLOC = p["tparam"][:5]
                strips, sq4 = p["arg"][:2]
                _x_strip_offsets_inside(g, 4 * NB, 1, NSLOT, 64 * NLOC, RV, sq4, NLOC, strips, 1, range(strips * g.LH))
                assert ((4 * NB - 1) * g.L + g.L - 1) * g.F + g.F - 1 < g.B * g.L * g.F
                assert ((g.L - 1) * g.K + (g.R - 1) * RC + 15 + 16 * (MTR - 1)) * g.F + g.F - 1 < g.L * g.K * g.F
            elif p["kernel"] == "lc_bwd_data_direct":
                MT, NT, NCELL, AP, NW = p["tparam"][:5]
                strips, RS, nbt = p["arg"][:3]
                BT, RV, NTHR = 16 * MT, RS // 4, 64 * NW
                R4, NV = RV - 1, 16 * MT * (RS // 4)
                NSLOT = cdiv(NV, NTHR)
                dyimg, nfh = g.L * g.F, g.F // 16
                tid = np.arange(NTHR)
                for ri in range(cdiv(g.H, g.S)):
                    a_lo, a_hi = max(0, ri - (g.LH - 1)), min(AP - 1, ri)
                    if a_hi < a_lo:
                        continue
                    for ws in range(strips):
                        jlo = ws * NCELL - (AP - 1)
                        for bt in range(nbt):
                            b0 = bt * BT
                            for q in range(NSLOT):
                                P = q * NTHR + tid
                                b, v = P // RV, P % RV
                                j = jlo + (v >> 2)
                                ok = (P < NV) & (v < R4) & (b0 + b < g.B) & (j >= 0) & (j < g.LW)
                                goff = np.where(ok, b * dyimg + j * g.F + (v & 3) * 4, 0)
                                live = ok | ~((P < NV) & (v < R4))
                                # every wave of every load has a live lane (the kernel's waits count on it)
                                assert live.reshape(-1, 64).any(axis=1).all()
                                for a in (a_lo, a_hi):
                                    for fh in (0, nfh - 1):
                                        ad = b0 * dyimg + (ri - a) * g.LW * g.F + fh * 16 + goff
                                        assert ad.min() >= 0 and ad.max() + 4 <= g.B * dyimg, (g, ri, ws, bt, q)
                        for wc in range(NCELL):
                            for a in (a_lo, a_hi):
                                for ap in range(AP):
                                    j = min(max(ws * NCELL + wc - ap, 0), g.LW - 1)
                                    base = (((ri - a) * g.LW + j) * g.K + g.S * a * RC + g.S * ap * g.C) * g.F
                                    nn = np.arange(g.S * SC)
                                    kn = ((nn // SC) * RC + nn % SC) * g.F
                                    assert base >= 0 and base + (nfh - 1) * 16 + kn.max() + 16 <= g.L * g.K * g.F
    if name == "cfg5_s1":
        assert {"lc_forward_direct", "lc_bwd_data_direct", "lc_bwd_weights_strip"} <= seen


# ------------------------------------------------------------------------------------ fused pooling + LCN forward
def replay_pool_lcn_band(shape, ks, p):
    """Replays pool_lcn_band_kernel's lane arithmetic for one image: which lane produces which pooled pixel, which
    rows of x it loads, which map cells and outputs it writes."""
    B, H, W, C = shape
    LPP, RPT = p["tparam"][:2]
    PB, bands, WPS, rpt = p["arg"][:4]
    assert p["arg"][4:8] == [H, W, ks, B] and LPP * 4 == C
    Hp, Wp, r = H - 2, W - 2, (ks - 1) // 2
    MH, MW = PB + 2 * r, Wp + 2 * r
    CPW, OPW = 64 // LPP, 64 // LPP - 2
    assert p["block"] == 1024 and p["grid"] == (B * bands, 1, 1)
    assert 1 <= rpt <= RPT <= 13 and 1 <= WPS <= 16 and WPS * OPW >= Wp and (16 // WPS) * rpt >= MH
    assert PB * bands >= Hp > PB * (bands - 1)
    assert p["lds_bytes"] >= (2 * MH * MW + 2 * PB * Wp + MH + Wp + 15) * 4 and p["lds_bytes"] <= 64 * 1024
    owned = np.zeros((Hp, Wp), dtype=np.int32)
    for band in range(bands):
        r0 = band * PB
        cells = np.zeros((MH, Wp), dtype=np.int32)
        for wave in range(16):
            seg, ws = divmod(wave, WPS)
            hrow0 = seg * rpt
            for cw in range(CPW):
                col = ws * OPW + cw
                for t in range(RPT):
                    hrow, prow = hrow0 + t, r0 - r + hrow0 + t
                    valid = t < rpt and hrow < MH and 0 <= prow < Hp and cw < OPW and col < Wp
                    if not valid:
                        continue
                    # the three rows of x under this pooled row are among the lane's loads, inside the image, and the
                    # two columns to the right come from lanes of the same wave
                    assert t + 2 < rpt + 2 and 0 <= prow and prow + 2 < H and col + 2 < W and cw + 2 < CPW
                    cells[hrow, col] += 1
                    if r0 <= prow < r0 + PB:
                        owned[prow, col] += 1
        rows = np.arange(MH) + r0 - r
        inside = (rows >= 0) & (rows < Hp)
        assert (cells[inside] == 1).all() and (cells[~inside] == 0).all(), (shape, ks, p)
    assert (owned == 1).all(), (shape, ks, p)


def test_fused_pool_lcn_plans_cover_every_pooled_pixel_once():
    rng = np.random.default_rng(11)
    named = [((128, 46, 46, 32), 5), ((128, 57, 57, 16), 5), ((128, 25, 25, 32), 5), ((128, 9, 9, 32), 5),
             ((192, 72, 72, 64), 5), ((1, 3, 3, 8), 3), ((7, 300, 90, 32), 7)]
    fused = 0
    for n in range(1500):
        if n < len(named):
            shape, ks = named[n]
        else:
            C_ = int(rng.choice([8, 16, 32, 64, 4, 12, 128]))
            shape = (int(rng.integers(1, 300)), int(rng.integers(3, 140)), int(rng.integers(3, 140)), C_)
            ks = int(rng.choice([1, 3, 5, 7, 9]))
        p = lc.l2pool_lcn_plan_query(shape, 3, 1, ks)
        if p is None:
            # the fused kernel's limits: 8 to 64 channels in whole quads of a power-of-two count, rows that 16 waves cover
            C_, Wp = shape[3], shape[2] - 2
            assert C_ not in (8, 16, 32, 64) or -(-Wp // (256 // C_ - 2)) > 16, (shape, ks)
            continue
        assert p["kernel"] == "pool_lcn_band"
        replay_pool_lcn_band(shape, ks, p)
        fused += 1
    assert fused > 500
    assert lc.l2pool_lcn_plan_query((4, 20, 20, 16), 2, 2, 5) is None      # other pooling windows: the two kernels
