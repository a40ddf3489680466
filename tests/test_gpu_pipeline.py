"""The layer pipeline of Sec. 3.1 (training paragraph, figure on semi-parallel training): every layer but the last
runs a training instance and a forward-only instance whose parameters are refreshed every P steps and which feeds
the next layer.  The streamed schedule (one HIP stream per stage) must reproduce the same schedule issued on one
stream bit for bit, and that must match the oracle driven through the same chain of stale parameters."""
import numpy as np
import pytest
import torch

import oracle
import paper_1502_03409_amd as lc
import workloads as wl
from conftest import rel_fro
from paper_1502_03409_amd.pipeline import SaePipeline
from test_gpu_parity import update_bar

pytestmark = pytest.mark.gpu

STAGES = [wl.LCGeom(B=24, H=40, W=40, C=3, R=8, S=2, F=16),     # -> 17x17 fields, pooled / normalised 15x15x16
          wl.LCGeom(B=24, H=15, W=15, C=16, R=4, S=1, F=16),    # -> 12x12, then 10x10x16
          wl.LCGeom(B=24, H=10, W=10, C=16, R=4, S=2, F=8)]     # last stage: no forward-only instance
LAMBDAS = [wl.SAE_LAMBDA, wl.SAE_LAMBDA, wl.SAE_LAMBDA_DENSE]
ALPHA0, STEPS = 0.9, 6
# (flags, lr): unit-norm rows with a step that keeps six steps stable; and learned alpha too, whose gradient sums over every
# unit of the layer and needs a far smaller step
MODES = {"project": (1, 5e-3), "project_alpha": (3, 1e-4)}
POOL = (wl.POOL_KSIZE, wl.POOL_STRIDE, wl.POOL_EPS)
LCN = (wl.LCN_KSIZE, wl.LCN_SIGMA, wl.LCN_EPS)


def initial_parameters():
    ws, bs = [], []
    for s, g in enumerate(STAGES):
        r = np.random.default_rng(200 + s)
        ws.append((r.standard_normal((g.LH, g.LW, g.K, g.F)) / np.sqrt(g.K)).astype(np.float32))
        bs.append((0.05 * r.standard_normal((g.H, g.W, g.C))).astype(np.float32))
    return ws, bs


def batches():
    return [wl.pink_images(np.random.default_rng(300 + t), 24, 40, 40, 3) for t in range(STEPS)]


def run_gpu(P, streams, mode="project"):
    FLAGS, LR = MODES[mode]
    ws, bs = initial_parameters()
    dev = lambda a: torch.from_numpy(a.copy()).cuda()
    pipe = SaePipeline([lc.geom(*g.as_tuple()) for g in STAGES], [dev(w) for w in ws], [dev(b) for b in bs],
                       [ALPHA0] * 3, LAMBDAS, sync_period=P, eps_sparse=wl.SAE_EPS, lr=LR, flags=FLAGS, pool=POOL,
                       lcn=LCN, streams=streams)
    xs = [dev(x) for x in batches()]
    costs = []
    for x in xs:
        pipe.step(x)
        if not streams:          # per-step costs from the one-stream run (reading them synchronises)
            torch.cuda.synchronize()
            costs.append([float(st.cost.item()) for st in pipe.stages])
    pipe.join()
    torch.cuda.synchronize()
    state = [(st.w.cpu().numpy(), st.b.cpu().numpy(), float(st.alpha.item()), float(st.cost.item())) for st in pipe.stages]
    return state, costs


def run_oracle(P, mode="project"):
    FLAGS, LR = MODES[mode]
    ws, bs = initial_parameters()
    W = [w.astype(np.float64) for w in ws]
    Bv = [b.astype(np.float64) for b in bs]
    A = [ALPHA0] * 3
    Wf, Af = [None] * 3, [None] * 3
    costs = []
    for t, x in enumerate(batches()):
        x_in, row = x.astype(np.float64), []
        for s, g in enumerate(STAGES):
            tg = g.as_tuple()
            nxt = None
            if s < 2:
                if t % P == 0:
                    Wf[s], Af[s] = W[s].copy(), A[s]
                hf = oracle.lc_forward(tg, x_in, Wf[s], None, Af[s])
                nxt = oracle.lcn_fwd(oracle.l2pool_fwd(hf, *POOL), *LCN)[0]
            J, W[s], Bv[s], A[s], _ = oracle.sae_step(tg, x_in, W[s], Bv[s], A[s], LAMBDAS[s], wl.SAE_EPS, LR, FLAGS)
            row.append(J)
            x_in = nxt
        costs.append(row)
    return list(zip(W, Bv, A)), costs


@pytest.mark.parametrize("P,mode", [(1, "project"), (2, "project"), (4, "project"), (2, "project_alpha")])
def test_pipeline_streams_match_one_stream_and_the_oracle(P, mode):
    print(f"case pipeline sync period {P} {mode}", flush=True)
    one, costs = run_gpu(P, streams=False, mode=mode)
    many, _ = run_gpu(P, streams=True, mode=mode)
    # (a) one stream per stage against everything on one stream: the same bits
    for s in range(3):
        np.testing.assert_array_equal(many[s][0], one[s][0])
        np.testing.assert_array_equal(many[s][1], one[s][1])
        assert many[s][2] == one[s][2] and many[s][3] == one[s][3]
    # (b) against the oracle run through the same chain of stale forward-only parameters
    ref, ref_costs = run_oracle(P, mode)
    w0, b0 = initial_parameters()
    for t in range(STEPS):
        for s in range(3):
            assert abs(costs[t][s] - ref_costs[t][s]) <= 1e-4 * abs(ref_costs[t][s]), (t, s)
    for s in range(3):
        for nm, got, want, base in (("dW", one[s][0], ref[s][0], w0[s]), ("db", one[s][1], ref[s][1], b0[s])):
            upd = want - base
            bar, floor = update_bar(got, upd, projected=nm == "dW")
            e = rel_fro(got.astype(np.float64) - base, upd)
            print(f"  stage {s + 1} {nm} over {STEPS} steps rel err {e:.2e} (bar {bar:.2e})", flush=True)
            assert e <= bar
        if MODES[mode][0] & 2:
            # alpha is stored in fp32 after every step: its change carries up to STEPS roundings of alpha itself
            bar = max(1e-4, 0.5e-4 + STEPS * 2.0 ** -24 * abs(ref[s][2]) / abs(ref[s][2] - ALPHA0))
            e = abs(one[s][2] - ref[s][2]) / abs(ref[s][2] - ALPHA0)
            print(f"  stage {s + 1} alpha rel err of the change {e:.2e} (bar {bar:.2e})", flush=True)
            assert e <= bar
        else:
            assert one[s][2] == np.float32(ALPHA0)


def test_stale_parameters_change_the_result():
    """The sync period is not a no-op: with P = 4 the second stage sees other features than with P = 1."""
    a, _ = run_gpu(1, streams=False)
    b, _ = run_gpu(4, streams=False)
    np.testing.assert_array_equal(a[0][0], b[0][0])          # the first stage never depends on the period
    assert rel_fro(b[1][0], a[1][0]) > 1e-7
