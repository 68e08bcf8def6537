"""The sharding planner (Section V-B): pins of the exhaustive oracle, and the library's pruned
search against it, exactly.  CPU only."""
import os

import numpy as np
import pytest

from oracle import planner as P
from paper_2311_00257_amd import binding as B
from paper_2311_00257_amd import build, workloads


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not build.built():
        build.build_all(verbose=False)


FLAT = [(op, 2, 1, v, 1e9) for op in range(4) for v in (1e3, 1e9)]
TINY = dict(phi=1e6, layers=1, module_params=[1e6], micro_batches=2, bucket_bytes=1e6, R=2, N=1,
            activation=0.0, tmp=0.0, table=FLAT)


def test_hand_evaluated_example(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "planner_tiny.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 5
    for r in rows:
        mem = float(r[0])
        best, count = P.plan(gpu_memory=mem, **TINY)
        if r[1] == "none":
            assert best is None and count == 0
            continue
        assert best["s"] == tuple(int(x) for x in r[1:7]) and count == int(r[8])
        assert best["t_comm"] == pytest.approx(float(r[7]), rel=1e-12)
    # activations and temporaries eat into the same limit (Section IV-D): 12e6 - 1.5e6 - 1e6 leaves 9.5e6
    best, count = P.plan(gpu_memory=12e6, **dict(TINY, activation=1.5e6, tmp=1e6))
    assert best["s"] == (1, 1, 2, 1, 2, 1) and count == 2


def test_cost_formulas_by_hand():
    """Phi = 4e6, L = 3, modules of 1e6 and 3e5 parameters, M = 3, U = 2e6 bytes, R = N = 2; flat
    bandwidths AG 2e9, RS 1e9, BC 1e9, AR 4e9 inside a node and 0.5e9 on any mesh that spans nodes."""
    table = []
    for mesh in ((2, 1), (1, 2), (2, 2)):
        for v in (1.0, 1e12):
            table += [(P.AG,) + mesh + (v, 2e9), (P.RS,) + mesh + (v, 1e9), (P.BC,) + mesh + (v, 1e9),
                      (P.AR,) + mesh + (v, 4e9 if mesh[1] == 1 else 0.5e9)]
    args = (4e6, 3, [1e6, 3e5], 3, 2e6, 2, 2, table)
    # s_p = s_g = 2x1, s_os = 2x2:
    #   T_p   = 3*3*[(2*2e6/2e9 + 2e6/1e9) + (2*6e5/2e9 + 6e5/1e9)] = 9 * 5.2e-3
    #   T_os0 = 8e6/(2e6*2) * t(AR, 2e6, 1x2) = 2 * 4e-3;  T_os1 = 4/2 * t(BC, 8e6/4, 1x2) = 2 * 2e-3;  T_g = 0
    c = P.evaluate((2, 1, 2, 1, 2, 2), *args)
    assert c["t_p"] == pytest.approx(46.8e-3, rel=1e-12) and c["t_os0"] == pytest.approx(8e-3, rel=1e-12)
    assert c["t_os1"] == pytest.approx(4e-3, rel=1e-12) and c["t_g"] == 0.0
    assert c["t_comm"] == pytest.approx(58.8e-3, rel=1e-12) and c["d_modelstate"] == 20e6
    # s_p = 1x1, s_g = s_os = 2x1:
    #   T_os0 = 8e6/2e6 * t(AR, 2e6, 2x2) = 4 * 4e-3;  T_os1 = 2 * t(BC, 4e6, 2x1) = 2 * 4e-3
    #   T_g   = (3-1) * 8e6/2e6 * t(AR, 2e6, 2x1) = 8 * 0.5e-3
    c = P.evaluate((1, 1, 2, 1, 2, 1), *args)
    assert c["t_p"] == 0.0 and c["t_os0"] == pytest.approx(16e-3, rel=1e-12)
    assert c["t_os1"] == pytest.approx(8e-3, rel=1e-12) and c["t_g"] == pytest.approx(4e-3, rel=1e-12)
    assert c["d_modelstate"] == 36e6
    # constraints, one violation each
    assert P.constraints_hold((2, 1, 2, 1, 2, 2), 2, 2) and P.constraints_hold((1, 1, 1, 1, 1, 1), 2, 2)
    assert not P.constraints_hold((2, 1, 1, 1, 2, 1), 2, 2)      # s_g below s_p (Eq. 3)
    assert not P.constraints_hold((2, 1, 2, 1, 1, 1), 2, 2)      # s_os below s_p (Eq. 3)
    assert not P.constraints_hold((1, 1, 1, 1, 1, 2), 2, 2)      # spans nodes before the node is full (Eq. 7)
    assert not P.constraints_hold((1, 1, 2, 1, 2, 2), 2, 2)      # s_g is neither s_p nor s_os
    assert not P.constraints_hold((1, 1, 1, 1, 3, 1), 4, 1)      # 3 does not divide 4 (Eq. 5)
    assert not P.constraints_hold((1, 1, 1, 1, 4, 3), 4, 4)      # 3 does not divide 4 (Eq. 6)
    assert not P.constraints_hold((1, 1, 1, 1, 4, 1), 2, 1)      # beyond the node (Eq. 3)
    # the search returns the cheapest tuple that fits, and the first one on a tie
    best, count = P.plan(4e6, 3, [1e6, 3e5], 3, 2e6, 2, 2, 21e6, 0.0, 0.0, table)
    # 21e6 bytes admit three tuples: (2x1, 2x1, 2x2) 20e6, (2x1, 2x2, 2x2) 18e6, (2x2, 2x2, 2x2) 16e6
    fits = [(2, 1, 2, 1, 2, 2), (2, 1, 2, 2, 2, 2), (2, 2, 2, 2, 2, 2)]
    costs = [P.evaluate(s, *args)["t_comm"] for s in fits]
    assert count == 3 and best["s"] == fits[costs.index(min(costs))] and best["t_comm"] == min(costs)
    # a true tie: with M = 1 the gradient mesh costs nothing, so (1x1, 1x1, 2x1) and (1x1, 2x1, 2x1) cost the
    # same; AllGather is left out of the table, which rules out s_p = 2x1, and 12e6 bytes rule out no sharding
    no_ag = [(op, 2, 1, v, 1e9) for op in (P.RS, P.AR, P.BC) for v in (1.0, 1e12)]
    tie, n_tie = P.plan(1e6, 1, [1e6], 1, 1e6, 2, 1, 12e6, 0.0, 0.0, no_ag)
    assert n_tie == 2 and tie["s"] == (1, 1, 1, 1, 2, 1)


def test_bandwidth_interpolation_and_missing_mesh():
    table = [(P.AR, 8, 1, 1e6, 10e9), (P.AR, 8, 1, 1e8, 30e9), (P.AR, 8, 1, 1e7, 20e9)]
    assert P.bandwidth(table, P.AR, 1e7, 8, 1) == 20e9
    assert P.bandwidth(table, P.AR, 5.5e6, 8, 1) == pytest.approx(15e9)          # halfway between 1e6 and 1e7
    assert P.bandwidth(table, P.AR, 1e3, 8, 1) == 10e9 and P.bandwidth(table, P.AR, 1e12, 8, 1) == 30e9
    assert P.bandwidth(table, P.AG, 1e7, 8, 1) is None and P.bandwidth(table, P.AR, 1e7, 4, 1) is None
    assert P.coll_time(table, P.AG, 1e7, 1, 1) == 0.0                            # one GPU: nothing to send
    assert P.coll_time(table, P.AR, 1e7, 8, 1) == pytest.approx(1e7 / 20e9)
    # a tuple whose meshes are not all in the table cannot be chosen
    best, count = P.plan(gpu_memory=1e9, **dict(TINY, table=[r for r in FLAT if r[0] != P.BC]))
    assert best["s"] == (1, 1, 1, 1, 1, 1) and count == 2                        # the two tuples with s_os > s_p need BC


def ring_table(R, N, intra=300e9, inter=25e9, alpha=10e-6):
    """A synthetic profile from the ring alpha-beta model of Section IV-A."""
    rows = []
    for op in range(4):
        for p0 in range(1, R + 1):
            for p1 in range(1, N + 1):
                if p0 * p1 == 1:
                    continue
                p = p0 * p1
                w = intra if p1 == 1 else inter
                for v in (1e5, 1e6, 1e7, 1e8, 1e9, 1e10):
                    steps = (p - 1) * (2 if op == P.AR else 1)
                    t = steps * (alpha + v / (w * p)) if op != P.BC else (p - 1) * alpha + v / w
                    rows.append((op, p0, p1, v, v / t))
    return rows


def _constraints_hold(s, R, N):
    """The constraints again, written independently of the oracle's own check."""
    sp0, sp1, sg0, sg1, so0, so1 = s
    ok = 1 <= sp0 <= sg0 <= so0 <= R and 1 <= sp1 <= sg1 <= so1 <= N
    ok &= all(R % a == 0 for a in (sp0, sg0, so0)) and all(N % a == 0 for a in (sp1, sg1, so1))
    ok &= all(b == 1 or a == R for a, b in ((sp0, sp1), (sg0, sg1), (so0, so1)))
    ok &= (sg0, sg1) in ((sp0, sp1), (so0, so1))
    return ok


@pytest.mark.parametrize("cfg,R,N,budget", [(1, 8, 4, 45e9), (3, 8, 4, 45e9), (4, 8, 4, 60e9), (1, 8, 1, 1e12)])
def test_llama_plans_obey_every_constraint_and_the_memory_limit(cfg, R, N, budget):
    w = workloads.get(cfg)
    phi = float(w.total_elems)
    mods = [float(x) for x in w.tensor_sizes[1:10]]
    best, count = P.plan(phi, w.layers, mods, 4, 256e6, R, N, budget, 0.0, 0.0, ring_table(R, N))
    assert best is not None and count >= 1
    assert _constraints_hold(best["s"], R, N)
    sp, sg, so = (best["s"][0] * best["s"][1], best["s"][2] * best["s"][3], best["s"][4] * best["s"][5])
    assert best["d_modelstate"] == pytest.approx(2 * phi / sp + 2 * phi / sg + 12 * phi / so)
    assert best["d_modelstate"] <= budget
    # more memory never makes the best plan slower; with unlimited memory on one node nothing is sharded
    roomy, _ = P.plan(phi, w.layers, mods, 4, 256e6, R, N, 10 * budget, 0.0, 0.0, ring_table(R, N))
    assert roomy["t_comm"] <= best["t_comm"]


def test_table_iv_rows_are_feasible_and_priced():
    """The meshes the paper reports for its own runs (Table IV: 7B -> 1x1,1x1,8x1; 13B -> 4x1,4x1,8x1;
    30B -> 8x1,8x1,8x4) pass every constraint of the program; whether they are optimal depends on the
    paper's measured bandwidths, which exist only as a figure."""
    for cfg, s in ((1, (1, 1, 1, 1, 8, 1)), (3, (4, 1, 4, 1, 8, 1)), (4, (8, 1, 8, 1, 8, 4))):
        assert _constraints_hold(s, 8, 128)
        w = workloads.get(cfg)
        phi = float(w.total_elems)
        sp, sg, so = s[0] * s[1], s[2] * s[3], s[4] * s[5]
        assert 2 * phi / sp + 2 * phi / sg + 12 * phi / so < 80e9       # fits an 80 GB GPU (Section VI)


def random_problems(trials=60, seed=21):
    """Seeded planner problems: argument tuples of P.plan / B.amsp_plan_sharding, with ring-model
    profiles, some of them with holes."""
    rng = np.random.default_rng(seed)
    for trial in range(trials):
        R = int(rng.choice([1, 2, 4, 6, 8]))
        N = int(rng.choice([1, 2, 3, 4, 6, 8]))
        table = ring_table(R, N, intra=float(rng.uniform(50e9, 400e9)), inter=float(rng.uniform(5e9, 60e9)),
                           alpha=float(rng.uniform(1e-6, 50e-6)))
        if trial % 5 == 0:      # holes in the profile
            table = [r for r in table if not (r[1] == R and r[2] == N and r[0] == P.BC)]
        phi = float(rng.uniform(1e8, 4e10))
        mods = [float(x) for x in rng.uniform(1e6, 2e8, int(rng.integers(1, 8)))]
        M = int(rng.integers(1, 9))
        U = float(rng.choice([25e6, 256e6, 1e9]))
        mem = float(rng.uniform(0.3, 18.0)) * phi
        yield (phi, int(rng.integers(1, 80)), mods, M, U, R, N, mem, float(rng.uniform(0, 0.2)) * phi, 1e8, table)


def test_library_search_equals_the_exhaustive_oracle():
    checked = 0
    for args in random_problems():
        want, count = P.plan(*args)
        if want is None:
            with pytest.raises(B.AmspError) as ei:
                B.amsp_plan_sharding(*args)
            assert ei.value.status == B.AMSP_ENOPLAN
            continue
        got, got_count = B.amsp_plan_sharding(*args)
        assert got["s"] == want["s"] and got_count == count
        for key in ("t_p", "t_g", "t_os0", "t_os1", "t_comm", "d_modelstate"):
            assert got[key] == pytest.approx(want[key], rel=1e-12, abs=0.0)
        checked += 1
    assert checked >= 30
    got, _ = B.amsp_plan_sharding(TINY["phi"], 1, TINY["module_params"], 2, 1e6, 2, 1, 9.5e6, 0.0, 0.0, FLAT)
    assert got["s"] == (1, 1, 2, 1, 2, 1) and got["t_comm"] == pytest.approx(6e-3, rel=1e-12)


def test_library_argument_errors():
    for bad in (dict(R=0), dict(N=0), dict(M=0), dict(phi=0.0), dict(U=0.0)):
        a = dict(phi=1e6, L=1, mods=[1e6], M=1, U=1e6, R=2, N=1)
        a.update(bad)
        with pytest.raises(B.AmspError) as ei:
            B.amsp_plan_sharding(a["phi"], a["L"], a["mods"], a["M"], a["U"], a["R"], a["N"], 1e9, 0.0, 0.0, FLAT)
        assert ei.value.status == B.AMSP_EINVAL
