"""Alg. 1 planning arithmetic: the oracle against the paper's worked example
(Sec. 4.1, fixture tests/golden/planner_example.txt) and against invariants;
the library's range-based planner against the oracle's set-based one."""
import os

import numpy as np

import oracle
import paper_2604_12171_amd as P

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "planner_example.txt")


def _parse_golden():
    d = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = line.split(":", 1)
        d[k.strip()] = v.split()
    rng = lambda t: tuple(int(x) for x in t.split("-"))
    cur = [rng(t) for t in d["current"]]
    tgt = [rng(t) for t in d["target"]]
    inter = [set(int(x) for x in t.split(",")) for t in d["intermediate"]]
    add = {int(t.split("=")[0][3:]): set(int(x) for x in t.split("=")[1].split(",") if x) for t in d["add"]}
    mig = {}
    for t in d["migrate"]:
        lhs, rhs = t.split("=")
        a, b = lhs.split(">")
        mig[(int(a[3:]), int(b[3:]))] = set(int(x) for x in rhs.split(","))
    dele = {int(t.split("=")[0][3:]): set(int(x) for x in t.split("=")[1].split(",") if x) for t in d["delete"]}
    return cur, tgt, inter, add, mig, dele


def test_oracle_reproduces_the_worked_example():
    cur, tgt, inter, add, mig, dele = _parse_golden()
    # the paper numbers layers and GPUs from 1; the oracle from 0
    cs = [set(range(a - 1, b)) for a, b in cur]
    ts = [set(range(a - 1, b)) for a, b in tgt]
    rc, out = oracle.plan_reconfig(cs, ts, 6, [80e9, 80e9, 80e9], 0.9, 2e9, 1e6, 10, 100000)
    assert rc == oracle.OK
    assert [set(l + 1 for l in s) for s in out["tmp"]] == inter
    assert {(a + 1, b + 1): set(l + 1 for l in v) for (a, b), v in out["mig"].items()} == mig
    assert [set(l + 1 for l in s) for s in out["dele"]] == [dele[1], dele[2], dele[3]]
    got_add = {}
    for (a, b), v in out["mig"].items():
        got_add.setdefault(b + 1, set()).update(l + 1 for l in v)
    assert got_add == {k: v for k, v in add.items() if v}
    # GPU 2 both receives (layer 2) and forwards (layer 4)
    assert any(b == 1 for (a, b) in out["mig"]) and any(a == 1 for (a, b) in out["mig"])
    # budgets: every intermediate set has 2..3 layers, the largest (3) fixes B_shrink
    assert out["b_shrink"] == oracle.max_blocks(80e9, 0.9, 3, 2e9, 1e6)
    assert out["b_new"] == oracle.max_blocks(80e9, 0.9, 3, 2e9, 1e6)      # GPU 3 ends with 3 layers
    assert out["feasible"] and out["need_shrink"]


def test_oracle_feasibility_and_identity_plan():
    cs = [set(range(0, 4)), set(range(4, 8))]
    rc, out = oracle.plan_reconfig(cs, cs, 8, [1e9, 1e9], 1.0, 1e8, 1e6, 0, 10**9)
    assert rc == oracle.OK and not out["mig"] and all(not d for d in out["dele"])
    assert out["b_shrink"] == out["b_new"] == int((1e9 - 4e8) // 4e6)
    ts = [set(range(0, 2)), set(range(2, 8))]
    b = oracle.max_blocks(1e9, 1.0, 6, 1e8, 1e6)
    rc, out = oracle.plan_reconfig(cs, ts, 8, [1e9, 1e9], 1.0, 1e8, 1e6, b + 1, 10**9)
    assert not out["feasible"]                           # B_used > B_shrink -> Alg. 1 returns false
    rc, out = oracle.plan_reconfig(cs, ts, 8, [1e9, 1e9], 1.0, 1e8, 1e6, b, 10**9)
    assert out["feasible"] and out["mig"] == {(0, 1): {2, 3}} and out["dele"] == [{2, 3}, set()]
    rc, out = oracle.plan_reconfig([set(), {1}], [{0}, {1}], 2, [1e9, 1e9], 1.0, 1e8, 1e6, 0, 1)
    assert rc == oracle.E_RANGE                          # layer 0 has no owner


def test_library_planner_equals_oracle_on_random_contiguous_configs():
    rng = np.random.default_rng(5)
    for case in range(300):
        n = int(rng.integers(2, 6))
        L = int(rng.integers(n, 40))

        def split():
            cuts = np.sort(rng.choice(np.arange(1, L), size=n - 1, replace=False)) if L > n - 1 else np.arange(1, n)
            edges = [0] + cuts.tolist() + [L]
            return [(edges[i], edges[i + 1] - 1) for i in range(n)]

        cur, tgt = split(), split()
        if case % 7 == 0:                                 # a GPU that ends up empty
            tgt = [(tgt[0][0], tgt[1][1])] + [(1, 0)] + tgt[2:] if n > 2 else tgt
        mem = rng.uniform(20e9, 200e9, size=n)
        used, curb = int(rng.integers(0, 200000)), int(rng.integers(1000, 400000))
        rc_o, o = oracle.plan_reconfig([set(range(a, b + 1)) for a, b in cur], [set(range(a, b + 1)) for a, b in tgt],
                                       L, mem, 0.9, 0.4e9, 65536.0, used, curb)
        rc_l, plan, mig, dele = P.pipelive_plan_reconfig(cur, tgt, mem, 0.9, 0.4e9, 65536.0, used, curb)
        assert rc_o == oracle.OK and rc_l == P.OK
        assert (bool(plan.feasible), bool(plan.need_shrink), plan.b_shrink, plan.b_new) == \
               (o["feasible"], o["need_shrink"], o["b_shrink"], o["b_new"])
        got = {}
        for s, d, l in mig:
            got.setdefault((s, d), set()).add(l)
        assert got == o["mig"]
        gd = [set() for _ in range(n)]
        for g, l in dele:
            gd[g].add(l)
        assert gd == o["dele"]
        assert plan.n_mig == sum(len(v) for v in o["mig"].values())


def test_convergence_predicate():
    assert P.pipelive_converged(1000, [960, 951], 50)
    assert not P.pipelive_converged(1000, [960, 950], 50)      # gap == tau is not yet converged
    assert P.pipelive_converged(10, [], 50)
