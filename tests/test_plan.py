"""The cost model of Section 4 and the (U, V) planner (include/zpp_plan.h): host arithmetic, no GPU.

The checks use what the paper fixes: the two communication volumes and the condition it derives from
them (Section 4.1), the bubble formula and the memory formula (Section 4.2), and the rows of its
comparison table, which must agree with the memory formula at the unit size U = 2P-1 that the table
assumes."""
import ctypes
import itertools

import pytest

import synth
import paper_2402_03791_amd as zpp
from paper_2402_03791_amd import binding


def model(**kw):
    base = dict(L=32, h=4096, s=2048, b=1, B=16, P=4, D=8, Mw=12 * 4096 ** 2 * 2.0, Ma=34.0 * 2048 * 4096)
    base.update(kw)
    return zpp.PlanModel(**base)


def test_communication_volumes_and_the_condition_derived_from_them():
    m = model()
    # Section 4.1: TP moves 8*B*b*s*h per block; a unit moves three times the ~12 h^2 parameters, B/U units
    assert zpp.plan_tp_comm(m) == 8 * 16 * 1 * 2048 * 4096
    assert zpp.plan_zeropp_comm(m, 16) == 3 * 12 * 4096 ** 2
    assert zpp.plan_zeropp_comm(m, 4) == 36 * 16 * 4096 ** 2 / 4
    # 36*B*h^2/U < 8*B*b*s*h  <=>  2*s*U*b > 9*h, over a grid that includes the boundary
    for h, s, b, U, B in itertools.product((4, 64, 4096, 5120), (9, 128, 2048, 4096), (1, 2, 4), (1, 2, 8, 16), (16, 48)):
        mm = model(h=h, s=s, b=b, B=B)
        assert zpp.plan_zeropp_wins(mm, U) == (zpp.plan_zeropp_comm(mm, U) < zpp.plan_tp_comm(mm)), (h, s, b, U)
    edge = model(h=4, s=9, b=2)                       # 2*9*1*2 = 9*4: equal volumes, not smaller
    assert zpp.plan_zeropp_comm(edge, 1) == zpp.plan_tp_comm(edge) and not zpp.plan_zeropp_wins(edge, 1)
    # at the 6.2B shape (h 4096, s 2048, b 1) the condition needs U > 9
    assert not zpp.plan_zeropp_wins(m, 9) and zpp.plan_zeropp_wins(m, 10)


def test_bubble_formula():
    m = model(P=4, B=12)
    assert zpp.plan_bubbles(m, 7) == 0 and zpp.plan_bubbles(m, 12) == 0     # U >= 2P-1
    assert zpp.plan_bubbles(m, 3) == 12 * (7 - 3) / 3
    assert zpp.plan_bubbles(m, 6) == 12 * 1 / 6
    assert zpp.plan_bubbles(model(P=1), 1) == 0                              # a single pipeline rank never waits
    # fewer bubbles as the unit grows
    vals = [zpp.plan_bubbles(m, U) for U in (1, 2, 3, 4, 6, 12)]
    assert vals == sorted(vals, reverse=True)


def test_memory_formula_and_the_comparison_table():
    m = model(L=32, P=4, D=8, B=16, Mw=3.0, Ma=5.0)
    mem = zpp.plan_max_memory(m, 7, 2)
    assert mem["weights_partitioned"] == 32 * 3.0 / (4 * 8)
    assert mem["weights_gathered"] == 32 * 3.0 / (4 * 2)
    assert mem["activations"] == 7 * 32 * 5.0 / 4
    assert mem["total"] == mem["weights_partitioned"] + mem["weights_gathered"] + mem["activations"]
    assert zpp.plan_max_memory(m, 64, 2)["activations"] == 16 * 32 * 5.0 / 4      # min(B, U)
    # the table's ZeroPP row is the formula at U = 2P-1; recomputation divides the activations by V
    for V in (1, 2, 4, 8):
        row = zpp.plan_pp_method(m, "zeropp", V)
        f = zpp.plan_max_memory(m, 2 * 4 - 1, V)
        assert row["bubble_ratio"] == 0
        assert row["weight_memory"] == pytest.approx(f["weights_partitioned"] + f["weights_gathered"], rel=1e-15)
        assert row["activation_memory"] == pytest.approx(f["activations"], rel=1e-15)
        rc = zpp.plan_pp_method(m, "zeropp_recompute", V)
        assert rc["activation_memory"] == pytest.approx(f["activations"] / V, rel=1e-15)
        assert rc["weight_memory"] == row["weight_memory"]
    g, f1, il = (zpp.plan_pp_method(m, k, 2) for k in ("gpipe", "1f1b", "interleaved_1f1b"))
    assert g["bubble_ratio"] == f1["bubble_ratio"] == 3 / 16 and il["bubble_ratio"] == 3 / 32
    assert g["weight_memory"] == f1["weight_memory"] == il["weight_memory"] == 32 * 3.0 / 4
    assert g["activation_memory"] == 16 * 32 * 5.0 / 4
    assert f1["activation_memory"] == 32 * 5.0
    assert il["activation_memory"] == 32 * 5.0 * (1 + 3 / 8)
    # the ordering the table's arrows state: ZeroPP holds the least weight memory
    assert zpp.plan_pp_method(m, "zeropp", 2)["weight_memory"] < g["weight_memory"]
    with pytest.raises(zpp.ZppError) as e:     # unknown method
        binding._check(zpp.lib().zpp_plan_pp_method(ctypes.byref(m), 9, 1, None, None, None))
    assert e.value.status == -1


def test_planner_picks_the_best_choice_that_fits():
    m = model(L=32, P=4, D=8, B=16, Mw=3.0, Ma=5.0)

    def candidates(limit):
        out = []
        for U in (1, 2, 4, 8, 16):
            for V in (1, 2, 4, 8):
                mem = zpp.plan_max_memory(m, U, V)["total"]
                if mem <= limit:
                    out.append((zpp.plan_bubbles(m, U), zpp.plan_zeropp_comm(m, U), mem, V, U))
        return out

    prev = None
    for limit in (60.0, 100.0, 200.0, 400.0, 1000.0):
        c = zpp.plan_choose(m, limit)
        cand = candidates(limit)
        assert c["memory"] <= limit and (zpp.plan_bubbles(m, c["U"]), c["comm"]) == min(cand)[:2]
        assert (c["bubbles"], c["comm"], c["memory"], c["V"], c["U"]) == min(cand)
        if prev:   # a larger budget never makes the plan worse
            assert (c["bubbles"], c["comm"]) <= (prev["bubbles"], prev["comm"])
        prev = c
    assert zpp.plan_choose(m, 1000.0)["U"] == 16            # everything fits: one unit, no bubbles
    tight = zpp.plan_choose(m, 60.0)
    assert tight["U"] < 7 and tight["bubbles"] > 0          # too little room for 2P-1 active micro-batches
    with pytest.raises(zpp.ZppError) as e:
        zpp.plan_choose(m, 1.0)
    assert e.value.status == -6
    with pytest.raises(zpp.ZppError) as e:
        zpp.plan_choose(model(L=30, P=4), 1e9)
    assert e.value.status == -1


def test_memory_formula_against_the_workspace_this_library_plans():
    """With P = D = 1 the gathered-stage and activation terms of the formula are what zpp_device plans,
    when M_w and M_a are the library's own per-block figures."""
    sh = synth.CONFIGS["cfg3_gpt_6p2b"]                  # L = 4 blocks, U = 16
    one = zpp.Device(sh.replace(n_blocks=1), 1, prefetch=False, allocate=False).memory_terms()
    Mw, Ma = one["working_copies"], one["stash"] / sh.unit_mbs
    m = zpp.PlanModel(L=4, h=sh.hidden, s=sh.seq, b=sh.micro_batch, B=sh.unit_mbs, P=1, D=1, Mw=float(Mw), Ma=float(Ma))
    for V in (1, 2, 4):
        dev = zpp.Device(sh.replace(n_blocks=4 // V), V, prefetch=False, allocate=False)
        t = dev.memory_terms()
        f = zpp.plan_max_memory(m, sh.unit_mbs, V)
        assert abs(t["working_copies"] - f["weights_gathered"]) <= 1e-4 * f["weights_gathered"]
        assert abs(t["stash"] - f["activations"]) <= 1e-4 * f["activations"]
        dev.close()
