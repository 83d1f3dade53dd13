"""Pins of the CPU checker's partition solvers (oracle/partition.py enumerator,
oracle/partition_oracle.c dynamic program): closed forms, hand-worked cases,
special cases and invariants from paper sections 3.2-3.3 and 5.2."""
import math

import numpy as np
import pytest

from oracle import partition as P
from paper_2110_14895_amd import synth


def args(inst):
    return inst.t_comp, inst.layer_mem, inst.dev_mem, inst.xfer_bytes, inst.bw


def make(t_comp, layer_mem=None, dev_mem=None, xfer=None, bw=None):
    t_comp = np.asarray(t_comp, dtype=np.float64)
    L, D = t_comp.shape
    return synth.PartitionInstance(
        t_comp,
        np.ones(L) if layer_mem is None else np.asarray(layer_mem, float),
        np.full(D, 1e9) if dev_mem is None else np.asarray(dev_mem, float),
        np.full(L, 1e-9) if xfer is None else np.asarray(xfer, float),
        np.ones((D, D)) if bw is None else np.asarray(bw, float))


@pytest.mark.parametrize("L,D", [(1, 1), (3, 2), (5, 3), (8, 3), (4, 4), (3, 5)])
def test_enumerator_visits_search_space_closed_form(L, D):
    # section 3.3: sum_i D!/(D-i)! * C(L-1, i-1)
    n = sum(1 for _ in P.all_strategies(L, D))
    want = sum(math.factorial(D) // math.factorial(D - i) * math.comb(L - 1, i - 1)
               for i in range(1, min(D, L) + 1))
    assert n == want == P.search_space_size(L, D)
    if (L, D) == (8, 3):
        assert n == 171
    keys = {P.canonical_key(s) for s in P.all_strategies(L, D)}
    assert len(keys) == n                         # all distinct
    for s in P.all_strategies(L, D):
        assert s[0][1] == 0 and s[-1][2] == L - 1
        assert all(s[k + 1][1] == s[k][2] + 1 for k in range(len(s) - 1))
        assert len({d for d, _, _ in s}) == len(s)


def test_hand_worked_three_layers_two_devices():
    # compute only: dev0 = [1,2,3], dev1 = [3,1,1]
    # {0}|{1,2}: dev0 then dev1 -> max(1, 2) = 2 is the best of the 6 two-stage
    # options and beats both single-device plans (6 and 5).
    inst = make([[1, 3], [2, 1], [3, 1]])
    t, s, n = P.brute_force(*args(inst))
    assert n == 2 + 2 * 2 and t == 2.0 and s == [(0, 0, 0), (1, 1, 2)]
    assert P.paper_dp(*args(inst))[0] == 2.0
    # add a link: P = 10 bytes, b_{0,1} = 4 B/s -> T_comm = 2.5 (Eq. 1); period of stage 1
    # = max(1, 2.5) (Eq. 2) -> T_opt = 2.5
    inst = make([[1, 3], [2, 1], [3, 1]], xfer=[10, 10, 10], bw=[[1, 4], [1, 1]])
    t, s, _ = P.brute_force(*args(inst))
    assert t == 2.5 and s == [(0, 0, 0), (1, 1, 2)]
    assert P.paper_dp(*args(inst))[0] == 2.5
    # a slower link (b = 2 -> 5 s) makes splitting worse than dev1 alone (5): tie at 5 ->
    # canonical = lexicographically smallest (u1, e1, ...) -> (0,0),(1,2)
    inst = make([[1, 3], [2, 1], [3, 1]], xfer=[10, 10, 10], bw=[[1, 2], [0.5, 1]])
    t, s, _ = P.brute_force(*args(inst))
    assert t == 5.0 and s == [(0, 0, 0), (1, 1, 2)]
    # memory: dev1 holds only one layer -> {0,1}|{2} (3) is the best feasible
    inst = make([[1, 3], [2, 1], [3, 1]], dev_mem=[1e9, 1.0])
    t, s, _ = P.brute_force(*args(inst))
    assert t == 3.0 and s == [(0, 0, 1), (1, 2, 2)]
    assert P.paper_dp(*args(inst))[0] == 3.0


def test_last_stage_has_no_communication_term():
    # one device, huge transfer sizes: period is compute only
    inst = make([[1.0], [2.0]], xfer=[1e12, 1e12], bw=[[1e-6]])
    assert P.brute_force(*args(inst))[0] == 3.0
    assert P.paper_dp(*args(inst))[0] == 3.0


@pytest.mark.parametrize("L,D", [(8, 3), (7, 2), (5, 4), (2, 3), (12, 2)])
def test_even_split_closed_form(L, D):
    # identical devices, equal layers, free links -> ceil(L / min(D, L)) * c
    c = 0.25
    inst = make(np.full((L, D), c))
    want = math.ceil(L / min(D, L)) * c
    assert P.brute_force(*args(inst))[0] == want
    assert P.paper_dp(*args(inst))[0] == want


def test_single_device_is_sum_or_infeasible():
    t = np.array([[0.3], [0.1], [0.7], [0.2]])
    inst = make(t, layer_mem=[1, 1, 1, 1], dev_mem=[4])
    acc = 0.0
    for v in t[:, 0]:
        acc = acc + v
    assert P.brute_force(*args(inst))[0] == acc == P.paper_dp(*args(inst))[0]
    inst = make(t, layer_mem=[1, 1, 1, 1], dev_mem=[3.5])
    assert P.brute_force(*args(inst))[0] is None
    assert P.paper_dp(*args(inst)) == (None, None)


def test_dead_links_force_single_stage_on_fastest_fitting_device():
    inst = synth.random_partition_instance(6, 3, 7)
    inst.bw[:] = 1e-12
    inst.dev_mem[:] = inst.layer_mem.sum()
    fastest = int(np.argmin(inst.t_comp.sum(axis=0)))
    inst.dev_mem[fastest] = 0.0        # ... but it cannot hold the model
    t, s, _ = P.brute_force(*args(inst))
    rest = [d for d in range(3) if d != fastest]
    best = min(rest, key=lambda d: sum(inst.t_comp[:, d]))
    assert s == [(best, 0, 5)]
    assert P.paper_dp(*args(inst))[0] == t


@pytest.mark.parametrize("kw", [dict(), dict(mem_tight=0.7), dict(comm_heavy=1.0),
                                dict(mem_tight=0.5, comm_heavy=0.3, quantize=4),
                                dict(quantize=2), dict(mem_tight=0.9, quantize=3)])
def test_dynamic_program_equals_enumeration(kw):
    n_inf = 0
    for seed in range(60):
        L, D = [(8, 3), (6, 3), (5, 2), (4, 4), (7, 3)][seed % 5]
        inst = synth.random_partition_instance(L, D, seed, **kw)
        bt, bs, _ = P.brute_force(*args(inst))
        dt, ds = P.paper_dp(*args(inst))
        if bt is None:
            n_inf += 1
            assert dt is None
            continue
        assert dt == bt                                      # bit-exact
        assert P.evaluate(ds, *args(inst)) == bt             # its plan reaches T_opt
        assert P.evaluate(bs, *args(inst)) == bt
    assert n_inf < 60


def test_monotone_in_devices_bandwidth_memory():
    for seed in range(25):
        inst = synth.random_partition_instance(6, 3, seed, mem_tight=0.6, comm_heavy=0.5)
        base = P.brute_force(*args(inst))[0]
        sub = synth.PartitionInstance(inst.t_comp[:, :2].copy(), inst.layer_mem, inst.dev_mem[:2],
                                      inst.xfer_bytes, inst.bw[:2, :2].copy())
        fewer = P.brute_force(*args(sub))[0]
        if fewer is not None:
            assert base is not None and base <= fewer
        if base is None:
            continue
        faster = synth.PartitionInstance(inst.t_comp, inst.layer_mem, inst.dev_mem, inst.xfer_bytes,
                                         inst.bw * 3.0)
        assert P.brute_force(*args(faster))[0] <= base
        roomier = synth.PartitionInstance(inst.t_comp, inst.layer_mem, inst.dev_mem * 2.0,
                                          inst.xfer_bytes, inst.bw)
        assert P.brute_force(*args(roomier))[0] <= base


def test_slow_egress_device_is_used_only_as_last_stage():
    # section 5.2 (the case with one low-bandwidth device among faster-linked ones): the
    # optimal plan places the device whose outgoing link is slow at the end of the pipeline
    L, D = 8, 3
    t = np.full((L, D), 1.0)
    bw = np.full((D, D), 100.0)
    bw[1, :] = 0.01                        # device 1 sends slowly, receives normally
    inst = make(t, xfer=np.full(L, 10.0), bw=bw)
    tb, s, _ = P.brute_force(*args(inst))
    assert [d for d, _, _ in s][-1] == 1 and len(s) == 3
    assert tb == 3.0


def test_weak_devices_are_left_out():
    # section 5.2: the optimal plan may use fewer devices than available
    L = 6
    t = np.stack([np.full(L, 1.0), np.full(L, 1.0), np.full(L, 50.0)], axis=1)
    inst = make(t)
    tb, s, _ = P.brute_force(*args(inst))
    assert tb == 3.0 and sorted(d for d, _, _ in s) == [0, 1]


def test_full_size_dynamic_program_invariants():
    # 32 layers, 16 devices: no enumeration possible (1.46e22 strategies); the plan must be
    # valid and re-evaluate to T_opt, and T_opt must not exceed simple constructive bounds
    sh = synth.SHAPES["vit_huge"]
    inst = synth.heterogeneous_cluster(np.ones(32), sh, batch=8)
    t, s = P.paper_dp(*args(inst))
    assert t is not None
    assert P.evaluate(s, *args(inst)) == t
    assert s[0][1] == 0 and s[-1][2] == 31
    assert len({d for d, _, _ in s}) == len(s)
    # upper bounds: any single device that fits; lower bound: perfect split over all devices
    for d in range(16):
        single = P.evaluate([(d, 0, 31)], *args(inst))
        if single is not None:
            assert t <= single
    lower = 1.0 / sum(1.0 / inst.t_comp[0, d] for d in range(16)) * 32
    assert t >= lower * (1 - 1e-12)
