"""Host logic of the HBM arena allocator (class-aware first fit), without a GPU: the probe
result is injected."""
import pytest
import torch

from paper_2511_17849_amd.hbm_arena import HbmArena


def fake_arena(classes, granule=1024):
    a = HbmArena.__new__(HbmArena)
    a.granule = granule
    a.buf = torch.empty(len(classes) * granule, dtype=torch.uint8)
    a.classes = list(classes)
    a.used = [False] * len(classes)
    a.n_classes = max(classes) + 1
    return a


def test_alloc_respects_classes_and_contiguity():
    a = fake_arena([0, 0, 0, 1, 1, 0, 2, 2, 2, 1])
    assert a.class_sizes() == [4096, 3072, 3072]
    t, c = a.alloc(512, torch.float32, cls=1)            # 2048 bytes = 2 granules -> granules 3, 4
    assert c == 1 and t.numel() == 512 and t.data_ptr() == a.buf.data_ptr() + 3 * 1024
    t2, c2 = a.alloc(700, torch.float32, cls=2)          # 2800 bytes -> 3 granules 6..8
    assert c2 == 2 and t2.data_ptr() == a.buf.data_ptr() + 6 * 1024
    t3, c3 = a.alloc(300, torch.bfloat16, cls=4)         # class taken modulo the class count: 4 % 3 = 1
    assert c3 == 1 and t3.dtype == torch.bfloat16 and t3.data_ptr() == a.buf.data_ptr() + 9 * 1024
    # class 1 has no run of 2 left: falls back to the class with most room that has one
    t4, c4 = a.alloc(512, torch.float32, cls=1)
    assert c4 == 0 and t4.data_ptr() == a.buf.data_ptr()
    # granule 2 and 5 (class 0) are free but not adjacent: a 2-granule request cannot be met
    with pytest.raises(MemoryError):
        a.alloc(512, torch.float32, cls=0)
    t5, c5 = a.alloc(256, torch.float32)                 # single granules still fit
    assert c5 == 0
    # no overlap between anything handed out
    spans = sorted((x.data_ptr(), x.data_ptr() + x.numel() * x.element_size()) for x in (t, t2, t3, t4, t5))
    assert all(e0 <= b1 for (_, e0), (b1, _) in zip(spans, spans[1:]))


def test_room_counts_disjoint_runs_per_class():
    a = fake_arena([0, 0, 0, 1, 1, 0, 2, 2, 2, 1])
    assert a.room(256) == [4, 3, 3]                       # one granule each
    assert a.room(512) == [1, 1, 1]                       # runs of two: 0-1, 3-4, 6-7
    assert a.room(768) == [1, 0, 1]
    a.alloc(256, torch.float32, cls=0)                    # takes granule 0
    assert a.room(512) == [1, 1, 1] and a.room(768) == [0, 0, 1]
    assert a.room(512, torch.bfloat16) == [3, 3, 3]       # 1024 bytes = one granule


def test_placement_plan_of_the_library():
    """pier_placement_plan (host arithmetic of libpier): every launch's buffers in two classes."""
    import paper_2511_17849_amd as pier
    reps, ca, cm = pier.pier_placement_plan([16, 16, 14], 8)
    assert [r["theta"] for r in reps] == [0, 1] * 4 and all(r["m"] == r["theta"] for r in reps)
    assert [r["v"] for r in reps] == [2] * 7 + [0] and all(r["grad"] == r["v"] for r in reps)
    assert sorted([ca, cm]) == [0, 1]
    # the 7B case: nine buffers fit; two gradient buffers cannot both be paired, one can
    reps, ca, cm = pier.pier_placement_plan([3, 3, 3], 2, outer_on_device=False)
    assert (ca, cm) == (-1, -1) and reps[0] == dict(theta=0, m=0, v=2, grad=2) and reps[1]["v"] == 2 and reps[1]["grad"] != 2
    reps, _, _ = pier.pier_placement_plan([3, 3, 3], 2, shared_grad=True, outer_on_device=False)
    assert all(r["v"] == 2 and r["grad"] == 2 for r in reps)
    # fewer classes
    reps, ca, cm = pier.pier_placement_plan([40], 2)
    assert all(set(r.values()) == {0} for r in reps) and (ca, cm) == (0, 0)
    reps, ca, cm = pier.pier_placement_plan([20, 20], 4)
    assert [(r["theta"], r["v"]) for r in reps] == [(0, 1), (1, 0), (0, 1), (1, 0)] and sorted([ca, cm]) == [0, 1]
    # odd group count: anchor and M even out the two classes
    reps, ca, cm = pier.pier_placement_plan([16, 16, 14], 3)
    assert (ca, cm) == (1, 0)
    # a full class hands its buffers on; too little room altogether is an error
    reps, ca, cm = pier.pier_placement_plan([2, 9, 9], 2)
    assert reps[0]["theta"] == 0 and (ca, cm) == (1, 1)
    with pytest.raises(pier.PierError, match="PIER_ERR_OOM"):
        pier.pier_placement_plan([3, 3, 2], 2)
    for bad in (dict(room=[], n_replicas=2), dict(room=[4, -1], n_replicas=1), dict(room=[4], n_replicas=0)):
        with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
            pier.pier_placement_plan(**bad)


def _placed(policy, G=8, classes=None, **kw):
    from pier_inputs import device as dev
    g = 4096                                             # granule bytes; one buffer = 3 granules
    a = fake_arena(classes or [0] * 48 + [1] * 48 + [2] * 44, granule=g)
    n = 3 * g // 4 - 8
    # PlacedState zeroes its buffers with torch ops, which is fine on the CPU tensors of the fake arena
    s = dev.PlacedState([n], G, arena=a, policy=policy, **kw)
    cls = lambda xs: [x.cls for x in xs]
    return s, cls(s.P), cls(s.M1), cls(s.V), cls(s.Gd), a


def _no_overlap(s):
    bufs = {id(x.flat): x.flat for x in s.P + s.M1 + s.V + s.Gd + [s.A, s.Mo]}.values()
    spans = sorted((x.data_ptr(), x.data_ptr() + x.numel() * x.element_size()) for x in bufs)
    assert all(e0 <= b1 for (_, e0), (b1, _) in zip(spans, spans[1:]))


def test_default_policy_keeps_every_launch_in_two_classes():
    """theta_g, m_g in class g mod 2; the outer step's ten buffers five and five in classes 0 and
    1; v_g, grad_g in class 2 until it is full (14 buffers of 3 granules in 44), then in the class
    theta_g is not in."""
    s, P, M, V, Gd, a = _placed("two_class")
    assert P == [0, 1, 0, 1, 0, 1, 0, 1] and M == P
    assert sorted([s.A.cls, s.Mo.cls]) == [0, 1]
    assert V == [2] * 7 + [0] and Gd == V
    for g in range(8):          # back to back: m_g follows theta_g, grad_g follows v_g
        assert s.M1[g].flat.data_ptr() - s.P[g].flat.data_ptr() == 3 * a.granule
        assert s.Gd[g].flat.data_ptr() - s.V[g].flat.data_ptr() == 3 * a.granule
    _no_overlap(s)
    # odd group count: anchor and M even the two classes out
    s, P, M, V, Gd, _ = _placed("two_class", G=3)
    assert P == [0, 1, 0] and [s.A.cls, s.Mo.cls] == [1, 0] and V == [2, 2, 2]
    # one shared gradient buffer
    s, P, M, V, Gd, _ = _placed("two_class", G=4, shared_grad=True)
    assert len({id(x) for x in s.Gd}) == 1 and Gd == [2] * 4
    # two classes only, and a single one
    s, P, M, V, Gd, _ = _placed("two_class", G=4, classes=[0] * 40 + [1] * 40)
    assert P == [0, 1, 0, 1] and V == [1, 0, 1, 0] and Gd == V
    s, P, M, V, Gd, _ = _placed("two_class", G=2, classes=[0] * 40)
    assert P + M + V + Gd == [0] * 8
    _no_overlap(s)
    with pytest.raises(ValueError):
        _placed("nonsense")


def test_pairs_and_spread_policies_on_a_linear_three_class_arena():
    """"pairs": theta_g and m_g share a class, v_g and grad_g the next one, the thetas rotate over
    the classes, anchor and M go where the fewest thetas are."""
    s, P, M, V, Gd, _ = _placed("pairs")
    assert P == [0, 1, 2, 0, 1, 2, 0, 1] and M == P
    assert V == [1, 2, 0, 1, 2, 0, 1, 2] and Gd == V
    assert s.A.cls == 2 and s.Mo.cls in (0, 1)           # class 2 holds two thetas, the others three
    _no_overlap(s)
    s, P, M, V, Gd, _ = _placed("spread", G=3)
    assert P == [0, 1, 2] and M == [1, 2, 0] and V == [2, 0, 1] and Gd == P


# ---------------------------------------------------------------- randomised host-logic checks

def test_plan_never_overfills_a_class_and_keeps_launches_in_two_classes_when_room_allows():
    import numpy as np
    import paper_2511_17849_amd as pier
    rng = np.random.default_rng(5)
    for _ in range(400):
        ncls = int(rng.integers(1, 5))
        G = int(rng.integers(1, 17))
        shared = bool(rng.integers(0, 2))
        outer = bool(rng.integers(0, 2))
        need = 3 * G + (1 if shared else G) + (2 if outer else 0)
        room = [int(x) for x in rng.integers(0, 2 * need // ncls + 3, ncls)]
        try:
            reps, ca, cm = pier.pier_placement_plan(room, G, shared_grad=shared, outer_on_device=outer)
        except pier.PierError as e:
            assert "PIER_ERR_OOM" in str(e)
            # the plan gives up only when whole buffers cannot be placed one by one either:
            # that can only happen when the total room is short
            assert sum(room) < need, (room, G, shared, outer)
            continue
        used = [0] * ncls
        grads = set()
        for g, r in enumerate(reps):
            for k in ("theta", "m", "v"):
                assert 0 <= r[k] < ncls
                used[r[k]] += 1
            assert 0 <= r["grad"] < ncls
            if shared:
                grads.add(r["grad"])
            else:
                used[r["grad"]] += 1
        if shared:
            assert len(grads) == 1
            used[grads.pop()] += 1
        if outer:
            used[ca] += 1
            used[cm] += 1
        else:
            assert (ca, cm) == (-1, -1)
        assert all(u <= r for u, r in zip(used, room)), (room, used)
        assert sum(used) == need
        # with generous room every AdamW launch is two-and-two over two classes (or one class
        # when there is only one), and the outer step's buffers split evenly over two
        if ncls >= 2 and min(room) >= need:
            for r in reps:
                assert r["theta"] == r["m"] and r["v"] == r["grad"] and r["v"] != r["theta"]
            if outer:
                o = [r["theta"] for r in reps] + [ca, cm]
                assert abs(o.count(0) - o.count(1)) <= 1 and o.count(0) + o.count(1) == G + 2


def test_arena_random_allocation_never_overlaps_and_room_is_honest():
    import numpy as np
    rng = np.random.default_rng(6)
    for _ in range(100):
        n = int(rng.integers(8, 80))
        classes = list(np.repeat(rng.integers(0, 3, 8), rng.integers(1, 12, 8))[:n])
        if len(set(classes)) != max(classes) + 1:
            continue                                        # class ids must be dense
        a = fake_arena(classes, granule=64)
        spans = []
        for _ in range(30):
            numel = int(rng.integers(1, 80))
            cls = None if rng.random() < 0.3 else int(rng.integers(0, 4))
            room = a.room(numel)
            try:
                t, c = a.alloc(numel, torch.float32, cls)
            except MemoryError:
                assert sum(room) == 0                       # nothing fitted anywhere
                continue
            assert sum(room) > 0
            if cls is not None and room[cls % a.n_classes] > 0:
                assert c == cls % a.n_classes               # the asked class when it had a run
            lo = t.data_ptr() - a.buf.data_ptr()
            hi = lo + numel * 4
            g0, g1 = lo // 64, (hi - 1) // 64
            assert lo % 64 == 0 and all(a.classes[g] == c for g in range(g0, g1 + 1))
            assert all(hi <= s or e <= lo for s, e in spans)
            spans.append((g0 * 64, (g1 + 1) * 64))
