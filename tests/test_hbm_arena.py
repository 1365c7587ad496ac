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


def _placed(G=8, classes=None, **kw):
    import paper_2511_17849_amd as pier
    g = 4096                                             # granule bytes; one buffer = 3 granules
    a = fake_arena(classes or [0] * 48 + [1] * 48 + [2] * 44, granule=g)
    n = 3 * g // 4 - 8
    s = pier.ModelBuffers(n, G, arena=a, device="cpu", **kw)
    c = s.classes
    return s, c["theta"], c["m"], c["v"], c["grad"], a


def _no_overlap(s):
    bufs = {id(x): x for x in s.theta + s.m + s.v + s.grad + [s.anchor, s.momentum] if x is not None}.values()
    spans = sorted((x.data_ptr(), x.data_ptr() + x.numel() * x.element_size()) for x in bufs)
    assert all(e0 <= b1 for (_, e0), (b1, _) in zip(spans, spans[1:]))


def test_model_buffers_keep_every_launch_in_two_classes():
    """theta_g, m_g in class g mod 2; the outer step's ten buffers five and five in classes 0 and
    1; v_g, grad_g in class 2 until it is full (14 buffers of 3 granules in 44), then in the class
    theta_g is not in."""
    s, P, M, V, Gd, a = _placed()
    assert P == [0, 1, 0, 1, 0, 1, 0, 1] and M == P
    assert sorted([s.classes["anchor"], s.classes["momentum"]]) == [0, 1]
    assert V == [2] * 7 + [0] and Gd == V
    for g in range(8):          # back to back: m_g follows theta_g, grad_g follows v_g
        assert s.m[g].data_ptr() - s.theta[g].data_ptr() == 3 * a.granule
        assert s.grad[g].data_ptr() - s.v[g].data_ptr() == 3 * a.granule
    _no_overlap(s)
    # odd group count: anchor and M even the two classes out
    s, P, M, V, Gd, _ = _placed(G=3)
    assert P == [0, 1, 0] and [s.classes["anchor"], s.classes["momentum"]] == [1, 0] and V == [2, 2, 2]
    # one shared gradient buffer
    s, P, M, V, Gd, _ = _placed(G=4, shared_grad=True)
    assert len({x.data_ptr() for x in s.grad}) == 1 and Gd == [2] * 4
    # outer state elsewhere (pinned host memory)
    s, P, M, V, Gd, _ = _placed(G=2, outer_on_device=False)
    assert s.anchor is None and s.momentum is None and P == [0, 1] and V == [2, 2]
    # bfloat16 gradients take half the granules
    import torch
    s, P, M, V, Gd, a = _placed(G=2, grad_dtype=torch.bfloat16)
    assert s.grad[0].dtype == torch.bfloat16 and s.grad[0].numel() == s.v[0].numel()
    # two classes only, and a single one
    s, P, M, V, Gd, _ = _placed(G=4, classes=[0] * 40 + [1] * 40)
    assert P == [0, 1, 0, 1] and V == [1, 0, 1, 0] and Gd == V
    s, P, M, V, Gd, _ = _placed(G=2, classes=[0] * 40)
    assert P + M + V + Gd == [0] * 8
    _no_overlap(s)
    # without an arena: plain allocations, no classes
    s = __import__("paper_2511_17849_amd").ModelBuffers(100, 2, device="cpu")
    assert s.classes["theta"] == [None, None] and s.anchor.numel() == 100 and len(s.grad) == 2


# ---------------------------------------------------------------- classification of probe rates
#
# pier_hbm_classify is the probe's decision logic on its own: these tables are synthetic, built
# from the behaviour the probe meets on MI355X - granules of different address classes stream
# together within a few per cent of the best rate, granules of one class clearly slower, at a
# rate that swings with their distance, neighbouring distances swinging in opposite directions.

def rate_table(classes, *, top=6.5, noise=0.0, seed=0, spikes=(), scale=1.0):
    import numpy as np
    rng = np.random.default_rng(seed)
    n = len(classes)
    R = np.zeros((n, n))
    for a in range(n):
        for b in range(a, n):
            d = b - a
            if classes[a] != classes[b]:
                r = top + 0.1 * np.cos(0.37 * d)                        # 6.4 .. 6.6
            else:
                swing = 0.25 + 0.15 * np.cos(0.05 * d)                  # 0.1 .. 0.4
                r = 5.85 + (swing if d % 2 == 0 else -swing)            # 5.45 .. 6.25
                if d in spikes and d > 0:
                    r = 6.42                                            # a same-class distance that streams fast
            r *= scale * (1.0 + noise * rng.uniform(-1, 1))
            R[a, b] = R[b, a] = r
    return R


def same_partition(got, want):
    pairs = set(zip(got, want))
    return len(pairs) == len(set(got)) == len(set(want))


def runs(spec):
    out = []
    for c, k in spec:
        out += [c] * k
    return out


@pytest.mark.parametrize("spec", [
    [(0, 30)],                                     # an arena inside one class
    [(0, 140)],
    [(0, 48), (1, 48), (2, 44)],                   # a fresh process: three classes of 96 GiB in 2 GiB granules
    [(0, 48), (1, 48)],
    [(0, 10), (1, 48), (2, 48)],                   # the arena starts near the end of a class
    [(0, 16), (1, 16), (2, 16), (0, 16), (1, 16), (2, 16), (0, 16), (1, 12)],   # a used process: 32 GiB runs
    [(0, 2), (1, 60)],                             # only the two reference granules in the first class
])
def test_classify_recovers_the_classes(spec):
    import paper_2511_17849_amd as pier
    want = runs(spec)
    for kw in (dict(), dict(noise=0.004, seed=1), dict(noise=0.004, seed=2), dict(scale=0.5), dict(scale=3.0),
               dict(spikes=(7, 22), noise=0.002, seed=3)):
        got = pier.pier_hbm_classify(rate_table(want, **kw))
        assert sorted(set(got)) == list(range(max(got) + 1))          # dense class ids
        assert same_partition(got, want), (kw, "".join(map(str, got)))
        assert got[0] == 0


def test_classify_is_relative_not_absolute():
    """The same table in other units (GB/s, or a part with slower memory) classifies the same; a
    table with a single level - everything equally fast, or everything equally slow - is one class."""
    import numpy as np
    import paper_2511_17849_amd as pier
    want = runs([(0, 48), (1, 48), (2, 44)])
    base = pier.pier_hbm_classify(rate_table(want))
    for scale in (1e3, 0.3, 7.0):
        assert pier.pier_hbm_classify(rate_table(want, scale=scale)) == base
    flat = np.full((40, 40), 6.5)
    # everything within the band of everything else: all pairings look "cross-class", which only a
    # model of 40 one-granule classes could explain; the class cap folds them - what matters here
    # is that the call returns dense ids and does not fail
    got = pier.pier_hbm_classify(flat)
    assert sorted(set(got)) == list(range(max(got) + 1)) and max(got) < 8
    slow = rate_table([0] * 40, scale=0.8)
    assert pier.pier_hbm_classify(slow) == [0] * 40


def test_classify_argument_errors():
    import numpy as np
    import paper_2511_17849_amd as pier
    bad = rate_table(runs([(0, 6), (1, 6)]))
    bad[0, 5] = bad[5, 0] = 0.0
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_hbm_classify(bad)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_hbm_classify(np.ones((1, 1)))
    assert pier.pier_hbm_classify(np.ones((2, 2))) == [0, 0]


def test_classify_replays_a_recorded_probe_of_an_mi355x():
    """The rates a real probe run measured (tests/golden/probe_rates_mi355x.txt: the 465 pairs it asked
    for, of 140 x 140) classify into the three contiguous classes of 96, 96 and 88 GiB that run reported;
    pairs the probe never measured are absent from the table (zero), so this also pins which pairs the
    classifier needs.  The same table in GB/s gives the same answer."""
    import os
    import numpy as np
    import paper_2511_17849_amd as pier
    path = os.path.join(os.path.dirname(__file__), "golden", "probe_rates_mi355x.txt")
    n, want, pairs = None, None, []
    for line in open(path):
        if line.startswith("# classes "):
            want = [int(c) for c in line.split()[2]]
        elif line.startswith("granules "):
            n = int(line.split()[1])
        elif line[0].isdigit():
            a, b, r = line.split()
            pairs.append((int(a), int(b), float(r)))
    assert n == 140 and len(want) == n and len(pairs) == 465
    R = np.zeros((n, n))
    for a, b, r in pairs:
        R[a, b] = R[b, a] = r
    same = [r for a, b, r in pairs if want[a] == want[b]]
    cross = [r for a, b, r in pairs if want[a] != want[b]]
    assert max(same) < min(cross)                         # the two levels of this machine do not overlap
    assert pier.pier_hbm_classify(R) == want
    summary = pier.pier_hbm_probe_summary()
    assert summary["n_classes"] == 3 and summary["n_pairs"] == 465 and summary["best_rate"] == max(cross)
    assert max(same) < summary["threshold"] < min(cross)
    assert pier.pier_hbm_classify(R * 1000.0) == want
    assert [want.count(c) for c in (0, 1, 2)] == [48, 48, 44]


def test_classify_and_plan_hold_their_contracts_on_random_input():
    """Whatever the table, classification returns dense class ids starting at 0 (at most 8 classes);
    whatever the room, a plan either fits - no class holds more buffers than it had room for, every
    buffer of the model is placed once - or is refused as PIER_ERR_OOM."""
    import numpy as np
    import paper_2511_17849_amd as pier
    rng = np.random.default_rng(2024)
    for _ in range(200):
        n = int(rng.integers(2, 60))
        R = rng.uniform(0.5, 7.0, (n, n))
        R = (R + R.T) / 2
        got = pier.pier_hbm_classify(R)
        assert got[0] == 0 and sorted(set(got)) == list(range(max(got) + 1)) and max(got) < 8
    for _ in range(300):
        ncls = int(rng.integers(1, 5))
        room = [int(x) for x in rng.integers(0, 14, ncls)]
        G = int(rng.integers(1, 9))
        shared, outer = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        need = 3 * G + (1 if shared else G) + (2 if outer else 0)
        try:
            reps, ca, cm = pier.pier_placement_plan(room, G, shared_grad=shared, outer_on_device=outer)
        except pier.PierError as e:
            assert "PIER_ERR_OOM" in str(e)
            # a refusal may also come from a split that first-fit could not make, never from ample room
            assert sum(room) < need + 2 * ncls, (room, G, shared, outer)
            continue
        used = [0] * ncls
        for r in reps:
            for k in ("theta", "m", "v"):
                used[r[k]] += 1
        grads = {reps[0]["grad"]} if shared else None
        if shared:
            assert all(r["grad"] == reps[0]["grad"] for r in reps)
            used[reps[0]["grad"]] += 1
        else:
            for r in reps:
                used[r["grad"]] += 1
        if outer:
            used[ca] += 1
            used[cm] += 1
        else:
            assert (ca, cm) == (-1, -1)
        assert sum(used) == need and all(u <= r for u, r in zip(used, room)), (room, used)
