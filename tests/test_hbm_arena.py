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


def test_placement_policy_on_a_linear_three_class_arena():
    """The policy PlacedState applies: theta_g and m_g share a class, v_g and grad_g the next one,
    the thetas rotate over the classes, anchor and M go where the fewest thetas are."""
    from pier_inputs import device as dev
    g = 4096                                             # granule bytes; one buffer = 3 granules
    a = fake_arena([0] * 48 + [1] * 48 + [2] * 44, granule=g)
    calls = []
    real_alloc = a.alloc

    def spy(numel, dtype=torch.float32, cls=None):
        t, c = real_alloc(numel, dtype, cls)
        calls.append(c)
        return t, c
    a.alloc = spy
    n = 3 * g // 4 - 8

    class S(dev.PlacedState):
        pass
    # PlacedState zeroes its buffers with torch ops, which is fine on the CPU tensors of the fake arena
    s = S([n], 8, arena=a)
    P, M, V, Gd = [x.cls for x in s.P], [x.cls for x in s.M1], [x.cls for x in s.V], [x.cls for x in s.Gd]
    assert P == [0, 1, 2, 0, 1, 2, 0, 1] and M == P
    assert V == [1, 2, 0, 1, 2, 0, 1, 2] and Gd == V
    assert s.A.cls == 2 and s.Mo.cls in (0, 1)           # class 2 holds two thetas, the others three
