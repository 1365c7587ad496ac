"""The seeded input generator: known-answer vectors of the published Philox4x32-10
test set, moments of the normal draw, random addressability, workload sizes."""
import numpy as np

from pier_inputs import generator as gen
from pier_inputs import shapes


def _kat(ctr, key):
    out = gen.philox4x32_10(*[np.uint32(c) for c in ctr], key[0], key[1])
    return [int(x) for x in out]


def test_philox_known_answers():
    # Random123 known-answer tests for philox4x32, 10 rounds
    assert _kat((0, 0, 0, 0), (0, 0)) == [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]
    assert _kat((0xFFFFFFFF,) * 4, (0xFFFFFFFF, 0xFFFFFFFF)) == [0x408F276D, 0x41C83B0E, 0xA20BC7C6, 0x6D5451FD]
    assert _kat((0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344), (0xA4093822, 0x299F31D0)) == \
        [0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1]


def test_normal_moments_and_streams():
    z = gen.normal(1 << 20, seed=0, stream=1, step=3, std=1e-3).astype(np.float64)
    assert abs(z.mean()) < 4e-6 and abs(z.std() - 1e-3) < 4e-6
    assert abs(((z / z.std()) ** 4).mean() - 3.0) < 0.03
    assert abs(np.mean(z[:-1] * z[1:])) < 1e-8                      # neighbours uncorrelated
    other = gen.normal(1 << 12, seed=0, stream=2, step=3, std=1e-3)
    later = gen.normal(1 << 12, seed=0, stream=1, step=4, std=1e-3)
    reseed = gen.normal(1 << 12, seed=1, stream=1, step=3, std=1e-3)
    for y in (other, later, reseed):
        assert abs(np.corrcoef(z[:1 << 12], y)[0, 1]) < 0.06
    assert np.all(np.isfinite(z))


def test_normal_is_randomly_addressable():
    full = gen.normal(10_001, seed=7, stream=3, step=9, std=0.02)
    idx = np.array([0, 1, 2, 3, 4, 5, 4095, 4096, 9999, 10_000])
    assert np.array_equal(gen.normal_at(idx, seed=7, stream=3, step=9, std=0.02), full[idx])
    assert np.array_equal(gen.normal(100, seed=7, stream=3, step=9, std=0.02, offset=5000), full[5000:5100])
    big = gen.normal_at(np.array([(1 << 34) + 5]), seed=7, stream=3, step=9, std=1.0)   # block index > 2^32
    assert np.isfinite(big[0])


def test_workload_sizes():
    w = shapes.workloads()
    assert [w[k].N for k in ("tiny", "gpt2_small", "gpt2_medium", "gpt2_xl", "gpt_7b")] == \
        [3_939_328, 124_439_808, 354_823_168, 1_557_611_200, 6_654_210_048]
    assert [len(w[k].tensors) for k in ("tiny", "gpt2_small", "gpt2_medium", "gpt2_xl", "gpt_7b")] == \
        [28, 148, 292, 580, 388]
    assert all(n % 4 == 0 for k in w for n in w[k].numels)


def test_input_package_does_not_import_the_product_or_the_oracle():
    """pier_inputs serves both sides, so it may lean on neither."""
    import os
    root = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "pier_inputs")
    for dirpath, _, files in os.walk(root):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "paper_2511_17849_amd" not in text and "oracle" not in text.lower(), f
