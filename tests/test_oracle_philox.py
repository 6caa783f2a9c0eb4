"""Pins for the oracle's Philox4x32-10 and for how the noise field is keyed."""
import os

import numpy as np

from oracle import flashdp_oracle as O


def _kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(golden_dir):
    rows = _kat(golden_dir)
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = O.philox4x32_10(np.array(ctr, dtype=np.uint32), key)
        assert [int(x) for x in got] == want


def test_philox_vectorised_equals_one_by_one(golden_dir):
    rows = _kat(golden_dir)
    # same key for a batch: take the zero-key row and two more counters
    ctrs = np.array([[0, 0, 0, 0], [1, 0, 0, 0], [0, 0, 7, 0], [0xFFFFFFFF, 3, 2, 0]], dtype=np.uint32)
    batch = O.philox4x32_10(ctrs, (5, 9))
    for k in range(len(ctrs)):
        assert np.array_equal(batch[k], O.philox4x32_10(ctrs[k], (5, 9)))
    # every counter word and every key word matters
    base = O.philox4x32_10(np.zeros(4, np.uint32), (0, 0))
    for j in range(4):
        c = np.zeros(4, np.uint32)
        c[j] = 1
        assert not np.array_equal(O.philox4x32_10(c, (0, 0)), base)
    assert not np.array_equal(O.philox4x32_10(np.zeros(4, np.uint32), (1, 0)), base)
    assert not np.array_equal(O.philox4x32_10(np.zeros(4, np.uint32), (0, 1)), base)


def test_philox_is_injective_on_a_counter_range():
    g = np.arange(1 << 16, dtype=np.uint32)
    ctr = np.zeros((g.size, 4), np.uint32)
    ctr[:, 0] = g
    out = O.philox4x32_10(ctr, (123, 456))
    packed = out.astype(np.uint64)
    keys = (packed[:, 0] << np.uint64(32)) | packed[:, 1]
    keys2 = (packed[:, 2] << np.uint64(32)) | packed[:, 3]
    assert len(set(zip(keys.tolist(), keys2.tolist()))) == g.size
    # word bits are balanced (a broken multiply/shift shows here)
    ones = np.unpackbits(out.view(np.uint8)).mean()
    assert abs(ones - 0.5) < 0.002


def test_field_keying_seed_layer_element():
    # key = (seed low word, seed high word); counter = (g low, g high, layer, 0); element e -> group e//4, slot e%4
    seed = (7 << 32) | 11
    layer = 5
    z = O.noise_field(seed, layer, 23)           # ragged tail: 23 is not a multiple of 4
    for g in range(6):
        words = O.philox4x32_10(np.array([g, 0, layer, 0], np.uint32), (11, 7))
        z4 = O.gaussians_from_words(words)
        for j in range(4):
            e = 4 * g + j
            if e < 23:
                assert z[e] == z4[j]
    # group index above 2^32 goes to counter word 1
    e_big = np.array([(1 << 34) + 5], dtype=np.uint64)   # g = 2^32 + 1, slot 1
    words = O.philox4x32_10(np.array([1, 1, layer, 0], np.uint32), (11, 7))
    assert O.noise_at(seed, layer, e_big)[0] == O.gaussians_from_words(words)[1]
    # noise_at agrees with the dense field, any order
    idx = np.array([22, 0, 7, 13, 4])
    assert np.array_equal(O.noise_at(seed, layer, idx), z[idx])
    # different layer or seed -> different field; same (seed, layer) -> same field whatever the length
    assert not np.array_equal(O.noise_field(seed, layer + 1, 23), z)
    assert not np.array_equal(O.noise_field(seed + 1, layer, 23), z)
    assert np.array_equal(O.noise_field(seed, layer, 1000)[:23], z)
    # chunking of the generator does not change values
    assert np.array_equal(O.noise_field(3, 1, 5003, chunk_groups=17), O.noise_field(3, 1, 5003))
