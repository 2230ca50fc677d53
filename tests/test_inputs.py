"""The seeded byte generator: numpy and torch forms agree with each other and
with SplitMix64 evaluated in plain Python integers.  CPU only."""

import numpy as np
import torch

from paper_1603_06809_amd import inputs as I


def test_splitmix64_known_values():
    # SplitMix64 seeded with 0 produces these first outputs (the published
    # reference sequence): state advances by the golden-ratio increment, then
    # the two multiply-xorshift rounds are applied.
    assert I.splitmix64_word(0, 0) == 0xE220A8397B1DCDAF
    assert I.splitmix64_word(0, 1) == 0x6E789E6AA1B965F4
    assert I.splitmix64_word(0, 2) == 0x06C45D188009454F


def test_numpy_torch_python_agree():
    for seed, stream, nbytes in [(1, 0, 0), (1, 0, 1), (160306809, 0, 1000), (160306813, 514, 4097), (7, 3, 64)]:
        a = I.bytes_numpy(seed, stream, nbytes)
        b = I.bytes_torch(seed, stream, nbytes).numpy()
        assert a.dtype == np.uint8 and a.shape == (nbytes,)
        assert np.array_equal(a, b)
        key = I.stream_key(seed, stream)
        ref = b"".join(I.splitmix64_word(key, k).to_bytes(8, "little") for k in range((nbytes + 7) // 8))
        assert a.tobytes() == ref[:nbytes]
        for start in (0, 1, 8, 13, nbytes // 2):
            if start <= nbytes:
                assert np.array_equal(I.bytes_numpy(seed, stream, nbytes - start, start), a[start:])


def test_streams_differ_and_are_uniform():
    w = I.workload("P10_n512K")
    msg = I.message_numpy(w)
    assert msg.shape == (w.n,)
    hist = np.bincount(msg, minlength=256)
    assert hist.min() > 0.8 * w.n / 256 and hist.max() < 1.2 * w.n / 256
    p3 = I.poison_numpy(w, 3, 4096)
    p4 = I.poison_numpy(w, 4, 4096)
    assert (p3 != p4).mean() > 0.98 and (p3 != msg[:4096]).mean() > 0.98
    assert np.array_equal(I.poison_torch(w, 3, 4096).numpy(), p3)


def test_workloads_are_the_five_configs():
    got = [(w.P, w.root, w.n) for w in I.WORKLOADS]
    assert got == [(10, 0, 524_288), (24, 3, 4_194_304), (64, 0, 16_777_216),
                   (96, 17, 12_345_677), (513, 256, 134_217_728)]
