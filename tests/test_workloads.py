"""Seeded input generators: determinism, piecewise regeneration, distribution shape."""
import numpy as np

import workloads as wl


def test_splitmix64_known_values():
    # First outputs of the published splitmix64 generator seeded with 0 are the
    # output function applied to the state after one, two and three additions of
    # the golden-gamma constant.
    g = 0x9E3779B97F4A7C15
    x = np.array([0, g, (2 * g) & (2**64 - 1)], dtype=np.uint64)
    got = wl.splitmix64(x)
    assert [int(v) for v in got] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_payload_is_piecewise_consistent():
    whole = wl.payload_bytes(5, 3, 1000)
    for a, n in ((0, 1000), (1, 7), (8, 8), (13, 900), (999, 1), (500, 0)):
        assert np.array_equal(wl.payload_bytes(5, 3, n, first_byte=a), whole[a:a + n])
    assert not np.array_equal(wl.payload_bytes(5, 2, 64), whole[:64])
    assert not np.array_equal(wl.payload_bytes(6, 3, 64), whole[:64])


def test_normal_bf16_shape():
    bits = wl.normal_bf16_bits(1, 0, 1 << 16)
    f = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.isfinite(f).all()
    assert abs(float(f.mean())) < 0.02 and abs(float(f.std()) - 1.0) < 0.02
    assert np.array_equal(wl.normal_bf16_bits(1, 0, 100, first=50), bits[50:150])


def test_zipf_topk_distinct_and_skewed():
    ids = wl.zipf_topk_expert_ids(wl.config_seed(3), 0, 2048, 8, 256)
    assert ids.shape == (2048, 8) and ids.dtype == np.int32
    assert ids.min() >= 0 and ids.max() < 256
    s = np.sort(ids, axis=1)
    assert (np.diff(s, axis=1) > 0).all(), "experts of one token must be distinct"
    cnt = np.bincount(ids.reshape(-1), minlength=256)
    assert cnt[0] > cnt[8] > cnt[64], "low ids must be the hot experts"
    per_rank = cnt.reshape(8, 32).sum(axis=1)
    assert per_rank.argmax() == 0
    assert np.array_equal(ids, wl.zipf_topk_expert_ids(wl.config_seed(3), 0, 2048, 8, 256))


def test_random_layout_is_consistent():
    for seed in range(5):
        lay = wl.random_layout(seed, 5, 200, align=16)
        assert np.array_equal(lay["recvcounts"], lay["sendcounts"].T)
        for cnt, dsp, size in ((lay["sendcounts"], lay["sdispls"], lay["send_sizes"]),
                               (lay["recvcounts"], lay["rdispls"], lay["recv_sizes"])):
            assert (cnt % 16 == 0).all() and (dsp % 16 == 0).all()
            for a in range(5):
                used = np.zeros(int(size[a]), dtype=bool)
                for b in range(5):
                    d, n = int(dsp[a, b]), int(cnt[a, b])
                    assert d + n <= size[a] and not used[d:d + n].any()
                    used[d:d + n] = True
