"""The seeded input generators: determinism, independence from chunking, moments."""
import numpy as np
import pytest

from inputs import synth


def test_deterministic_and_tag_seed_dependent():
    a = synth.uniform(3, "A", 50, 70)
    assert np.array_equal(a, synth.uniform(3, "A", 50, 70))
    assert not np.array_equal(a, synth.uniform(4, "A", 50, 70))
    assert not np.array_equal(a, synth.uniform(3, "B", 50, 70))
    # value depends on the logical index only: a sub-block of a larger draw starts the same
    big = synth.uniform(3, "A", 80, 70)
    assert np.array_equal(big[:50], a)
    # batch b of a stack is not batch 0
    st = synth.normal(3, "A", 8, 8, batch=3)
    assert not np.array_equal(st[0], st[1])


def test_chunked_generation_matches_single_chunk():
    # 3000 x 1500 exceeds one chunk (2^21 elements) and is split over threads
    x = synth.normal(5, "B", 3000, 1500)
    for r in (0, 1397, 1398, 1399, 2999):
        assert np.array_equal(x[r], synth.normal(5, "B", r + 1, 1500)[r])


@pytest.mark.parametrize("kind", ["uniform", "normal", "normal_small", "integers"])
def test_moments(kind):
    n = 1 << 20
    if kind == "uniform":
        x = synth.uniform(7, "A", 1024, 1024).astype(np.float64); mean, var = 0.0, 1.0 / 3.0
        assert x.min() >= -1.0 and x.max() < 1.0
    elif kind == "normal":
        x = synth.normal(7, "A", 1024, 1024).astype(np.float64); mean, var = 0.0, 1.0
        assert abs(np.mean(x ** 4) - 3.0) < 0.05          # kurtosis of a Gaussian
        assert abs(np.mean(np.abs(x) < 1.0) - 0.682689) < 0.003
    elif kind == "normal_small":
        K = 16384
        x = synth.normal(7, "A", 1024, 1024, 0.0, K ** -0.5).astype(np.float64); mean, var = 0.0, 1.0 / K
    else:
        x = synth.integers(7, "A", 1024, 1024, -3, 3).astype(np.float64); mean, var = 0.0, 4.0
        assert set(np.unique(x)) == {-3.0, -2.0, -1.0, 0.0, 1.0, 2.0, 3.0}
    sd = np.sqrt(var)
    assert abs(x.mean() - mean) < 5 * sd / np.sqrt(n)
    assert abs(x.var() - var) < 5 * var * np.sqrt(3.0 / n)   # generous for all four
    # neighbouring entries are uncorrelated
    c = np.mean((x[:, 1:] - mean) * (x[:, :-1] - mean)) / var
    assert abs(c) < 5 / np.sqrt(n)


def test_bf16_round_trip_and_ties():
    bits = np.arange(0, 0x7F80, dtype=np.uint16)
    f = synth.bf16_bits_to_f32(bits)
    assert np.array_equal(synth.f32_to_bf16_bits(f), bits)
    one = np.array([1.0, 1.00390625, 1.01171875, 1.0039064], dtype=np.float32)
    assert list(synth.f32_to_bf16_bits(one)) == [0x3F80, 0x3F80, 0x3F82, 0x3F81]
    assert synth.f32_to_bf16_bits(np.array([np.inf, -np.inf, 3.4e38], dtype=np.float32)).tolist() == [0x7F80, 0xFF80, 0x7F80]
    assert synth.f32_to_bf16_bits(np.array([np.nan], dtype=np.float32))[0] & 0x7FFF > 0x7F80


def test_sample_entries_cover_tiles_and_are_in_range():
    b, i, j = synth.sample_entries(3, 1000, 4, 700, 900, tile_m=256, tile_n=256)
    assert len(b) == len(i) == len(j) >= 1000
    assert b.min() >= 0 and b.max() < 4 and i.min() >= 0 and i.max() < 700 and j.min() >= 0 and j.max() < 900
    pts = set(zip(b.tolist(), i.tolist(), j.tolist()))
    for bb in (0, 3):
        for ii in (0, 255, 511, 699):
            for jj in (0, 255, 511, 767, 899):
                if ii in (0,) and jj not in (0, 899):
                    continue
                if jj in (0,) and ii not in (0, 699):
                    continue
                assert (bb, ii, jj) in pts


@pytest.mark.parametrize("name", synth.WORKLOADS)
def test_workloads_scaled_down(name):
    w = synth.make_workload(name, scale=16)
    es = np.float32 if w.dtype == synth.DTYPE_F32 else np.uint16
    assert w.A.dtype == es and w.B.dtype == es and w.bias.dtype == np.float32
    a_shape = (w.K, w.M) if w.layout & 2 else (w.M, w.K)
    b_shape = (w.N, w.K) if w.layout & 1 else (w.K, w.N)
    lead = (w.batch,) if w.batch > 1 else ()
    assert w.A.shape == lead + a_shape and w.B.shape == lead + b_shape and w.bias.shape == (w.batch, w.N)
    assert w.flops == 2 * w.batch * w.M * w.N * w.K


def test_full_size_workload_accounting():
    # flop and byte counts of the five workloads at full size (no arrays are built here)
    def bytes_(batch, M, N, K, es):
        return batch * ((M * K + K * N + M * N) * es + 4 * N)
    assert bytes_(1, 256, 256, 256, 4) == 787456
    assert bytes_(1, 16, 16384, 16384, 4) == 1075904512
    assert bytes_(1, 4096, 4096, 4096, 4) == 201342976
    assert bytes_(1, 8192, 8192, 8192, 2) == 402685952
    assert bytes_(32, 2048, 2048, 512, 2) == 402915328
    w = synth.make_workload("c1_f32_256_relu")
    assert w.algorithmic_bytes == 787456 and w.flops == 2 * 256 ** 3


def test_workload_specs_match_the_workloads_they_describe():
    assert sorted(synth.SPECS) == sorted(synth.WORKLOADS + synth.BREADTH_WORKLOADS)
    for name, (batch, M, N, K, layout, dtype, act) in synth.SPECS.items():
        s = 64 if M >= 4096 or N >= 4096 else 1
        w = synth.make_workload(name, scale=s)
        assert (w.batch, w.layout, w.dtype, w.act) == (batch, layout, dtype, act), name
        assert (w.M * (s if M > 16 else 1), w.N * s, w.K * s) == (M, N, K), name
