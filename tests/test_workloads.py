"""Host-side checks of the seeded input generator (no GPU)."""
import numpy as np

from paper_2208_08124_amd import workloads as wl


def test_config1_is_the_stated_pack():
    b = wl.make_workload(1)
    assert b["lengths"].tolist() == [3, 17, 64, 128]
    assert b["cu_seqlens"].tolist() == [0, 3, 20, 84, 212]
    assert b["q"].shape == (212, 2, 64) and b["q"].dtype == np.uint16
    assert b["scale"] == 0.125 and "do" not in b


def test_configs_2_and_3_share_inputs_and_are_reproducible():
    a, b = wl.make_workload(2), wl.make_workload(3)
    assert a["lengths"].tolist() == b["lengths"].tolist()
    for n in ("q", "k", "v"):
        assert np.array_equal(a[n], b[n])
    assert "do" in b and "do" not in a
    c = wl.make_workload(3)
    assert np.array_equal(b["do"], c["do"])
    L = a["lengths"]
    assert len(L) == 56 and L.min() >= 1 and L.max() <= 512
    assert (L == 512).sum() >= 8          # about 30% sit at the maximum length


def test_length_mixtures():
    rng = np.random.default_rng(0)
    L4 = wl.draw_lengths(4, rng)
    assert len(L4) == 256 and set(np.unique(L4[L4 > 256])) == {512}
    L5 = wl.draw_lengths(5, rng)
    assert len(L5) == 2048 and L5.min() >= 1 and L5.max() == 512


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], dtype=np.float32)
    b = wl.f32_to_bf16_bits(x)
    y = wl.bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie -> rounds to even (1.0); 1 + 3*2^-8 is a tie -> rounds to 1 + 2^-6
    assert y.tolist() == [1.0, 1.0, 1.015625, -2.5, 0.0]
    assert np.array_equal(wl.f32_to_bf16_bits(y), b)
    assert wl.bits_to_f64(b, "bf16").dtype == np.float64


def test_padding_layout():
    b = wl.make_batch([3, 1, 5], 2, "f16", 7)
    p = wl.pad_batch(b, 8)
    assert p["cu_seqlens"].tolist() == [0, 8, 16, 24] and p["seqused"].tolist() == [3, 1, 5]
    rows = wl.valid_row_index(b["lengths"], 8)
    assert rows.tolist() == [0, 1, 2, 8, 16, 17, 18, 19, 20]
    assert np.array_equal(p["k"][rows], b["k"])
    mask = np.ones(24, bool)
    mask[rows] = False
    assert not p["v"][mask].any()


def test_useful_flops():
    assert wl.useful_flops([3, 17, 64, 128], 2, False) == 4 * 20778 * 2 * 64
    assert wl.useful_flops([2], 1, True) == 14 * 4 * 64


def test_zipf_token_ids_are_seeded_in_range_and_skewed():
    a = wl.zipf_token_ids(20000, 30522, 7)
    b = wl.zipf_token_ids(20000, 30522, 7)
    assert np.array_equal(a, b) and a.dtype == np.int32 and a.min() >= 0 and a.max() < 30522
    counts = np.sort(np.bincount(a, minlength=30522))[::-1]
    # Zipf(1) over 30 522 ids: the most frequent id has about 1/H(V) = 9 % of the tokens,
    # and a long tail of ids appears once or not at all
    assert 0.06 < counts[0] / 20000 < 0.13 and counts[0] > 1.5 * counts[1] > 0
    assert (counts <= 1).sum() > 20000
