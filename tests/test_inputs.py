"""Host-side checks of the seeded workload generator (recipe, determinism, bf16 rounding)."""
import numpy as np

from paper_2601_02609_amd import inputs as I


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0, 0.0], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to the even mantissa (1.0);
    # 1 + 3*2^-8 is a tie between 1 + 2^-7 and 1 + 2^-6: goes to 1 + 2^-6.
    got = I.bf16_bits_to_f32(I.f32_to_bf16_bits(x))
    assert list(got) == [1.0, 1.0, 1.015625, -3.0, 0.0]


def test_tiny_config_recipe():
    w = I.make_config("tiny")
    s = w.spec
    assert (s.N, s.D, s.V) == (256, 64, 1000)
    assert w.hidden.shape == (256, 64) and w.hidden.dtype == np.uint16
    assert w.weight.shape == (1000, 64) and w.labels.dtype == np.int32
    assert int((w.labels == -100).sum()) == 26 and w.n_valid == 230
    lab = w.labels[w.labels != -100]
    assert lab.min() >= 0 and lab.max() < 1000
    Wf = I.bf16_bits_to_f32(w.weight)
    assert abs(Wf.std() - 2.5 / 8.0) < 0.01
    assert np.all(w.dloss_mean == np.float32(1.0 / 230))
    assert np.all(np.isnan(w.dloss_var[w.labels == -100]))
    assert np.all(np.isfinite(w.dloss_var[w.labels != -100]))
    w2 = I.make_config("tiny")
    assert np.array_equal(w.hidden, w2.hidden) and np.array_equal(w.labels, w2.labels)


def test_rms_rows_and_zipf_labels():
    spec = I.custom_spec(512, 128, 5000, seed=1, ignore_frac=0.25)
    w = I.make_workload(spec)
    Hf = I.bf16_bits_to_f32(w.hidden).astype(np.float64)
    rms = np.sqrt((Hf ** 2).mean(axis=1))
    assert np.all(np.abs(rms - 1.0) < 0.01)
    lab = w.labels[w.labels != -100]
    assert int((w.labels == -100).sum()) == 128
    # Zipf: id 0 is the most frequent and low ids dominate
    counts = np.bincount(lab, minlength=5000)
    assert counts[0] == counts.max()
    assert (lab < 50).mean() > 0.4
