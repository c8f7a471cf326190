"""The synthetic input recipe: shapes, determinism, storage rounding, planted coverage."""
import numpy as np
import pytest

from workloads import baseline_case, baseline_spec, bf16_bits_to_f32, f32_to_bf16_bits, make_case

SMALL = {"d": 64, "V_t": 6000, "V_d": 2000, "n_direct": 1500, "n_ngram": 800}


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7, -3.3, 0.0], np.float32)
    b = f32_to_bf16_bits(x)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: even mantissa (1.0) wins; 1 + 3*2^-8 ties up to 1 + 2^-6
    assert bf16_bits_to_f32(b)[:4].tolist() == [1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]
    r = bf16_bits_to_f32(b)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(f32_to_bf16_bits(r), b)


def test_config1_shapes():
    c = baseline_case(1)
    assert (c.B, c.M, c.K, c.d, c.V_t, c.V_d, c.dtype) == (1, 5, 4, 256, 1024, 512, "f32")
    assert c.hidden.shape == (5, 256) and c.W.shape == (256, 1024) and c.draft_logits.shape == (4, 512)
    assert (c.direct_map >= 0).sum() == 400
    img = c.direct_map[c.direct_map >= 0]
    assert len(set(img.tolist())) == 400
    assert c.ngram_target_ids.size == 64 and not set(c.ngram_target_ids.tolist()) & set(img.tolist())
    lens = np.diff(c.ngram_key_off)
    assert lens.min() >= 2 and lens.max() <= 3
    assert abs(float(c.W.std()) - 0.02) < 0.001 and abs(float(c.draft_logits.std()) - 2.0) < 0.1


def test_determinism():
    a, b = baseline_case(1), baseline_case(1)
    for f in ("hidden", "W", "draft_logits", "draft_ids", "direct_map", "ngram_key_ids", "ngram_target_ids"):
        assert np.array_equal(getattr(a, f), getattr(b, f))


@pytest.mark.parametrize("i", [3, 4, 5])
def test_scaled_configs_structure(i):
    spec = baseline_spec(i, scale=SMALL)
    c = make_case(spec)
    assert c.dtype == "bf16" and c.hidden.dtype == np.uint16 and c.W.dtype == np.uint16
    assert c.row_off[-1] == c.M == int((c.k + 1).sum())
    assert c.draft_logits.shape == (c.K, c.V_d) and c.draft_ids.shape == (c.K,)
    assert c.draft_ids.min() >= 0 and c.draft_ids.max() < c.V_d
    lens = np.diff(c.ngram_key_off)
    assert lens.min() >= 2 and lens.max() <= spec.ngram_len[1] and c.max_ngram_len == spec.ngram_len[1]
    keys = {tuple(c.ngram_key_ids[c.ngram_key_off[e]:c.ngram_key_off[e + 1]]) for e in range(lens.size)}
    assert len(keys) == lens.size                      # keys are unique
    if i == 5:
        assert c.B == 64 and c.k.min() >= 1 and c.k.max() <= 10 and set(c.temperature.tolist()) == {0.0, 1.0}
    if i == 4:
        assert c.B == 16 and np.all(c.k == 8) and np.allclose(c.temperature, 0.7)


def test_planted_coverage_is_about_thirty_percent():
    spec = baseline_spec(4, scale=dict(SMALL, k=[8] * 400, temperature=[0.7] * 400))
    c = make_case(spec)
    covered = sum(L for pl in c.planted for _, L in pl)
    assert 0.24 < covered / c.K < 0.36


def test_identity_map_with_permuted_fraction():
    spec = baseline_spec(2, scale={"d": 32, "V_t": 5000, "V_d": 5000})
    c = make_case(spec)
    moved = (c.direct_map != np.arange(5000)).sum()
    assert 80 <= moved <= 100 and sorted(c.direct_map.tolist()) == list(range(5000))
