"""The seeded input generator: determinism, chunk independence, stated distributions."""
import numpy as np

import synth


def test_rows_do_not_depend_on_chunking_or_threads():
    w = synth.WORKLOADS["1p5b"].scaled(V=4099)
    tk = synth.token_arrays(w.scaled(S=2, L=16, len_lo=4, len_hi=16, G=2))
    ch = tk["chosen"]
    a = synth.logit_rows(w, 0, 32, ch)
    b = np.concatenate([synth.logit_rows(w, 0, 5, ch), synth.logit_rows(w, 5, 27, ch)])
    assert np.array_equal(a, b)
    assert np.array_equal(a, synth.logit_rows(w, 0, 32, ch))


def test_value_distribution_and_boost():
    w = synth.WORKLOADS["1p5b"]
    tk = synth.token_arrays(w)
    z = synth.bf16_bits_to_f64(synth.logit_rows(w, 0, 64, tk["chosen"]))
    assert abs(z.std() - 3.0) < 0.02 and abs(z.mean()) < 0.02
    at_y = z[np.arange(64), tk["chosen"][:64]]
    boosted = (at_y > 4.0).mean()           # N(8, 9) vs N(0, 9) mixture with weight 0.7
    assert 0.45 < boosted < 0.9


def test_padding_sentinel_and_stride():
    w = synth.WORKLOADS["tiny"].scaled(V=1001)
    z = synth.logit_rows(w, 0, 3, None, ld=1008)
    assert z.shape == (3, 1008) and (z[:, 1001:] > 1e29).all() and (np.abs(z[:, :1001]) < 20).all()
    assert np.array_equal(z[:, :1001], synth.logit_rows(w, 0, 3, None))


def test_token_arrays_follow_the_recipe():
    for name, w in synth.WORKLOADS.items():
        tk = synth.token_arrays(w)
        assert tk["chosen"].min() >= 0 and tk["chosen"].max() < w.V
        d = tk["current_version"] - tk["versions"]
        assert d.min() >= 0 and d.max() <= w.stale_max
        # staleness is per sequence
        assert (d.reshape(w.S, w.L) == d.reshape(w.S, w.L)[:, :1]).all()
        m = tk["mask"].reshape(w.S, w.L)
        assert (m.sum(axis=1) == tk["lengths"]).all()
        assert ((np.diff(m.astype(np.int8), axis=1) <= 0).all())   # ones then zeros
        g = tk["rewards"].reshape(-1, w.G)
        assert (g.max(axis=1) != g.min(axis=1)).any()
        assert abs(tk["noise"].std() - w.noise_std) < 0.05 * w.noise_std + 1e-3
    assert abs(synth.token_arrays(synth.WORKLOADS["long"])["mask"].mean() - 0.6) < 0.15


def test_behaviour_logprobs_are_clamped():
    lt = np.array([-0.01, -5.0])
    lb = synth.behav_from_target(lt, np.array([0.5, 0.25], dtype=np.float32))
    assert lb[0] == 0.0 and abs(lb[1] + 4.75) < 1e-6 and lb.dtype == np.float32
