"""Pins for the oracle's teacher head + greedy choice: numpy's float64 matmul on the same exact values, closed
forms (one-hot hidden states pick a weight column, a planted multiple of the hidden state wins by a known
margin), the tie rule, padding, and fp32 / bf16 input handling."""
import numpy as np

import oracle
from paper_2603_08088_amd import synth


def _vals(rng, shape, dtype):
    x = rng.standard_normal(shape).astype(np.float32)
    return synth.f32_to_bf16_bits(x) if dtype == "bf16" else x


def _f64(x, dtype):
    return (synth.bf16_bits_to_f32(x) if dtype == "bf16" else x).astype(np.float64)


def test_against_numpy_float64_matmul():
    rng = np.random.default_rng(11)
    for dtype in ("f32", "bf16"):
        B, T, D, V = 3, 5, 96, 203
        h, w = _vals(rng, (B, T, D), dtype), _vals(rng, (V, D), dtype)
        n = np.asarray([5, 2, 0], dtype=np.int32)
        r = oracle.lm_head_argmax(h, w, n, dtype=dtype, want_logits=True)
        ref = _f64(h, dtype) @ _f64(w, dtype).T
        for b in range(B):
            nb = int(n[b])
            assert np.allclose(r["logits"][b, :nb], ref[b, :nb], rtol=1e-12, atol=1e-12)
            assert r["argmax"][b, :nb].tolist() == ref[b, :nb].argmax(axis=1).tolist()
            assert np.allclose(r["maxval"][b, :nb], ref[b, :nb].max(axis=1), rtol=1e-12)
            assert np.all(r["argmax"][b, nb:] == -1) and np.all(np.isneginf(r["maxval"][b, nb:]))


def test_one_hot_hidden_state_reads_a_weight_column_and_ties_take_the_lowest_index():
    D, V = 8, 15
    w = np.arange(V * D, dtype=np.float32).reshape(V, D) % 7.0      # column c: values (v*D + c) % 7
    h = np.zeros((1, D, D), dtype=np.float32)
    for c in range(D):
        h[0, c, c] = 1.0                                             # row c is the one-hot e_c
    r = oracle.lm_head_argmax(h, w, [D], dtype="f32", want_logits=True)
    for c in range(D):
        col = w[:, c].astype(np.float64)
        assert np.array_equal(r["logits"][0, c], col)
        assert r["argmax"][0, c] == int(np.flatnonzero(col == col.max())[0])   # 6 occurs more than once: lowest wins
    assert len(set(np.flatnonzero(w[:, 0] == w[:, 0].max()).tolist())) > 1


def test_planted_winner_has_the_planted_margin():
    rng = np.random.default_rng(12)
    B, T, D, V = 2, 4, 64, 300
    h = rng.standard_normal((B, T, D)).astype(np.float32)
    w = (rng.standard_normal((V, D)) / np.sqrt(D)).astype(np.float32)
    target = rng.permutation(V)[: B * T].reshape(B, T)               # distinct rows of w
    for b in range(B):
        for k in range(T):
            hv = h[b, k].astype(np.float64)
            w[target[b, k]] = (9.0 * hv / (hv @ hv)).astype(np.float32)   # logit of the target = 9 up to rounding
    r = oracle.lm_head_argmax(h, w, [T, T], dtype="f32", want_logits=True)
    assert np.array_equal(r["argmax"], target)
    assert np.allclose(r["maxval"], 9.0, atol=1e-5)
