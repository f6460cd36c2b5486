"""The error-analysis harness (Section 3.2, Table 2) on synthetic heads: the orderings the paper
reports must come out, and the harness must agree with a direct evaluation of its definitions.
The paper's numbers themselves need Llama-2-13B activations: parity unpinned."""
import numpy as np

from oracle import error_analysis as ea
from oracle import kivi_oracle as ko


def test_fake_quantize_directions_and_identity():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((64, 128)).astype(np.float16)
    # a per-token group never looks at other tokens, a per-channel group never at other channels
    y = x.copy(); y[5] *= 7
    a, b = ea.fake_quantize(x, 2, 32, "token"), ea.fake_quantize(y, 2, 32, "token")
    assert np.array_equal(np.delete(a, 5, 0), np.delete(b, 5, 0))
    y = x.copy(); y[:, 9] *= 7
    a, b = ea.fake_quantize(x, 2, 32, "channel"), ea.fake_quantize(y, 2, 32, "channel")
    assert np.array_equal(np.delete(a, 9, 1), np.delete(b, 9, 1))
    # 16 bits reproduce the input up to the fp16 rounding of the scale
    assert ea.relative_error(x, ea.fake_quantize(x, 16, 32, "token")) < 1e-3
    # definitions, written out once more by hand on a tiny case
    t = np.array([[1.0, 2.0], [3.0, 4.0]])
    assert abs(ea.relative_error(t, t + 0.5) - np.sqrt(4 * 0.25) / np.sqrt(30.0)) < 1e-15
    assert ea.attention_sparsity(np.array([[0.97, 0.02, 0.005, 0.005]])) == 0.5


def test_table2_orderings_on_synthetic_heads():
    stats = []
    for seed in range(4):
        q, k, v = ea.synthetic_head(seed)
        stats.append(ea.analyze_head(q, k, v, bits=2, group=32, scale=1 / np.sqrt(128)))
    mean = lambda path: float(np.mean([s[path[0]][path[1]] for s in stats]))
    assert np.mean([s["sparsity"] for s in stats]) > 0.8                 # the regime the paper measures
    # keys: per-channel beats per-token on both statistics (fixed outlier channels)
    assert mean(("k_channel", "reconstruction")) < 0.8 * mean(("k_token", "reconstruction"))
    assert mean(("k_channel", "attention_score")) < 0.4 * mean(("k_token", "attention_score"))
    # values: similar reconstruction error either way, but the attention output is far better
    # per-token (sparse attention picks single rows; a per-channel group spreads the range of
    # its heaviest token over all 32)
    assert mean(("v_token", "attention_output")) < 0.3 * mean(("v_channel", "attention_output"))
    ratio = mean(("v_token", "reconstruction")) / mean(("v_channel", "reconstruction"))
    assert 0.3 < ratio < 3.0


def test_analysis_matches_the_decode_path_definition():
    """The per-channel-K / per-token-V column is what the decode path computes with everything
    quantised and no residual: the harness' reconstruction fed through plain attention must equal
    the oracle's mixed-precision decode attention."""
    q, k, v = ea.synthetic_head(9, tokens=256, n_queries=1)
    sc = 1 / np.sqrt(128)
    kq = ea.fake_quantize(k, 2, 32, "channel")
    vq = ea.fake_quantize(v, 2, 32, "token")
    plain = ko.softmax(sc * (q.astype(np.float64) @ kq.T)) @ vq
    empty = np.zeros((1, 1, 0, 128), np.float16)
    o = ko.decode_attention(q[None], ko.quantize_key(k[None, None], 2, 32), empty,
                            ko.quantize_value(v[None, None], 2, 32), empty, 32, sc)
    assert np.allclose(o[0], plain, rtol=1e-12, atol=1e-12)
