"""Pins for the speculative-sampling oracle: its defining property (the emitted token is distributed as q,
whatever p is) by exact integration over the uniform inputs on a tiny vocabulary, special cases, and
the inverse-CDF draw against its definition."""
import numpy as np

import oracle


def test_inverse_cdf_definition():
    w = [0.0, 2.0, 0.0, 1.0, 1.0]                    # cumulative 0 2 2 3 4
    assert oracle.inverse_cdf(w, 0.0)[0] == 1
    assert oracle.inverse_cdf(w, 0.49)[0] == 1
    assert oracle.inverse_cdf(w, 0.5)[0] == 3         # target 2.0: the first cumulative sum above it is 3
    assert oracle.inverse_cdf(w, 0.74)[0] == 3
    assert oracle.inverse_cdf(w, 0.75)[0] == 4
    assert oracle.inverse_cdf(w, 0.999)[0] == 4
    rng = np.random.default_rng(0)
    w = rng.random(1000)
    u = rng.random(2000)
    got = np.array([oracle.inverse_cdf(w, x)[0] for x in u])
    counts = np.bincount(got, minlength=1000) / len(u)
    assert np.abs(counts - w / w.sum()).max() < 0.01   # draws follow the weights


def test_emitted_token_is_distributed_as_q():
    """k = 1 on a 5-token vocabulary.  The draft is distributed as p; integrate the rule over the two uniform
    inputs exactly: for a draft x the accept region has length min(1, q_x / p_x), where the emitted token is
    the bonus draw from q_2 (ignored here: we look at position 1, which is then x itself); the reject region
    emits the residual draw.  Position 1's token must come out distributed exactly as q_1."""
    rng = np.random.default_rng(1)
    for _ in range(6):
        V = 5
        q1 = rng.dirichlet(np.ones(V))
        q2 = rng.dirichlet(np.ones(V))
        full = rng.dirichlet(np.ones(V) * 0.7)
        ids = np.argsort(-full)[:3]                    # the device sends its top 3
        probs = full[ids]
        p = oracle.compressed_to_dense(ids, probs, V)
        out = np.zeros(V)
        n_grid = 400
        us = (np.arange(n_grid) + 0.5) / n_grid
        for x in ids:
            for ua in us:                              # uniform grid over u_accept
                n, tok, _ = oracle.speculative_accept(np.stack([q1, q2]), [(ids, probs)], [x], [ua], 0.0)
                if n == 1:
                    out[x] += p[x] / n_grid            # position 1 = the accepted draft
                else:                                  # rejected: integrate the residual draw over u_sample
                    for us2 in us[::4]:
                        _, tok, _ = oracle.speculative_accept(np.stack([q1, q2]), [(ids, probs)], [x], [ua], us2)
                        out[tok] += p[x] / n_grid / len(us[::4])
        assert np.abs(out - q1).max() < 1.5e-2, (out, q1)


def test_special_cases():
    V = 6
    q = np.array([[0.1, 0.2, 0.3, 0.1, 0.2, 0.1], [0.0, 0.0, 1.0, 0.0, 0.0, 0.0]])
    ids, probs = np.arange(V), q[0]
    # p == q: every draft is accepted whatever the uniform number; the bonus token comes from q_2
    for u in (0.0, 0.5, 0.999999):
        assert oracle.speculative_accept(q, [(ids, probs)], [4], [u], 0.3)[:2] == (1, 2)
    # a draft outside its own list cannot have been sampled from it: rejected; the residual is then q - p over
    # the list and q elsewhere
    n, tok, _ = oracle.speculative_accept(q, [([0, 1], [0.5, 0.5])], [3], [0.0], 0.0)
    assert n == 0 and tok == 2                      # q - p = (-.4, -.3, .3, .1, .2, .1) -> first positive weight
    # p concentrated where q is small: ratio q/p
    n, _, info = oracle.speculative_accept(q, [([0], [1.0])], [0], [0.0999], 0.5)
    assert n == 1
    n, tok, _ = oracle.speculative_accept(q, [([0], [1.0])], [0], [0.1001], 0.0)
    assert n == 0 and tok == 1                      # residual (0, .2, .3, .1, .2, .1)
    # two drafts, second rejected: the count is 1
    q3 = np.vstack([q[0], q[0], q[1]])
    n, tok, _ = oracle.speculative_accept(q3, [(ids, probs), ([5], [1.0])], [1, 5], [0.9, 0.5], 0.0)
    assert n == 1 and tok == 0                      # ratio for draft 5 is 0.1 < 0.5; residual q - e_5, first positive
