"""Pins of the oracle's relaxed acceptance rule (paper Section 3.2, Eq. 9-12 with threshold tau; tau = 0.75 is the
paper's operating point, Section 4.1): things the rule must satisfy that do not come from the oracle's own code."""
import math

import numpy as np
import pytest

import oracle as O
import workloads as W


def _softmax(x):
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def _brute_relaxed(logits, draft, tau):
    """Eq. 11 written with probabilities: accept while p(u*) / p(u_hat) >= tau."""
    p = _softmax(logits.astype(np.float64))
    alpha = 0
    for i, d in enumerate(draft):
        if p[i, d] / p[i].max() >= tau:
            alpha += 1
        else:
            break
    return alpha, int(np.argmax(p[alpha]))


@pytest.mark.parametrize("tau", [0.9, 0.75, 0.3, 0.05])
def test_relaxed_rule_equals_probability_ratio_form(tau):
    rng = np.random.default_rng(5)
    for trial in range(200):
        k, V = int(rng.integers(1, 40)), 50
        logits = rng.normal(0, 1.5, size=(k + 1, V))
        top = np.argsort(-logits, axis=1)
        # drafts made of top-1 / top-2 / random tokens so that all three outcomes occur
        pick = rng.integers(0, 3, size=k)
        draft = np.where(pick == 0, top[:k, 0], np.where(pick == 1, top[:k, 1], rng.integers(0, V, size=k)))
        assert O.accept_relaxed(logits, draft, math.log(tau)) == _brute_relaxed(logits, draft, tau)


def test_tau_to_one_is_exact_match_and_acceptance_is_monotone_in_tau():
    rng = np.random.default_rng(6)
    for trial in range(200):
        k, V = int(rng.integers(1, 30)), 40
        logits = rng.normal(0, 1, size=(k + 1, V))
        top = np.argsort(-logits, axis=1)
        draft = np.where(rng.random(k) < 0.7, top[:k, 0], top[:k, 1])
        exact = O.accept_longest_prefix(O.argmax_lowest_index(logits), draft)
        assert O.accept_relaxed(logits, draft, -1e-300) == exact          # no exact ties in continuous data
        alphas = [O.accept_relaxed(logits, draft, math.log(t))[0] for t in (0.99, 0.75, 0.5, 0.1, 1e-6)]
        assert alphas == sorted(alphas) and alphas[0] >= exact[0]
        assert O.accept_relaxed(logits, draft, -np.inf)[0] == k            # tau -> 0 accepts everything


def test_near_miss_draft_closed_form():
    """A draft equal to the greedy target except that some positions carry the model's SECOND choice: position i
    is accepted iff the top-1/top-2 margin there is at most -log tau, so alpha is the first near-miss position
    whose margin exceeds -log tau.  Uses the full decoder (teacher-forced rows equal the greedy rows)."""
    desc = W.tiny_model(2, 64, 2, 1, 32, 128, 96, "fp32")
    seed = 31
    weights = W.make_weights(desc, seed)
    vis, prompt = W.make_prefix(desc, seed, 0, 12, 3)
    cache, pending = O.prefill(desc, weights, vis, prompt)
    base = len(cache)
    k = 40
    target = O.greedy_decode(desc, weights, cache, pending, k)
    cache.truncate(base)
    _, _, u_hat, logits = O.verify_block(desc, weights, cache, pending, target)
    cache.truncate(base)
    assert (u_hat[:k] == target).all()
    margin = O.top2_margin(logits)
    second = np.argsort(-logits, axis=1)[:, 1]
    for tau in (0.9, 0.75, 0.4):
        lt = math.log(tau)
        # a near-miss changes the context of the rows after it, so the closed form covers the FIRST one only
        for pos in (0, 7, 23, k - 1):
            draft = target.copy()
            draft[pos] = second[pos]
            alpha, bonus, _, lg = O.verify_block(desc, weights, cache, pending, draft, log_tau=lt)
            cache.truncate(base)
            if margin[pos] <= -lt:
                assert alpha > pos            # accepted; what follows depends on the new context
            else:
                assert (alpha, bonus) == (pos, int(target[pos]))


def test_relaxed_spec_decode_commits_only_tau_admissible_tokens():
    """Analogue of the lossless invariant for tau < 1: replaying the committed sequence token by token, every
    committed token must pass the rule in its own context (bonus tokens are the arg-max itself), and with an
    uncorrupted greedy draft the result is the greedy sequence."""
    desc = W.tiny_model(2, 64, 2, 2, 32, 128, 80, "fp32")
    seed = 32
    weights = W.make_weights(desc, seed)
    vis, prompt = W.make_prefix(desc, seed, 1, 9, 2)
    lt = math.log(0.75)
    cache, pending = O.prefill(desc, weights, vis, prompt)
    base = len(cache)
    n = 48
    target = O.greedy_decode(desc, weights, cache, pending, n)
    cache.truncate(base)
    same, _ = O.spec_decode(desc, weights, cache, pending, target, n, log_tau=lt)
    np.testing.assert_array_equal(same, target)
    cache.truncate(base)
    draft, _ = W.corrupt_draft(target, 0.3, desc.vocab, seed, "relaxed")
    committed, rounds = O.spec_decode(desc, weights, cache, pending, draft, n, log_tau=lt)
    cache.truncate(base)
    tok = pending
    for t in committed:
        lg = O.decoder_forward(desc, weights, O.embed_tokens(weights, [tok]), cache)[0]
        assert lg[t] - lg.max() >= lt - 1e-9
        tok = int(t)
    assert len(rounds) >= 2
