"""Pins of the oracle's sampling-mode verification (Sec. 4.3 "sampling strategies", Table 3).
The paper reports temperature and top-p sampling without the rule; the rule taken -- accept the
deterministic draft x with probability P(x), else draw from P without x -- is pinned here by
what fixes it: every emitted token must be distributed as the full model's own sample.  CPU only."""
import numpy as np
import pytest
from scipy import stats

import sb_inputs as si
import oracle as orc
from helpers import tiny_model, params, linear_T, oracle_with_mistake
from oracle import Oracle, OrcParams


def test_sampling_distribution_closed_forms():
    g = np.random.default_rng(3)
    z = g.standard_normal(200) * 2.0
    for temp in (0.3, 1.0, 2.5):
        p = orc.sample_dist(z, temp)
        e = np.exp((z - z.max()) / temp)
        np.testing.assert_allclose(p, e / e.sum(), rtol=1e-12)
    # nucleus: brute force by a full sort
    for top_p in (0.1, 0.5, 0.9, 0.999):
        p = orc.sample_dist(z, 1.0, top_p)
        full = np.exp(z - z.max()); full /= full.sum()
        order = np.argsort(-full)
        k = int(np.searchsorted(np.cumsum(full[order]), top_p - 1e-15)) + 1
        keep = np.zeros_like(full, bool); keep[order[:k]] = True
        want = np.where(keep, full, 0.0); want /= want.sum()
        np.testing.assert_allclose(p, want, rtol=1e-12, atol=0)
        assert abs(p.sum() - 1) < 1e-12 and (p > 0).sum() == k
    # ties at the edge of the nucleus are kept together
    zt = np.array([2.0, 1.0, 1.0, 1.0, -3.0])
    pt = orc.sample_dist(zt, 1.0, 0.7)           # 0.45 + 0.17 < 0.7: a second token is needed, all three tie
    assert (pt > 0).tolist() == [True, True, True, True, False]
    # top_p = 1 keeps everything; temperature -> 0 is a point mass on the arg max
    assert (orc.sample_dist(z, 1.0, 1.0) > 0).all()
    cold = orc.sample_dist(z, 1e-3)
    assert cold[np.argmax(z)] == 1.0 and cold.sum() == 1.0


def test_inverse_cdf_draw():
    p = np.array([0.1, 0.0, 0.4, 0.2, 0.3])
    cdf = np.cumsum(p)
    for u in (0.0, 0.05, 0.0999, 0.1, 0.3, 0.4999, 0.5, 0.69, 0.7, 0.99999):
        assert orc.sample_token(p, u) == int(np.searchsorted(cdf, u, side="right"))
    # without token 2: the rest renormalised (0.1, 0.2, 0.3) / 0.6
    q = p.copy(); q[2] = 0; q /= q.sum()
    cq = np.cumsum(q)
    for u in (0.0, 0.16, 0.17, 0.49, 0.51, 0.999):
        t = orc.sample_token(p, u, exclude=2)
        assert t == int(np.searchsorted(cq, u, side="right")) and t != 2
    # never a token without mass, never the excluded one
    g = np.random.default_rng(0)
    for u in g.random(200):
        assert orc.sample_token(p, u, exclude=0) in (2, 3, 4)


def _peaked_model():
    """Tiny model whose final distribution has a few dominant tokens (norm gains scaled up)."""
    shape = si.tiny_shape(n_layers=5, n_exit_heads=3, vocab=64)
    w = si.make_weights(shape, 91, gain_jitter=0.1)
    w["final_norm"] = (w["final_norm"] * 14.0).astype(np.float32)
    for l in range(3):      # exit heads: the final head, so that drafts are often the likely token
        w[f"exit_head.{l}"] = w["lm_head"]
        w[f"exit_norm.{l}"] = w["final_norm"]
    return shape, w, Oracle(shape, w, 64)


def pin_distribution(temp=1.0, top_p=1.0):
    """Chi-square of the first two tokens a round emits against the full model's own sampling
    distribution (computed from its logits): token 1 ~ P(. | prefix), token 2 ~ P(. | prefix, a)
    for the most frequent first token a."""
    shape, w, m = _peaked_model()
    V = shape.vocab
    prompt = si.make_prompt(V, 7, 501)
    s = m.session()
    first = s.prefill(prompt)
    P0 = len(prompt)
    # reference distributions from teacher-forced logits of the full model
    _, z1 = s.step(first)
    p1 = orc.sample_dist(z1, temp, top_p)
    a = int(np.argmax(p1))
    _, z2 = s.step(a)
    p2 = orc.sample_dist(z2, temp, top_p)
    assert 0.15 < p1[a] < 0.9            # both the acceptance and the rejection branch are taken often
    N = 3000
    g = np.random.default_rng(77)
    c1, c2 = np.zeros(V), np.zeros(V)
    n_acc = 0
    for it in range(N):
        U = g.random(2 * 64).astype(np.float32)
        p = OrcParams(3, 4, linear_T(3), 0.5, forced_exit=[1, 2, 3, 1], sample_temperature=temp, top_p=top_p, sample_u=U)
        s.rewind(P0, first)
        while s.draft_step(p)["status"] == orc.EXITED:
            pass
        v = s.verify(p)
        toks = v["tokens"][: v["n_emit"]]
        c1[toks[0]] += 1
        n_acc += v["n_matched"] >= 1
        if toks[0] == a and len(toks) >= 2:
            c2[toks[1]] += 1
    assert 0.05 * N < n_acc < 0.95 * N

    def chi2_ok(counts, p):
        n = counts.sum()
        big = p * n >= 5
        obs = np.append(counts[big], counts[~big].sum())
        exp = np.append(p[big] * n, p[~big].sum() * n)
        keep = exp > 0
        assert obs[~keep].sum() == 0                       # nothing outside the support (nucleus)
        stat = ((obs[keep] - exp[keep]) ** 2 / exp[keep]).sum()
        return stats.chi2.sf(stat, keep.sum() - 1)
    assert chi2_ok(c1, p1) > 1e-3
    assert c2.sum() > 200 and chi2_ok(c2, p2) > 1e-3
    # a wrong rule would show: e.g. emitting the draft whenever it is the arg max gives p(a) = 1
    assert abs(c1[a] / N - p1[a]) < 0.04


@pytest.mark.parametrize("temp,top_p", [(1.0, 1.0), (0.6, 0.9)])
def test_emitted_tokens_are_distributed_as_the_full_models_samples(temp, top_p):
    pin_distribution(temp, top_p)


SAMPLING_MISTAKES = {
    "rejected_draft_can_be_drawn_again": ("m < s->n_drafts ? s->drafts[m] : -1);\n        for (int32_t i = m + 1", "-1);\n        for (int32_t i = m + 1"),
    "draft_accepted_whenever_it_has_mass": ("p->sample_u[2 * (int64_t)s->slots[m].pos] < P[s->drafts[m]]", "0 < P[s->drafts[m]]"),
    "same_uniform_for_test_and_draw": ("p->sample_u[2 * (int64_t)s->slots[m].pos + 1]", "p->sample_u[2 * (int64_t)s->slots[m].pos]"),
    "temperature_ignored": ("(real)p->sample_temperature,\n", "(real)1,\n"),
}


@pytest.mark.parametrize("name", sorted(SAMPLING_MISTAKES))
def test_planted_sampling_mistake_fails_the_distribution_pin(name, tmp_path, monkeypatch):
    oracle_with_mistake(monkeypatch, tmp_path, *SAMPLING_MISTAKES[name])
    red = 0
    for temp, top_p in ((1.0, 1.0), (0.6, 0.9)):
        try:
            pin_distribution(temp, top_p)
        except AssertionError:
            red += 1
    assert red >= 1, f"the distribution pin does not notice '{name}'"


def test_cold_sampling_is_greedy_decoding():
    """Temperature towards 0: the distribution is a point mass on the arg max, so the rounds,
    accept lengths and tokens are those of greedy verification, whatever the uniforms."""
    shape, w, m = tiny_model(n_layers=6, n_exit_heads=3, seed=21)
    prompt = si.make_prompt(shape.vocab, 8, 100)
    fe = si.forced_exit_schedule(5, 300, 0, 3)
    U = np.random.default_rng(1).random(2 * 160).astype(np.float32)
    ref_s = m.session()
    ref = ref_s.generate(prompt, 30, params(3, 4, 0.5, forced_exit=fe))
    s = m.session()
    out = s.generate(prompt, 30, OrcParams(3, 4, linear_T(3), 0.5, forced_exit=fe, sample_temperature=1e-4, sample_u=U))
    assert out.tolist() == ref.tolist()
    assert s.stats()["accept_hist"] == ref_s.stats()["accept_hist"]


def test_sampling_parameter_errors():
    shape, w, m = tiny_model(n_layers=4, n_exit_heads=2, seed=3)
    s = m.session()
    s.prefill(si.make_prompt(shape.vocab, 5, 1))
    bad = [dict(sample_temperature=-1.0), dict(sample_temperature=1.0), dict(sample_temperature=1.0, top_p=0.0, sample_u=np.zeros(400)),
           dict(sample_temperature=1.0, top_p=1.5, sample_u=np.zeros(400))]
    for kw in bad:
        assert s.draft_step(OrcParams(2, 2, linear_T(2), 0.5, **kw), check=False) == -1
    # too few uniforms for the positions of the round
    p = OrcParams(2, 2, linear_T(2), 0.5, forced_exit=[1, 1], sample_temperature=1.0, sample_u=np.zeros(6))
    while s.draft_step(p)["status"] == orc.EXITED:
        pass
    assert s.verify(p, check=False) == -1
