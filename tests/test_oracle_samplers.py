"""Pins for the oracle's samplers: the special cases and invariants the paper states."""
import math

import numpy as np
import pytest

import synth_inputs as S
from oracle import rdlm_oracle as O


@pytest.fixture(scope="module")
def tiny():
    shape = S.TINY
    return shape, O.RecurrentDepthLM(shape, S.make_weights(shape, 1)), S.make_prompt(shape.vocab, 16, 1)


@pytest.fixture(scope="module")
def tiny_conditioned():
    """Same shape with a 6x larger embedding: the conditioning e then outweighs the state in the
    adapter input and the recurrence settles, so that a threshold on delta_i can fire."""
    shape = S.TINY
    w = S.make_weights(shape, 1)
    w["emb"] = w["emb"] * 6.0
    return shape, O.RecurrentDepthLM(shape, w), S.make_prompt(shape.vocab, 16, 1)


def _same_run(a: O.Trace, b: O.Trace):
    assert np.array_equal(a.tokens, b.tokens)
    assert a.final_states.keys() == b.final_states.keys()
    for p in a.final_states:
        assert np.array_equal(a.final_states[p], b.final_states[p])
        assert a.recurrences[p] == b.recurrences[p]


@pytest.mark.parametrize("temperature", [0.0, 1.0])
def test_inner_recurrence_equal_to_r_recovers_autoregressive(tiny, temperature):
    """End of Sec. 3.3: with the fixed exit rule, r' = r is exactly the autoregressive sampler."""
    _, m, prompt = tiny
    ar = O.generate_autoregressive(m, prompt, 12, 4, temperature=temperature, seed=3)
    df = O.generate_diffusion_forcing(m, prompt, 12, 4, 4, temperature=temperature, seed=3)
    _same_run(ar, df)
    assert df.steps == 12 and max(df.window_sizes) == 1


@pytest.mark.parametrize("r_inner", [1, 2])
def test_wavefront_of_one_recovers_adaptive_compute(tiny_conditioned, r_inner):
    """Sec. 3.5: a wavefront of one token is the token-per-token adaptive-compute sampler."""
    _, m, prompt = tiny_conditioned
    kw = dict(r_inner=r_inner, r_cap=24, eps=0.05, temperature=1.0, seed=4)
    a = O.generate_adaptive_autoregressive(m, prompt, 10, **kw)
    d = O.generate_diffusion_forcing_adaptive(m, prompt, 10, w_max=1, **kw)
    _same_run(a, d)
    assert a.steps == d.steps
    recs = list(a.recurrences.values())
    assert min(recs) < 24, "the threshold never fired: the test would not exercise early exit"
    assert all(r % r_inner == 0 for r in recs)


@pytest.mark.parametrize("r,r_inner,headway", [(4, 1, 1), (6, 2, 1), (5, 2, 1), (4, 1, 3)])
def test_adaptive_with_zero_threshold_is_the_fixed_exit_sampler(tiny, r, r_inner, headway):
    """eps = 0 never converges, so only the recurrence cap freezes: Alg. 2 must then walk exactly
    like Alg. 1 (whose rule is that cap)."""
    _, m, prompt = tiny
    w = -(-r // r_inner) * headway
    a = O.generate_diffusion_forcing(m, prompt, 12, r_inner, r, headway=headway, seed=2)
    b = O.generate_diffusion_forcing_adaptive(m, prompt, 12, r_inner, r, 0.0, w, headway=headway, seed=2)
    _same_run(a, b)
    assert a.steps == b.steps and a.window_sizes == b.window_sizes


@pytest.mark.parametrize("r,r_inner", [(4, 1), (8, 2), (7, 3)])
def test_fixed_exit_wave_shape(tiny, r, r_inner):
    """Sec. 3.3: the wave holds ceil(r/r') states, advances one token per step once full, and a
    token is frozen exactly when its position has had ceil(r/r') sampler steps."""
    _, m, prompt = tiny
    n_new = 10
    w = -(-r // r_inner)
    tr = O.generate_diffusion_forcing(m, prompt, n_new, r_inner, r)
    assert tr.steps == n_new + w - 1
    assert max(tr.window_sizes) == w
    assert tr.window_sizes[:w] == list(range(1, w + 1))
    assert tr.frozen_per_step == [0] * (w - 1) + [1] * n_new
    assert all(v == w * r_inner for v in tr.recurrences.values())
    assert sorted(tr.final_states) == list(range(15, 15 + n_new))


def test_headway_wave_shape(tiny):
    """Sec. 4.2 (moving forward multiple steps): headway g appends g states per step, so the wave
    holds g*r states and g tokens are frozen per step."""
    _, m, prompt = tiny
    tr = O.generate_diffusion_forcing(m, prompt, 12, 1, 4, headway=3, pad_token=7)
    assert max(tr.window_sizes) == 3 * 4 and tr.window_sizes[:6] == [1, 4, 7, 10, 12, 12]
    assert tr.frozen_per_step[:4] == [0, 0, 0, 1]
    assert set(tr.frozen_per_step[4:]) == {3}
    # the first generated token never sees a pad input: it cannot depend on the pad token
    tr2 = O.generate_diffusion_forcing(m, prompt, 12, 1, 4, headway=3, pad_token=9)
    assert tr.tokens[16] == tr2.tokens[16]
    assert np.array_equal(tr.final_states[15], tr2.final_states[15])


def test_wavefront_limit_stalls_and_bounds_memory(tiny):
    """Sec. 3.5: the limiter bounds the number of states in flight; when nothing converges the
    wave stalls at that size until the cap frees its head."""
    _, m, prompt = tiny
    tr = O.generate_diffusion_forcing_adaptive(m, prompt, 8, 1, 6, 0.0, 3)
    assert max(tr.window_sizes) == 3
    assert 3 in tr.window_sizes and tr.frozen_per_step.count(0) > 3
    assert all(v == 6 for v in tr.recurrences.values())
    assert len(tr.tokens) == 16 + 8


def test_adaptive_freezes_only_converged_prefixes(tiny_conditioned):
    _, m, prompt = tiny_conditioned
    eps, cap = 0.05, 400
    tr = O.generate_diffusion_forcing_adaptive(m, prompt, 10, 1, cap, eps, 8)
    assert any(k > 0 for k in tr.frozen_per_step)
    assert max(tr.recurrences.values()) < cap, "the cap fired: the prefix rule below would not hold"
    for d, k in zip(tr.deltas, tr.frozen_per_step):
        assert all(x < eps for x in d[:k])          # every frozen state was below the threshold
        if k < len(d):
            assert not d[k] < eps                   # and the first one kept was not
    assert min(tr.recurrences.values()) < cap, "threshold never fired"
    assert max(tr.window_sizes) <= 8
    # a brand-new state is compared with its random initialisation: it cannot look converged
    assert all(d[-1] > 0.5 for d in tr.deltas[1:] if len(d) > 1)


def test_contraction_gives_the_autoregressive_solution():
    """Remark of Sec. 3.5: if R is a contraction, the adaptive sampler converges to what
    autoregressive sampling (run to its fixed point) produces."""
    shape = S.TINY
    w = S.make_weights(shape, 6)
    w["wa"] = w["wa"].copy()
    w["wa"][:, shape.hidden:] *= 0.02          # the state half of the adapter barely feeds back
    w["emb"] = w["emb"] * 8.0                   # conditioning dominates
    m = O.RecurrentDepthLM(shape, w)
    prompt = S.make_prompt(shape.vocab, 12, 5)
    ar = O.generate_autoregressive(m, prompt, 10, 48)
    df = O.generate_diffusion_forcing_adaptive(m, prompt, 10, 1, 200, 1e-9, 6, r_prefill=48)
    assert np.array_equal(ar.tokens, df.tokens)
    for p in ar.final_states:
        assert np.allclose(ar.final_states[p], df.final_states[p], rtol=0, atol=1e-6)
    assert max(df.recurrences.values()) < 200, "only the cap fired: not a convergence test"


def test_cost_remark(tiny):
    """Remark of Sec. 3.5: one sampler iteration costs (cost of P and C) + r' * f per in-flight
    token; over w tokens the fixed-exit sampler spends (r + r/r') f w against (r + 1) f w when
    P and C together cost f."""
    shape, m, prompt = tiny
    h, Fm, V = shape.hidden, shape.mlp, shape.vocab
    layer = 2 * (4 * h * h + 3 * h * Fm)
    f_R = shape.n_core * layer + 2 * (2 * h * h)
    f_PC = (shape.n_prelude + shape.n_coda) * layer + 2 * V * h
    r, r_inner, n_new = 4, 2, 9
    m.counter.flops = 0
    O.generate_diffusion_forcing(m, prompt, n_new, r_inner, r, r_prefill=0)
    got_df = m.counter.flops
    m.counter.flops = 0
    tr = O.generate_diffusion_forcing(m, prompt, n_new, r_inner, r, r_prefill=0)
    prefill_part = (len(prompt) - 1) * (f_PC - 2 * V * h)
    assert got_df == sum(tr.window_sizes) * (f_PC + r_inner * f_R) + prefill_part
    m.counter.flops = 0
    O.generate_autoregressive(m, prompt, n_new, r, r_prefill=0)
    assert m.counter.flops == n_new * (f_PC + r * f_R) + prefill_part
    # steady state: each token spends r/r' iterations in flight
    per_token = (r // r_inner) * (f_PC + r_inner * f_R)
    assert per_token == (r // r_inner) * f_PC + r * f_R


def test_streams_are_not_degenerate(tiny):
    """Parity on token ids means little if every run emits the same few tokens, or if the prompt
    does not matter."""
    _, m, prompt = tiny
    tr = O.generate_diffusion_forcing(m, prompt, 32, 1, 4)
    assert len(set(tr.tokens[16:].tolist())) >= 16
    p2 = prompt.copy()
    p2[3] = (p2[3] + 1) % 256
    tr2 = O.generate_diffusion_forcing(m, p2, 32, 1, 4)
    assert (tr.tokens[16:] != tr2.tokens[16:]).sum() >= 2


# ---------------------------------------------------------------------------------------------
# Stabilising components (Sec. 3.4): momentum on the conditioning (Eq. 1), state noise (Eq. 2)

def test_noise_schedule_is_linear_and_ends_low():
    """Sec. 3.4: beta_t falls linearly with the steps a position has received."""
    levels = [O.noise_level(0.5, c, 8) for c in range(8)]
    assert levels[0] == 0.5
    assert np.allclose(np.diff(levels), -0.5 / 8)
    assert all(l > 0 for l in levels) and O.noise_level(0.5, 8, 8) == 0.0 and O.noise_level(0.5, 11, 8) == 0.0
    assert O.noise_level(0.0, 0, 8) == 0.0


def test_mix_noise_is_the_convex_combination_of_eq_2():
    z = np.linspace(-1, 1, 128)
    zn = O.init_state(128, 9, 2, 0.7, 5, step=3, tag=O.TAG_NOISE)
    out = O.mix_noise(z, 0.25, 9, 2, 3, 0.7, 5)
    assert np.allclose(out, 0.75 * z + 0.25 * zn, rtol=0, atol=1e-15)
    assert O.mix_noise(z, 0.0, 9, 2, 3, 0.7, 5) is z
    assert np.array_equal(O.mix_noise(z, 1.0, 9, 2, 3, 0.7, 5), zn)
    # the noise stream is its own: not the InitState draw of the same position, and new every step
    assert not np.allclose(zn, O.init_state(128, 9, 2, 0.7, 5))
    assert not np.allclose(zn, O.init_state(128, 9, 2, 0.7, 5, step=4, tag=O.TAG_NOISE))


def test_momentum_is_an_exponential_average_of_the_preludes(tiny):
    """Eq. 1 unrolled: e_k = eta^k P_0 + (1 - eta) sum_{j=1..k} eta^(k-j) P_j over the steps a
    position has been in flight (P_j = its raw prelude output at step j)."""
    eta = 0.3
    rng = np.random.default_rng(0)
    P = rng.standard_normal((5, 16))
    e = None
    for k in range(5):
        e = O.momentum(P[k], e, eta)
        want = eta ** k * P[0] + (1 - eta) * sum(eta ** (k - j) * P[j] for j in range(1, k + 1))
        assert np.allclose(e, want, rtol=0, atol=1e-14)
    assert np.array_equal(O.momentum(P[1], P[0], 0.0), P[1])
    # in the sampler: the first state reads the last prompt token, which never changes, so its
    # conditioning stays P(token) for any eta; later positions see changing drafts and do move
    _, m, prompt = tiny
    seen = {}

    def hook(t, z_pos, zz, logits, y, e):
        for i, p in enumerate(z_pos):
            seen.setdefault(p, []).append(e[i].copy())

    O.generate_diffusion_forcing(m, prompt, 6, 1, 4, seed=2, eta=eta, hook=hook)
    first = seen[len(prompt) - 1]
    assert len(first) == 4
    for k in range(1, len(first)):
        assert np.allclose(first[k], first[0], rtol=0, atol=1e-12)
    plain = {}

    def hook0(t, z_pos, zz, logits, y, e):
        for i, p in enumerate(z_pos):
            plain.setdefault(p, []).append(e[i].copy())

    O.generate_diffusion_forcing(m, prompt, 6, 1, 4, seed=2, eta=0.0, hook=hook0)
    later = len(prompt) + 1
    assert np.allclose(seen[later][0], plain[later][0])          # first step of a position: no memory
    assert any(not np.allclose(a, b) for a, b in zip(seen[later][1:], plain[later][1:]))


def test_eta_and_beta_zero_change_nothing(tiny):
    _, m, prompt = tiny
    a = O.generate_diffusion_forcing(m, prompt, 8, 1, 4, seed=2)
    b = O.generate_diffusion_forcing(m, prompt, 8, 1, 4, seed=2, eta=0.0, beta=0.0)
    _same_run(a, b)


def test_momentum_and_noise_change_the_run_but_not_its_shape(tiny):
    _, m, prompt = tiny
    base = O.generate_diffusion_forcing(m, prompt, 8, 1, 4, seed=2)
    for kw in (dict(eta=0.5), dict(beta=0.5), dict(eta=0.1, beta=0.3)):
        tr = O.generate_diffusion_forcing(m, prompt, 8, 1, 4, seed=2, **kw)
        assert tr.steps == base.steps and tr.window_sizes == base.window_sizes
        assert any(not np.allclose(tr.final_states[p], base.final_states[p]) for p in base.final_states)


def test_full_noise_with_window_one_is_autoregressive_from_the_noise_draw(tiny):
    """r' = r (window 1, one step per position) with beta = 1: the state a position starts from is
    exactly the TAG_NOISE draw of that step, so the run equals an autoregressive loop seeded with
    those draws."""
    _, m, prompt = tiny
    r, n_new, seed = 3, 5, 7
    tr = O.generate_diffusion_forcing(m, prompt, n_new, r, r, seed=seed, beta=1.0)
    L = len(prompt)
    cache = m.new_cache(L + n_new + 4)
    y = list(int(t) for t in prompt)
    m.prefill(np.asarray(y[: L - 1]), r, 1.0, seed, 0, cache)
    for t in range(1, n_new + 1):
        p = len(y) - 1
        pos = np.array([p])
        s = O.init_state(m.h, p, 0, 1.0, seed, step=t, tag=O.TAG_NOISE)[None, :]
        e = m.prelude(np.array([y[p]]), pos, cache)
        for _ in range(r):
            s = m.core(e, s, pos, cache)
        y.append(O.sample(m.coda(s, pos, cache)[0], 0.0, p, 0, t, seed))
        assert np.allclose(tr.final_states[p], s[0], rtol=0, atol=1e-12)
    assert np.array_equal(tr.tokens, np.asarray(y))


def test_adaptive_sampler_takes_momentum_and_noise(tiny_conditioned):
    """Alg. 2 with eta, beta: delta_i still compares against the noise-free end of the previous
    step, so with beta > 0 a state needs more steps to pass the threshold (or runs to the cap)."""
    _, m, prompt = tiny_conditioned
    kw = dict(r_inner=1, r_cap=12, eps=0.05, w_max=6, seed=4)
    a = O.generate_diffusion_forcing_adaptive(m, prompt, 6, **kw)
    b = O.generate_diffusion_forcing_adaptive(m, prompt, 6, beta=0.5, **kw)
    assert sum(b.recurrences.values()) > sum(a.recurrences.values())
    c = O.generate_diffusion_forcing_adaptive(m, prompt, 6, eta=0.0, beta=0.0, **kw)
    _same_run(a, c)


def test_continuous_compute_with_window_one_carries_the_state_across_tokens(tiny):
    """App., additional hyperparameter sweeps: appended states start from the latest state of the
    position to the left.  With r' = r (window 1) that is the plain token-by-token loop whose
    state is never re-drawn -- written out here without the sampler's bookkeeping."""
    _, m, prompt = tiny
    r, n_new, seed = 3, 9, 5
    df = O.generate_diffusion_forcing(m, prompt, n_new, r, r, temperature=1.0, seed=seed, continuous_compute=True)
    L = len(prompt)
    cache = m.new_cache(L + n_new)
    y = [int(t) for t in prompt]
    m.prefill(np.asarray(y[: L - 1]), r, 1.0, seed, 0, cache)
    s = O.init_state(m.h, L - 1, 0, 1.0, seed)[None, :]          # drawn once
    for t in range(1, n_new + 1):
        p = len(y) - 1
        e = m.prelude(np.array([y[p]]), np.array([p]), cache)
        for _ in range(r):
            s = m.core(e, s, np.array([p]), cache)
        y.append(O.sample(m.coda(s, np.array([p]), cache)[0], 1.0, p, 0, t, seed))
        assert np.array_equal(df.final_states[p], s[0])
    assert np.array_equal(df.tokens, np.asarray(y))
    plain = O.generate_diffusion_forcing(m, prompt, n_new, r, r, temperature=1.0, seed=seed)
    assert np.array_equal(plain.final_states[L - 1], df.final_states[L - 1])      # the first state is a draw
    assert not np.array_equal(plain.final_states[L], df.final_states[L])


@pytest.mark.parametrize("headway", [1, 2])
def test_continuous_compute_starts_from_the_left_neighbours_latest_state(tiny, headway):
    """In a wavefront the copied state is the one the left neighbour ended the step on: the first
    delta_i of an appended state (Eq. 3, against its initial value) must equal its distance to
    that neighbour state, as recorded by the hook one step earlier."""
    _, m, prompt = tiny
    states = {}

    def hook(t, z_pos, zz, logits, y, e):
        states[t] = {p: zz[i].copy() for i, p in enumerate(z_pos)}

    tr = O.generate_diffusion_forcing_adaptive(m, prompt, 8, 1, 4, 0.0, 16, seed=2, headway=headway,
                                               continuous_compute=True, hook=hook)
    checked = 0
    for t in range(2, tr.steps + 1):
        prev, cur = states[t - 1], states[t]
        last_prev = max(prev)                                   # right-most position of the previous window
        fresh = [p for p in cur if p not in prev]
        assert all(p > last_prev for p in fresh)
        pos = sorted(cur)
        for p in fresh:
            want = np.linalg.norm(cur[p] - prev[last_prev]) / np.linalg.norm(cur[p])
            assert math.isclose(tr.deltas[t - 1][pos.index(p)], want, rel_tol=1e-12)
            checked += 1
    assert checked >= 6
    base = O.generate_diffusion_forcing_adaptive(m, prompt, 8, 1, 4, 0.0, 16, seed=2, headway=headway)
    assert base.steps == tr.steps and base.window_sizes == tr.window_sizes      # same wave, other values
    assert not np.array_equal(base.final_states[len(prompt)], tr.final_states[len(prompt)])
