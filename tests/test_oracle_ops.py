"""Pins for the oracle's building blocks: each compares the oracle with something that is not the
oracle (published vectors, a library routine, a scalar brute force, a closed form, a statistic)."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F
from scipy import stats

import synth_inputs as S
from oracle import rdlm_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ counter-based generator
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 2
    for r in rows:
        v = [int(x, 16) for x in r]
        out = O.philox4x32_10(v[0], v[1], v[2], v[3], v[4], v[5])
        assert [int(o) for o in out] == v[6:10]


def test_philox_vectorised_matches_scalar_calls():
    c0 = np.arange(7)
    out = O.philox4x32_10(c0, 5, 9, 33, 123, 456)
    for i in range(7):
        one = O.philox4x32_10(i, 5, 9, 33, 123, 456)
        assert [int(o[i]) for o in out] == [int(o) for o in one]


def test_init_state_is_standard_normal():
    z = np.concatenate([O.init_state(4096, p, 0, 1.0, seed=7) for p in range(32)])
    assert abs(z.mean()) < 4 / math.sqrt(z.size)
    assert abs(z.var() - 1.0) < 0.02
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # pairs produced by one Box-Muller draw must be uncorrelated, and so must neighbours
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 0.02
    assert abs(stats.kurtosis(z)) < 0.1


def test_init_state_keys():
    a = O.init_state(64, 3, 0, 1.0, seed=1)
    assert np.array_equal(a, O.init_state(64, 3, 0, 1.0, seed=1))          # reproducible
    assert not np.allclose(a, O.init_state(64, 4, 0, 1.0, seed=1))         # position
    assert not np.allclose(a, O.init_state(64, 3, 1, 1.0, seed=1))         # sequence
    assert not np.allclose(a, O.init_state(64, 3, 0, 1.0, seed=2))         # seed
    assert not np.allclose(a, O.init_state(64, 3, 0, 1.0, seed=1 << 32))   # high key word
    assert np.allclose(2.5 * a, O.init_state(64, 3, 0, 2.5, seed=1))       # alpha scales
    assert np.array_equal(a[:30], O.init_state(30, 3, 0, 1.0, seed=1))     # prefix-stable, ragged


def test_gumbel_max_draws_from_softmax():
    logits = np.array([0.0, 1.0, -0.5, 2.0, 0.3, -2.0, 1.5])
    for temp in (1.0, 0.5):
        p = np.exp(logits / temp)
        p /= p.sum()
        n = 6000
        counts = np.zeros(len(logits))
        for step in range(n):
            counts[O.sample(logits, temp, position=11, seq=2, step=step, seed=5)] += 1
        chi2 = ((counts - n * p) ** 2 / (n * p)).sum()
        assert stats.chi2.sf(chi2, len(logits) - 1) > 1e-3


def test_greedy_lowest_index_wins_ties():
    assert O.sample(np.array([1.0, 3.0, 3.0, 2.0]), 0.0, 0, 0, 0, 0) == 1


# ------------------------------------------------------------------ layer pieces
def test_rmsnorm_against_library_and_invariants():
    x = S.make_rows(5, 48, 3).astype(np.float64)
    g = 1.0 + 0.1 * S.make_rows(1, 48, 4)[0].astype(np.float64)
    ref = F.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-6).numpy()
    got = O.rmsnorm(x, g, 1e-6)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)
    # unit gains give rows of unit mean square; scaling the input changes nothing
    y = O.rmsnorm(x, np.ones(48), 0.0)
    assert np.allclose((y * y).mean(-1), 1.0)
    assert np.allclose(O.rmsnorm(7.0 * x, g, 0.0), O.rmsnorm(x, g, 0.0))
    # hand value: x = (3,4) -> mean square 12.5
    assert np.allclose(O.rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0),
                       [[3 / math.sqrt(12.5), 8 / math.sqrt(12.5)]])


def test_silu_against_library():
    x = np.linspace(-6, 6, 41)
    assert np.allclose(O.silu(x), F.silu(torch.from_numpy(x)).numpy(), rtol=1e-12)
    assert O.silu(np.array([0.0]))[0] == 0.0


def test_rope_closed_forms():
    # d = 2: one pair, theta = 1: (1,0) at position p becomes (cos p, sin p)
    x = np.array([[[1.0, 0.0]]])
    for p in (0, 1, 5):
        assert np.allclose(O.rope(x, np.array([p]), 10000.0)[0, 0], [math.cos(p), math.sin(p)])
    # d = 4: pairs are (0,2) and (1,3); second pair turns by p * base^(-1/2)
    x = np.array([[[0.0, 1.0, 0.0, 0.0]]])
    got = O.rope(x, np.array([3]), 100.0)[0, 0]
    assert np.allclose(got, [0.0, math.cos(0.3), 0.0, math.sin(0.3)])


def test_rope_relative_position_and_norm():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((1, 1, 16))
    k = rng.standard_normal((1, 1, 16))
    def dot(m, n):
        return float((O.rope(q, np.array([m]), 10000.0) * O.rope(k, np.array([n]), 10000.0)).sum())
    assert np.isclose(dot(7, 3), dot(104, 100))
    assert np.isclose(dot(0, 0), float((q * k).sum()))
    assert not np.isclose(dot(7, 3), dot(7, 4))
    assert np.isclose(np.linalg.norm(O.rope(q, np.array([9]), 10000.0)), np.linalg.norm(q))


def test_rope_against_complex_multiplication():
    rng = np.random.default_rng(1)
    n, H, d = 4, 3, 8
    x = rng.standard_normal((n, H, d))
    pos = np.array([0, 2, 5, 11])
    zc = x[..., : d // 2] + 1j * x[..., d // 2:]
    ang = pos[:, None] * (10000.0 ** (-2.0 * np.arange(d // 2) / d))[None, :]
    zr = zc * np.exp(1j * ang)[:, None, :]
    ref = np.concatenate([zr.real, zr.imag], -1)
    assert np.allclose(O.rope(x, pos, 10000.0), ref)


def test_attention_against_scalar_loops():
    rng = np.random.default_rng(2)
    P, H, d = 6, 2, 4
    K = rng.standard_normal((P, H, d))
    V = rng.standard_normal((P, H, d))
    q = rng.standard_normal((3, H, d))
    pos = np.array([1, 3, 5])
    got = O.causal_attention(q, pos, K, V)
    for i in range(3):
        for hd in range(H):
            sc = []
            for j in range(pos[i] + 1):
                sc.append(sum(q[i, hd, t] * K[j, hd, t] for t in range(d)) / math.sqrt(d))
            m = max(sc)
            w = [math.exp(s - m) for s in sc]
            tot = sum(w)
            for t in range(d):
                ref = sum(w[j] / tot * V[j, hd, t] for j in range(len(sc)))
                assert math.isclose(got[i, hd, t], ref, rel_tol=1e-12, abs_tol=1e-14)


def test_attention_against_library_sdpa():
    rng = np.random.default_rng(3)
    n, H, d = 9, 3, 8
    q, K, V = (rng.standard_normal((n, H, d)) for _ in range(3))
    got = O.causal_attention(q, np.arange(n), K, V)
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, K, V))
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_attention_special_cases():
    rng = np.random.default_rng(4)
    K = rng.standard_normal((5, 1, 4))
    V = rng.standard_normal((5, 1, 4))
    # position 0 sees only itself
    assert np.allclose(O.causal_attention(rng.standard_normal((1, 1, 4)), np.array([0]), K, V)[0, 0], V[0, 0])
    # a zero query averages the visible values
    assert np.allclose(O.causal_attention(np.zeros((1, 1, 4)), np.array([3]), K, V)[0, 0], V[:4, 0].mean(0))
    # entries beyond the row's position are never read
    K2, V2 = K.copy(), V.copy()
    K2[4] += 100.0
    V2[4] -= 100.0
    qq = rng.standard_normal((1, 1, 4))
    assert np.array_equal(O.causal_attention(qq, np.array([3]), K, V), O.causal_attention(qq, np.array([3]), K2, V2))


# ------------------------------------------------------------------ whole layer / model
SMALL = S.ModelShape(vocab=11, hidden=8, n_heads=2, head_dim=4, mlp=6, n_prelude=1, n_core=2, n_coda=1,
                     dtype="f32")


def _scalar_layer(w, name, x, pos, ck, cv, H, d, base, eps):
    """Pre-norm layer written with Python scalars only (brute force for tiny shapes)."""
    n, h = len(x), len(x[0])
    Fm = len(w[name + ".wg"])
    def norm(row, g):
        ms = sum(v * v for v in row) / h
        return [v / math.sqrt(ms + eps) * g[i] for i, v in enumerate(row)]
    def lin(W, row):
        return [sum(W[o][i] * row[i] for i in range(len(row))) for o in range(len(W))]
    def rot(vec, p):
        out = list(vec)
        for i in range(d // 2):
            a = p * base ** (-2.0 * i / d)
            out[i] = vec[i] * math.cos(a) - vec[i + d // 2] * math.sin(a)
            out[i + d // 2] = vec[i + d // 2] * math.cos(a) + vec[i] * math.sin(a)
        return out
    qs = []
    for r_ in range(n):
        qkv = lin(w[name + ".wqkv"], norm(x[r_], w[name + ".g1"]))
        qrow = []
        for hd in range(H):
            qrow.append(rot(qkv[hd * d:(hd + 1) * d], pos[r_]))
            ck[pos[r_]][hd] = rot(qkv[h + hd * d: h + (hd + 1) * d], pos[r_])
            cv[pos[r_]][hd] = qkv[2 * h + hd * d: 2 * h + (hd + 1) * d]
        qs.append(qrow)
    out = []
    for r_ in range(n):
        att = []
        for hd in range(H):
            sc = [sum(qs[r_][hd][t] * ck[j][hd][t] for t in range(d)) / math.sqrt(d) for j in range(pos[r_] + 1)]
            m = max(sc)
            e = [math.exp(s - m) for s in sc]
            z = sum(e)
            att += [sum(e[j] / z * cv[j][hd][t] for j in range(len(sc))) for t in range(d)]
        y = [a + b for a, b in zip(x[r_], lin(w[name + ".wo"], att))]
        nb = norm(y, w[name + ".g2"])
        g = lin(w[name + ".wg"], nb)
        u = lin(w[name + ".wu"], nb)
        act = [gi / (1 + math.exp(-gi)) * ui for gi, ui in zip(g, u)]
        assert len(act) == Fm
        out.append([a + b for a, b in zip(y, lin(w[name + ".wd"], act))])
    return out


def test_layer_against_scalar_brute_force():
    w = S.make_weights(SMALL, 3, std=0.5, gain_jitter=0.2)
    m = O.RecurrentDepthLM(SMALL, w)
    cache = m.new_cache(8)
    rng = np.random.default_rng(5)
    # warm the cache at positions 0..2, then run rows at 3,4 (a window against a cache)
    x0 = rng.standard_normal((3, 8))
    x1 = rng.standard_normal((2, 8))
    wl = {k: v.astype(np.float64).tolist() for k, v in w.items()}
    ck = [[None] * 2 for _ in range(8)]
    cv = [[None] * 2 for _ in range(8)]
    ref0 = _scalar_layer(wl, "R1", x0.tolist(), [0, 1, 2], ck, cv, 2, 4, 10000.0, 1e-6)
    ref1 = _scalar_layer(wl, "R1", x1.tolist(), [3, 4], ck, cv, 2, 4, 10000.0, 1e-6)
    got0 = m.layer("R1", x0, np.array([0, 1, 2]), cache)
    got1 = m.layer("R1", x1, np.array([3, 4]), cache)
    assert np.allclose(got0, ref0, rtol=1e-10, atol=1e-12)
    assert np.allclose(got1, ref1, rtol=1e-10, atol=1e-12)


def _torch_forward(shape, w, tokens, s0, r):
    """Independent whole-model forward with library ops (linear, rms_norm, SDPA, silu) for the
    case that has a plain definition: all positions processed together from position 0."""
    tw = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    h, H, d = shape.hidden, shape.n_heads, shape.head_dim
    n = len(tokens)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * (shape.rope_base ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d))[None]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    def rope(t):
        c = torch.complex(t[..., : d // 2], t[..., d // 2:]) * rot
        return torch.cat([c.real, c.imag], -1)
    def layer(name, x):
        a = F.rms_norm(x, (h,), tw[name + ".g1"], eps=shape.rms_eps)
        q, k, v = F.linear(a, tw[name + ".wqkv"]).view(n, 3, H, d).unbind(1)
        o = F.scaled_dot_product_attention(rope(q).transpose(0, 1)[None], rope(k).transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True)[0].transpose(0, 1).reshape(n, h)
        x = x + F.linear(o, tw[name + ".wo"])
        b = F.rms_norm(x, (h,), tw[name + ".g2"], eps=shape.rms_eps)
        return x + F.linear(F.silu(F.linear(b, tw[name + ".wg"])) * F.linear(b, tw[name + ".wu"]), tw[name + ".wd"])
    x = tw["emb"][torch.as_tensor(tokens, dtype=torch.long)] * shape.emb_scale
    for i in range(shape.n_prelude):
        x = layer(f"P{i}", x)
    e, s = x, torch.from_numpy(s0)
    for _ in range(r):
        x = F.linear(torch.cat([e, s], -1), tw["wa"])
        for i in range(shape.n_core):
            x = layer(f"R{i}", x)
        s = F.rms_norm(x, (h,), tw["gf"], eps=shape.rms_eps)
    x = s
    for i in range(shape.n_coda):
        x = layer(f"C{i}", x)
    return s.numpy(), F.linear(F.rms_norm(x, (h,), tw["gout"], eps=shape.rms_eps), tw["emb"]).numpy()


@pytest.mark.parametrize("shape", [SMALL, S.reduced(S.TINY, hidden=64, n_heads=2, head_dim=32, mlp=96, vocab=50)])
def test_model_against_library_forward(shape):
    w = S.make_weights(shape, 9, std=0.3, gain_jitter=0.2)
    m = O.RecurrentDepthLM(shape, w)
    tokens = S.make_prompt(shape.vocab, 7, 2)
    cache = m.new_cache(7)
    pos = np.arange(7)
    s0 = np.stack([O.init_state(shape.hidden, p, 0, 1.0, 3) for p in pos])
    e = m.prelude(tokens, pos, cache)
    s = s0
    for _ in range(3):
        s = m.core(e, s, pos, cache)
    logits = m.coda(s, pos, cache)
    ref_s, ref_logits = _torch_forward(shape, w, tokens, s0, 3)
    assert np.allclose(s, ref_s, rtol=1e-9, atol=1e-11)
    assert np.allclose(logits, ref_logits, rtol=1e-9, atol=1e-11)
    # prefill() is the same computation: its returned states must equal them
    cache2 = m.new_cache(7)
    s_pf = m.prefill(tokens, 3, 1.0, 3, 0, cache2)
    assert np.array_equal(s_pf, s)
    for name in cache.k:
        assert np.array_equal(cache.k[name], cache2.k[name])
        assert np.array_equal(cache.v[name], cache2.v[name])


def test_incremental_window_equals_full_pass():
    """Rows processed in two batches against the cache give what one batch over all rows gives
    (the cache is the only coupling between positions)."""
    shape = SMALL
    w = S.make_weights(shape, 4, std=0.4)
    m = O.RecurrentDepthLM(shape, w)
    rng = np.random.default_rng(7)
    x = rng.standard_normal((6, 8))
    c1, c2 = m.new_cache(6), m.new_cache(6)
    full = m.layer("P0", x, np.arange(6), c1)
    a = m.layer("P0", x[:4], np.arange(4), c2)
    b = m.layer("P0", x[4:], np.arange(4, 6), c2)
    assert np.allclose(np.concatenate([a, b]), full, rtol=1e-12, atol=1e-13)


def test_causality_of_every_block():
    """Sec. 1: information moves strictly left to right -- changing a later token or state leaves
    every earlier row bit-identical."""
    shape = SMALL
    w = S.make_weights(shape, 5, std=0.4)
    m = O.RecurrentDepthLM(shape, w)
    tokens = S.make_prompt(shape.vocab, 6, 1)
    pos = np.arange(6)
    s0 = np.stack([O.init_state(8, p, 0, 1.0, 1) for p in pos])
    def run(tok, st):
        c = m.new_cache(6)
        e = m.prelude(tok, pos, c)
        s = m.core(e, st, pos, c)
        return e, s, m.coda(s, pos, c)
    base = run(tokens, s0)
    tok2 = tokens.copy()
    tok2[4] = (tok2[4] + 1) % shape.vocab
    st2 = s0.copy()
    st2[4] += 1.0
    for other, first in ((run(tok2, s0), 0), (run(tokens, st2), 1)):   # a state change cannot reach e
        for a, b in list(zip(base, other))[first:]:
            assert np.array_equal(a[:4], b[:4])
            assert not np.allclose(a[4:], b[4:])


def test_kv_cache_size_is_that_of_a_fixed_depth_model():
    """Footnote of Sec. 3.2: the shared cache needs what a fixed-depth model needs: one K and one V
    row per layer and position, whatever the number of recurrences."""
    shape = S.TINY
    m = O.RecurrentDepthLM(shape, S.make_weights(shape, 1))
    cache = m.new_cache(24)
    expect = shape.n_layers * 2 * 24 * shape.hidden * 8
    assert cache.nbytes() == expect
    m.prefill(S.make_prompt(256, 10, 1), 5, 1.0, 1, 0, cache)
    assert cache.nbytes() == expect


# ------------------------------------------------------------------ Eq. 3
def test_delta_closed_forms():
    z = np.array([[3.0, 4.0], [1.0, 0.0], [2.0, 2.0], [0.0, 0.0]])
    zp = np.array([[0.0, 0.0], [1.0, 0.0], [2.0, 0.0], [1.0, 0.0]])
    d = O.delta(z, zp)
    assert np.allclose(d[:3], [1.0, 0.0, 2.0 / math.sqrt(8.0)])
    assert not np.isfinite(d[3])
    rng = np.random.default_rng(0)
    a, b = rng.standard_normal((2, 5, 33))
    assert np.allclose(O.delta(a, b), np.linalg.norm(a - b, axis=1) / np.linalg.norm(a, axis=1))


def test_k_star_is_the_longest_prefix():
    assert O.k_star([True, True, False, True]) == 2          # a gap stops the prefix
    assert O.k_star([False, True, True]) == 0
    assert O.k_star([True, True, True]) == 3
    assert O.k_star([]) == 0
    f = O.freezable_flags(np.array([0.5, 1e-4, np.nan, np.inf, 1e-4]), [9, 1, 1, 1, 1], 1, 1e-3, 9)
    assert f == [True, True, False, False, True]              # cap, converged, nan, inf, converged
    assert O.freezable_flags(np.array([np.nan]), [4], 2, 1e-3, 8) == [True]   # the cap still applies


# ---------------------------------------------------------------------------------------------
# Top-p (nucleus) filter of Sample

def test_nucleus_is_the_smallest_descending_prefix_reaching_top_p():
    rng = np.random.default_rng(3)
    for trial in range(50):
        v = int(rng.integers(2, 9))
        logits = rng.standard_normal(v) * 2.0
        T, top_p = float(rng.uniform(0.2, 1.5)), float(rng.uniform(0.05, 0.99))
        keep = O.nucleus(logits, T, top_p)
        p = np.exp(logits / T - np.max(logits / T))
        p /= p.sum()
        # brute force: over all subsets, the kept one is closed under "at least as probable as a
        # member", reaches top_p, and dropping its least probable member falls below top_p
        assert keep.any()
        assert p[keep].min() >= p[~keep].max() if (~keep).any() else True
        assert p[keep].sum() >= top_p - 1e-12
        least = np.argmin(np.where(keep, p, np.inf))
        assert p[keep].sum() - p[least] < top_p + 1e-12
    assert O.nucleus(np.array([0.0, 1.0, 2.0]), 1.0, 1.0).all()
    assert O.nucleus(np.array([0.0, 1.0, 2.0]), 1.0, 0.0).all()          # off
    assert list(O.nucleus(np.array([0.0, 1.0, 5.0]), 1.0, 0.5)) == [False, False, True]
    assert list(O.nucleus(np.array([1.0, 1.0, -9.0]), 1.0, 0.4)) == [True, True, False]   # equal probabilities stay together


def test_top_p_sampling_draws_from_the_renormalised_nucleus():
    """Gumbel-max restricted to the nucleus is sampling from the truncated, renormalised softmax
    (chi-square on a small vocabulary), and never leaves the nucleus."""
    logits = np.array([2.0, 1.0, 0.5, 0.0, -1.0, -3.0])
    T, top_p = 0.7, 0.97
    keep = O.nucleus(logits, T, top_p)
    p = np.exp(logits / T)
    p = np.where(keep, p, 0.0)
    p /= p.sum()
    n = 4000
    counts = np.zeros(6)
    for step in range(n):
        counts[O.sample(logits, T, 3, 1, step, 11, top_p)] += 1
    assert counts[~keep].sum() == 0
    chi2 = np.sum((counts[keep] - n * p[keep]) ** 2 / (n * p[keep]))
    assert chi2 < 16.27                                  # chi-square 0.999 quantile, 3 degrees of freedom
    assert keep.sum() == 4
    # top_p = 1 is plain temperature sampling, a tiny top_p is greedy
    for step in range(20):
        assert O.sample(logits, T, 3, 1, step, 11, 1.0) == O.sample(logits, T, 3, 1, step, 11)
        assert O.sample(logits, T, 3, 1, step, 11, 1e-6) == 0
