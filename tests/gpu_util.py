"""Shared helpers of the GPU parity tests: build both sides from the same seeded inputs."""
from __future__ import annotations

import numpy as np

import synth_inputs as S
from oracle import rdlm_oracle as O

# small shapes that still span several MFMA tiles and ragged tails
SMALL_BF16_D64 = S.ModelShape(vocab=512, hidden=256, n_heads=4, head_dim=64, mlp=512,
                              n_prelude=1, n_core=2, n_coda=1, dtype="bf16")
SMALL_BF16_D96 = S.ModelShape(vocab=384, hidden=288, n_heads=3, head_dim=96, mlp=608,
                              n_prelude=1, n_core=2, n_coda=1, dtype="bf16")
SMALL_BF16_D32 = S.ModelShape(vocab=256, hidden=160, n_heads=5, head_dim=32, mlp=224,
                              n_prelude=1, n_core=1, n_coda=1, dtype="bf16")
SMALL_BF16_D128 = S.ModelShape(vocab=256, hidden=256, n_heads=2, head_dim=128, mlp=384,
                               n_prelude=1, n_core=2, n_coda=1, dtype="bf16")


def rel_l2(a, b) -> float:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def tol_latent(shape) -> float:
    """Bound of the benchmark spec: rel-L2 1e-4 in fp32, 2e-2 in bf16."""
    return 1e-4 if shape.dtype == "f32" else 2e-2


def assert_rows_close(got, ref, tol, what=""):
    """Row-wise comparison of a [n, width] result with the oracle's: the whole matrix and every single
    row within the rel-L2 bound, and no single element further off than 10 x tol x rms(ref) -- one
    wrong element of ordinary size (1 rms) in an otherwise exact matrix fails the last bound, which
    a norm over the matrix would not notice.  Returns (worst row rel-L2, worst element / rms)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    whole = rel_l2(got, ref)
    rows = max(rel_l2(got[i], ref[i]) for i in range(got.shape[0]))
    rms = float(np.sqrt(np.mean(ref * ref)))
    worst = float(np.max(np.abs(got - ref))) / max(rms, 1e-300)
    assert whole < tol, (what, "whole matrix", whole)
    assert rows < tol, (what, "worst row", rows)
    assert worst < 10 * tol, (what, "worst element / rms", worst)
    return rows, worst


# Token tolerance tau (score units) of the tie-aware check, per shape family: four times the largest
# logit error measured once for that family on MI355X (bf16 operands, float32 accumulation), as
# constants -- not derived from the run under test.  Logit standard deviation: 0.02 sqrt(h) (unit-RMS
# final hidden state against N(0, 0.02) embedding rows).
#   small bf16 test shapes (h 160..288, vocab <= 512): measured max |logit error| 0.0024 for the coda
#                                                       alone, about twice that through P, R and C
#   workload 2 shape (h 1024, vocab 32768):             measured 0.0075 (largest near-tie gap seen in
#                                                       4216 drafted tokens: 0.0069)
#   3.5B shape (h 5280, vocab 65536):                   measured 0.167 behind a prefix cache each side
#                                                       filled itself
# (A legitimate near-tie has a gap of at most twice the logit error: the GPU preferred t' to the
# oracle's best b, so oracle(b) - oracle(t') <= err(b) + err(t').)
TAU_SMALL_BF16 = 0.02
TAU_MID_BF16 = 0.03
TAU_BIG_BF16 = 0.7
TAU_F32 = 1e-4


def tau_for(shape) -> float:
    if shape.dtype == "f32":
        return TAU_F32
    return TAU_SMALL_BF16 if shape.hidden < 1024 else TAU_MID_BF16 if shape.hidden < 4096 else TAU_BIG_BF16


def make_pair(shape, seed=1, max_seqs=1, max_positions=128, max_rows=64, gain_jitter=0.1, emb_mul=1.0, **ctx_kw):
    """(Context on the GPU, oracle model, numpy weights) from one weight draw."""
    import torch
    import paper_2510_14961_amd as R
    w = S.make_weights(shape, seed, gain_jitter=gain_jitter)
    if emb_mul != 1.0:
        w["emb"] = w["emb"] * np.float32(emb_mul)
        if shape.dtype == "bf16":
            w["emb"] = S.bf16_bits_to_f32(S.f32_to_bf16_bits(w["emb"]))
    dev = R.upload_weights(shape, w)
    ctx = R.Context(shape, dev, max_seqs, max_positions, max_rows, **ctx_kw)
    del dev
    torch.cuda.synchronize()
    return ctx, O.RecurrentDepthLM(shape, w), w


LAST_TIE_GAP = [0.0]     # largest gap among the near-ties the last calls accepted (reported by the tests)


def tie_aware_token_check(gpu_tokens, oracle_scores, tau):
    """A GPU token is accepted iff the oracle's score of it is within tau of the oracle's best.
    Returns (number of exact matches, number accepted as near-ties); raises on a real mismatch."""
    exact = ties = 0
    for i, t in enumerate(gpu_tokens):
        sc = oracle_scores[i]
        best = int(np.argmax(sc))
        if int(t) == best:
            exact += 1
        else:
            gap = float(sc[best] - sc[int(t)])
            assert gap <= tau, f"row {i}: GPU token {int(t)} scores {gap:.4g} below the oracle's best {best} (tau {tau:.3g})"
            LAST_TIE_GAP[0] = max(LAST_TIE_GAP[0], gap)
            ties += 1
    return exact, ties


def top_p_token_check(gpu_tokens, logits, temperature, top_p, positions, seq, step, seed, tau=1e-5, slack=1e-4):
    """Tokens sampled with a top-p filter, judged on the logits the GPU itself returned (float32
    values, exact in the oracle's float64), so both sides decide on the same numbers.  A token
    is accepted iff it lies in the oracle's top-p set and its Gumbel score is within tau of the
    best in that set -- for top_p itself or top_p (1 +- slack): the GPU sums probabilities in
    float32, which can move a token sitting exactly on the boundary.
    Returns (matches at the nominal top_p, tokens accepted otherwise); raises on a mismatch."""
    exact = other = 0
    for i, t in enumerate(gpu_tokens):
        t = int(t)
        lg = np.asarray(logits[i], dtype=np.float64)
        if t == O.sample(lg, temperature, int(positions[i]), seq, step, seed, top_p):
            exact += 1
            continue
        score = lg / temperature + O.gumbel_noise(lg.shape[0], int(positions[i]), seq, step, seed)
        ok = False
        for tp in (top_p, top_p * (1 - slack), min(top_p * (1 + slack), 1 - 1e-12)):
            keep = O.nucleus(lg, temperature, tp)
            ok = ok or (keep[t] and float(np.max(score[keep]) - score[t]) <= tau)
        assert ok, f"row {i}: GPU token {t} is not the oracle's top-p sample (top_p {top_p})"
        other += 1
    return exact, other


def teacher_forced_sampler_run(ctx, m, shape, prompt, r, n_new, seed, tol, max_positions):
    """Drive the GPU sampler (fixed exit, r' = 1) step by step; before each step read the GPU's own
    inputs (tokens, in-flight states), run the same step in the oracle from them, and compare the
    new latents, the deltas' count and the drafted tokens (tie-aware).  Returns (exact, ties)."""
    L = len(prompt)
    ctx.set_tokens(0, prompt)
    ctx.prefill(0, L - 1, r, 1.0, seed)
    cache = m.new_cache(max_positions)
    m.prefill(prompt[: L - 1], r, 1.0, seed, 0, cache)
    ctx.sampler_begin(1, n_new=n_new, r_inner=1, r_total=r, seed=seed)
    win_pos0, win_n, n_frozen = L - 1, 1, L
    total_exact = total_ties = 0
    for t in range(1, n_new + r):
        y_before, _ = ctx.read_tokens(0)
        z_before = ctx.read_states(0, win_pos0, win_n).astype(np.float64)
        ctx.sample_step()
        pos = np.arange(win_pos0, win_pos0 + win_n)
        e = m.prelude(y_before[pos], pos, cache)
        z_ref = m.core(e, z_before, pos, cache)
        logits = m.coda(z_ref, pos, cache)
        z_gpu = ctx.read_states(0, win_pos0, win_n)
        assert_rows_close(z_gpu, z_ref, tol, f"step {t}")
        d_gpu = ctx.read_deltas(0)
        assert len(d_gpu) == win_n
        d_ref = O.delta(z_ref, z_before)
        assert np.max(np.abs(d_gpu - d_ref)) < 4 * tol, t
        y_after, nf = ctx.read_tokens(0)
        ex, ti = tie_aware_token_check(y_after[pos + 1], logits, tau=tau_for(shape))
        total_exact += ex
        total_ties += ti
        k = 1 if t >= r else 0                      # the oldest state has had r recurrences
        assert nf == n_frozen + k
        n_frozen += k
        win_pos0 += k
        win_n = win_n - k + (1 if n_frozen - L < n_new else 0)
        if n_frozen - L >= n_new:
            break
    return total_exact, total_ties


def teacher_forced_step(ctx, m, shape, spec, n_seqs, t, tol=None, tau=None, label=""):
    """Sampler step number `t` (1-based, counted from sampler_begin) of a running GPU sampler against
    one oracle step started from the GPU's own inputs: for every unfinished sequence the tokens, the
    in-flight states, z_prev, the step counters and the K/V entries of every layer up to the end of
    the window are read back, the GPU takes the step, and the oracle recomputes it (P, r' x R, C,
    Sample, delta_i, k*) from those inputs.  Compared per sequence: the new latents row by row, delta_i
    (within what the latent error of the row allows), the freeze count
    k* (from the GPU's own delta_i, so that both sides take the decision on the same numbers; exact),
    the drafted tokens (tie-aware, fixed tau) and the window the bookkeeping leaves behind (exact).
    spec: the keyword arguments given to sampler_begin.  Returns a dict of what was measured."""
    tol = tol_latent(shape) if tol is None else tol
    tau = tau_for(shape) if tau is None else tau
    r_inner, cap = spec["r_inner"], spec["r_total"]
    adaptive = bool(spec.get("adaptive", False))
    eps = float(spec.get("eps", 0.0)) if adaptive else 0.0
    headway = spec.get("headway", 1)
    wave = -(-cap // r_inner)
    w_max = spec.get("w_max", 0) if (adaptive and spec.get("w_max", 0) > 0) else wave * headway
    temp, seed = float(spec.get("temperature", 0.0)), spec.get("seed", 1)
    layers = m.P_layers + m.R_layers + m.C_layers
    pre = []
    for q in range(n_seqs):
        p0, n, done = ctx.read_window(q)
        if done or n == 0:
            pre.append(None)
            continue
        y, nf = ctx.read_tokens(q)
        cache = m.new_cache(p0 + n)
        for li, name in enumerate(layers):
            k, v = ctx.read_kv(li, q, 0, p0 + n)
            cache.k[name][:] = k
            cache.v[name][:] = v
        pre.append(dict(p0=p0, n=n, y=y.copy(), nf=nf, z=ctx.read_states(q, p0, n).astype(np.float64),
                        zp=ctx.read_prev_states(q, p0, n).astype(np.float64), cnt=ctx.read_counts(q, p0, n).copy(),
                        cache=cache))
    ctx.sample_step()
    out = dict(rows=0, worst_row=0.0, worst_delta=0.0, exact=0, ties=0, frozen=0, max_keys=0)
    for q in range(n_seqs):
        s = pre[q]
        if s is None:
            continue
        p0, n = s["p0"], s["n"]
        pos = np.arange(p0, p0 + n)
        e = m.prelude(s["y"][pos], pos, s["cache"])
        z1 = s["z"]
        for _ in range(r_inner):
            z1 = m.core(e, z1, pos, s["cache"])
        logits = m.coda(z1, pos, s["cache"])
        z_gpu = ctx.read_states(q, p0, n)
        rows, _ = assert_rows_close(z_gpu, z1, tol, f"{label} step {t} seq {q}: latents")
        d_gpu = ctx.read_deltas(q).astype(np.float64)
        assert len(d_gpu) == n, (label, t, q)
        d_ref = O.delta(z1, s["zp"])
        row_err = np.array([rel_l2(z_gpu[i], z1[i]) for i in range(n)])
        d_err = np.abs(d_gpu - d_ref)
        # with ||a - b|| = rho ||b||:  delta_a <= (delta_b + rho) / (1 - rho), and the same the other way round
        assert np.all(d_err <= 1.1 * (1.0 + d_ref) * row_err + 1e-5), (label, t, q, float(np.max(d_err)),
                                                                       float(np.max(row_err)))
        cnt_after = s["cnt"] + 1
        assert np.array_equal(ctx.read_counts(q, p0, n), cnt_after), (label, t, q)
        k = O.k_star(O.freezable_flags(d_gpu, cnt_after, r_inner, eps, cap))
        y_after, nf_after = ctx.read_tokens(q)
        assert nf_after == s["nf"] + k, (label, t, q, nf_after, s["nf"], k)
        scores = logits if temp == 0.0 else np.stack(
            [logits[i] / temp + O.gumbel_noise(shape.vocab, int(pos[i]), q, t, seed) for i in range(n)])
        ex, ti = tie_aware_token_check(y_after[pos + 1], scores, tau)
        assert np.array_equal(y_after[: p0 + 1], s["y"][: p0 + 1]), (label, t, q, "frozen text changed")
        p0_after, n_after, done_after = ctx.read_window(q)
        if not done_after:
            left = n - k
            n_app = max(0, min(headway, w_max - left))
            assert n_after == left + n_app, (label, t, q, n_after, left, n_app)
            assert p0_after == (p0 + k if left > 0 else nf_after - 1), (label, t, q)
        out["rows"] += n
        out["worst_row"] = max(out["worst_row"], rows)
        out["worst_delta"] = max(out["worst_delta"], float(np.max(d_err)))
        out["exact"] += ex
        out["ties"] += ti
        out["frozen"] += k
        out["max_keys"] = max(out["max_keys"], p0 + n)
    return out

