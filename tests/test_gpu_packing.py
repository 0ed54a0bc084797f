"""GPU: rows of several sequences in one 32-row tile (App. "Larger batch sizes": many sequences with short
windows in one forward call).  Windows of up to 32 rows are packed one after the other into row tiles, so a
batch of short windows costs the matrix products one row tile instead of one per sequence; sequences never
interact, so each must still come out as the oracle's run of that sequence alone.
"""
import numpy as np
import pytest

import synth_inputs as S
from oracle import rdlm_oracle as O
from gpu_util import SMALL_BF16_D64, SMALL_BF16_D96, assert_rows_close, make_pair, rel_l2, teacher_forced_step, tol_latent

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def _begin(ctx, prompts, spec, r_prefill):
    for q, p in enumerate(prompts):
        ctx.set_tokens(q, p)
        ctx.prefill(q, len(p) - 1, r_prefill, spec.get("alpha", 1.0), spec.get("seed", 1))
    ctx.sampler_begin(len(prompts), **spec)


@pytest.mark.parametrize("temp,beta,eta", [(0.0, 0.0, 0.0), (0.9, 0.3, 0.1)])
def test_seven_short_windows_share_one_row_tile_fp32(temp, beta, eta):
    """Seven sequences, fixed exit with r = 4: 28 rows in steady state, one row tile.  Random draws (Gumbel,
    state noise, initial states) are keyed by each row's own sequence and position."""
    shape = S.TINY
    n_new, r = 9, 4
    ctx, m, _ = make_pair(shape, seed=3, max_seqs=7, max_positions=64, max_rows=224)
    prompts = [S.make_prompt(shape.vocab, 5 + 3 * q, 50 + q, seq=q) for q in range(7)]
    spec = dict(n_new=n_new, r_inner=1, r_total=r, temperature=temp, seed=11, beta=beta, eta=eta)
    _begin(ctx, prompts, spec, r)
    ctx.generate(1000)
    for q, p in enumerate(prompts):
        ref = O.generate_diffusion_forcing(m, p, n_new, 1, r, seq=q, temperature=temp, seed=11, beta=beta, eta=eta)
        toks, nf = ctx.read_tokens(q)
        assert nf == len(p) + n_new, q
        assert np.array_equal(toks[:nf], ref.tokens), q
        for pos, st in ref.final_states.items():
            assert rel_l2(ctx.read_states(q, pos, 1)[0], st) < 1e-4, (q, pos)
    ctx.close()


def test_long_and_short_windows_in_one_step_fp32():
    """One sequence whose window spans two row tiles (its own tiles, grouped attention) between short ones that
    are packed around it; adaptive exit, so the windows change size from step to step."""
    shape = S.TINY
    ctx, m, _ = make_pair(shape, seed=5, max_seqs=4, max_positions=128, max_rows=256)
    prompts = [S.make_prompt(shape.vocab, n, 60 + q, seq=q) for q, n in enumerate((7, 12, 9, 15))]
    spec = dict(n_new=30, r_inner=1, r_total=48, eps=0.02, w_max=40, headway=3, adaptive=True, temperature=0.6, seed=4)
    _begin(ctx, prompts, spec, 4)
    ctx.generate(2000)
    widest = 0
    for q, p in enumerate(prompts):
        ref = O.generate_diffusion_forcing_adaptive(m, p, 30, 1, 48, 0.02, 40, temperature=0.6, seed=4, seq=q, headway=3,
                                                    r_prefill=4)
        toks, nf = ctx.read_tokens(q)
        assert nf >= len(p) + 30, q
        assert np.array_equal(toks[: len(p) + 30], ref.tokens), q
        widest = max(widest, max(ref.window_sizes))
    assert widest > 32                                   # some window really needed two row tiles
    ctx.close()


@pytest.mark.parametrize("shape", [SMALL_BF16_D64, SMALL_BF16_D96], ids=["bf16_d64", "bf16_d96"])
def test_packed_rows_on_the_matrix_core_path(shape):
    """bf16 model: six sequences with windows of up to 6 rows in one or two row tiles.  The QKV product writes
    each row's K/V into its own sequence's cache, attention runs per sequence on rows that start anywhere in a
    tile, the LM head draws each row's Gumbel noise for its own (sequence, position): single steps recomputed
    by the oracle from the GPU's inputs, sequence by sequence."""
    ctx, m, _ = make_pair(shape, seed=4, max_seqs=6, max_positions=128, max_rows=192)
    prompts = [S.make_prompt(shape.vocab, 20 + 7 * q, 70 + q, seq=q) for q in range(6)]
    spec = dict(n_new=16, r_inner=1, r_total=6, seed=2)
    _begin(ctx, prompts, spec, 6)
    rows = 0
    for t in range(1, 13):
        out = teacher_forced_step(ctx, m, shape, spec, 6, t, label="packed")
        rows += out["rows"]
    assert rows == 6 * (1 + 2 + 3 + 4 + 5 + 6 * 7)
    ctx.close()


def test_ragged_core_step_packs_short_windows():
    """rdlm_core_step with windows of 3, 40, 7 and 12 rows: the 40-row window owns two row tiles, the others
    share one; against the oracle, sequence by sequence, and against the unpacked layout."""
    torch = _torch()
    shape = SMALL_BF16_D64
    ctx, m, _ = make_pair(shape, seed=6, max_seqs=4, max_positions=128, max_rows=128)
    rows = (3, 40, 7, 12)
    L = (30, 20, 41, 25)
    caches, es, zs, refs = [], [], [], []
    for q, (n, l) in enumerate(zip(rows, L)):
        tokens = S.make_prompt(shape.vocab, l + n, 80 + q, seq=q)
        ctx.set_tokens(q, tokens[:l])
        ctx.prefill(q, l, 2, 1.0, 5)
        cache = m.new_cache(128)
        m.prefill(tokens[:l], 2, 1.0, 5, q, cache)
        pos = np.arange(l, l + n)
        e = m.prelude(tokens[l:], pos, cache)
        z0 = np.stack([O.init_state(shape.hidden, p, q, 1.0, 5) for p in pos])
        refs.append(m.core(e, z0, pos, cache))
        es.append(e); zs.append(z0)
        # (the GPU's prelude caches for the window rows are not written here: the core step does not read them)
    e_dev = torch.from_numpy(np.concatenate(es).astype(np.float32)).cuda()
    got = {}
    for no_pack in ("0", "1"):
        ctx.set_tuning("no_pack", no_pack)
        z_dev = torch.from_numpy(np.concatenate(zs).astype(np.float32)).cuda()
        d = torch.zeros(sum(rows), device="cuda")
        ctx.core_step(list(range(4)), list(L), list(rows), e_dev, z_dev, 1, d)
        got[no_pack] = z_dev.cpu().numpy()
    off = 0
    for q, n in enumerate(rows):
        assert_rows_close(got["0"][off: off + n], refs[q], tol_latent(shape), f"packed, sequence {q}")
        assert_rows_close(got["1"][off: off + n], refs[q], tol_latent(shape), f"unpacked, sequence {q}")
        off += n
    ctx.close()
