"""Error paths and repeatability of the HIP path that need a device but no oracle arithmetic:
status codes that come back from inside a step, the caller-owned workspace, and bitwise
repeatability of the hand-overs between workgroups with several sequences in a step."""
import numpy as np
import pytest

import synth_inputs as S
from oracle import rdlm_oracle as O
from gpu_util import SMALL_BF16_D64, SMALL_BF16_D96, make_pair, rel_l2

pytestmark = pytest.mark.gpu


def test_a_launch_shape_without_a_kernel_is_reported_by_the_call():
    """A projection whose launch shape has no kernel instance makes the ABI call return
    RDLM_EINVAL (nothing of that projection is launched) instead of carrying on with stale buffers."""
    import torch
    import paper_2510_14961_amd as R
    shape = SMALL_BF16_D64
    ctx, m, _ = make_pair(shape, max_positions=192, max_rows=128)
    n = 70                                                   # three row tiles: the several-tile plans
    e = torch.from_numpy(S.make_rows(n, shape.hidden, 3)).cuda()
    z = torch.from_numpy(S.make_rows(n, shape.hidden, 4)).cuda()
    ctx.core_step([0], [0], [n], e, z.clone())               # fine with the default shapes
    ctx.set_tuning("planr_gu", "3,1,4,4,1")                  # three row tiles per workgroup: no such instance
    with pytest.raises(R.RdlmError) as ei:
        ctx.core_step([0], [0], [n], e, z.clone())
    assert ei.value.status == R.STATUS["EINVAL"]
    # inside a sampler step the failure also ends the sampler
    prompt = S.make_prompt(shape.vocab, 8, 1)
    ctx.set_tokens(0, prompt)
    ctx.prefill(0, 7, 2, 1.0, 1)
    ctx.sampler_begin(1, n_new=4, r_inner=1, r_total=40, headway=3)
    with pytest.raises(R.RdlmError) as ei:
        for _ in range(30):                                  # the window reaches a second row tile at step 12
            ctx.sample_step()
    assert ei.value.status == R.STATUS["EINVAL"]
    with pytest.raises(R.RdlmError, match="out of order"):
        ctx.sample_step()
    ctx.set_tuning("planr_gu", "")                           # default shapes again
    ctx.core_step([0], [0], [n], e, z.clone())
    with pytest.raises(R.RdlmError, match="invalid"):
        ctx.set_tuning("no_such_knob", "1")
    torch.cuda.synchronize()
    ctx.close()


def test_a_non_finite_latent_is_reported_not_frozen():
    """Eq. 3 on a latent that is not finite: delta_i is NaN, the state is never frozen by the exit
    rule (only by the cap), and rdlm_generate says so with RDLM_ENUMERIC."""
    import torch
    import paper_2510_14961_amd as R
    shape = S.TINY
    w = S.make_weights(shape, 1)
    w["gf"] = w["gf"].copy()
    w["gf"][5] = np.nan                                      # the closing norm of R writes NaN into z[:, 5]
    ctx = R.Context(shape, R.upload_weights(shape, w), 1, 96, 32)
    prompt = S.make_prompt(shape.vocab, 8, 1)
    ctx.set_tokens(0, prompt)
    ctx.prefill(0, 7, 2, 1.0, 1)
    ctx.sampler_begin(1, n_new=4, r_inner=1, r_total=6, adaptive=True, eps=0.5, w_max=4)
    with pytest.raises(R.RdlmError) as ei:
        ctx.generate(200)
    assert ei.value.status == R.STATUS["ENUMERIC"]
    active, nonfinite = ctx.sampler_status()
    assert nonfinite
    ctx.sample_step()                                        # the sampler itself goes on (cap-bound)
    cnt = ctx.read_counts(0, 7, 1)
    assert cnt[0] >= 1
    # a healthy run reports nothing
    ctx.close()
    ctx, m, _ = make_pair(shape, max_positions=96, max_rows=32)
    ctx.set_tokens(0, prompt)
    ctx.prefill(0, 7, 2, 1.0, 1)
    ctx.sampler_begin(1, n_new=4, r_inner=1, r_total=6, adaptive=True, eps=0.5, w_max=4)
    steps = ctx.generate(200)
    assert steps > 0 and ctx.sampler_status() == (0, False)
    # steps_out counts the steps of the call: a second call after the end takes none that matter
    ctx.close()


def test_generate_reports_the_steps_of_the_call():
    shape = S.TINY
    ctx, m, _ = make_pair(shape, max_positions=96, max_rows=32)
    prompt = S.make_prompt(shape.vocab, 8, 1)
    ref = O.generate_diffusion_forcing(m, prompt, 10, 1, 4)
    ctx.set_tokens(0, prompt)
    ctx.prefill(0, 7, 4, 1.0, 1)
    ctx.sampler_begin(1, n_new=10, r_inner=1, r_total=4)
    first = ctx.generate(5)                                   # stops at its step limit
    rest = ctx.generate(1000)
    assert first == 5 and first + rest == ref.steps
    assert np.array_equal(ctx.read_tokens(0)[0][:18], ref.tokens)
    ctx.close()


def test_caller_owned_workspace_gives_the_same_run():
    import torch
    import paper_2510_14961_amd as R
    shape = SMALL_BF16_D96
    w = S.make_weights(shape, 2, gain_jitter=0.1)
    prompt = S.make_prompt(shape.vocab, 20, 2)
    need = R.workspace_bytes(shape, 1, 64)
    assert need > 0
    outs = []
    for own in (False, True):
        ws = torch.full((need + 256,), 0x5A, dtype=torch.uint8, device="cuda") if own else None   # dirty on purpose
        if own:
            off = (-ws.data_ptr()) % 256
            ws = ws[off: off + need]
        ctx = R.Context(shape, R.upload_weights(shape, w), 1, 128, 64, workspace=ws)
        ctx.set_tokens(0, prompt)
        ctx.prefill(0, 19, 3, 1.0, 4)
        ctx.sampler_begin(1, n_new=12, r_inner=1, r_total=5, temperature=1.0, seed=9)
        ctx.generate(100)
        outs.append((ctx.read_tokens(0)[0][:32].copy(), ctx.read_states(0, 19, 12).copy()))
        ctx.close()
    assert np.array_equal(outs[0][0], outs[1][0])
    assert np.array_equal(outs[0][1], outs[1][1])
    too_small = torch.zeros(need - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(R.RdlmError) as ei:
        R.Context(shape, R.upload_weights(shape, w), 1, 128, 64, workspace=too_small)
    assert ei.value.status == R.STATUS["ECAPACITY"]


def test_multi_sequence_steps_are_bitwise_repeatable():
    """Four sequences, adaptive exit, temperature sampling, windows that span two row tiles: the
    step-end bookkeeping (one workgroup per sequence, tile list built by the last to arrive), the
    folding GEMMs and the KV-split merges all hand data between workgroups.  Two runs from the same
    seeds must agree bit for bit; a hand-over read too early would show the previous step's values."""
    shape = SMALL_BF16_D64
    ctx, m, _ = make_pair(shape, seed=4, max_seqs=4, max_positions=160, max_rows=4 * 64)
    prompts = [S.make_prompt(shape.vocab, L, 5, seq=q) for q, L in enumerate((20, 9, 33, 14))]
    spec = dict(n_new=24, r_inner=1, r_total=40, eps=0.02, w_max=40, adaptive=True, temperature=1.0, seed=3)
    outs = []
    for _ in range(2):
        for q, p in enumerate(prompts):
            ctx.set_tokens(q, p)
            ctx.prefill(q, len(p) - 1, 3, 1.0, 3)
        ctx.sampler_begin(4, **spec)
        steps = ctx.generate(2000)
        run = [steps]
        for q, p in enumerate(prompts):
            toks, nf = ctx.read_tokens(q)
            run += [toks.copy(), nf, ctx.read_states(q, len(p) - 1, 24).copy(), ctx.read_counts(q, len(p) - 1, 24).copy()]
        outs.append(run)
    for a, b in zip(*outs):
        assert np.array_equal(a, b)
    ctx.close()
