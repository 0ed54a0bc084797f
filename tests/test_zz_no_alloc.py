"""rdlm_core_step_static -- the core step for callers that cannot allocate -- against rdlm_core_step
through the C ABI: same inputs, same cache prefix, two calls in a row, the second on a smaller
window; then the same on a second context (another model shape sharing the GPU's static array)."""
import numpy as np
import pytest

import synth_inputs as S
from oracle import rdlm_oracle as O
from gpu_util import SMALL_BF16_D96, assert_rows_close, make_pair, tol_latent

pytestmark = pytest.mark.gpu


def _pair_of_calls(ctx, m, shape, cases, seed):
    """For every (pos0, rows) case: rdlm_core_step on a copy of the inputs, then rdlm_core_step_static
    on another copy.  Both overwrite the same cache positions with the same values, so the second
    sees exactly the cache the first saw.  Returns nothing; asserts."""
    import torch
    h = shape.hidden
    for pos0, n in cases:
        e = torch.from_numpy(S.make_rows(n, h, seed + n, scale=2.0)).cuda()
        z0 = np.stack([O.init_state(h, pos0 + j, 0, 1.0, seed) for j in range(n)]).astype(np.float32)
        z_a, z_b = torch.from_numpy(z0).cuda(), torch.from_numpy(z0).cuda()
        d_a, d_b = torch.zeros(n, device="cuda"), torch.full((n,), -1.0, device="cuda")
        ctx.core_step([0], [pos0], [n], e, z_a, 2, d_a)
        ctx.core_step_static([0], [pos0], [n], e, z_b, 2, d_b)
        torch.cuda.synchronize()
        got, want = z_b.cpu().numpy(), z_a.cpu().numpy()
        # same kernels, same launch shapes, fixed summation orders: the bar is the latent tolerance,
        # the expectation is equality
        assert_rows_close(got, want, tol_latent(shape), f"static vs allocated, {n} rows at {pos0}")
        assert np.array_equal(got, want), (pos0, n, float(np.max(np.abs(got - want))))
        assert np.array_equal(d_b.cpu().numpy(), d_a.cpu().numpy())
        assert not np.array_equal(got, z0)                   # the step did something
        # and against the oracle, to the bar of every other parity test
        cache = m.new_cache(256)
        k_all = [ctx.read_kv(li, 0, 0, pos0 + n) for li in range(shape.n_layers)]
        for li, name in enumerate(m.P_layers + m.R_layers + m.C_layers):
            cache.k[name][: pos0 + n] = k_all[li][0]
            cache.v[name][: pos0 + n] = k_all[li][1]
        pos = np.arange(pos0, pos0 + n)
        e64 = e.cpu().numpy().astype(np.float64)
        ref = m.core(e64, m.core(e64, z0.astype(np.float64), pos, cache), pos, cache)
        assert_rows_close(got, ref, tol_latent(shape), "static vs oracle")


@pytest.mark.parametrize("shape", [S.TINY, SMALL_BF16_D96], ids=["tiny_f32", "bf16_d96"])
def test_core_step_static_equals_core_step(shape):
    import paper_2510_14961_amd as R
    ctx, m, _ = make_pair(shape, seed=5, max_positions=256, max_rows=96)
    L = 40
    prompt = S.make_prompt(shape.vocab, L + 1, 3)
    ctx.set_tokens(0, prompt)
    ctx.prefill(0, L, 2, 1.0, 7)
    # a three-tile ragged window, then a smaller one (one ragged tile) further on
    _pair_of_calls(ctx, m, shape, [(L, 70), (L + 70, 9)], seed=11)
    # sizes beyond the array are refused before anything is enqueued
    assert 0 < ctx.core_step_static_bytes(1) < ctx.core_step_static_bytes(2)
    too_many = 1
    while ctx.core_step_static_bytes(too_many) <= R.STATIC_SCRATCH_BYTES:
        too_many *= 2
    import torch
    if too_many * 32 <= 4096:
        big = torch.zeros(too_many * 32, shape.hidden, device="cuda")
        with pytest.raises(R.RdlmError) as ei:
            ctx.core_step_static([0], [0], [too_many * 32], big, big.clone())
        assert ei.value.status == R.STATUS["ECAPACITY"]
    ctx.close()


def test_core_step_static_is_shared_by_contexts_of_different_shapes():
    """Two contexts (different models) use the GPU's one static array in turn: each call clears the
    ticket words it needs, so what the other left behind does not matter."""
    a, ma, _ = make_pair(SMALL_BF16_D96, seed=5, max_positions=256, max_rows=64)
    b, mb, _ = make_pair(S.TINY, seed=6, max_positions=256, max_rows=64)
    for ctx, m, shape in ((a, ma, SMALL_BF16_D96), (b, mb, S.TINY), (a, ma, SMALL_BF16_D96)):
        _pair_of_calls(ctx, m, shape, [(0, 33), (33, 5)], seed=13)
    a.close()
    b.close()
