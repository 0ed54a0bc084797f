"""GPU: the paged KV cache, eviction of a sequence to host memory and its re-admission into another
slot (App. "Larger batch sizes": the slots of a batch are fungible, a sequence's states can leave the
device and be bundled into a later forward call).

Sequences never interact and a sequence's random draws are keyed by its own step count and the slot
it started in, so whatever happens around it -- blocks handed out in any order, neighbours coming
and going, a stay in host memory, another slot afterwards -- each sequence must come out as the
oracle's run of that sequence alone: token ids exact and latents to the fp32 bar on the float32
model; on the bf16 model single steps are recomputed by the oracle from the GPU's own inputs, read
back through the block table.
"""
import numpy as np
import pytest

import synth_inputs as S
from oracle import rdlm_oracle as O
from gpu_util import SMALL_BF16_D64, make_pair, rel_l2, teacher_forced_step

pytestmark = pytest.mark.gpu


def _start(ctx, slot, prompt, r, seed):
    ctx.set_tokens(slot, prompt)
    ctx.prefill(slot, len(prompt) - 1, r, 1.0, seed)


def _check_against_own_run(ctx, m, slot, prompt, ident, n_new, r, kw, states=True):
    ref = O.generate_diffusion_forcing(m, prompt, n_new, 1, r, seq=ident, **kw)
    toks, nf = ctx.read_tokens(slot)
    assert nf == len(prompt) + n_new, (slot, nf)
    assert np.array_equal(toks[:nf], ref.tokens), slot
    if states:
        for p, st in ref.final_states.items():
            assert rel_l2(ctx.read_states(slot, p, 1)[0], st) < 1e-4, (slot, p)


def test_blocks_are_handed_out_lazily_and_come_back():
    shape = S.TINY
    ctx, m, _ = make_pair(shape, seed=3, max_seqs=2, max_positions=160, max_rows=64, kv_pool_positions=200)
    total, free = ctx.kv_blocks()
    assert total == 7 and free == 7                      # 200 positions round up to 7 blocks of 32
    p = S.make_prompt(shape.vocab, 40, 5)
    _start(ctx, 0, p, 4, 1)
    assert ctx.kv_blocks() == (7, 5)                     # 39 prefilled positions: 2 blocks
    ctx.sampler_begin(1, n_new=30, r_inner=1, r_total=4, seed=1)
    ctx.generate(1000)
    used = 7 - ctx.kv_blocks()[1]
    assert 3 <= used <= 4                                # 70 positions, plus at most one block ahead
    ctx.seq_release(0)
    assert ctx.kv_blocks() == (7, 7)
    toks, nf = ctx.read_tokens(0)                        # the text outlives the cache
    ref = O.generate_diffusion_forcing(m, p, 30, 1, 4, seed=1, seq=0)
    assert nf == 70 and np.array_equal(toks[:nf], ref.tokens)
    import paper_2510_14961_amd as R
    with pytest.raises(R.RdlmError) as e:                # a released slot has no cache to read
        ctx.read_kv(0, 0, 0, 8)
    assert e.value.status == R.STATUS["ESTATE"]
    ctx.close()
    ctx2, _, _ = make_pair(shape, seed=3, max_seqs=2, max_positions=160, max_rows=64)
    assert ctx2.kv_blocks() == (10, 10)                  # the default pool lets every slot reach max_positions
    ctx2.close()


@pytest.mark.parametrize("temp,beta", [(0.0, 0.0), (0.8, 0.3)])
def test_evicted_sequence_continues_in_another_slot_fp32(temp, beta):
    """Three sequences share a pool too small for all of them at full length; one is evicted in
    mid-flight, a fourth takes its slot, and the evicted one comes back later into the slot of a
    finished sequence."""
    shape = S.TINY
    n_new, r, seed = 20, 4, 9
    # each sequence ends near 60 positions = 2 blocks; 4 sequences would need 8, the pool has 6
    ctx, m, _ = make_pair(shape, seed=3, max_seqs=3, max_positions=96, max_rows=96, kv_pool_positions=6 * 32)
    pa = S.make_prompt(shape.vocab, 30, 31, seq=0)
    pb = S.make_prompt(shape.vocab, 38, 32, seq=1)
    pc = S.make_prompt(shape.vocab, 27, 33, seq=2)
    pd = S.make_prompt(shape.vocab, 35, 34, seq=1)
    spec = dict(n_new=n_new, r_inner=1, r_total=r, temperature=temp, seed=seed, beta=beta)
    kw = dict(temperature=temp, seed=seed, beta=beta)
    for q, p in enumerate((pa, pb, pc)):
        _start(ctx, q, p, r, seed)
    ctx.sampler_begin(3, **spec)
    for _ in range(6):
        ctx.sample_step()
    free_before = ctx.kv_blocks()[1]
    record = ctx.seq_evict(1)                           # B leaves in mid-flight
    assert ctx.kv_blocks()[1] == free_before + 2
    assert ctx.read_window(1)[2] == 1                   # its slot contributes no rows
    _start(ctx, 1, pd, r, seed)                         # D takes the slot (and B's old blocks)
    ctx.sampler_join(1)
    for _ in range(n_new + r - 1 - 6):                  # A and C finish in here
        ctx.sample_step()
    _check_against_own_run(ctx, m, 0, pa, 0, n_new, r, kw)
    _check_against_own_run(ctx, m, 2, pc, 2, n_new, r, kw)
    import paper_2510_14961_amd as R
    with pytest.raises(R.RdlmError) as e:               # slot 0 still holds A
        ctx.seq_admit(0, record)
    assert e.value.status == R.STATUS["ESTATE"]
    ctx.seq_release(0)
    ctx.seq_admit(0, record)                            # B comes back into A's slot
    p0, n, done = ctx.read_window(0)
    assert not done and n == min(r, 6 + 1) and p0 == len(pb) - 1 + (6 - r + 1)
    ctx.generate(1000)
    _check_against_own_run(ctx, m, 0, pb, 1, n_new, r, kw)      # B: identity 1, now in slot 0
    _check_against_own_run(ctx, m, 1, pd, 1, n_new, r, kw)
    ctx.close()


def test_a_dry_pool_refuses_the_step_and_eviction_lets_the_rest_go_on():
    shape = S.TINY
    n_new, r, seed = 30, 4, 4
    ctx, m, _ = make_pair(shape, seed=5, max_seqs=2, max_positions=96, max_rows=64, kv_pool_positions=3 * 32)
    pa = S.make_prompt(shape.vocab, 25, 41, seq=0)
    pb = S.make_prompt(shape.vocab, 20, 42, seq=1)
    kw = dict(temperature=0.6, seed=seed)
    for q, p in enumerate((pa, pb)):
        _start(ctx, q, p, r, seed)
    ctx.sampler_begin(2, n_new=n_new, r_inner=1, r_total=r, **kw)
    import paper_2510_14961_amd as R
    steps = 0
    with pytest.raises(R.RdlmError) as e:
        for _ in range(200):
            ctx.sample_step()
            steps += 1
    assert e.value.status == R.STATUS["ECAPACITY"]
    assert 7 <= steps <= 13                              # A reaches position 32 after 8 steps, B after 13; 3 blocks
    assert ctx.kv_blocks()[1] == 0
    with pytest.raises(R.RdlmError):                     # refused again, nothing has changed
        ctx.sample_step()
    record = ctx.seq_evict(1)
    assert ctx.kv_blocks()[1] >= 1
    ctx.generate(1000)
    _check_against_own_run(ctx, m, 0, pa, 0, n_new, r, kw)
    ctx.seq_release(0)
    ctx.seq_admit(0, record)                             # B goes on in A's slot
    ctx.generate(1000)
    _check_against_own_run(ctx, m, 0, pb, 1, n_new, r, kw)
    ctx.close()


def test_a_record_moves_between_contexts_and_bad_records_are_refused():
    shape = S.TINY
    n_new, r, seed = 12, 4, 2
    a, m, _ = make_pair(shape, seed=7, max_seqs=1, max_positions=96, max_rows=32)
    b, _, _ = make_pair(shape, seed=7, max_seqs=2, max_positions=128, max_rows=64, kv_pool_positions=96)
    p = S.make_prompt(shape.vocab, 33, 8)
    kw = dict(temperature=0.9, seed=seed, beta=0.2)
    _start(a, 0, p, r, seed)
    a.sampler_begin(1, n_new=n_new, r_inner=1, r_total=r, **kw)
    for _ in range(5):
        a.sample_step()
    rec = a.seq_evict(0)
    import paper_2510_14961_amd as R
    with pytest.raises(R.RdlmError) as e:                # no sampler runs in b yet
        b.seq_admit(1, rec)
    assert e.value.status == R.STATUS["ESTATE"]
    q = S.make_prompt(shape.vocab, 10, 9)
    _start(b, 0, q, r, seed)
    b.sampler_begin(1, n_new=n_new, r_inner=1, r_total=r, **kw)
    b.sample_step()
    bad = rec.copy()
    bad[0] ^= 0xFF
    with pytest.raises(R.RdlmError) as e:
        b.seq_admit(1, bad)
    assert e.value.status == R.STATUS["EINVAL"]
    with pytest.raises(R.RdlmError) as e:                # cut short
        b.seq_admit(1, rec[: len(rec) // 2])
    assert e.value.status == R.STATUS["EINVAL"]
    # a record whose fields contradict each other never reaches the device: 32-bit words of the header are
    # magic, version, the model (12 words), then n_pos, n_blocks, prompt_len (word 16), ..., pos_bound (word 20), and the window record from
    # word 22 on (prompt_len, n_frozen, win_pos0, win_n, ...)
    for word, value in ((16, -1), (25, 1 << 20), (24, -5), (20, 1 << 30)):
        bad = rec.copy()
        bad.view(np.int32)[word] = value
        with pytest.raises(R.RdlmError) as e:
            b.seq_admit(1, bad)
        assert e.value.status == R.STATUS["EINVAL"], (word, value)
    b.seq_admit(1, rec)                                  # the sequence started as number 0 of context a
    b.generate(1000)
    _check_against_own_run(b, m, 1, p, 0, n_new, r, kw)
    _check_against_own_run(b, m, 0, q, 0, n_new, r, kw)
    a.close()
    b.close()


def test_bf16_steps_through_the_block_table_and_across_an_eviction():
    """bf16 model (matrix-core GEMMs write K/V through the block table, grouped attention reads
    through it): single steps recomputed by the oracle from the GPU's inputs, before an eviction
    and after re-admission into another slot; blocks are interleaved between the two sequences."""
    shape = SMALL_BF16_D64
    r, n_new = 8, 40
    ctx, m, _ = make_pair(shape, seed=4, max_seqs=3, max_positions=192, max_rows=96, kv_pool_positions=10 * 32)
    pa = S.make_prompt(shape.vocab, 50, 21, seq=0)
    pb = S.make_prompt(shape.vocab, 70, 22, seq=1)
    spec = dict(n_new=n_new, r_inner=1, r_total=r, seed=3)
    # interleave the blocks: A's first block, B's blocks, then A's second
    ctx.set_tokens(0, pa)
    ctx.set_tokens(1, pb)
    ctx.prefill(0, 20, r, 1.0, 3)
    ctx.prefill(1, len(pb) - 1, r, 1.0, 3)
    ctx.set_tokens(0, pa)
    ctx.prefill(0, len(pa) - 1, r, 1.0, 3)
    ctx.sampler_begin(2, **spec)
    t = 0
    for _ in range(10):
        t += 1
        out = teacher_forced_step(ctx, m, shape, spec, 2, t, label="paged")
    assert out["rows"] == 16
    rec = ctx.seq_evict(0)
    for _ in range(3):
        t += 1
        teacher_forced_step(ctx, m, shape, spec, 3, t, label="paged, A away")
    ctx.seq_admit(2, rec)
    rows = 0
    for _ in range(12):
        t += 1
        out = teacher_forced_step(ctx, m, shape, spec, 3, t, label="paged, A back in slot 2")
        rows += out["rows"]
    assert rows == 12 * 16
    ctx.generate(1000)
    for slot, p in ((2, pa), (1, pb)):
        toks, nf = ctx.read_tokens(slot)
        assert nf == len(p) + n_new
        assert np.array_equal(toks[: len(p)], p)
    ctx.close()
