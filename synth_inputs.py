"""Seeded synthetic inputs for the recurrent-depth LM sampler: model shapes, weights, prompts.

This module is the only thing the CPU oracle's tests and the HIP path's tests have in common.
It holds none of the method's arithmetic: it only draws random arrays (numpy bit generators)
and names the five workload configurations.  Random numbers that the *method* draws (latent
state initialisation, Gumbel noise) are NOT produced here: each side implements the same
counter-based generator on its own.

Weights are N(0, 0.02) matrices (config text of the workloads); norm gains are 1 by default,
or 1 + jitter*N(0,1) when a test wants gain handling to be visible.  For bf16 models the values
are rounded to bf16 (round-to-nearest-even) here, so that both consumers see identical numbers.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Iterator, List, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Shape of a recurrent-depth LM: prelude P, recurrent block R (core), coda C (Sec. 3.1)."""
    vocab: int
    hidden: int
    n_heads: int
    head_dim: int
    mlp: int
    n_prelude: int
    n_core: int
    n_coda: int
    dtype: str = "bf16"          # storage type of the matrices: "f32" or "bf16"
    rope_base: float = 10000.0
    rms_eps: float = 1e-6
    emb_scale: float = 0.0       # factor on gathered embedding rows; 0 = sqrt(hidden)

    def __post_init__(self):
        if self.emb_scale == 0.0:
            object.__setattr__(self, "emb_scale", float(self.hidden) ** 0.5)
        assert self.n_heads * self.head_dim == self.hidden
        assert self.head_dim % 2 == 0
        assert self.dtype in ("f32", "bf16")

    @property
    def n_layers(self) -> int:
        return self.n_prelude + self.n_core + self.n_coda


@dataclasses.dataclass(frozen=True)
class SamplerSpec:
    """Hyper-parameters of the diffusion-forcing sampler (Alg. 1 / Alg. 2 inputs)."""
    n_new: int                  # N, max new tokens (per sequence)
    r: int                      # total recurrences per token (fixed exit) or cap (adaptive)
    r_inner: int = 1            # r'
    w_max: int = 0              # wavefront limiter; 0 = ceil(r/r')*headway
    headway: int = 1
    adaptive: bool = False      # Alg. 2 exit rule
    eps: float = 0.0            # exit threshold on delta_i
    alpha: float = 1.0          # init scale
    temperature: float = 0.0    # 0 = greedy
    seed: int = 1               # seed of the method's own draws (state init, Gumbel)
    pad_token: int = 0          # input token of headway positions beyond the first


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    sampler: SamplerSpec
    n_seqs: int
    prompt_len: int
    weight_seed: int = 1
    prompt_seed: int = 1


TINY = ModelShape(vocab=256, hidden=128, n_heads=2, head_dim=64, mlp=512,
                  n_prelude=1, n_core=2, n_coda=1, dtype="f32")
MID = ModelShape(vocab=32768, hidden=1024, n_heads=16, head_dim=64, mlp=2816,
                 n_prelude=2, n_core=4, n_coda=2, dtype="bf16")
BIG = ModelShape(vocab=65536, hidden=5280, n_heads=55, head_dim=96, mlp=17920,
                 n_prelude=2, n_core=4, n_coda=2, dtype="bf16")

WORKLOADS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", TINY, SamplerSpec(n_new=32, r=4), 1, 16),
    "cfg2": Workload("cfg2", MID, SamplerSpec(n_new=256, r=16), 1, 128),
    "cfg3": Workload("cfg3", BIG, SamplerSpec(n_new=512, r=32), 1, 512),
    "cfg4": Workload("cfg4", BIG, SamplerSpec(n_new=256, r=64, w_max=64, adaptive=True, eps=1e-3,
                                               temperature=1.0), 8, 1024),
    "cfg5": Workload("cfg5", BIG, SamplerSpec(n_new=256, r=32, headway=4), 1, 4096),
}


def reduced(shape: ModelShape, **kw) -> ModelShape:
    """A copy of a shape with some fields replaced (tests use scaled-down variants)."""
    return dataclasses.replace(shape, **kw)


# --------------------------------------------------------------------------------------------
# bf16 helpers (bit manipulation only)

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 with round-to-nearest-even; returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------------
# tensors

def tensor_specs(shape: ModelShape) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) for every parameter; kind is "matrix" or "gain".

    Matrices are stored [out_features, in_features].  Per layer: wqkv [3h,h] (rows: q heads,
    then k heads, then v heads), wo [h,h], wg [F,h], wu [F,h], wd [h,F], gains g1,g2 [h].
    Global: emb [V,h] (also the LM head, tied), wa [h,2h] (adapter on concat(e, s)),
    gf [h] (norm closing each recurrence), gout [h] (norm before the LM head).
    """
    h, F, V = shape.hidden, shape.mlp, shape.vocab
    out: List[Tuple[str, Tuple[int, ...], str]] = [("emb", (V, h), "matrix")]
    for blk, n in (("P", shape.n_prelude), ("R", shape.n_core), ("C", shape.n_coda)):
        for i in range(n):
            p = f"{blk}{i}."
            out += [(p + "g1", (h,), "gain"), (p + "wqkv", (3 * h, h), "matrix"),
                    (p + "wo", (h, h), "matrix"), (p + "g2", (h,), "gain"),
                    (p + "wg", (F, h), "matrix"), (p + "wu", (F, h), "matrix"),
                    (p + "wd", (h, F), "matrix")]
    out += [("wa", (h, 2 * h), "matrix"), ("gf", (h,), "gain"), ("gout", (h,), "gain")]
    return out


def _draw(seed: int, index: int, shp: Tuple[int, ...], kind: str, std: float, gain_jitter: float,
          bf16: bool) -> np.ndarray:
    rng = np.random.Generator(np.random.SFC64(np.random.SeedSequence([int(seed), int(index), 0xD1FF])))
    if kind == "gain":
        g = np.ones(shp, dtype=np.float32)
        if gain_jitter:
            g += np.float32(gain_jitter) * rng.standard_normal(shp, dtype=np.float32)
        return g            # gains stay f32 on both sides
    w = rng.standard_normal(shp, dtype=np.float32)
    w *= np.float32(std)
    if bf16:
        w = bf16_bits_to_f32(f32_to_bf16_bits(w))
    return w


def iter_weights(shape: ModelShape, seed: int, std: float = 0.02, gain_jitter: float = 0.0,
                 threads: int = 8) -> Iterator[Tuple[str, np.ndarray]]:
    """Yield (name, float32 array) one tensor at a time (values bf16-exact for bf16 shapes)."""
    specs = tensor_specs(shape)
    bf16 = shape.dtype == "bf16"
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        pending = []
        it = iter(enumerate(specs))
        # keep a few tensors in flight so big models generate in parallel without holding all
        def submit():
            try:
                i, (name, shp, kind) = next(it)
            except StopIteration:
                return False
            pending.append((name, ex.submit(_draw, seed, i, shp, kind, std, gain_jitter, bf16)))
            return True
        for _ in range(max(1, threads)):
            if not submit():
                break
        while pending:
            name, fut = pending.pop(0)
            arr = fut.result()
            submit()
            yield name, arr


def make_weights(shape: ModelShape, seed: int, std: float = 0.02, gain_jitter: float = 0.0,
                 threads: int = 8) -> Dict[str, np.ndarray]:
    return dict(iter_weights(shape, seed, std, gain_jitter, threads))


def make_prompt(vocab: int, length: int, seed: int, seq: int = 0) -> np.ndarray:
    """Uniform token ids over the vocabulary (int32)."""
    rng = np.random.Generator(np.random.SFC64(np.random.SeedSequence([int(seed), int(seq), 0x70B0])))
    return rng.integers(0, vocab, size=length, dtype=np.int32)


def make_rows(n: int, width: int, seed: int, scale: float = 1.0) -> np.ndarray:
    """Generic N(0, scale^2) float32 rows for kernel-level tests."""
    rng = np.random.Generator(np.random.SFC64(np.random.SeedSequence([int(seed), n, width, 0xA11])))
    return (rng.standard_normal((n, width), dtype=np.float32) * np.float32(scale))
