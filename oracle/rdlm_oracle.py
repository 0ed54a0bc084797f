"""CPU oracle for the recurrent-depth LM and its samplers.  TEST INFRASTRUCTURE ONLY.

Plain numpy, float64 arithmetic throughout, no blocking, no fusion: every function follows the
passage of the paper it cites so that it can be checked against the paper by eye.  Nothing in
the product path may import this module; it shares no code with the HIP implementation.

What the paper fixes and what it leaves open:
  * Sec. 3.1 fixes the block structure  e = P(x), s_0 ~ N(0, sigma^2 I), s_i = R(e, s_{i-1}),
    p = C(s_r); Sec. 3.2 fixes input injection and the depth-shared KV cache (one K/V entry per
    layer and position, overwritten by every recurrence); Alg. 1 and Alg. 2 fix the samplers.
  * The internals of a transformer layer are not in the paper.  The workload text fixes the
    ingredients (RMSNorm, QKV projection, RoPE base 10000, causal attention, output projection,
    SwiGLU MLP, adapter Linear(2h -> h) on [embedding, state]); the arrangement used here is
    the pre-norm residual layer, rotate-half RoPE on absolute positions, 1/sqrt(d) scaling,
    a gain-only RMSNorm closing each recurrence, a final RMSNorm and a tied LM head; gathered
    embedding rows are multiplied by sqrt(h) (with N(0, 0.02) matrices the conditioning e would
    otherwise be ~50x smaller than the unit-RMS state and the prompt would not matter).

Pins (tests/test_oracle_*.py): Philox known-answer vectors, Box-Muller statistics, brute-force
loops for matmul orientation / attention / RoPE, library routines (torch SDPA, rms_norm, silu),
"r' = r recovers the autoregressive sampler" (end of Sec. 3.3), "wavefront 1 recovers the
adaptive-compute sampler" (Sec. 3.5), causality (Sec. 1), the contraction remark (Sec. 3.5),
the cost remark (Sec. 3.5), closed forms for delta_i and k* (Eq. 3).
Parity unpinned: the actual token values and latents of the five workloads (random weights; the
paper prints no worked numeric example) -- only the invariants above constrain them.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64

# ---------------------------------------------------------------------------------------------
# Counter-based random numbers the method draws (state init, Sec. 3.1 s_0; Sample; state noise).
# Philox4x32-10 (Salmon et al., SC'11, "Parallel random numbers: as easy as 1, 2, 3").

_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)

TAG_INIT_STATE = 1
TAG_SAMPLE = 2
TAG_NOISE = 3


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Ten Philox rounds on arrays of 4x32-bit counters with one 2x32-bit key."""
    c0 = np.asarray(c0, dtype=np.uint64) & _MASK32
    c1 = np.asarray(c1, dtype=np.uint64) & _MASK32
    c2 = np.asarray(c2, dtype=np.uint64) & _MASK32
    c3 = np.asarray(c3, dtype=np.uint64) & _MASK32
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 &= 0xFFFFFFFF
    k1 &= 0xFFFFFFFF
    for _ in range(10):
        p0 = _PHILOX_M0 * c0            # 32x32 -> 64 bit products
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0
        k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return (c0.astype(np.uint32), c1.astype(np.uint32), c2.astype(np.uint32), c3.astype(np.uint32))


def _uniform_open(x: np.ndarray) -> np.ndarray:
    """23 high bits -> u in (0,1): u = (x>>9 + 1/2) * 2^-23 (never 0, never 1; 24 significant bits,
    so the value is exact in float32 as well)."""
    return ((x >> np.uint32(9)).astype(F64) + 0.5) * (2.0 ** -23)


def _draw_block(n_blocks: int, position: int, seq: int, step: int, tag: int, seed: int):
    c0 = np.arange(n_blocks, dtype=np.uint64)
    c3 = (int(step) << 4) | int(tag)
    return philox4x32_10(c0, np.uint64(position), np.uint64(seq), np.uint64(c3),
                         seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)


def init_state(hidden: int, position: int, seq: int, alpha: float, seed: int,
               step: int = 0, tag: int = TAG_INIT_STATE) -> np.ndarray:
    """InitState(1, alpha): one latent s_0 ~ N(0, alpha^2 I) for a sequence position (Sec. 3.1).

    Element 4b+j comes from Philox block b of counter (b, position, seq, step*16+tag):
    words (x0,x1) and (x2,x3) each feed one Box-Muller pair
    (sqrt(-2 ln u_a) cos(2 pi u_b), sqrt(-2 ln u_a) sin(2 pi u_b)).
    """
    nb = (hidden + 3) // 4
    x0, x1, x2, x3 = _draw_block(nb, position, seq, step, tag, seed)
    out = np.empty((nb, 4), dtype=F64)
    for j, (xa, xb) in enumerate(((x0, x1), (x2, x3))):
        ua, ub = _uniform_open(xa), _uniform_open(xb)
        rad = np.sqrt(-2.0 * np.log(ua))
        out[:, 2 * j] = rad * np.cos(2.0 * math.pi * ub)
        out[:, 2 * j + 1] = rad * np.sin(2.0 * math.pi * ub)
    return alpha * out.reshape(-1)[:hidden]


def gumbel_noise(vocab: int, position: int, seq: int, step: int, seed: int) -> np.ndarray:
    """g_v = -ln(-ln u_v), u_v word (v mod 4) of Philox block v//4, counter tagged TAG_SAMPLE."""
    nb = (vocab + 3) // 4
    xs = _draw_block(nb, position, seq, step, TAG_SAMPLE, seed)
    u = np.stack([_uniform_open(x) for x in xs], axis=1).reshape(-1)[:vocab]
    return -np.log(-np.log(u))


def nucleus(logits: np.ndarray, temperature: float, top_p: float) -> np.ndarray:
    """Top-p filter (the paper's runs sample at temperature 0.2 with top-p 0.95, App. "Dataset
    details"): boolean mask of the smallest set of tokens, taken in order of decreasing probability
    under softmax(logits / T), whose total probability reaches top_p.  Tokens exactly as probable
    as the last one taken are all kept, so the set depends on the probabilities only."""
    if not (0.0 < top_p < 1.0):
        return np.ones(logits.shape[0], dtype=bool)
    s = logits / temperature
    p = np.exp(s - np.max(s))
    p = p / np.sum(p)
    order = np.argsort(-p, kind="stable")
    c = np.cumsum(p[order])
    k = int(np.searchsorted(c, top_p, side="left"))        # first prefix with mass >= top_p
    k = min(k, len(order) - 1)
    return p >= p[order[k]]


def sample(logits: np.ndarray, temperature: float, position: int, seq: int, step: int,
           seed: int, top_p: float = 1.0) -> int:
    """Sample(p) (Alg. 1): greedy at temperature 0, else Gumbel-max, which draws from
    softmax(logits / T) -- restricted to the top-p set and renormalised when 0 < top_p < 1 (the
    Gumbel race among the kept tokens draws from exactly that).  Ties go to the lowest token id."""
    if temperature > 0.0:
        score = logits / temperature + gumbel_noise(logits.shape[0], position, seq, step, seed)
        score = np.where(nucleus(logits, temperature, top_p), score, -np.inf)
    else:
        score = logits
    return int(np.argmax(score))            # numpy returns the first maximum


# ---------------------------------------------------------------------------------------------
# Layer pieces

def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * gain / sqrt(mean(x^2) + eps), row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing: for i < d/2 the pair (x_i, x_{i+d/2}) is rotated
    by the angle pos * base^(-2i/d).  x: [n, H, d], pos: [n]."""
    d = x.shape[-1]
    half = d // 2
    theta = base ** (-2.0 * np.arange(half, dtype=F64) / d)
    ang = pos.astype(F64)[:, None] * theta[None, :]            # [n, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def causal_attention(q: np.ndarray, pos: np.ndarray, cache_k: np.ndarray, cache_v: np.ndarray
                     ) -> np.ndarray:
    """Row i (absolute position pos[i]) attends to cache positions 0..pos[i] inclusive:
    softmax_j(q_i . k_j / sqrt(d)) v_j, one head at a time.  q: [n, H, d]; caches [P, H, d]."""
    n, H, d = q.shape
    out = np.empty_like(q)
    for i in range(n):
        p = int(pos[i])
        K = cache_k[: p + 1]                                   # [p+1, H, d]
        V = cache_v[: p + 1]
        for hd in range(H):
            sc = K[:, hd, :] @ q[i, hd, :] / math.sqrt(d)
            sc = sc - np.max(sc)
            w = np.exp(sc)
            w = w / np.sum(w)
            out[i, hd, :] = w @ V[:, hd, :]
    return out


class FlopCounter:
    """Counts 2*m*n*k for every projection (attention excluded), for the cost remark of Sec. 3.5."""
    def __init__(self):
        self.flops = 0

    def add(self, m, n, k):
        self.flops += 2 * m * n * k


class KVCache:
    """Depth-shared KV cache (Sec. 3.2): one K and one V entry per (layer, position); a later
    recurrence or sampler step at the same position overwrites the entry."""
    def __init__(self, layer_names: Sequence[str], max_positions: int, n_heads: int, head_dim: int):
        self.k = {n: np.zeros((max_positions, n_heads, head_dim), dtype=F64) for n in layer_names}
        self.v = {n: np.zeros((max_positions, n_heads, head_dim), dtype=F64) for n in layer_names}

    def nbytes(self) -> int:
        return sum(a.nbytes for a in self.k.values()) + sum(a.nbytes for a in self.v.values())

    def copy(self) -> "KVCache":
        c = KVCache.__new__(KVCache)
        c.k = {n: a.copy() for n, a in self.k.items()}
        c.v = {n: a.copy() for n, a in self.v.items()}
        return c


class RecurrentDepthLM:
    """Prelude P, recurrent block R, coda C (Sec. 3.1) over float64 copies of the weights."""

    def __init__(self, shape, weights: Dict[str, np.ndarray]):
        self.shape = shape
        self.w = {k: np.asarray(v, dtype=F64) for k, v in weights.items()}
        self.h = shape.hidden
        self.H = shape.n_heads
        self.d = shape.head_dim
        self.eps = float(shape.rms_eps)
        self.base = float(shape.rope_base)
        self.emb_scale = float(shape.emb_scale)
        self.P_layers = [f"P{i}" for i in range(shape.n_prelude)]
        self.R_layers = [f"R{i}" for i in range(shape.n_core)]
        self.C_layers = [f"C{i}" for i in range(shape.n_coda)]
        self.counter = FlopCounter()

    def new_cache(self, max_positions: int) -> KVCache:
        return KVCache(self.P_layers + self.R_layers + self.C_layers, max_positions, self.H, self.d)

    def _proj(self, x: np.ndarray, name: str) -> np.ndarray:
        W = self.w[name]                                       # [out, in]
        self.counter.add(x.shape[0], W.shape[0], W.shape[1])
        return x @ W.T

    def layer(self, name: str, x: np.ndarray, pos: np.ndarray, cache: KVCache) -> np.ndarray:
        """Pre-norm transformer layer on rows x [n,h] at absolute positions pos [n].
        Writes this pass's K/V at those positions before attending, so a row sees earlier rows
        of the same pass (that is what makes a batched window or prefill pass causal)."""
        n = x.shape[0]
        a = rmsnorm(x, self.w[name + ".g1"], self.eps)
        qkv = self._proj(a, name + ".wqkv").reshape(n, 3, self.H, self.d)
        q = rope(qkv[:, 0], pos, self.base)
        k = rope(qkv[:, 1], pos, self.base)
        v = qkv[:, 2]
        cache.k[name][pos] = k
        cache.v[name][pos] = v
        att = causal_attention(q, pos, cache.k[name], cache.v[name]).reshape(n, self.h)
        x = x + self._proj(att, name + ".wo")
        b = rmsnorm(x, self.w[name + ".g2"], self.eps)
        act = silu(self._proj(b, name + ".wg")) * self._proj(b, name + ".wu")
        return x + self._proj(act, name + ".wd")

    def prelude(self, tokens: np.ndarray, pos: np.ndarray, cache: KVCache) -> np.ndarray:
        """e = P(x): embedding rows (times the model's embedding scale) through the prelude layers."""
        x = self.w["emb"][np.asarray(tokens, dtype=np.int64)] * self.emb_scale
        for name in self.P_layers:
            x = self.layer(name, x, pos, cache)
        return x

    def core(self, e: np.ndarray, s: np.ndarray, pos: np.ndarray, cache: KVCache) -> np.ndarray:
        """One recurrence s_i = R(e, s_{i-1}): adapter on concat(e, s), the core layers, and the
        gain-only RMSNorm that closes the recurrence."""
        x = self._proj(np.concatenate([e, s], axis=-1), "wa")
        for name in self.R_layers:
            x = self.layer(name, x, pos, cache)
        return rmsnorm(x, self.w["gf"], self.eps)

    def coda_hidden(self, s: np.ndarray, pos: np.ndarray, cache: KVCache) -> np.ndarray:
        x = s
        for name in self.C_layers:
            x = self.layer(name, x, pos, cache)
        return rmsnorm(x, self.w["gout"], self.eps)

    def coda(self, s: np.ndarray, pos: np.ndarray, cache: KVCache) -> np.ndarray:
        """p = C(s) as logits: coda layers, final norm, tied LM head."""
        out = self.coda_hidden(s, pos, cache)
        return self._proj(out, "emb")

    # -----------------------------------------------------------------------------------------
    def prefill(self, tokens: np.ndarray, r: int, alpha: float, seed: int, seq: int,
                cache: KVCache) -> np.ndarray:
        """Parallel prefill (Sec. 3.3): all given prompt positions at once, r recurrences from
        fresh random states, then the coda layers so their caches hold the prompt as well.
        Returns the final latent states [n, h]."""
        n = len(tokens)
        pos = np.arange(n)
        if n == 0:
            return np.zeros((0, self.h), dtype=F64)
        e = self.prelude(tokens, pos, cache)
        s = np.stack([init_state(self.h, p, seq, alpha, seed) for p in pos])
        for _ in range(r):
            s = self.core(e, s, pos, cache)
        self.coda_hidden(s, pos, cache)
        return s


# ---------------------------------------------------------------------------------------------
# Eq. 3: exit criterion

def delta(z: np.ndarray, z_prev: np.ndarray) -> np.ndarray:
    """delta_i = ||z_i - z_prev,i||_2 / ||z_i||_2 per row."""
    num = np.sqrt(np.sum((z - z_prev) ** 2, axis=-1))
    den = np.sqrt(np.sum(z * z, axis=-1))
    with np.errstate(divide="ignore", invalid="ignore"):
        return num / den


def k_star(freezable: Sequence[bool]) -> int:
    """Length of the longest prefix of freezable positions (k* of Eq. 3; 0 = none)."""
    k = 0
    for f in freezable:
        if not f:
            break
        k += 1
    return k


def freezable_flags(deltas: np.ndarray, counts: Sequence[int], r_inner: int, eps: float,
                    r_cap: int) -> List[bool]:
    """A state may be frozen when delta_i < eps (non-finite delta never qualifies) or when it has
    received r_cap recurrences."""
    out = []
    for dlt, c in zip(deltas, counts):
        conv = bool(np.isfinite(dlt) and dlt < eps)
        out.append(conv or (c * r_inner >= r_cap))
    return out


# ---------------------------------------------------------------------------------------------
# Samplers.  All start from the same split: the first L-1 prompt tokens are prefilled with r
# recurrences; generation starts with one fresh state at the last prompt position.

class Trace:
    """What a sampler run leaves behind for tests."""
    def __init__(self):
        self.tokens: Optional[np.ndarray] = None      # prompt + generated
        self.steps = 0                                 # sampler steps taken
        self.window_sizes: List[int] = []              # |z| during each step
        self.frozen_per_step: List[int] = []
        self.final_states: Dict[int, np.ndarray] = {}  # position -> latent when frozen
        self.recurrences: Dict[int, int] = {}          # position -> recurrences received
        self.deltas: List[np.ndarray] = []


def noise_level(beta: float, steps_done: int, n_steps: int) -> float:
    """beta_t of Eq. 2, scheduled linearly in the sampler steps a position has already received
    (Sec. 3.4: "the latter steps are naturally less noisy"): beta on a position's first step,
    falling by beta / n_steps per step, where n_steps = ceil(r / r') is the number of steps a
    position stays in flight under the fixed exit rule (the cap, for the adaptive rule)."""
    return beta * max(0.0, 1.0 - steps_done / float(n_steps))


def mix_noise(z: np.ndarray, level: float, position: int, seq: int, step: int, alpha: float,
              seed: int) -> np.ndarray:
    """z' = (1 - beta_t) z + beta_t z_noise, z_noise = InitState(1, alpha) drawn afresh at every
    sampler step (Eq. 2; Alg. 1, noise on the conditioning): counter (., position, seq, step) tagged TAG_NOISE."""
    if level == 0.0:
        return z
    noise = init_state(z.shape[0], position, seq, alpha, seed, step=step, tag=TAG_NOISE)
    return (1.0 - level) * z + level * noise


def momentum(e_new: np.ndarray, e_prev: Optional[np.ndarray], eta: float) -> np.ndarray:
    """e = eta e_prev + (1 - eta) P(y_current) (Eq. 1).  A position that has no previous
    conditioning yet (its first sampler step) takes P(y_current) as it is."""
    if e_prev is None or eta == 0.0:
        return e_new
    return eta * e_prev + (1.0 - eta) * e_new


def generate_autoregressive(model: RecurrentDepthLM, prompt: np.ndarray, n_new: int, r: int,
                            alpha: float = 1.0, temperature: float = 0.0, seed: int = 1,
                            seq: int = 0, r_prefill: Optional[int] = None, top_p: float = 1.0) -> Trace:
    """Baseline sampler (Sec. 1): one token at a time, r sequential recurrences per token."""
    L = len(prompt)
    cache = model.new_cache(L + n_new)
    y = list(int(t) for t in prompt)
    model.prefill(np.asarray(y[: L - 1]), r if r_prefill is None else r_prefill, alpha, seed, seq, cache)
    tr = Trace()
    for t in range(1, n_new + 1):
        p = len(y) - 1
        pos = np.array([p])
        s = init_state(model.h, p, seq, alpha, seed)[None, :]
        e = model.prelude(np.array([y[p]]), pos, cache)
        for _ in range(r):
            s = model.core(e, s, pos, cache)
        logits = model.coda(s, pos, cache)[0]
        y.append(sample(logits, temperature, p, seq, t, seed, top_p))
        tr.final_states[p] = s[0]
        tr.recurrences[p] = r
        tr.steps += 1
    tr.tokens = np.asarray(y, dtype=np.int64)
    return tr


def generate_adaptive_autoregressive(model: RecurrentDepthLM, prompt: np.ndarray, n_new: int,
                                     r_inner: int, r_cap: int, eps: float, alpha: float = 1.0,
                                     temperature: float = 0.0, seed: int = 1, seq: int = 0,
                                     r_prefill: Optional[int] = None, top_p: float = 1.0) -> Trace:
    """Token-per-token adaptive-compute sampler (Sec. 4): recur on one position, r' recurrences
    at a time, until the latent's relative change drops below eps (or r_cap is reached)."""
    L = len(prompt)
    cache = model.new_cache(L + n_new)
    y = list(int(t) for t in prompt)
    model.prefill(np.asarray(y[: L - 1]), r_cap if r_prefill is None else r_prefill, alpha, seed, seq, cache)
    tr = Trace()
    t = 0
    for _ in range(n_new):
        p = len(y) - 1
        pos = np.array([p])
        s = init_state(model.h, p, seq, alpha, seed)[None, :]
        e = model.prelude(np.array([y[p]]), pos, cache)
        c = 0
        while True:
            t += 1
            s_prev = s
            for _ in range(r_inner):
                s = model.core(e, s, pos, cache)
            c += 1
            d = delta(s, s_prev)[0]
            if (np.isfinite(d) and d < eps) or c * r_inner >= r_cap:
                break
        logits = model.coda(s, pos, cache)[0]
        y.append(sample(logits, temperature, p, seq, t, seed, top_p))
        tr.final_states[p] = s[0]
        tr.recurrences[p] = c * r_inner
    tr.steps = t
    tr.tokens = np.asarray(y, dtype=np.int64)
    return tr


def appended_state(h: int, position: int, seq: int, alpha: float, seed: int,
                   left_state: np.ndarray, continuous_compute: bool) -> np.ndarray:
    """State of a position that enters the window: a random InitState draw (Alg. 1), or, with
    "continuous compute" (App., additional hyperparameter sweeps), a copy of the latest state of
    the position one step to its left."""
    if continuous_compute:
        return np.array(left_state, dtype=np.float64, copy=True)
    return init_state(h, position, seq, alpha, seed)


def generate_diffusion_forcing(model: RecurrentDepthLM, prompt: np.ndarray, n_new: int,
                               r_inner: int, r: int, alpha: float = 1.0,
                               temperature: float = 0.0, seed: int = 1, seq: int = 0,
                               headway: int = 1, pad_token: int = 0, T: Optional[int] = None,
                               r_prefill: Optional[int] = None, hook=None, eta: float = 0.0,
                               beta: float = 0.0, top_p: float = 1.0,
                               continuous_compute: bool = False) -> Trace:
    """Alg. 1: diffusion-forcing sampler with the fixed exit rule; optional momentum on the
    conditioning (Eq. 1, eta), scheduled state noise (Eq. 2, beta) and continuous-compute
    initialisation of appended states (the very first state is always a random draw).

    y_current is kept as one array over absolute positions: frozen tokens, then the drafts of the
    in-flight positions, then pad tokens for headway positions that have no draft yet.  The
    state at position p reads token y[p] and drafts token y[p+1].  A state is frozen once it has
    received r recurrences; its token becomes final and its K/V entries stay in the caches.
    """
    L = len(prompt)
    max_pos = L + n_new + (-(-r // r_inner)) * headway + headway
    cache = model.new_cache(max_pos)
    y = np.full(max_pos + 1, pad_token, dtype=np.int64)      # y_current
    y[:L] = prompt
    n_frozen = L                                             # |y_frozen|
    model.prefill(y[: L - 1], r if r_prefill is None else r_prefill, alpha, seed, seq, cache)
    # z <- InitState(1, alpha): one state at the last prompt position
    z_pos: List[int] = [L - 1]
    z: List[np.ndarray] = [init_state(model.h, L - 1, seq, alpha, seed)]
    count: List[int] = [0]
    e_prev: Dict[int, np.ndarray] = {}
    n_steps = -(-r // r_inner)
    tr = Trace()
    t = 0
    while T is None or t < T:
        t += 1
        pos = np.asarray(z_pos)
        tr.window_sizes.append(len(z_pos))
        e = model.prelude(y[pos], pos, cache)                # e <- P(y_current)
        e = np.stack([momentum(e[i], e_prev.get(p), eta) for i, p in enumerate(z_pos)])
        for i, p in enumerate(z_pos):
            e_prev[p] = e[i]
        # z <- (1 - beta_t) z + beta_t z_noise
        zz = np.stack([mix_noise(z[i], noise_level(beta, count[i], n_steps), p, seq, t, alpha, seed)
                       for i, p in enumerate(z_pos)])
        for _ in range(r_inner):                             # inner recurrence
            zz = model.core(e, zz, pos, cache)
        count = [c + 1 for c in count]
        logits = model.coda(zz, pos, cache)                  # p <- C(z)
        for i, p in enumerate(z_pos):                        # y_hat <- Sample(p)
            y[p + 1] = sample(logits[i], temperature, p, seq, t, seed, top_p)
        z = [zz[i] for i in range(len(z_pos))]
        if hook is not None:
            hook(t, list(z_pos), zz, logits, y.copy(), e)
        # freeze completed tokens: states that have had r recurrences (always a prefix)
        k = 0
        while k < len(z_pos) and count[k] * r_inner >= r:
            k += 1
        for i in range(k):
            tr.final_states[z_pos[i]] = z[i]
            tr.recurrences[z_pos[i]] = count[i] * r_inner
        n_frozen += k
        tr.frozen_per_step.append(k)
        left = z[-1]                                         # latest state at position nxt - 1 (see below)
        z_pos, z, count = z_pos[k:], z[k:], count[k:]
        if n_frozen - L >= n_new:
            break
        # the next state sits after the last in-flight one, or, when none is left, at the
        # position of the newest frozen token (which it reads); either way the position to its
        # left is the last row of this step's window
        nxt = (z_pos[-1] + 1) if z_pos else n_frozen - 1
        for j in range(headway):                             # append new latent state(s)
            z_pos.append(nxt + j)
            z.append(appended_state(model.h, nxt + j, seq, alpha, seed, left, continuous_compute))
            count.append(0)
    tr.steps = t
    tr.tokens = y[: L + n_new].copy()
    return tr


def generate_diffusion_forcing_adaptive(model: RecurrentDepthLM, prompt: np.ndarray, n_new: int,
                                        r_inner: int, r_cap: int, eps: float, w_max: int,
                                        alpha: float = 1.0, temperature: float = 0.0,
                                        seed: int = 1, seq: int = 0, headway: int = 1,
                                        pad_token: int = 0, T: Optional[int] = None,
                                        r_prefill: Optional[int] = None, hook=None,
                                        eta: float = 0.0, beta: float = 0.0, top_p: float = 1.0,
                                        continuous_compute: bool = False) -> Trace:
    """Alg. 2: diffusion-forcing sampler with latent-difference freezing and a wavefront limit;
    optional momentum (Eq. 1) and scheduled state noise (Eq. 2; delta_i still compares the state
    after the recurrences with the state the previous step ended on, before any noise).

    After the r' recurrences of a step, delta_i compares each state with what it was at the end of
    the previous step (a new state's previous value is its random initialisation).  The longest
    prefix of freezable states is frozen (k* of Eq. 3); a new state is appended only while the
    wavefront holds fewer than w_max states.
    """
    L = len(prompt)
    max_pos = L + n_new + w_max + headway + 1
    cache = model.new_cache(max_pos)
    y = np.full(max_pos + 1, pad_token, dtype=np.int64)
    y[:L] = prompt
    n_frozen = L
    model.prefill(y[: L - 1], r_cap if r_prefill is None else r_prefill, alpha, seed, seq, cache)
    z_pos: List[int] = [L - 1]
    z: List[np.ndarray] = [init_state(model.h, L - 1, seq, alpha, seed)]
    z_prev: List[np.ndarray] = [z[0]]
    count: List[int] = [0]
    e_prev: Dict[int, np.ndarray] = {}
    n_steps = -(-r_cap // r_inner)
    tr = Trace()
    t = 0
    while T is None or t < T:
        t += 1
        pos = np.asarray(z_pos)
        tr.window_sizes.append(len(z_pos))
        e = model.prelude(y[pos], pos, cache)
        e = np.stack([momentum(e[i], e_prev.get(p), eta) for i, p in enumerate(z_pos)])
        for i, p in enumerate(z_pos):
            e_prev[p] = e[i]
        zz = np.stack([mix_noise(z[i], noise_level(beta, count[i], n_steps), p, seq, t, alpha, seed)
                       for i, p in enumerate(z_pos)])
        for _ in range(r_inner):
            zz = model.core(e, zz, pos, cache)
        count = [c + 1 for c in count]
        logits = model.coda(zz, pos, cache)
        for i, p in enumerate(z_pos):
            y[p + 1] = sample(logits[i], temperature, p, seq, t, seed, top_p)
        d = delta(zz, np.stack(z_prev))
        tr.deltas.append(d)
        z = [zz[i] for i in range(len(z_pos))]
        if hook is not None:
            hook(t, list(z_pos), zz, logits, y.copy(), e)
        k = k_star(freezable_flags(d, count, r_inner, eps, r_cap))
        for i in range(k):
            tr.final_states[z_pos[i]] = z[i]
            tr.recurrences[z_pos[i]] = count[i] * r_inner
        n_frozen += k
        tr.frozen_per_step.append(k)
        left = z[-1]
        z_pos, z, count = z_pos[k:], z[k:], count[k:]
        if n_frozen - L >= n_new:
            break
        n_app = min(headway, w_max - len(z_pos))             # wavefront limiter
        nxt = (z_pos[-1] + 1) if z_pos else n_frozen - 1
        for j in range(max(0, n_app)):
            z_pos.append(nxt + j)
            z.append(appended_state(model.h, nxt + j, seq, alpha, seed, left, continuous_compute))
            count.append(0)
        z_prev = list(z)                                     # z_prev <- z
    tr.steps = t
    tr.tokens = y[: L + n_new].copy()
    return tr
