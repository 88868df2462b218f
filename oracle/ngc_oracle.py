"""ctypes front end of the C oracle (``ngc_oracle.c``) plus the few host-integer
parts of the method that need no C (keep counts, cache-size trajectory).

TEST INFRASTRUCTURE ONLY -- see the header of ``ngc_oracle.c``.  All arrays are
numpy; bf16 tensors travel as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ngc_oracle.c")
_SO = os.path.join(_HERE, "libngc_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Contraction is off so that the defined
    logarithm is the stated operation sequence and nothing else."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        u32p, i32p, f32p, u16p = (C.POINTER(C.c_uint32), C.POINTER(C.c_int32),
                                  C.POINTER(C.c_float), C.POINTER(C.c_uint16))
        lib.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
        lib.orc_philox4x32_10.restype = None
        lib.orc_item_word.argtypes = [C.c_uint64] + [C.c_uint32] * 5
        lib.orc_item_word.restype = C.c_uint32
        lib.orc_log.argtypes = [C.c_double]
        lib.orc_log.restype = C.c_double
        lib.orc_gumbel_u32.argtypes = [C.c_uint32]
        lib.orc_gumbel_u32.restype = C.c_double
        lib.orc_perturbed_keys.argtypes = [f32p, C.c_int32, C.c_float, C.c_uint64,
                                           C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, f32p]
        lib.orc_perturbed_keys.restype = None
        lib.orc_select.argtypes = [f32p, C.c_int32, C.c_int32, i32p, i32p]
        lib.orc_select.restype = C.c_int
        for name in ("orc_logprob_literal", "orc_logprob_suffix"):
            fn = getattr(lib, name)
            fn.argtypes = [f32p, C.c_int32, i32p, C.c_int32]
            fn.restype = C.c_double
        lib.orc_compact_rows.argtypes = [u16p, u16p, C.c_int32, C.c_int32, C.c_int32, i32p, C.c_int32]
        lib.orc_compact_rows.restype = C.c_int32
        lib.orc_compact_rows_unordered.argtypes = [u16p, u16p, C.c_int32, C.c_int32, i32p, C.c_int32]
        lib.orc_compact_rows_unordered.restype = C.c_int32
        lib.orc_compact_i32.argtypes = [i32p, i32p, C.c_int32, C.c_int32, i32p, C.c_int32]
        lib.orc_compact_i32.restype = C.c_int32
        lib.orc_decode_attn.argtypes = [u16p, u16p, u16p, C.c_int32, C.c_int32, C.c_int32,
                                        C.c_double, f32p]
        lib.orc_decode_attn.restype = None
        f64p = C.POINTER(C.c_double)
        lib.orc_logprob_grad_literal.argtypes = [f32p, C.c_int32, i32p, C.c_int32, f64p]
        lib.orc_logprob_grad_literal.restype = None
        lib.orc_decode_lse.argtypes = [u16p, u16p, C.c_int32, C.c_int32, C.c_int32, C.c_double, f64p]
        lib.orc_decode_lse.restype = None
        lib.orc_replay_attn.argtypes = [u16p, u16p, u16p, i32p, C.c_int32, C.c_int32, C.c_int32, C.c_double, f32p]
        lib.orc_replay_attn.restype = None
        lib.orc_score_keys.argtypes = [u16p, u16p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                       C.c_double, C.c_int32, f64p]
        lib.orc_score_keys.restype = None
        lib.orc_block_means.argtypes = [f64p, C.c_int32, C.c_int32, f64p]
        lib.orc_block_means.restype = None
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _arr(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


# ---------------------------------------------------------------- RNG -----

def philox4x32_10(ctr, key) -> np.ndarray:
    c = _arr(ctr, np.uint32)
    k = _arr(key, np.uint32)
    out = np.zeros(4, np.uint32)
    _L().orc_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def item_word(seed: int, rnd: int, l: int, b: int, hsel: int, t: int) -> int:
    return int(_L().orc_item_word(seed, rnd, l, b, hsel, t))


def defined_log(x: float) -> float:
    return float(_L().orc_log(float(x)))


def gumbel_u32(r: int) -> float:
    return float(_L().orc_gumbel_u32(int(r)))


# ------------------------------------------------------------- sampling ---

def perturbed_keys(logits, tau: float, seed: int, rnd: int, l: int, b: int, hsel: int) -> np.ndarray:
    s = _arr(logits, np.float32)
    keys = np.empty_like(s)
    _L().orc_perturbed_keys(_p(s, C.c_float), s.size, tau, seed, rnd, l, b, hsel, _p(keys, C.c_float))
    return keys


def select(keys, K: int):
    k = _arr(keys, np.float32)
    kept = np.empty(K, np.int32)
    sigma = np.empty(K, np.int32)
    rc = _L().orc_select(_p(k, C.c_float), k.size, K, _p(kept, C.c_int32), _p(sigma, C.c_int32))
    if rc != 0:
        raise ValueError("orc_select: bad arguments or NaN key")
    return kept, sigma


def evict_select(logits, K: int, tau: float, seed: int, rnd: int, l: int, b: int, hsel: int):
    """Sample which K items of one segment survive: (kept ascending, sigma in
    sampled order)."""
    return select(perturbed_keys(logits, tau, seed, rnd, l, b, hsel), K)


def evict_select_pooled(logits_per_head, K_total: int, tau: float, seed: int, rnd: int, l: int, b: int):
    """One selection over the items of all KV heads of a (layer, sequence): the
    heads' items are laid end to end in (head, row) order, every item keeps the
    noise it would draw in its own head, and the K_total largest keys win.
    Returns (kept rows per head, sigma as a list of (head, row), concatenated
    logits, sigma as indices into the concatenation)."""
    keys = [perturbed_keys(s, tau, seed, rnd, l, b, h) for h, s in enumerate(logits_per_head)]
    sizes = [k.size for k in keys]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    kept, sigma = select(np.concatenate(keys) if keys else np.zeros(0, np.float32), K_total)
    head_of = np.searchsorted(offs, kept, side="right") - 1
    kept_per_head = [(kept[head_of == h] - offs[h]).astype(np.int32) for h in range(len(keys))]
    sh = np.searchsorted(offs, sigma, side="right") - 1
    sigma_pairs = [(int(h), int(i - offs[h])) for h, i in zip(sh, sigma)]
    return kept_per_head, sigma_pairs, np.concatenate([_arr(s, np.float32) for s in logits_per_head]), sigma


# ------------------------------------------------------------- log-prob ---

def logprob_literal(logits, sigma) -> float:
    s = _arr(logits, np.float32)
    sg = _arr(sigma, np.int32)
    return float(_L().orc_logprob_literal(_p(s, C.c_float), s.size, _p(sg, C.c_int32), sg.size))


def logprob_suffix(logits, sigma) -> float:
    s = _arr(logits, np.float32)
    sg = _arr(sigma, np.int32)
    return float(_L().orc_logprob_suffix(_p(s, C.c_float), s.size, _p(sg, C.c_int32), sg.size))


def logprob_grad(logits, sigma) -> np.ndarray:
    """d log p(sigma | logits) / d logits, fp64 [n]."""
    s = _arr(logits, np.float32)
    sg = _arr(sigma, np.int32)
    g = np.zeros(max(s.size, 1), np.float64)
    _L().orc_logprob_grad_literal(_p(s, C.c_float), s.size, _p(sg, C.c_int32), sg.size, _p(g, C.c_double))
    return g[:s.size]


# ----------------------------------------------- eviction loss (Eq. 4) ------

def advantages(reward, group: int) -> np.ndarray:
    """A_i = r_i - mean of r over the rollouts of the same prompt (groups of `group` consecutive rollouts)."""
    r = np.asarray(reward, np.float64)
    assert r.size % group == 0
    out = np.zeros_like(r)
    for g0 in range(0, r.size, group):
        out[g0:g0 + group] = r[g0:g0 + group] - r[g0:g0 + group].sum() / group
    return out


def lmem(logp, rounds, reward, group: int):
    """Eq. 4 written out.  logp: [R, L, B, H] log-probabilities of the eviction decisions (round, layer,
    rollout, KV head: the decision of a layer is the joint one over its heads, so their log-probabilities
    add); rounds[i] = number of rounds that fired for rollout i.  The expectation is the mean over the
    prompts of the batch.  Returns (per-layer losses [L], total loss)."""
    lp = np.asarray(logp, np.float64)
    R, L, B, H = lp.shape
    adv = advantages(reward, group)
    prompts = B // group
    per_layer = np.zeros(L, np.float64)
    for l in range(L):
        acc = 0.0
        for p in range(prompts):
            inner = 0.0
            for i in range(p * group, (p + 1) * group):
                n = int(rounds[i])
                if n == 0:
                    continue
                mean_rounds = 0.0
                for t in range(n):
                    for h in range(H):
                        mean_rounds += lp[t, l, i, h]
                inner += (mean_rounds / n) * adv[i]
            acc += inner / group
        per_layer[l] = -acc / prompts
    return per_layer, float(per_layer.sum())


# ------------------------------------------------------------ compaction --

def compact_rows(rows_u16, kept, block: int = 1) -> np.ndarray:
    """rows_u16: [n, D] uint16.  Returns the packed surviving rows [n_new, D]."""
    src = _arr(rows_u16, np.uint16)
    n, D = src.shape
    kp = _arr(kept, np.int32)
    dst = np.zeros_like(src)
    n_new = _L().orc_compact_rows(_p(src, C.c_uint16), _p(dst, C.c_uint16), n, D, block,
                                  _p(kp, C.c_int32), kp.size)
    return dst[:n_new].copy()


def compact_rows_unordered(rows_u16, kept) -> np.ndarray:
    """Hole-filling arrangement of the same survivors (single rows): [K, D]."""
    src = _arr(rows_u16, np.uint16)
    n, D = src.shape
    kp = _arr(kept, np.int32)
    dst = np.zeros_like(src)
    n_new = _L().orc_compact_rows_unordered(_p(src, C.c_uint16), _p(dst, C.c_uint16), n, D,
                                            _p(kp, C.c_int32), kp.size)
    if n_new < 0:
        raise MemoryError
    return dst[:n_new].copy()


def compact_i32(vals, kept, block: int = 1) -> np.ndarray:
    src = _arr(vals, np.int32)
    kp = _arr(kept, np.int32)
    dst = np.zeros_like(src)
    n_new = _L().orc_compact_i32(_p(src, C.c_int32), _p(dst, C.c_int32), src.size, block,
                                 _p(kp, C.c_int32), kp.size)
    return dst[:n_new].copy()


# ------------------------------------------------------------- attention --

def decode_attn(q_u16, k_u16, v_u16, scale: float) -> np.ndarray:
    """q: [G, D], k, v: [n, D] (bf16 bit patterns).  Returns fp32 [G, D]."""
    q = _arr(q_u16, np.uint16)
    k = _arr(k_u16, np.uint16)
    v = _arr(v_u16, np.uint16)
    G, D = q.shape
    n = k.shape[0]
    assert k.shape == v.shape and (n == 0 or k.shape[1] == D)
    out = np.zeros((G, D), np.float32)
    _L().orc_decode_attn(_p(q, C.c_uint16), _p(k, C.c_uint16), _p(v, C.c_uint16), n, G, D,
                         float(scale), _p(out, C.c_float))
    return out


def decode_lse(q_u16, k_u16, scale: float) -> np.ndarray:
    """Log-sum-exp of the scaled scores per query head: fp64 [G]."""
    q = _arr(q_u16, np.uint16)
    k = _arr(k_u16, np.uint16)
    G, D = q.shape
    out = np.zeros(G, np.float64)
    _L().orc_decode_lse(_p(q, C.c_uint16), _p(k, C.c_uint16), k.shape[0], G, D, float(scale), _p(out, C.c_double))
    return out


# --------------------------------------------------------------- scoring --

def score_keys(q_u16, k_u16, scale: float, causal: bool = True) -> np.ndarray:
    """q: [w, G, D], k: [n, D] (bf16 bit patterns).  Returns psi, fp64 [n]."""
    q = _arr(q_u16, np.uint16)
    k = _arr(k_u16, np.uint16)
    w, G, D = q.shape
    n = k.shape[0]
    psi = np.zeros(max(n, 1), np.float64)
    _L().orc_score_keys(_p(q, C.c_uint16), _p(k, C.c_uint16), n, w, G, D, float(scale), int(bool(causal)),
                        _p(psi, C.c_double))
    return psi[:n]


def block_means(psi, block: int) -> np.ndarray:
    x = _arr(psi, np.float64)
    N = (x.size + block - 1) // block
    s = np.zeros(max(N, 1), np.float64)
    _L().orc_block_means(_p(x, C.c_double), x.size, block, _p(s, C.c_double))
    return s[:N]


# ---------------------------------------------------------------- replay --

def replay_death(T: int, boundaries, decisions) -> np.ndarray:
    """Turn per-round retention decisions into one number per token (Appendix
    A.3): round r fires when `boundaries[r]` tokens exist; `decisions[r]` is a
    0/1 vector over the tokens alive at that moment (ascending); a token that a
    round drops is invisible to every query from position boundaries[r] on.
    Returns death[T]: first query position that cannot see the token (T if
    it survives to the end)."""
    death = np.full(T, T, np.int32)
    alive = []
    nxt = 0
    for bnd, dec in zip(boundaries, decisions):
        alive.extend(range(nxt, bnd))
        nxt = bnd
        dec = np.asarray(dec).astype(bool)
        assert dec.size == len(alive), "one decision per alive token"
        for tok, keep in zip(alive, dec):
            if not keep:
                death[tok] = bnd
        alive = [tok for tok, keep in zip(alive, dec) if keep]
    return death


def replay_mask(death) -> np.ndarray:
    """Dense replay mask: M[i, j] = (j <= i < death[j])."""
    d = np.asarray(death)
    T = d.size
    i = np.arange(T)[:, None]
    j = np.arange(T)[None, :]
    return (j <= i) & (i < d[None, :])


def replay_attn(q_u16, k_u16, v_u16, death, scale: float) -> np.ndarray:
    """q: [T, G, D], k, v: [T, D], death: [T].  Returns fp32 [T, G, D]."""
    q = _arr(q_u16, np.uint16)
    k = _arr(k_u16, np.uint16)
    v = _arr(v_u16, np.uint16)
    dd = _arr(death, np.int32)
    T, G, D = q.shape
    out = np.zeros((T, G, D), np.float32)
    _L().orc_replay_attn(_p(q, C.c_uint16), _p(k, C.c_uint16), _p(v, C.c_uint16), _p(dd, C.c_int32), T, G, D,
                         float(scale), _p(out, C.c_float))
    return out


# ------------------------------------------------- host-integer schedule --

def keep_count(n: int, num: int, den: int) -> int:
    """Items kept out of n at retention rate num/den (= 1 - eviction rate):
    the ceiling, at least 1 and at most n (Sec. 4.1 leaves the rounding open)."""
    if n <= 0:
        return 0
    k = -((-n * num) // den)
    return max(1, min(n, k))


def trajectory_fraction(c0: int, delta: int, num: int, den: int, rounds: int):
    """Cache sizes immediately before each eviction round when every round
    keeps the fraction num/den of the cache and delta tokens follow
    (Appendix A.2: c_{t+1} = (1 - eps) c_t + delta)."""
    sizes, c = [], c0
    for _ in range(rounds):
        sizes.append(c)
        c = keep_count(c, num, den) + delta
    return sizes


def steady_state(delta: int, num: int, den: int) -> Fraction:
    """Fixed point delta / eps of the recursion above (Appendix A.2)."""
    eps = 1 - Fraction(num, den)
    return Fraction(delta) / eps
