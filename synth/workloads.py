"""Synthetic workload generator: shapes and skew of Switch-base-128/256 MoE layers.

Every tensor is drawn from ``numpy.random`` generators seeded from one integer, in fixed
size chunks, so the same seed gives the same bits whatever the number of worker threads.
Low-precision ("bf16") tensors are stored as ``uint16`` bit patterns (the upper half of an
IEEE binary32, rounded to nearest-even), so that every consumer reads identical bits.

Nothing here evaluates the method (see the package docstring).
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

SEED0 = 1153700
_CHUNK = 1 << 22  # elements per independently seeded chunk

F32 = 0
BF16 = 1

# The five workloads (T tokens, d model width, F hidden width, E experts, C slot capacity,
# R replica budget, s Zipf exponent).  C = capacity_factor * T / E is an integer in each.
CONFIGS = {
    1: dict(dtype=F32, T=512, d=64, F=256, E=8, C=80, R=4, zipf_s=1.2, seq=512),
    2: dict(dtype=BF16, T=4096, d=768, F=3072, E=128, C=40, R=16, zipf_s=1.0, seq=512),
    3: dict(dtype=BF16, T=4096, d=768, F=3072, E=128, C=40, R=16, zipf_s=1.0, seq=512,
            sru=dict(B=8, L=512, n_in=768, n_hidden=256, n_layers=2, n_out=128),
            agree=0.85, alpha=8.0, beta=1.0),
    4: dict(dtype=BF16, T=16384, d=768, F=3072, E=256, C=64, R=32, zipf_s=1.1, seq=512,
            C_alt=128),
    5: dict(dtype=BF16, T=65536, d=768, F=3072, E=256, C=1024, R=64, zipf_s=1.0, seq=512,
            n_layers=6, hot_share=0.5, alpha=8.0, beta=1.0),
}


# ----------------------------------------------------------------------------- storage
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """binary32 -> upper-16-bit pattern, round to nearest, ties to even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_storage(a: np.ndarray, dtype: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return bf16_bits(a) if dtype == BF16 else a


def storage_to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of either storage format to float64."""
    if a.dtype == np.uint16:
        return bf16_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# ----------------------------------------------------------------------------- draws
def _n_threads() -> int:
    env = os.environ.get("OMP_NUM_THREADS")
    n = int(env) if env and env.isdigit() else (os.cpu_count() or 1)
    return max(1, min(n, 16))


def normal_tensor(shape, std: float, seed, dtype: int) -> np.ndarray:
    """N(0, std^2) tensor in the storage format of ``dtype``; chunk-seeded, thread-parallel."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16 if dtype == BF16 else np.float32)
    n_chunks = (n + _CHUNK - 1) // _CHUNK
    children = np.random.SeedSequence(seed).spawn(max(n_chunks, 1))

    def fill(i: int) -> None:
        lo = i * _CHUNK
        hi = min(n, lo + _CHUNK)
        g = np.random.Generator(np.random.Philox(children[i]))
        v = g.standard_normal(hi - lo, dtype=np.float32)
        v *= np.float32(std)
        out[lo:hi] = bf16_bits(v) if dtype == BF16 else v

    if n_chunks <= 1:
        if n:
            fill(0)
    else:
        with ThreadPoolExecutor(_n_threads()) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


def zipf_weights(n: int, s: float) -> np.ndarray:
    """Normalised Zipf popularity w_k ~ k^-s, k = 1..n (float64)."""
    w = np.arange(1, n + 1, dtype=np.float64) ** (-float(s))
    return w / w.sum()


def _rng(seed, stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream)])


# ----------------------------------------------------------------------------- MoE layer
def moe_layer_inputs(T: int, d: int, F: int, E: int, dtype: int, zipf_s: float, seed: int,
                     weights: bool = True) -> dict:
    """Tokens, router and expert weights with a Zipf popularity bias on the router logits.

    x ~ N(0,1); Wr, W1, W2 ~ N(0, 0.02^2).  Popularity rank k (1 = hottest) is mapped to an
    expert id by a seeded permutation, and expert e gets the logit bias
    ``kappa * ln(w_rank(e) / w_1)`` with ``kappa = 0.5 * 0.02*sqrt(d)``: the Gaussian spread of
    one logit (standard deviation 0.02*sqrt(d)) plays the role of Gumbel noise, so the share of
    tokens whose largest logit is e comes out close to the Zipf share.  (The Gumbel-equivalent
    factor sqrt(6)/pi = 0.78 over-concentrates, a Gaussian tail being lighter; 0.5 was calibrated by
    simulation: the hottest expert's share lands within ~2 points of its Zipf share at E = 128/256.)
    """
    out = dict(T=T, d=d, F=F, E=E, dtype=dtype, seed=seed)
    out["x"] = normal_tensor((T, d), 1.0, [seed, 1], dtype)
    out["w_router"] = normal_tensor((d, E), 0.02, [seed, 2], dtype)
    g = _rng(seed, 3)
    rank_of = g.permutation(E)              # expert e has popularity rank rank_of[e] (0 = hottest)
    w = zipf_weights(E, zipf_s)
    kappa = 0.5 * 0.02 * math.sqrt(d)
    out["b_router"] = (kappa * np.log(w[rank_of] / w[0])).astype(np.float32)
    out["rank_of"] = rank_of.astype(np.int32)
    if weights:
        out["w1"] = normal_tensor((E, d, F), 0.02, [seed, 4], dtype)
        out["w2"] = normal_tensor((E, F, d), 0.02, [seed, 5], dtype)
    return out


def planted_ids_hot_zipf(T: int, E: int, hot_share: float, zipf_s: float, seed: int) -> np.ndarray:
    """Per-token planted expert id: exactly round(hot_share*T) tokens (at random positions)
    carry one hot id, the others are drawn Zipf(s) over the remaining E-1 ids; popularity
    ranks are mapped to ids by a seeded permutation."""
    g = _rng(seed, 11)
    id_of_rank = g.permutation(E)
    n_hot = int(round(hot_share * T))
    z = np.empty(T, dtype=np.int64)
    pos = g.permutation(T)
    z[pos[:n_hot]] = 0
    z[pos[n_hot:]] = 1 + g.choice(E - 1, size=T - n_hot, p=zipf_weights(E - 1, zipf_s))
    return id_of_rank[z].astype(np.int32)


def mix_ids(pred: np.ndarray, E: int, agree: float, zipf_s: float, seed: int) -> np.ndarray:
    """Ids that equal ``pred`` on a Bernoulli(agree) subset of tokens and are redrawn from a
    Zipf(s) popularity over E ids (seeded rank->id permutation) elsewhere."""
    g = _rng(seed, 12)
    T = pred.shape[0]
    id_of_rank = g.permutation(E)
    redraw = id_of_rank[g.choice(E, size=T, p=zipf_weights(E, zipf_s))]
    keep = g.random(T) < agree
    return np.where(keep, pred, redraw).astype(np.int32)


def planted_layer_inputs(z: np.ndarray, d: int, F: int, E: int, dtype: int, seed: int,
                         alpha: float, beta: float, n_layers: int = 1, weights: bool = True,
                         x_only_first: bool = True) -> dict:
    """Tokens and router weights in which id z[s] is planted as token s's largest logit.

    u_0..u_{E-1} are orthonormal directions of R^d (QR of a seeded Gaussian, needs E <= d).
    x_s = g_s + alpha*u_{z_s} with g ~ N(0,1).  Layer l has Wr_l[:, e] = N(0, 0.02^2) +
    beta*u_{sigma_l(e)} with sigma_0 the identity and sigma_l a seeded permutation, so the
    planted logit alpha*beta sits on expert sigma_l^-1(z_s) and the per-expert load is the
    same multiset of counts in every layer.  Router bias is zero.
    """
    assert E <= d
    T = z.shape[0]
    g = _rng(seed, 21)
    q, _ = np.linalg.qr(g.standard_normal((d, E)))
    u = q.T.astype(np.float32)                       # [E, d]
    xg = bf16_to_f32(normal_tensor((T, d), 1.0, [seed, 22], BF16)) if dtype == BF16 else \
        normal_tensor((T, d), 1.0, [seed, 22], F32)
    x = xg + np.float32(alpha) * u[z]
    out = dict(T=T, d=d, F=F, E=E, dtype=dtype, seed=seed, z=z.astype(np.int32),
               x=f32_to_storage(x, dtype), layers=[])
    for l in range(n_layers):
        sigma = np.arange(E) if l == 0 else _rng(seed, 30 + l).permutation(E)
        wr = normal_tensor((d, E), 0.02, [seed, 40 + l], F32) + np.float32(beta) * u[sigma].T
        lay = dict(w_router=f32_to_storage(wr, dtype), b_router=np.zeros(E, np.float32),
                   sigma=sigma.astype(np.int32))
        if weights:
            lay["w1"] = normal_tensor((E, d, F), 0.02, [seed, 50 + l], dtype)
            lay["w2"] = normal_tensor((E, F, d), 0.02, [seed, 60 + l], dtype)
        out["layers"].append(lay)
    return out


# ----------------------------------------------------------------------------- SRU predictor
def sru_inputs(B: int, L: int, n_in: int, n_hidden: int, n_layers: int, n_out: int, dtype: int,
               seed: int, bias_std: float = 0.0, w_std: float = 0.05) -> dict:
    """Embeddings ~N(0,1) and SRU weights ~N(0, w_std^2).

    Layer l's ``w_cat`` is [n_in_l, k_l*n_hidden]: column blocks W | W_f | W_r, then W_h
    when n_in_l != n_hidden (k_l = 4), else k_l = 3.  Biases are zero unless bias_std > 0.
    """
    out = dict(B=B, L=L, n_in=n_in, n_hidden=n_hidden, n_layers=n_layers, n_out=n_out,
               dtype=dtype, seed=seed)
    out["emb"] = normal_tensor((B, L, n_in), 1.0, [seed, 70], dtype)
    out["w_cat"], out["b_f"], out["b_r"] = [], [], []
    g = _rng(seed, 71)
    for l in range(n_layers):
        nin = n_in if l == 0 else n_hidden
        k = 3 if nin == n_hidden else 4
        out["w_cat"].append(normal_tensor((nin, k * n_hidden), w_std, [seed, 72 + l], dtype))
        out["b_f"].append((bias_std * g.standard_normal(n_hidden)).astype(np.float32))
        out["b_r"].append((bias_std * g.standard_normal(n_hidden)).astype(np.float32))
    out["w_head"] = normal_tensor((n_hidden, n_out), w_std, [seed, 90], dtype)
    out["b_head"] = (bias_std * g.standard_normal(n_out)).astype(np.float32)
    return out


# ----------------------------------------------------------------------------- named configs
def config_inputs(cfg_id: int, weights: bool = True, pred: np.ndarray | None = None) -> dict:
    """Inputs of one of the five named workloads.

    Configs 1, 2, 4: Zipf-biased router (``moe_layer_inputs``).
    Config 3: returns the SRU inputs under key ``sru``; when ``pred`` (the predictor's ids,
    computed by the caller) is given, also the planted layer whose router agrees with
    ``pred`` on ~85% of tokens.
    Config 5: planted ids with one hot expert at 50%, 6 layers of independent weights.
    """
    c = dict(CONFIGS[cfg_id])
    seed = SEED0 + cfg_id
    if cfg_id in (1, 2, 4):
        out = moe_layer_inputs(c["T"], c["d"], c["F"], c["E"], c["dtype"], c["zipf_s"], seed,
                               weights=weights)
    elif cfg_id == 3:
        s = c["sru"]
        out = dict(sru=sru_inputs(s["B"], s["L"], s["n_in"], s["n_hidden"], s["n_layers"],
                                  s["n_out"], c["dtype"], seed))
        if pred is not None:
            z = mix_ids(np.asarray(pred, dtype=np.int32), c["E"], c["agree"], c["zipf_s"], seed)
            lay = planted_layer_inputs(z, c["d"], c["F"], c["E"], c["dtype"], seed, c["alpha"],
                                       c["beta"], 1, weights=weights)
            out.update({k: v for k, v in lay.items() if k != "layers"})
            out.update(lay["layers"][0])
    elif cfg_id == 5:
        z = planted_ids_hot_zipf(c["T"], c["E"], c["hot_share"], c["zipf_s"], seed)
        out = planted_layer_inputs(z, c["d"], c["F"], c["E"], c["dtype"], seed, c["alpha"],
                                   c["beta"], c["n_layers"], weights=weights)
    else:
        raise KeyError(cfg_id)
    out.update({k: v for k, v in c.items() if k not in out})
    out["cfg"] = cfg_id
    return out
