"""fp64 CPU oracle of PaTH's decode path (paper Sec. 3.4 "Efficient Inference").

TEST INFRASTRUCTURE.  Only the tests may import this module; the GPU library and its
Python binding never do.  Plain numpy, written from the paper's two formulas:

* in-place key-cache update (the section's first equation): when token t arrives, every
  cached key is refreshed with that step's transition, k_i <- (I - beta_t w_t w_t^T) k_i for
  i < t, and k_t itself enters the cache untouched;
* after that, decoding IS ordinary softmax attention of q_t over the cache;
* key prefill (the section's second formula): the cache a prompt of length l leaves behind
  holds k_i^(l) = H_l ... H_{i+1} k_i -- here by applying the update token by token, which
  is the definition; the blockwise suffix-product form is the GPU's business.
"""
from __future__ import annotations

import numpy as np


def cache_update(kc, w_t, beta_t):
    """kc [..., n, d] -> keys after the transition of the arriving token (w_t [..., d], beta_t [...])."""
    kc = np.asarray(kc, dtype=np.float64)
    w_t = np.asarray(w_t, dtype=np.float64)
    beta_t = np.asarray(beta_t, dtype=np.float64)
    proj = np.einsum("...nd,...d->...n", kc, w_t)                       # w_t . k_i
    return kc - beta_t[..., None, None] * proj[..., None] * w_t[..., None, :]


def key_prefill(k, w, beta):
    """Cache after a prompt: k, w [..., l, d], beta [..., l] -> k^(l) [..., l, d]."""
    k = np.asarray(k, dtype=np.float64)
    l = k.shape[-2]
    kc = k[..., :0, :]
    for t in range(l):
        kc = cache_update(kc, np.asarray(w)[..., t, :], np.asarray(beta)[..., t])
        kc = np.concatenate([kc, k[..., t:t + 1, :]], axis=-2)
    return kc


def decode_step(q_t, k_t, v_t, w_t, beta_t, kc, vc, scale, round_cache=None):
    """One decoding step.  kc, vc [..., n, d]: caches before the step.

    Returns o_t [..., d], lse_t [...], and the caches after the step ([..., n+1, d]).
    ``round_cache`` (optional) is applied to the refreshed keys before they are used and
    stored: it models a cache kept in a narrower storage type, where the rounding of every
    in-place update is part of the method as run.
    """
    q_t = np.asarray(q_t, dtype=np.float64)
    kc = cache_update(kc, w_t, beta_t)
    kc = np.concatenate([kc, np.asarray(k_t, dtype=np.float64)[..., None, :]], axis=-2)
    if round_cache is not None:
        kc = round_cache(kc)
    vc = np.concatenate([np.asarray(vc, dtype=np.float64), np.asarray(v_t, dtype=np.float64)[..., None, :]], axis=-2)
    s = scale * np.einsum("...nd,...d->...n", kc, q_t)
    m = s.max(axis=-1, keepdims=True)
    p = np.exp(s - m)
    z = p.sum(axis=-1, keepdims=True)
    o = np.einsum("...n,...nd->...d", p / z, vc)
    lse = (m + np.log(z))[..., 0]
    return o, lse, kc, vc
