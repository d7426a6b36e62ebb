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


def decode_step(q_t, k_t, v_t, w_t, beta_t, kc, vc, scale, round_cache=None, logf_t=None, cc=None):
    """One decoding step.  kc, vc [..., n, d]: caches before the step.

    Returns o_t [..., d], lse_t [...], and the caches after the step ([..., n+1, d]).
    ``round_cache`` (optional) is applied to the refreshed keys before they are used and
    stored: it models a cache kept in a narrower storage type, where the rounding of every
    in-place update is part of the method as run.

    PaTH-FoX (Sec. 2.2 extension, at decode time): ``logf_t`` [...] is the arriving token's log gate and ``cc``
    [..., n] the running sums c_i = sum_{s<=i} log f_s of the cached tokens.  The arriving token's sum is
    c_t = c_{t-1} + log f_t, key i's logit gets c_t - c_i = sum_{s=i+1..t} log f_s (the token's own gets 0), and
    the sums after the step, [..., n+1], are returned as a fifth value.
    """
    q_t = np.asarray(q_t, dtype=np.float64)
    kc = cache_update(kc, w_t, beta_t)
    kc = np.concatenate([kc, np.asarray(k_t, dtype=np.float64)[..., None, :]], axis=-2)
    if round_cache is not None:
        kc = round_cache(kc)
    vc = np.concatenate([np.asarray(vc, dtype=np.float64), np.asarray(v_t, dtype=np.float64)[..., None, :]], axis=-2)
    s = scale * np.einsum("...nd,...d->...n", kc, q_t)
    if logf_t is not None:
        cc = np.asarray(cc, dtype=np.float64)
        prev = cc[..., -1] if cc.shape[-1] else np.zeros(cc.shape[:-1])
        cc = np.concatenate([cc, (prev + np.asarray(logf_t, dtype=np.float64))[..., None]], axis=-1)
        s = s + (cc[..., -1:] - cc)
    m = s.max(axis=-1, keepdims=True)
    p = np.exp(s - m)
    z = p.sum(axis=-1, keepdims=True)
    o = np.einsum("...n,...nd->...d", p / z, vc)
    lse = (m + np.log(z))[..., 0]
    if logf_t is not None:
        return o, lse, kc, vc, cc
    return o, lse, kc, vc
