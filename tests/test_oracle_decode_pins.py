"""Pins of the decode oracle (CPU).  The cache formulation (keys refreshed as tokens arrive,
paper Sec. 3.4) is checked against things it does not share code with: the forward oracle's
query-side walk (paper Sec. 2.2 definition), closed forms, and special cases."""
import numpy as np

from oracle import decode_oracle as dec
from oracle import path_oracle
from paper_2505_16381_amd import synth_inputs as si


def _x(L=37, d=8, seed=11, B=1, H=2):
    return si.make_inputs(B, H, L, d, "fp32", seed, 0.0)


def test_prefilled_cache_reproduces_the_walk_logits_of_the_last_query():
    # q_l . k_i^(l) * scale must equal the definition's logit s_{l,i}, which the forward oracle
    # gets by transforming the QUERY leftwards -- a different order of the same product.
    x = _x()
    scale = 0.3
    kc = dec.key_prefill(x["k"], x["w"], x["beta"])
    last = x["q"].shape[2] - 1
    got = scale * np.einsum("bhnd,bhd->bhn", kc, x["q"][:, :, last].astype(np.float64))
    for b in range(x["q"].shape[0]):
        for h in range(x["q"].shape[1]):
            S = path_oracle.logits(x["q"][b, h], x["k"][b, h], x["w"][b, h], x["beta"][b, h], scale)   # [L,L], row i = query i
            assert np.abs(got[b, h] - S[last, :]).max() <= 1e-12


def test_decode_steps_equal_forward_rows():
    # prefill on the first l0 tokens, then decode the rest one by one: every step's output and
    # log-sum-exp equal the forward oracle's row.
    x = _x(L=29, d=8, seed=5)
    scale = 8 ** -0.5
    o_ref, lse_ref = path_oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale)
    l0 = 10
    kc = dec.key_prefill(x["k"][:, :, :l0 - 1], x["w"][:, :, :l0 - 1], x["beta"][:, :, :l0 - 1])
    vc = x["v"][:, :, :l0 - 1].astype(np.float64)
    for t in range(l0 - 1, 29):
        o, lse, kc, vc = dec.decode_step(x["q"][:, :, t], x["k"][:, :, t], x["v"][:, :, t], x["w"][:, :, t],
                                         x["beta"][:, :, t], kc, vc, scale)
        assert np.abs(o - o_ref[:, :, t]).max() <= 1e-12
        assert np.abs(lse - lse_ref[:, :, t]).max() <= 1e-12


def test_gated_decode_steps_equal_gated_forward_rows():
    # PaTH-FoX at decode time: with the running gate sums of the cached tokens, prefill + decoding reproduces the
    # gated forward oracle's rows (code the decode oracle shares nothing with); gates of exactly 1 (log f = 0)
    # reproduce the plain steps.
    x = _x(L=31, d=8, seed=6)
    scale = 8 ** -0.5
    rng = np.random.default_rng(6)
    logf = -np.log1p(np.exp(-rng.normal(1.0, 1.0, size=x["beta"].shape)))
    o_ref, lse_ref = path_oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, logf=logf)
    l0 = 12
    kc = dec.key_prefill(x["k"][:, :, :l0], x["w"][:, :, :l0], x["beta"][:, :, :l0])
    vc = x["v"][:, :, :l0].astype(np.float64)
    cc = np.cumsum(logf[:, :, :l0], axis=-1)
    kc0, vc0 = kc.copy(), vc.copy()
    for t in range(l0, 31):
        o, lse, kc, vc, cc = dec.decode_step(x["q"][:, :, t], x["k"][:, :, t], x["v"][:, :, t], x["w"][:, :, t],
                                             x["beta"][:, :, t], kc, vc, scale, logf_t=logf[:, :, t], cc=cc)
        assert np.abs(o - o_ref[:, :, t]).max() <= 1e-12
        assert np.abs(lse - lse_ref[:, :, t]).max() <= 1e-12
    assert np.abs(cc - np.cumsum(logf, axis=-1)).max() <= 1e-12
    plain = dec.decode_step(x["q"][:, :, l0], x["k"][:, :, l0], x["v"][:, :, l0], x["w"][:, :, l0], x["beta"][:, :, l0], kc0, vc0, scale)
    unit = dec.decode_step(x["q"][:, :, l0], x["k"][:, :, l0], x["v"][:, :, l0], x["w"][:, :, l0], x["beta"][:, :, l0], kc0, vc0, scale,
                           logf_t=np.zeros(x["beta"].shape[:2]), cc=np.zeros(x["beta"].shape[:2] + (l0,)))
    assert np.array_equal(plain[0], unit[0]) and np.array_equal(plain[1], unit[1])
    # an empty cache: the first token attends only itself, whatever its gate
    e = dec.decode_step(x["q"][:, :, 0], x["k"][:, :, 0], x["v"][:, :, 0], x["w"][:, :, 0], x["beta"][:, :, 0],
                        x["k"][:, :, :0].astype(np.float64), x["v"][:, :, :0].astype(np.float64), scale,
                        logf_t=logf[:, :, 0], cc=logf[:, :, :0])
    assert np.abs(e[0] - x["v"][:, :, 0]).max() <= 1e-12 and np.abs(e[4][..., 0] - logf[:, :, 0]).max() <= 1e-15


def test_beta_zero_leaves_the_cache_alone_and_beta_two_reflects():
    x = _x(L=12, d=6, seed=3)
    kc = x["k"].astype(np.float64)
    w = x["w"][:, :, 0].astype(np.float64)
    w = w / np.linalg.norm(w, axis=-1, keepdims=True)          # unit in fp64, not just in fp32
    assert np.array_equal(dec.cache_update(kc, w, np.zeros(w.shape[:-1])), kc)
    # beta = 2 with unit w is a reflection: applying it twice is the identity, norms are kept
    r1 = dec.cache_update(kc, w, 2 * np.ones(w.shape[:-1]))
    r2 = dec.cache_update(r1, w, 2 * np.ones(w.shape[:-1]))
    assert np.abs(r2 - kc).max() <= 1e-12
    assert np.abs(np.linalg.norm(r1, axis=-1) - np.linalg.norm(kc, axis=-1)).max() <= 1e-12


def test_one_update_closed_form_and_transposed_operand_trap():
    # k' = k - beta (w.k) w, written out for one key; an update with w and k swapped, or with the
    # outer product transposed, gives a different vector for these numbers.
    k = np.array([[1.0, 2.0, -1.0]])
    w = np.array([0.6, 0.0, 0.8])
    beta = np.array(1.5)
    got = dec.cache_update(k, w, beta)
    want = np.array([[1.0 - 1.5 * (-0.2) * 0.6, 2.0, -1.0 - 1.5 * (-0.2) * 0.8]])
    assert np.abs(got - want).max() <= 1e-15
    wrong = k - 1.5 * (k @ k.T) * w          # (k.k) instead of (w.k)
    assert np.abs(wrong - want).max() > 0.1


def test_last_key_enters_untouched_and_order_of_transitions_matters():
    x = _x(L=9, d=5, seed=21)
    kc = dec.key_prefill(x["k"], x["w"], x["beta"])
    assert np.array_equal(kc[:, :, -1], x["k"][:, :, -1].astype(np.float64))
    # k_0^(l) = H_{l-1} ... H_1 k_0 (later transitions applied last): brute force with explicit matrices
    b, h = 0, 1
    u = x["k"][b, h, 0].astype(np.float64)
    for t in range(1, 9):
        wt = x["w"][b, h, t].astype(np.float64)
        Ht = np.eye(5) - float(x["beta"][b, h, t]) * np.outer(wt, wt)
        u = Ht @ u
    assert np.abs(kc[b, h, 0] - u).max() <= 1e-13
    # the reversed order is a different vector (the transitions do not commute)
    u2 = x["k"][b, h, 0].astype(np.float64)
    for t in range(8, 0, -1):
        wt = x["w"][b, h, t].astype(np.float64)
        u2 = (np.eye(5) - float(x["beta"][b, h, t]) * np.outer(wt, wt)) @ u2
    assert np.abs(u2 - u).max() > 1e-3


def test_round_cache_hook_rounds_what_is_stored_and_what_is_used():
    # The hook models a cache kept in a narrower type.  Pinned against the un-hooked step (itself pinned
    # above) and against plain softmax attention written out here: (1) it is called once per step, on the
    # refreshed keys with the arriving key appended, i.e. on exactly what the un-hooked step returns;
    # (2) what the step returns as the new cache is the hook's result, a fixed point of the rounding;
    # (3) the logits use the ROUNDED keys -- o and lse equal softmax attention over the returned cache,
    # and differ from the un-hooked step's; (4) an identity hook changes nothing; (5) with beta = 0 and
    # keys that the narrow type holds exactly, rounding is invisible.
    x = _x(L=14, d=8, seed=33)
    scale = 0.4
    rnd = lambda a: si.round_to_bf16(a.astype(np.float32)).astype(np.float64)
    n = 9
    kc0 = dec.key_prefill(x["k"][:, :, :n], x["w"][:, :, :n], x["beta"][:, :, :n])
    vc0 = x["v"][:, :, :n].astype(np.float64)
    a = (x["q"][:, :, n], x["k"][:, :, n], x["v"][:, :, n], x["w"][:, :, n], x["beta"][:, :, n])
    o_plain, lse_plain, kc_plain, vc_plain = dec.decode_step(*a, kc0, vc0, scale)
    seen = []
    def hook(k):
        seen.append(k.copy())
        return rnd(k)
    o_r, lse_r, kc_r, vc_r = dec.decode_step(*a, kc0, vc0, scale, round_cache=hook)
    assert len(seen) == 1 and np.array_equal(seen[0], kc_plain)                       # (1)
    assert np.array_equal(kc_r, rnd(kc_plain)) and np.array_equal(rnd(kc_r), kc_r)    # (2)
    assert np.array_equal(vc_r, vc_plain)                                             # values are not touched
    s = scale * np.einsum("bhnd,bhd->bhn", kc_r, a[0].astype(np.float64))             # (3)
    p = np.exp(s - s.max(-1, keepdims=True)); z = p.sum(-1, keepdims=True)
    assert np.abs(np.einsum("bhn,bhnd->bhd", p / z, vc_r) - o_r).max() <= 1e-14
    assert np.abs(np.log(z[..., 0]) + s.max(-1) - lse_r).max() <= 1e-14
    assert np.abs(o_r - o_plain).max() > 1e-5                                         # the rounding is visible
    o_i, lse_i, kc_i, _ = dec.decode_step(*a, kc0, vc0, scale, round_cache=lambda k: k)   # (4)
    assert np.array_equal(o_i, o_plain) and np.array_equal(lse_i, lse_plain) and np.array_equal(kc_i, kc_plain)
    kb = rnd(x["k"][:, :, :n + 1].astype(np.float64))                                 # (5)
    zero = np.zeros_like(x["beta"][:, :, n])
    o5, l5, k5, _ = dec.decode_step(a[0], kb[:, :, n], a[2], a[3], zero, kb[:, :, :n], vc0, scale, round_cache=rnd)
    o6, l6, k6, _ = dec.decode_step(a[0], kb[:, :, n], a[2], a[3], zero, kb[:, :, :n], vc0, scale)
    assert np.array_equal(o5, o6) and np.array_equal(l5, l6) and np.array_equal(k5, k6)
