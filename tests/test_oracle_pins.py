"""Pins for the CPU oracle's building blocks: hand-worked values, closed forms, invariants,
an explicit T x T brute force, and torch CPU library routines (independent of the oracle)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import dsk_oracle as O

rng = np.random.default_rng(1234)


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_hand_example():
    # x = (3,4,0,0): mean square 25/4, root 2.5 -> (1.2, 1.6, 0, 0), then the gains
    y = O.rmsnorm(np.array([[3.0, 4.0, 0.0, 0.0]]), np.array([1.0, 2.0, 5.0, 7.0]), 0.0)
    assert np.allclose(y, [[1.2, 3.2, 0.0, 0.0]], rtol=0, atol=1e-15)


def test_rmsnorm_eps_inside_root():
    # x = 0 except eps: y = x/sqrt(eps) -> with x=(1,1,1,1), eps=3: 1/sqrt(1+3) = 0.5
    y = O.rmsnorm(np.ones((1, 4)), np.ones(4), 3.0)
    assert np.allclose(y, 0.5, atol=1e-15)


def test_rmsnorm_properties_and_library():
    x = rng.standard_normal((7, 48))
    g = rng.standard_normal(48)
    y = O.rmsnorm(x, np.ones(48), 0.0)
    assert np.allclose((y * y).mean(-1), 1.0, atol=1e-12)
    assert np.allclose(O.rmsnorm(17.0 * x, g, 0.0), O.rmsnorm(x, g, 0.0), atol=1e-12)
    ref = F.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), 1e-5).numpy()
    assert np.allclose(O.rmsnorm(x, g, 1e-5), ref, atol=1e-13)


# ---------------------------------------------------------------- RoPE
def test_rope_dh2_closed_form():
    # dh=2: one pair, theta_0 = 1; (1,0) at position 1 -> (cos 1, sin 1); (0,1) -> (-sin 1, cos 1)
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    y = O.rope(x, np.array([1, 1]), 10000.0)
    assert np.allclose(y[0, 0], [0.5403023058681398, 0.8414709848078965], atol=1e-15)
    assert np.allclose(y[1, 0], [-0.8414709848078965, 0.5403023058681398], atol=1e-15)


def test_rope_pairing_and_frequencies():
    # dh=4, base 10000: pairs (0,2) and (1,3); theta = (1, 10000^(-1/2) = 0.01)
    x = np.array([[[0.0, 1.0, 0.0, 0.0]]])
    y = O.rope(x, np.array([50]), 10000.0)  # angle 0.5 on pair (1,3)
    assert np.allclose(y[0, 0], [0.0, math.cos(0.5), 0.0, math.sin(0.5)], atol=1e-15)
    x = np.array([[[2.0, 0.0, 0.0, 0.0]]])
    y = O.rope(x, np.array([3]), 10000.0)   # angle 3 on pair (0,2)
    assert np.allclose(y[0, 0], [2 * math.cos(3.0), 0.0, 2 * math.sin(3.0), 0.0], atol=1e-15)


def test_rope_invariants():
    T, H, dh = 9, 3, 16
    q = rng.standard_normal((T, H, dh))
    k = rng.standard_normal((T, H, dh))
    pos = np.arange(T)
    assert np.array_equal(O.rope(q, np.zeros(T, dtype=np.int64), 5e5), q)          # position 0: identity
    rq = O.rope(q, pos, 5e5)
    half = dh // 2
    assert np.allclose(rq[..., :half] ** 2 + rq[..., half:] ** 2,
                       q[..., :half] ** 2 + q[..., half:] ** 2, atol=1e-12)        # per-pair norm kept
    # <R_m q, R_n k> depends only on m - n
    a = np.einsum("hd,hd->h", O.rope(q[:1], [7], 5e5)[0], O.rope(k[:1], [3], 5e5)[0])
    b = np.einsum("hd,hd->h", O.rope(q[:1], [104], 5e5)[0], O.rope(k[:1], [100], 5e5)[0])
    assert np.allclose(a, b, atol=1e-10)


# ---------------------------------------------------------------- SiLU
def test_silu_values():
    assert O.silu(np.array(0.0)) == 0.0
    assert np.isclose(O.silu(np.array(1.0)), 0.7310585786300049, atol=1e-15)   # 1/(1+e^-1)
    assert np.isclose(O.silu(np.array(-2.0)), -0.2384058440442351, atol=1e-15)
    z = rng.standard_normal(100) * 4
    assert np.allclose(O.silu(z), F.silu(torch.from_numpy(z)).numpy(), atol=1e-14)


# ---------------------------------------------------------------- attention
def brute_force_causal_gqa(q, k, v):
    """Explicit masked T x T scores per head, written independently of the oracle."""
    T, Hq, dh = q.shape
    Hkv = k.shape[1]
    rep = Hq // Hkv
    kk = np.repeat(k, rep, axis=1)
    vv = np.repeat(v, rep, axis=1)
    out = np.zeros_like(q)
    for h in range(Hq):
        S = np.zeros((T, T))
        for i in range(T):
            for j in range(T):
                S[i, j] = sum(q[i, h, e] * kk[j, h, e] for e in range(dh)) / math.sqrt(dh) if j <= i else -math.inf
        P = np.exp(S - S.max(axis=1, keepdims=True))
        P /= P.sum(axis=1, keepdims=True)
        out[:, h, :] = P @ vv[:, h, :]
    return out


def oracle_causal(q, k, v):
    return np.stack([O.attend_row(q[t], k[:t + 1], v[:t + 1]) for t in range(q.shape[0])])


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (6, 1), (8, 2)])
def test_attention_vs_brute_force(Hq, Hkv):
    T, dh = 11, 8
    q = rng.standard_normal((T, Hq, dh)) * 2
    k = rng.standard_normal((T, Hkv, dh)) * 2
    v = rng.standard_normal((T, Hkv, dh))
    assert np.allclose(oracle_causal(q, k, v), brute_force_causal_gqa(q, k, v), atol=1e-12)


@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (8, 1)])
def test_attention_vs_torch_sdpa(Hq, Hkv):
    T, dh = 33, 16
    q = rng.standard_normal((T, Hq, dh))
    k = rng.standard_normal((T, Hkv, dh))
    v = rng.standard_normal((T, Hkv, dh))
    rep = Hq // Hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None].repeat_interleave(rep, dim=1)
    tv = torch.from_numpy(v).permute(1, 0, 2)[None].repeat_interleave(rep, dim=1)
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(oracle_causal(q, k, v), ref, atol=1e-12)


def test_attention_special_cases():
    T, Hq, Hkv, dh = 6, 4, 2, 8
    q = rng.standard_normal((T, Hq, dh))
    k = rng.standard_normal((T, Hkv, dh))
    v = rng.standard_normal((T, Hkv, dh))
    assert np.allclose(oracle_causal(q, k, np.ones_like(v)), 1.0, atol=1e-14)       # weights sum to 1
    assert np.allclose(O.attend_row(q[0], k[:1], v[:1]), np.repeat(v[0], 2, axis=0))  # one key: out = v_0
    out = oracle_causal(np.zeros_like(q), k, v)                                        # uniform scores: running mean
    run_mean = np.cumsum(v, axis=0) / np.arange(1, T + 1)[:, None, None]
    assert np.allclose(out, np.repeat(run_mean, 2, axis=1), atol=1e-14)
    # scale is 1/sqrt(dh): with a single nonzero score of ln(3)*sqrt(dh), weights are (3/4, 1/4) for the later key
    qq = np.zeros((1, dh)); qq[0, 0] = math.log(3.0) * math.sqrt(dh)
    kk = np.zeros((2, 1, dh)); kk[1, 0, 0] = 1.0
    vv = np.zeros((2, 1, dh)); vv[0, 0, :] = 4.0
    assert np.allclose(O.attend_row(qq, kk, vv), 1.0, atol=1e-14)   # 0.25 * 4


def test_gqa_head_mapping_is_contiguous():
    # q heads 0,1 -> kv head 0 ; q heads 2,3 -> kv head 1
    dh = 4
    q = np.zeros((4, dh))
    k = np.zeros((1, 2, dh))
    v = np.zeros((1, 2, dh)); v[0, 0] = 1.0; v[0, 1] = 2.0
    out = O.attend_row(q, k, v)
    assert np.array_equal(out[:, 0], [1.0, 1.0, 2.0, 2.0])
