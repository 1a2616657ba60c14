"""Pins of the fp64 oracle against things other than itself.

The paper prints no worked numeric example for the block, so there are no
printed values to match.  The oracle is pinned by:
  * the bijection statement under Eq. 1-2 (inverse o forward = identity as the
    fixed point converges; stream 2 exactly),
  * central finite differences of the forward pass for every parameter group
    and both inputs (the backward pass shares no code path with this check),
  * equality of the stored-activation and the reconstruction gradient routes,
  * special cases with a textbook value (uniform attention = running mean,
    S = 1, one expert = dense SwiGLU MLP, zero down-projection = identity),
  * library routines (torch scaled_dot_product_attention, scipy expit/softmax),
  * brute force on tiny inputs (all experts computed densely and masked; top-k
    by exhaustive python selection).
"""
import numpy as np
import pytest
import scipy.special
import torch

import synth
from oracle import revffn_oracle as O


def cfg_of(wl, **kw):
    c = O.Config(wl.d_model, wl.n_heads, wl.head_dim, wl.n_experts, wl.top_k,
                 wl.d_expert, wl.d_shared)
    return O.replace(c, **kw)


def rand_weights(cfg, rng, scale, biases=True, router_bias=True):
    d, h, E, I, Is = cfg.d_model, cfg.h, cfg.n_experts, cfg.d_expert, cfg.d_shared
    W = {
        "norm_a1": 1 + 0.1 * rng.standard_normal(h), "norm_a2": 1 + 0.1 * rng.standard_normal(h),
        "norm_m": 1 + 0.1 * rng.standard_normal(h),
        "pup_a": scale * rng.standard_normal((d, h)), "pdn_a": scale * rng.standard_normal((h, d)),
        "pup_m": scale * rng.standard_normal((d, h)), "pdn_m": scale * rng.standard_normal((h, d)),
        "wq": scale * rng.standard_normal((d, d)), "wk": scale * rng.standard_normal((d, d)),
        "wv": scale * rng.standard_normal((d, d)), "wo": scale * rng.standard_normal((d, d)),
        "bq": scale * rng.standard_normal(d) if biases else None,
        "bk": scale * rng.standard_normal(d) if biases else None,
        "bv": scale * rng.standard_normal(d) if biases else None,
        "w_router": scale * rng.standard_normal((E, d)),
        "b_router": 0.3 * rng.standard_normal(E) if router_bias else None,
        "w_gate_up": scale * rng.standard_normal((E, 2 * I, d)),
        "w_down": scale * rng.standard_normal((E, d, I)),
        "ws_gate_up": scale * rng.standard_normal((2 * Is, d)) if Is else None,
        "ws_down": scale * rng.standard_normal((d, Is)) if Is else None,
        "ws_gate": scale * rng.standard_normal(d) if Is else None,
    }
    return W


SMALL = O.Config(d_model=16, n_heads=2, head_dim=8, n_experts=5, top_k=2, d_expert=6, d_shared=7)


# --------------------------------------------------------------------------
# inverse (bijection statement under Eq. 1-2; fixed-point remark at the end of 3.1)
# --------------------------------------------------------------------------
def test_inverse_recovers_input_tiny():
    wl = synth.WORKLOADS["tiny_f32"]
    cfg = cfg_of(wl)
    W = synth.make_weights(wl)
    x1, x2, _, _ = synth.make_inputs(wl)
    y1, y2 = O.forward(x1, x2, W, cfg, wl.B, wl.S)
    assert np.abs(y1 - x1).max() > 1e-4 and np.abs(y2 - x2).max() > 1e-7   # branches are small (weights N(0, 0.02)) but not zero
    r1, r2 = O.inverse(y1, y2, W, cfg, wl.B, wl.S, n_iters=0)
    assert np.abs(r2 - x2).max() < 1e-14            # stream 2 has no implicit term
    assert np.array_equal(r1, y1)                   # zero iterations = the starting point
    e1 = np.abs(O.inverse(y1, y2, W, cfg, wl.B, wl.S, n_iters=1)[0] - x1).max()
    e2 = np.abs(O.inverse(y1, y2, W, cfg, wl.B, wl.S, n_iters=2)[0] - x1).max()
    assert e1 < 1e-8 and e2 < 1e-12 and e2 < e1     # contraction
    xc, _, info = O.inverse(y1, y2, W, cfg, wl.B, wl.S, converge=True, return_info=True)
    assert np.abs(xc - x1).max() < 1e-13 and info["iters"] <= 6


def test_inverse_exact_where_attention_ignores_query():
    """Causal position 0 attends to one key, and S = 1 has one key: the branch then
    does not depend on the query, so one iteration is exact even with big weights."""
    rng = np.random.default_rng(3)
    cfg = SMALL
    W = rand_weights(cfg, rng, 0.5)
    B, S = 2, 6
    x1, x2 = rng.standard_normal((B * S, cfg.h)), rng.standard_normal((B * S, cfg.h))
    y1, y2 = O.forward(x1, x2, W, cfg, B, S)
    r1, r2 = O.inverse(y1, y2, W, cfg, B, S, n_iters=1)
    first = np.arange(B) * S
    assert np.abs(r1[first] - x1[first]).max() < 1e-13
    assert np.abs(r1 - x1).max() > 1e-6             # the other positions are not exact yet
    x1, x2 = rng.standard_normal((3, cfg.h)), rng.standard_normal((3, cfg.h))
    y1, y2 = O.forward(x1, x2, W, cfg, 3, 1)
    r1, r2 = O.inverse(y1, y2, W, cfg, 3, 1, n_iters=1)
    assert np.abs(r1 - x1).max() < 1e-13 and np.abs(r2 - x2).max() < 1e-13


def test_symmetric_variant_closed_form_inverse_and_reduction():
    """The symmetric comparison block of section 3.1 (queries from stream 2 too): its branch ignores stream 1, its
    inverse is exact without any iteration, and where both streams and both norm gains coincide it is the
    asymmetric block's branch."""
    rng = np.random.default_rng(5)
    cfg = O.replace(SMALL, symmetric=True)
    W = rand_weights(cfg, rng, 0.5)                     # far too large for the fixed point to contract
    B, S = 2, 6
    x1, x2 = rng.standard_normal((B * S, cfg.h)), rng.standard_normal((B * S, cfg.h))
    y1, y2 = O.forward(x1, x2, W, cfg, B, S)
    assert np.abs(y1 - x1).max() > 0.1
    r1, r2, info = O.inverse(y1, y2, W, cfg, B, S, n_iters=0, return_info=True)
    assert np.abs(r1 - x1).max() < 1e-13 and np.abs(r2 - x2).max() < 1e-13 and info["iters"] == 0
    # the branch is a function of stream 2 alone
    A, _ = O.attn_half_forward(x1, x2, W, cfg, B, S)
    A2, _ = O.attn_half_forward(rng.standard_normal(x1.shape), x2, W, cfg, B, S)
    assert np.array_equal(A, A2)
    # reduction to the asymmetric branch at X1 = X2 with equal gains
    Wq = dict(W)
    Wq["norm_a1"] = W["norm_a2"]
    A3, _ = O.attn_half_forward(x2, x2, Wq, SMALL, B, S)
    assert np.abs(A - A3).max() < 1e-14 and np.abs(A).max() > 0.1
    # and it is not the asymmetric branch otherwise
    A4, _ = O.attn_half_forward(x1, x2, W, SMALL, B, S)
    assert np.abs(A - A4).max() > 1e-2
    # stored and reconstructed gradient routes agree exactly (the rebuilt input is exact)
    dy1, dy2 = rng.standard_normal(x1.shape), rng.standard_normal(x1.shape)
    dx1, dx2, g = O.grads_stored(x1, x2, dy1, dy2, W, cfg, B, S)
    _, _, qx1, qx2, qg = O.grads_reconstructed(y1, y2, dy1, dy2, W, cfg, B, S)
    assert np.abs(qx1 - dx1).max() < 1e-10 and np.abs(qx2 - dx2).max() < 1e-10
    assert np.abs(g["norm_a1"]).max() == 0.0


def test_zero_down_projection_is_identity():
    """P_dn = 0 on both halves: Y = X, inverse exact, dX = dY (section 3.2 display)."""
    rng = np.random.default_rng(4)
    cfg = SMALL
    W = rand_weights(cfg, rng, 0.3)
    W["pdn_a"] = np.zeros_like(W["pdn_a"])
    W["pdn_m"] = np.zeros_like(W["pdn_m"])
    B, S = 1, 5
    x1, x2 = rng.standard_normal((5, cfg.h)), rng.standard_normal((5, cfg.h))
    y1, y2 = O.forward(x1, x2, W, cfg, B, S)
    assert np.array_equal(y1, x1) and np.array_equal(y2, x2)
    dy1, dy2 = rng.standard_normal((5, cfg.h)), rng.standard_normal((5, cfg.h))
    dx1, dx2, g = O.backward(x1, x2, y1, dy1, dy2, W, cfg, B, S)
    assert np.array_equal(dx1, dy1) and np.array_equal(dx2, dy2)
    assert np.abs(g["wq"]).max() == 0 and np.abs(g["pdn_a"]).max() > 0
    # only the MoE side switched off: classic additive coupling on stream 1 alone
    W["pdn_a"] = 0.3 * rng.standard_normal(W["pdn_a"].shape)
    y1, y2 = O.forward(x1, x2, W, cfg, B, S)
    assert np.array_equal(y2, x2) and np.abs(y1 - x1).max() > 1e-3


# --------------------------------------------------------------------------
# gradients
# --------------------------------------------------------------------------
def test_stored_and_reconstructed_routes_agree():
    wl = synth.WORKLOADS["tiny_shared_f32"]
    cfg = cfg_of(wl)
    W = synth.make_weights(wl)
    x1, x2, dy1, dy2 = synth.make_inputs(wl)
    y1, y2 = O.forward(x1, x2, W, cfg, wl.B, wl.S)
    dx1, dx2, g = O.grads_stored(x1, x2, dy1, dy2, W, cfg, wl.B, wl.S)
    _, _, rx1, rx2, rg = O.grads_reconstructed(y1, y2, dy1, dy2, W, cfg, wl.B, wl.S, n_iters=2)
    assert np.abs(rx1 - dx1).max() < 1e-10 and np.abs(rx2 - dx2).max() < 1e-10
    for k in g:
        assert np.abs(rg[k] - g[k]).max() < 1e-10 * max(1.0, np.abs(g[k]).max()), k
    # with one iteration the routes differ by about (reconstruction error) x (Lipschitz constant)
    _, _, qx1, _, _ = O.grads_reconstructed(y1, y2, dy1, dy2, W, cfg, wl.B, wl.S, n_iters=1)
    assert 0 < np.abs(qx1 - dx1).max() < 1e-6


FD_CASES = [
    dict(),                                                        # causal, rope, biases, shared
    dict(causal=False, use_rope=False, norm_topk_prob=True),
    dict(d_shared=0, norm_topk_prob=True),
    dict(top_k=5),                                                 # k = E: no selection at all
    dict(symmetric=True),                                          # comparison block: queries from stream 2
]


@pytest.mark.parametrize("case", range(len(FD_CASES)))
def test_finite_differences_every_group(case):
    """Central differences of L = <Y1, dY1> + <Y2, dY2> along a random direction in
    each parameter group and each input, plus single entries, against backward()."""
    kw = FD_CASES[case]
    cfg = O.replace(SMALL, **kw)
    rng = np.random.default_rng(10 + case)
    W = rand_weights(cfg, rng, 0.25)
    B, S = 2, 5
    T = B * S
    x1, x2 = rng.standard_normal((T, cfg.h)), rng.standard_normal((T, cfg.h))
    dy1, dy2 = rng.standard_normal((T, cfg.h)), rng.standard_normal((T, cfg.h))

    def loss(W_, a, b):
        y1, y2 = O.forward(a, b, W_, cfg, B, S)
        return float(np.sum(y1 * dy1) + np.sum(y2 * dy2))

    y1, y2, cache = O.forward(x1, x2, W, cfg, B, S, return_cache=True)
    margin = O.topk_margin(cache["moe"]["z"], cfg.top_k).min()
    eps = 1e-6
    assert margin > 1e-3            # perturbations of size eps cannot change the selected set
    dx1, dx2, g = O.backward(x1, x2, None, dy1, dy2, W, cfg, B, S)
    names = [k for k in O.PARAM_NAMES if W.get(k) is not None]
    assert set(names) == set(g.keys())
    for k in names:
        v = rng.standard_normal(W[k].shape)
        Wp, Wm = dict(W), dict(W)
        Wp[k], Wm[k] = W[k] + eps * v, W[k] - eps * v
        fd = (loss(Wp, x1, x2) - loss(Wm, x1, x2)) / (2 * eps)
        an = float(np.sum(g[k] * v))
        assert abs(fd - an) < 2e-7 * max(1.0, abs(an)) + 1e-6 * abs(an), (k, fd, an)
        if k == "bk" and not cfg.use_rope:
            # without rotary encoding a key bias shifts every score of a row equally: softmax ignores it
            assert np.abs(g[k]).max() < 1e-14
            continue
        if k == "norm_a1" and cfg.symmetric:
            assert np.abs(g[k]).max() == 0.0 and fd == 0.0      # stream 1 is not normalised anywhere in that block
            continue
        assert abs(an) > 1e-4, (k, "direction too weak to pin anything")
        # one single entry (catches transposed gradients that a random direction could hide)
        idx = tuple(rng.integers(0, s) for s in W[k].shape)
        Wp, Wm = dict(W), dict(W)
        Wp[k], Wm[k] = W[k].copy(), W[k].copy()
        Wp[k][idx] += eps
        Wm[k][idx] -= eps
        fd = (loss(Wp, x1, x2) - loss(Wm, x1, x2)) / (2 * eps)
        assert abs(fd - g[k][idx]) < 2e-7 * max(1.0, abs(fd)) + 1e-6 * abs(fd), (k, idx, fd, g[k][idx])
    for which, dx in ((0, dx1), (1, dx2)):
        v = rng.standard_normal(x1.shape)
        a = (x1 + eps * v, x2) if which == 0 else (x1, x2 + eps * v)
        b = (x1 - eps * v, x2) if which == 0 else (x1, x2 - eps * v)
        fd = (loss(W, *a) - loss(W, *b)) / (2 * eps)
        an = float(np.sum(dx * v))
        assert abs(fd - an) < 1e-6 * max(1.0, abs(an)), (which, fd, an)


def test_rmsnorm_closed_form_and_gradient():
    g = np.array([1.0, 2.0, -1.0, 0.5])
    x = np.full((1, 4), 3.0)
    assert np.allclose(O.rmsnorm(x, g, 0.0), g[None, :], atol=1e-15)     # x/|x|_rms = 1
    x = np.array([[3.0, -4.0, 0.0, 0.0]])                                # mean square = 25/4
    assert np.allclose(O.rmsnorm(x, np.ones(4), 0.0), x / 2.5, atol=1e-15)
    rng = np.random.default_rng(0)
    x, dy, g = rng.standard_normal((3, 6)), rng.standard_normal((3, 6)), rng.standard_normal(6)
    dx, dg = O.rmsnorm_bwd(dy, x, g, 1e-6)
    eps = 1e-6
    for i in range(3):
        for j in range(6):
            xp, xm = x.copy(), x.copy()
            xp[i, j] += eps
            xm[i, j] -= eps
            fd = np.sum((O.rmsnorm(xp, g, 1e-6) - O.rmsnorm(xm, g, 1e-6)) * dy) / (2 * eps)
            assert abs(fd - dx[i, j]) < 1e-8
    for j in range(6):
        gp, gm = g.copy(), g.copy()
        gp[j] += eps
        gm[j] -= eps
        fd = np.sum((O.rmsnorm(x, gp, 1e-6) - O.rmsnorm(x, gm, 1e-6)) * dy) / (2 * eps)
        assert abs(fd - dg[j]) < 1e-8


# --------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------
@pytest.mark.parametrize("causal", [True, False])
def test_attention_core_matches_library_sdpa(causal):
    rng = np.random.default_rng(1)
    B, S, H, dh = 2, 9, 3, 8
    Q, K, V = (rng.standard_normal((B, S, H, dh)) for _ in range(3))
    Oo, P = O.attention_core(Q, K, V, causal)
    tq, tk, tv = (torch.tensor(a).permute(0, 2, 1, 3) for a in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)
    assert np.abs(Oo - ref.permute(0, 2, 1, 3).numpy()).max() < 1e-13
    assert np.abs(P.sum(-1) - 1).max() < 1e-14
    if causal:
        assert np.all(P[:, :, np.triu_indices(S, 1)[0], np.triu_indices(S, 1)[1]] == 0)


def test_uniform_attention_is_running_mean():
    """Wq = 0, bq = 0 makes every score zero: O is the causal running mean of V."""
    rng = np.random.default_rng(2)
    cfg = O.replace(SMALL, d_shared=0)
    W = rand_weights(cfg, rng, 0.3)
    W["wq"] = np.zeros_like(W["wq"])
    W["bq"] = None
    B, S = 2, 7
    x1, x2 = rng.standard_normal((B * S, cfg.h)), rng.standard_normal((B * S, cfg.h))
    A, c = O.attn_half_forward(x1, x2, W, cfg, B, S)
    V = (O.rmsnorm(x2, W["norm_a2"], cfg.rms_eps) @ W["pup_a"].T @ W["wv"].T + W["bv"]).reshape(B, S, -1)
    mean = np.cumsum(V, axis=1) / np.arange(1, S + 1)[None, :, None]
    expect = mean.reshape(B * S, -1) @ W["wo"].T @ W["pdn_a"].T
    assert np.abs(A - expect).max() < 1e-13
    # queries come from stream 1 only: with uniform attention stream 1 has no influence at all
    A2, _ = O.attn_half_forward(rng.standard_normal(x1.shape), x2, W, cfg, B, S)
    assert np.abs(A2 - A).max() < 1e-13


def test_attention_single_position_returns_value():
    rng = np.random.default_rng(5)
    cfg = SMALL
    W = rand_weights(cfg, rng, 0.3)
    x1, x2 = rng.standard_normal((4, cfg.h)), rng.standard_normal((4, cfg.h))
    A, c = O.attn_half_forward(x1, x2, W, cfg, 4, 1)
    assert np.abs(c["O"] - c["V"].reshape(4, -1)).max() < 1e-14
    # position 0 gets angle 0: rope leaves K untouched there
    Kl = O.rmsnorm(x2, W["norm_a2"], cfg.rms_eps) @ W["pup_a"].T @ W["wk"].T + W["bk"]
    assert np.abs(c["K"].reshape(4, -1) - Kl).max() < 1e-14


def test_attention_causality_batch_independence_and_cross_stream():
    rng = np.random.default_rng(6)
    cfg = SMALL
    W = rand_weights(cfg, rng, 0.3)
    B, S = 2, 6
    x1, x2 = rng.standard_normal((B * S, cfg.h)), rng.standard_normal((B * S, cfg.h))
    A, _ = O.attn_half_forward(x1, x2, W, cfg, B, S)
    # perturb keys/values at position 4 of batch 0: rows 0..3 of batch 0 and all of batch 1 unchanged
    x2p = x2.copy()
    x2p[4] += 1.0
    Ap, _ = O.attn_half_forward(x1, x2p, W, cfg, B, S)
    assert np.abs(Ap[:4] - A[:4]).max() == 0 and np.abs(Ap[S:] - A[S:]).max() == 0
    assert np.abs(Ap[4:S] - A[4:S]).max() > 1e-6
    # perturb the query stream at one token: only that token's row changes
    x1p = x1.copy()
    x1p[3] += 1.0
    Aq, _ = O.attn_half_forward(x1p, x2, W, cfg, B, S)
    changed = np.abs(Aq - A).max(axis=1) > 0
    assert changed.tolist() == [i == 3 for i in range(B * S)]
    # non-causal: a later key does reach earlier rows
    An, _ = O.attn_half_forward(x1, x2, W, O.replace(cfg, causal=False), B, S)
    Anp, _ = O.attn_half_forward(x1, x2p, W, O.replace(cfg, causal=False), B, S)
    assert np.abs(Anp[:4] - An[:4]).max() > 1e-6


def test_rope_is_a_relative_rotation():
    rng = np.random.default_rng(7)
    B, S, H, dh = 1, 12, 2, 8
    q, k = rng.standard_normal((B, S, H, dh)), rng.standard_normal((B, S, H, dh))
    rq, rk = O.rope(q, 1e4), O.rope(k, 1e4)
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), atol=1e-13)
    assert np.abs(rq[:, 0] - q[:, 0]).max() == 0                      # angle 0 at position 0
    assert np.abs(O.rope(rq, 1e4, sign=-1.0) - q).max() < 1e-14        # the inverse rotation
    # <rope(q,s), rope(k,s')> depends only on s - s': same vector placed at shifted positions
    qq = np.broadcast_to(q[:, :1], q.shape).copy()
    kk = np.broadcast_to(k[:, :1], k.shape).copy()
    dots = np.einsum("bshd,bthd->bhst", O.rope(qq, 1e4), O.rope(kk, 1e4))
    for off in range(-3, 4):
        diag = np.diagonal(dots, offset=off, axis1=2, axis2=3)
        assert np.abs(diag - diag[..., :1]).max() < 1e-12
    # the pairing is half-split: element 0 pairs with element dh/2, frequency theta^0 = 1
    e0 = np.zeros((1, 2, 1, dh))
    e0[0, :, 0, 0] = 1.0
    r = O.rope(e0, 1e4)[0, 1, 0]
    expect = np.zeros(dh)
    expect[0], expect[dh // 2] = np.cos(1.0), np.sin(1.0)
    assert np.abs(r - expect).max() < 1e-15
    # last pair uses frequency theta^(-2(dh/2-1)/dh)
    e1 = np.zeros((1, 4, 1, dh))
    e1[0, :, 0, dh // 2 - 1] = 1.0
    ang = 3 * 1e4 ** (-2.0 * (dh // 2 - 1) / dh)
    r = O.rope(e1, 1e4)[0, 3, 0]
    assert abs(r[dh // 2 - 1] - np.cos(ang)) < 1e-15 and abs(r[dh - 1] - np.sin(ang)) < 1e-15


# --------------------------------------------------------------------------
# routing and MoE
# --------------------------------------------------------------------------
def test_element_functions_match_scipy():
    x = np.linspace(-20, 20, 401)
    assert np.abs(O.sigmoid(x) - scipy.special.expit(x)).max() < 1e-15
    assert np.abs(O.silu(x) - x * scipy.special.expit(x)).max() < 1e-14
    eps = 1e-6
    fd = (O.silu(x + eps) - O.silu(x - eps)) / (2 * eps)
    assert np.abs(fd - O.silu_grad(x)).max() < 1e-8


def test_route_against_exhaustive_selection():
    rng = np.random.default_rng(8)
    cfg = O.replace(SMALL, n_experts=7, top_k=3)
    z = rng.standard_normal((40, 7))
    z[0, :] = 0.5                       # all tied: lowest indices win, in index order
    z[1, [2, 5]] = 9.0                  # a tie at the top
    z[2, [6, 1, 3]] = [1.0, 1.0, 1.0]
    z[2, [0, 2, 4, 5]] = -1.0
    idx, w, p = O.route(z, cfg)
    assert np.abs(p - scipy.special.softmax(z, axis=-1)).max() < 1e-15
    assert idx[0].tolist() == [0, 1, 2] and idx[1, :2].tolist() == [2, 5] and idx[2].tolist() == [1, 3, 6]
    for t in range(40):
        remaining, chosen = list(range(7)), []
        for _ in range(3):
            best = remaining[0]
            for e in remaining:
                if z[t, e] > z[t, best]:
                    best = e
            chosen.append(best)
            remaining.remove(best)
        assert idx[t].tolist() == chosen
        assert np.allclose(w[t], p[t, chosen], atol=0)
    _, wn, _ = O.route(z, O.replace(cfg, norm_topk_prob=True))
    assert np.abs(wn.sum(-1) - 1).max() < 1e-15
    assert np.allclose(wn * w.sum(-1, keepdims=True), w, atol=1e-15)


def test_permutation_is_stable_grouping():
    rng = np.random.default_rng(9)
    T, k, E = 37, 3, 6
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    idx[idx == 4] = 5                   # expert 4 gets nothing (and duplicates appear: still valid grouping)
    counts, offsets, row_map = O.permutation(idx, E)
    assert counts.sum() == T * k and counts[4] == 0
    assert offsets[0] == 0 and np.array_equal(offsets[1:], np.cumsum(counts))
    assert sorted(row_map.tolist()) == list(range(T * k))
    flat = idx.reshape(-1)
    for e in range(E):
        rows = row_map[offsets[e]:offsets[e + 1]]
        assert np.all(flat[rows] == e)
        assert np.all(np.diff(rows) > 0)                # (token, slot) order kept inside an expert


@pytest.mark.parametrize("norm", [False, True])
def test_moe_equals_dense_all_experts_masked(norm):
    rng = np.random.default_rng(11)
    cfg = O.replace(SMALL, norm_topk_prob=norm)
    W = rand_weights(cfg, rng, 0.3)
    T = 13
    y1 = rng.standard_normal((T, cfg.h))
    M, c = O.moe_half_forward(y1, W, cfg)
    Um = O.rmsnorm(y1, W["norm_m"], cfg.rms_eps) @ W["pup_m"].T
    z = Um @ W["w_router"].T + W["b_router"]
    p = scipy.special.softmax(z, axis=-1)
    I = cfg.d_expert
    R = np.zeros((T, cfg.d_model))
    for t in range(T):
        sel = sorted(range(cfg.n_experts), key=lambda e: (-z[t, e], e))[:cfg.top_k]
        tot = sum(p[t, e] for e in sel) if norm else 1.0
        for e in range(cfg.n_experts):                  # every expert, masked
            gte = W["w_gate_up"][e, :I] @ Um[t]
            upe = W["w_gate_up"][e, I:] @ Um[t]
            out = W["w_down"][e] @ (gte / (1 + np.exp(-gte)) * upe)
            R[t] += (p[t, e] / tot if e in sel else 0.0) * out
    Is = cfg.d_shared
    gs, us = Um @ W["ws_gate_up"][:Is].T, Um @ W["ws_gate_up"][Is:].T
    Sh = scipy.special.expit(Um @ W["ws_gate"])[:, None] * ((gs * scipy.special.expit(gs) * us) @ W["ws_down"].T)
    assert np.abs(c["R"] - R).max() < 1e-13
    assert np.abs(M - (R + Sh) @ W["pdn_m"].T).max() < 1e-13


def test_single_expert_is_dense_swiglu_and_tokens_are_independent():
    rng = np.random.default_rng(12)
    cfg = O.replace(SMALL, n_experts=1, top_k=1, d_shared=0)
    W = rand_weights(cfg, rng, 0.3)
    T = 9
    y1 = rng.standard_normal((T, cfg.h))
    M, c = O.moe_half_forward(y1, W, cfg)
    Um = c["Um"]
    I = cfg.d_expert
    gte, upe = Um @ W["w_gate_up"][0, :I].T, Um @ W["w_gate_up"][0, I:].T
    dense = (gte * scipy.special.expit(gte) * upe) @ W["w_down"][0].T      # routing weight is 1
    assert np.abs(c["w"] - 1).max() == 0
    assert np.abs(M - dense @ W["pdn_m"].T).max() < 1e-13
    # position-wise: permuting tokens permutes the output
    cfg2 = SMALL
    W2 = rand_weights(cfg2, rng, 0.3)
    perm = rng.permutation(T)
    M2, _ = O.moe_half_forward(y1, W2, cfg2)
    M2p, _ = O.moe_half_forward(y1[perm], W2, cfg2)
    assert np.abs(M2p - M2[perm]).max() < 1e-14


def test_router_bias_shifts_selection_and_weights():
    rng = np.random.default_rng(13)
    cfg = O.replace(SMALL, d_shared=0)
    W = rand_weights(cfg, rng, 0.3, router_bias=False)
    y1 = rng.standard_normal((50, cfg.h))
    _, c0 = O.moe_half_forward(y1, W, cfg)
    W["b_router"] = np.array([10.0, 0, 0, 0, 0])
    _, c1 = O.moe_half_forward(y1, W, cfg)
    assert np.all(c1["idx"][:, 0] == 0) and c1["counts"][0] == 50
    assert np.all(c1["w"][:, 0] > 0.99)
    assert c0["counts"][0] < 50


def test_stack_sweep_matches_blockwise_chain():
    rng = np.random.default_rng(14)
    cfg = O.replace(SMALL, n_inv_iters=3)
    Ws = [rand_weights(cfg, rng, 0.1) for _ in range(3)]
    B, S = 1, 4
    x1, x2 = rng.standard_normal((4, cfg.h)), rng.standard_normal((4, cfg.h))
    y1, y2, states = O.stack_forward(x1, x2, Ws, cfg, B, S, keep_all=True)
    dy1, dy2 = rng.standard_normal((4, cfg.h)), rng.standard_normal((4, cfg.h))
    dx1, dx2, grads, rebuilt = O.stack_backward_sweep(y1, y2, dy1, dy2, Ws, cfg, B, S, n_iters=8)
    # stored route through the whole stack
    g1, g2 = dy1, dy2
    for l in (2, 1, 0):
        a, b = states[l]
        g1, g2, gl = O.backward(a, b, states[l + 1][0], g1, g2, Ws[l], cfg, B, S)
        assert np.abs(rebuilt[l][0] - a).max() < 1e-9 and np.abs(rebuilt[l][1] - b).max() < 1e-9
        for k in gl:
            assert np.abs(gl[k] - grads[l][k]).max() < 1e-8 * max(1.0, np.abs(gl[k]).max()), (l, k)
    assert np.abs(g1 - dx1).max() < 1e-8 and np.abs(g2 - dx2).max() < 1e-8


def test_row_sums_and_token_permutation_equivariance():
    """Attention probabilities sum to one over the admissible keys; renormalised routing weights sum to one; the MoE
    half acts on each token alone, so permuting the tokens permutes its output (and its routing) the same way."""
    rng = np.random.default_rng(21)
    cfg = O.replace(SMALL, norm_topk_prob=True)
    W = rand_weights(cfg, rng, 0.3)
    B, S = 2, 7
    T = B * S
    x1, x2 = rng.standard_normal((T, cfg.h)), rng.standard_normal((T, cfg.h))
    _, ca = O.attn_half_forward(x1, x2, W, cfg, B, S, keep_probs=True)
    P = ca["P"]                                              # [B, H, S, S]
    assert np.abs(P.sum(axis=-1) - 1.0).max() < 1e-14
    assert np.abs(np.triu(P, k=1)).max() == 0.0              # causal: nothing above the diagonal
    M, cm = O.moe_half_forward(x1, W, cfg)
    assert np.abs(cm["w"].sum(axis=-1) - 1.0).max() < 1e-14
    perm = rng.permutation(T)
    Mp, cp = O.moe_half_forward(x1[perm], W, cfg)
    assert np.abs(Mp - M[perm]).max() < 1e-13
    assert np.array_equal(cp["idx"], cm["idx"][perm])
    assert cp["counts"].sum() == T * cfg.top_k and np.array_equal(cp["counts"], cm["counts"])


# --------------------------------------------------------------------------
# helpers the GPU parity tests lean on: margin, forced selection, streaming attention backward
# --------------------------------------------------------------------------
def test_topk_margin_on_constructed_logits():
    """The margin decides which tokens the GPU routing comparison may skip, so it is pinned on logits whose k-th and
    (k+1)-th largest values are known by construction, and against a python sort."""
    rng = np.random.default_rng(31)
    E, k = 9, 3
    z = np.zeros((6, E))
    gaps = [0.5, 1e-3, 0.0, 2.5e-4, 7.0, 1e-9]
    for t, gap in enumerate(gaps):
        top = 3.0 + rng.random(k - 1)                   # k - 1 clearly larger logits
        kth = 1.0
        rest = kth - gap - np.concatenate([[0.0], rng.random(E - k - 1)])   # the (k+1)-th is kth - gap exactly
        row = np.concatenate([top, [kth], rest])
        z[t] = row[rng.permutation(E)]
    m = O.topk_margin(z, k)
    for t, gap in enumerate(gaps):
        assert abs(m[t] - gap) <= 1e-15, (t, m[t], gap)
        srt = sorted(z[t].tolist(), reverse=True)
        assert m[t] == srt[k - 1] - srt[k]
    # k = E: nothing can flip
    assert np.all(np.isinf(O.topk_margin(z, E))) and np.all(O.topk_margin(z, E) > 0)
    # a dropped "-1" or a margin taken between the wrong ranks would show here
    z2 = np.array([[5.0, 4.0, 2.0, 1.5]])
    assert O.topk_margin(z2, 1)[0] == 1.0 and O.topk_margin(z2, 2)[0] == 2.0 and O.topk_margin(z2, 3)[0] == 0.5


def test_forced_selection_is_the_identity_on_own_selection_and_swaps_experts_otherwise():
    """forced_idx bypasses the ranking only: forcing the block's own selection reproduces every output and gradient
    bit for bit; forcing another selection equals the dense all-experts computation masked with that selection."""
    rng = np.random.default_rng(32)
    cfg = SMALL
    W = rand_weights(cfg, rng, 0.3)
    B, S = 2, 5
    T = B * S
    x1, x2 = rng.standard_normal((T, cfg.h)), rng.standard_normal((T, cfg.h))
    dy1, dy2 = rng.standard_normal((T, cfg.h)), rng.standard_normal((T, cfg.h))
    y1, y2, cache = O.forward(x1, x2, W, cfg, B, S, return_cache=True)
    own = cache["moe"]["idx"]
    y1f, y2f = O.forward(x1, x2, W, cfg, B, S, forced_idx=own)
    assert np.array_equal(y1, y1f) and np.array_equal(y2, y2f)
    a = O.backward(x1, x2, y1, dy1, dy2, W, cfg, B, S)
    b = O.backward(x1, x2, y1, dy1, dy2, W, cfg, B, S, forced_idx=own)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    for k in a[2]:
        assert np.array_equal(a[2][k], b[2][k]), k
    xa = O.inverse(y1, y2, W, cfg, B, S, n_iters=2)
    xb = O.inverse(y1, y2, W, cfg, B, S, n_iters=2, forced_idx=own)
    assert np.array_equal(xa[0], xb[0]) and np.array_equal(xa[1], xb[1])
    # another selection: token 3 takes its two LOWEST-ranked experts instead
    other = own.copy()
    z = cache["moe"]["z"]
    other[3] = np.argsort(z[3], kind="stable")[:cfg.top_k]
    M, cm = O.moe_half_forward(y1, W, cfg, forced_idx=other)
    assert np.array_equal(cm["idx"], other)
    Wf = O.as_f64(W)
    Um, p, I = cm["Um"], cm["p"], cfg.d_expert
    assert np.abs(p - scipy.special.softmax(z, axis=-1)).max() < 1e-15       # weights are still this softmax's
    R = np.zeros((T, cfg.d_model))
    for t in range(T):
        for e in other[t]:
            hh = O.silu(Um[t] @ Wf["w_gate_up"][e, :I].T) * (Um[t] @ Wf["w_gate_up"][e, I:].T)
            R[t] += p[t, e] * (hh @ Wf["w_down"][e].T)
    assert np.abs(cm["R"] - R).max() < 1e-13
    M0 = cache["M"]
    assert np.abs(M[3] - M0[3]).max() > 1e-6                                # the forced token changed ...
    keep = np.arange(T) != 3
    assert np.array_equal(M[keep], M0[keep])                                # ... and only that token


def test_route_ranks_not_a_number_as_minus_infinity():
    cfg = O.replace(SMALL, n_experts=6, top_k=3)
    z = np.array([[0.1, np.nan, 0.7, -0.2, np.nan, 0.3],
                  [np.nan] * 6,
                  [np.nan, -np.inf, np.nan, 2.0, -np.inf, np.nan],
                  [0.4, 0.9, 0.1, 0.2, 0.3, 0.8]])
    idx, w, p = O.route(z, cfg)
    assert idx[0].tolist() == [2, 5, 0]                 # finite logits first
    assert idx[1].tolist() == [0, 1, 2]                 # all equal (minus infinity): lower index first
    assert idx[2].tolist() == [3, 0, 1]                 # the finite one, then the tie of NaN and -inf by index
    assert idx[3].tolist() == [1, 5, 0]                 # a clean row is untouched
    for t in range(4):
        assert len(set(idx[t].tolist())) == 3 and idx[t].min() >= 0 and idx[t].max() < 6
    assert np.all(np.isfinite(w[3]))
    # the stable grouping of such indices is still a permutation of all (token, slot) pairs
    counts, offsets, row_map = O.permutation(idx, 6)
    assert counts.sum() == 12 and sorted(row_map.tolist()) == list(range(12))


@pytest.mark.parametrize("causal", [True, False])
def test_streaming_attention_backward_equals_stored_probabilities(causal):
    rng = np.random.default_rng(33)
    B, S, H, dh = 2, 19, 3, 8
    Q, K, V, dO = (rng.standard_normal((B, S, H, dh)) for _ in range(4))
    O4, P = O.attention_core(Q, K, V, causal)
    O4n, none = O.attention_core(Q, K, V, causal, keep_probs=False)
    assert none is None and np.array_equal(O4, O4n)
    a = O.attention_core_backward(dO, Q, K, V, P)
    b = O.attention_core_backward_streaming(dO, Q, K, V, causal)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    # and against autograd through the library attention (an independent route to the same gradients)
    tq, tk, tv = (torch.tensor(np.transpose(t, (0, 2, 1, 3)), dtype=torch.float64, requires_grad=True) for t in (Q, K, V))
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)
    out.backward(torch.tensor(np.transpose(dO, (0, 2, 1, 3))))
    for g, t in zip(b, (tq, tk, tv)):
        assert np.abs(g - np.transpose(t.grad.numpy(), (0, 2, 1, 3))).max() < 1e-12


def test_block_backward_without_stored_probabilities():
    rng = np.random.default_rng(34)
    cfg = SMALL
    W = rand_weights(cfg, rng, 0.3)
    B, S = 2, 6
    T = B * S
    x1, x2, dy1, dy2 = (rng.standard_normal((T, cfg.h)) for _ in range(4))
    y1, _ = O.forward(x1, x2, W, cfg, B, S)
    a = O.backward(x1, x2, y1, dy1, dy2, W, cfg, B, S)
    b = O.backward(x1, x2, y1, dy1, dy2, W, cfg, B, S, keep_probs=False)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    for k in a[2]:
        assert np.array_equal(a[2][k], b[2][k]), k


def test_blockwise_stopping_rule_lands_on_fixed_counts():
    """The per-block stopping rule of the inverse: every block's rebuilt rows are bit for bit those of the fixed-count
    iteration run as many times as that block ran (a row's iterate depends on that row alone), counts are 1 under a
    huge tolerance and the cap under a zero one."""
    rng = np.random.default_rng(41)
    cfg = O.replace(SMALL, n_heads=2, head_dim=8)
    W = rand_weights(cfg, rng, 0.25)
    B, S, bp = 2, 12, 4
    T = B * S
    x1, x2 = rng.standard_normal((T, cfg.h)), rng.standard_normal((T, cfg.h))
    y1, y2 = O.forward(x1, x2, W, cfg, B, S)
    _, _, whole = O.inverse(y1, y2, W, cfg, B, S, tol=0.0, max_iters=6, return_info=True)
    r = whole["residuals"]
    assert len(r) == 6 and r[1] < r[0]
    tol = float(np.sqrt(r[2] * r[3]))
    xb, x2b, info = O.inverse(y1, y2, W, cfg, B, S, tol=tol, max_iters=12, return_info=True, block_positions=bp)
    its = info["block_iters"]
    assert len(its) == B * 3 and max(its) == info["iters"] and min(its) >= 1
    assert len(set(its)) > 1, its                       # the blocks do stop at different counts here
    fixed = {n: O.inverse(y1, y2, W, cfg, B, S, n_iters=n)[0] for n in set(its)}
    for q, n in enumerate(its):
        b, j = divmod(q, 3)
        rows = slice(b * S + j * bp, b * S + (j + 1) * bp)
        assert np.array_equal(xb[rows], fixed[n][rows]), (q, n)
        assert info["block_residuals"][q] <= tol
    assert np.array_equal(x2b, O.inverse(y1, y2, W, cfg, B, S, n_iters=1)[1])
    # limits of the rule
    _, _, big = O.inverse(y1, y2, W, cfg, B, S, tol=1e9, max_iters=12, return_info=True, block_positions=bp)
    assert big["block_iters"] == [1] * 6
    _, _, cap = O.inverse(y1, y2, W, cfg, B, S, tol=0.0, max_iters=5, return_info=True, block_positions=bp)
    assert cap["block_iters"] == [5] * 6
    # one block covering everything is the whole-call rule
    xa, _, ia = O.inverse(y1, y2, W, cfg, B, S, tol=tol, max_iters=12, return_info=True)
    xw, _, iw = O.inverse(y1, y2, W, cfg, B, S, tol=tol, max_iters=12, return_info=True, block_positions=10 ** 6)
    # (block_positions >= S: one block per sequence; the whole-call count is the largest of them)
    assert max(iw["block_iters"]) == ia["iters"]


def test_merged_adapters_are_the_same_function():
    """Section 3.2: P_dn(module(P_up x)) with the products formed first is the same map (associativity), so forward
    and inverse agree to fp64 rounding; a transposed or misplaced adapter in the merge changes them at once."""
    wl = synth.WORKLOADS["tiny_shared_f32"]
    cfg = cfg_of(wl)
    W = synth.make_weights(wl)
    x1, x2, _, _ = synth.make_inputs(wl)
    M = O.merge_adapters(W)
    h = wl.d_model // 2
    assert M["wq"].shape == (wl.d_model, h) and M["wo"].shape == (h, wl.d_model)
    assert M["w_gate_up"].shape == (wl.n_experts, 2 * wl.d_expert, h) and M["w_down"].shape == (wl.n_experts, h, wl.d_expert)
    y1, y2 = O.forward(x1, x2, W, cfg, wl.B, wl.S)
    z1, z2 = O.forward(x1, x2, M, cfg, wl.B, wl.S)
    assert np.abs(z1 - y1).max() < 1e-12 * max(1.0, np.abs(y1).max())
    assert np.abs(z2 - y2).max() < 1e-12 * max(1.0, np.abs(y2).max())
    a1, a2 = O.inverse(y1, y2, W, cfg, wl.B, wl.S, n_iters=2)
    b1, b2 = O.inverse(y1, y2, M, cfg, wl.B, wl.S, n_iters=2)
    assert np.abs(a1 - b1).max() < 1e-12 and np.abs(a2 - b2).max() < 1e-12
    # one element by hand: (Wq P_up)[i, j] = sum_c Wq[i, c] P_up[c, j]
    Wf = O.as_f64(W)
    assert abs(M["wq"][3, 5] - sum(Wf["wq"][3, c] * Wf["pup_a"][c, 5] for c in range(wl.d_model))) < 1e-15
    assert abs(M["w_down"][1, 2, 4] - sum(Wf["pdn_m"][2, c] * Wf["w_down"][1, c, 4] for c in range(wl.d_model))) < 1e-15
