"""GPU parity: the HIP library against the fp64 oracle, element by element, through the C ABI.

Tolerance (max |gpu - ref| / max |ref| per tensor): 1e-4 for the float32 path, 2e-2 for the
bfloat16 path.  It is applied to the branch outputs (the terms added in Eq. 1-2), to the
rebuilt-input deltas and to every weight gradient, not only to Y, because with N(0, 0.02)
weights Y ~ X would pass a check on Y alone.  Integer routing results must be bit-exact
wherever the oracle's top-k logit margin exceeds 1e-3.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import revffn_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2512_20920_amd as R
    from paper_2512_20920_amd import harness as Hn
    from helpers import Case, relerr, TOL, check_routing, delta_err


def _forward_checks(case, tol, min_same=0.97):
    wl, cfg, W = case.wl, case.ocfg, case.W
    y1d, y2d = case.forward()
    y1g, y2g = Hn.download(y1d), Hn.download(y2d)
    a_gpu, m_gpu = case.branches()
    A_ref, _ = O.attn_half_forward(case.x1, case.x2, W, cfg, wl.B, wl.S, keep_probs=False)
    assert relerr(a_gpu, A_ref) < tol, "attention branch"
    assert relerr(y1g, case.x1 + A_ref) < tol
    # the MoE half is a function of Y1 alone: compare it at the GPU's own (stored) Y1
    rep = {}
    cm, safe, idx_gpu = check_routing(case, y1g, rep)
    # every token is compared: on a near-tie the oracle evaluates the GPU's selection
    M_ref, _ = O.moe_half_forward(y1g, W, cfg, forced_idx=idx_gpu)
    assert relerr(m_gpu, M_ref) < tol, "MoE branch"
    assert relerr(y2g, case.x2 + M_ref) < tol
    # end to end against the oracle's own Y1 as well (routing flips near ties are excluded)
    y1o, y2o, cache = O.forward(case.x1, case.x2, W, cfg, wl.B, wl.S, return_cache=True)
    same = (cache["moe"]["idx"] == cm["idx"]).all(axis=-1)
    assert same.mean() > min_same
    assert relerr(m_gpu[same & safe], cache["M"][same & safe]) < tol
    return y1d, y2d, rep


def _inverse_checks(case, y1d, y2d, tol, n_iters):
    wl, cfg, W = case.wl, case.ocfg, case.W
    y1h, y2h = Hn.download(y1d), Hn.download(y2d)
    x1d, x2d, res = case.inverse(y1d, y2d, n_iters=n_iters, want_residual=True)
    a_gpu, m_gpu = case.branches()
    cm, safe, idx_gpu = check_routing(case, y1h)
    x1o, x2o, info = O.inverse(y1h, y2h, W, cfg, wl.B, wl.S, n_iters=n_iters, return_info=True, forced_idx=idx_gpu)
    assert relerr(m_gpu, y2h - x2o) < tol, "MoE branch in the inverse"
    if n_iters > 0:
        assert relerr(a_gpu, y1h - x1o) < tol, "attention branch in the inverse"
        assert abs(res - info["residual"]) <= max(tol * info["residual"], 2 * np.abs(y1h).max() * (2.0 ** -8 if case.dt == "bf16" else 2.0 ** -22))
    assert relerr(Hn.download(x2d), x2o) < tol
    assert relerr(Hn.download(x1d), x1o) < tol
    return x1d, x2d


def _backward_checks(case, x1d, x2d, y1d, tol):
    wl, cfg, W = case.wl, case.ocfg, case.W
    x1h, x2h, y1h = Hn.download(x1d), Hn.download(x2d), Hn.download(y1d)
    dx1d, dx2d, G = case.backward(x1d, x2d, y1d)
    # routing of the backward call: no flip where the margin is clear; the oracle then takes the GPU's selection,
    # so that every gradient is compared whatever a near-tie did (forcing its own selection changes nothing)
    rep = {}
    _, _, idx = check_routing(case, y1h, rep)
    dx1o, dx2o, go = O.backward(x1h, x2h, y1h, case.dy1, case.dy2, W, cfg, wl.B, wl.S, forced_idx=idx)
    errs, bad = {}, {}
    # dX = dY + (branch gradient): as stored, the update is resolvable only down to the rounding of dX
    for name, gd, ref, base in (("dx1", dx1d, dx1o, case.dy1), ("dx2", dx2d, dx2o, case.dy2)):
        e, bnd = delta_err(Hn.download(gd), ref, base, case.dt)
        errs[name] = e / bnd * tol
        if not e <= bnd:
            bad[name] = (e, bnd)
    for k, ref in go.items():
        assert G[k] is not None, k
        if k == "bk" and not cfg.use_rope:
            # exactly zero in exact arithmetic (a key bias shifts every score of a row equally);
            # measure the GPU value against the scale of the query-bias gradient instead
            errs[k] = float(np.abs(Hn.download(G[k])).max() / np.abs(go["bq"]).max())
        else:
            errs[k] = relerr(Hn.download(G[k]), ref)
        if not errs[k] < tol:
            bad[k] = errs[k]
    assert not bad, (bad, errs, rep)
    # the branch gradients alone, at full tolerance: with dY1 = 0 the stream-1 input gradient has no
    # residual term in front of it, and with dY2 = 0 neither has the stream-2 one
    zero = np.zeros_like(case.dy1)
    dxa, _, _ = case.backward(x1d, x2d, y1d, dy1=zero)
    ra, _, _ = O.backward(x1h, x2h, y1h, zero, case.dy2, W, cfg, wl.B, wl.S, forced_idx=idx)
    errs["dx1|dy1=0"] = relerr(Hn.download(dxa), ra)
    _, dxb, _ = case.backward(x1d, x2d, y1d, dy2=zero)
    _, rb, _ = O.backward(x1h, x2h, y1h, case.dy1, zero, W, cfg, wl.B, wl.S, forced_idx=idx)
    errs["dx2|dy2=0"] = relerr(Hn.download(dxb), rb)
    assert errs["dx1|dy1=0"] < tol and errs["dx2|dy2=0"] < tol, errs
    return errs


@pytest.mark.parametrize("name,mode", [("tiny_f32", 0), ("tiny_shared_f32", 0), ("mid_f32", 0),
                                       ("mid_bf16", 1), ("mid_bf16", 0), ("mid_fewbig_bf16", 0),
                                       ("mid_rows137_bf16", 0)])
def test_block_parity(name, mode):
    wl = synth.WORKLOADS[name]
    tol = TOL[wl.dtype]
    case = Case(wl, mode=mode)
    y1d, y2d, rep = _forward_checks(case, tol)
    for n in (1, 2, 0):
        _inverse_checks(case, y1d, y2d, tol, n)
    x1d, x2d = case.inverse(y1d, y2d, n_iters=2)
    errs = _backward_checks(case, x1d, x2d, y1d, tol)
    print(name, "mode", mode, "ties", rep, {k: f"{v:.2e}" for k, v in errs.items()})


def _drawn_geometries(n, seed=11):
    """Seeded draw of block geometries that the fixed workloads do not cover: odd head counts, head widths with and
    without the flash-attention kernels, expert widths that end inside a tile, with and without a shared expert."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        dh = 64 if i % 3 == 2 else 128          # 64: no flash-attention kernel, generic attention
        H = int(rng.integers(2, 5))
        E = int(rng.integers(3, 21))
        k = int(rng.integers(1, min(4, E) + 1))
        I = 8 * int(rng.integers(5, 66))
        Is = 0 if rng.random() < 0.3 else 8 * int(rng.integers(5, 90))
        B, S = int(rng.integers(1, 4)), int(rng.integers(17, 261))
        out.append(synth.Workload(f"drawn{i}", H * dh, H, dh, E, k, I, Is, B, S, "bf16", gain_jitter=0.02, seed=100 + i))
    return out


@pytest.mark.parametrize("wl", _drawn_geometries(6), ids=lambda w: f"{w.name}_d{w.d_model}_dh{w.head_dim}_E{w.n_experts}k{w.top_k}_I{w.d_expert}_Is{w.d_shared}_B{w.B}S{w.S}")
def test_block_parity_drawn_geometries(wl):
    """Forward, inverse and backward against the oracle on seeded random geometries (bf16, matrix-core kernels)."""
    tol = TOL[wl.dtype]
    case = Case(wl)
    y1d, y2d, rep = _forward_checks(case, tol, min_same=0.9)
    x1d, x2d = _inverse_checks(case, y1d, y2d, tol, 1)
    errs = _backward_checks(case, x1d, x2d, y1d, tol)
    print(wl.name, "ties", rep, {k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("flags", [dict(causal=False, use_rope=False, norm_topk_prob=True),
                                   dict(causal=True, use_rope=True, norm_topk_prob=True)])
@pytest.mark.parametrize("name", ["mid_f32", "mid_bf16"])
def test_block_parity_flag_variants(name, flags):
    wl = synth.WORKLOADS[name]
    tol = TOL[wl.dtype]
    case = Case(wl, flags=flags)
    y1d, y2d, _ = _forward_checks(case, tol)
    x1d, x2d = _inverse_checks(case, y1d, y2d, tol, 2)
    _backward_checks(case, x1d, x2d, y1d, tol)


def test_zipf_bias_and_no_qkv_bias():
    """Router bias present (load imbalance) and q/k/v biases absent (NULL pointers)."""
    wl = synth.WORKLOADS["mid_f32"]
    W = synth.make_weights(wl)
    rng = np.random.default_rng(5)
    W["b_router"] = np.float32(0.8 * rng.standard_normal(wl.n_experts)).astype(np.float64)
    W["bq"] = W["bk"] = W["bv"] = None
    case = Case(wl, weights=W)
    y1d, y2d, _ = _forward_checks(case, 1e-4)
    x1d, x2d = _inverse_checks(case, y1d, y2d, 1e-4, 2)
    errs = _backward_checks(case, x1d, x2d, y1d, 1e-4)
    assert "b_router" in errs and "bq" not in errs
    counts = case.routing()[2]
    assert counts.max() > 2 * counts.mean()


@pytest.mark.parametrize("name", ["mid_f32", "mid_bf16"])
def test_deterministic_and_in_place_and_strided(name):
    wl = synth.WORKLOADS[name]
    case = Case(wl)
    T, h, d = wl.T, wl.h, wl.d_model
    y1a, y2a = case.forward()
    y1b, y2b = case.forward()
    assert torch.equal(y1a, y1b) and torch.equal(y2a, y2b)
    # the two halves of one [T, d] hidden tensor, row stride d, updated in place
    H = torch.cat([case.up(case.x1), case.up(case.x2)], dim=1).contiguous()
    es = H.element_size()
    p1, p2 = H.data_ptr(), H.data_ptr() + h * es
    R.revffn_forward(case.ctx, case.Wd, p1, p2, p1, p2, wl.B, wl.S, d)
    torch.cuda.synchronize()
    assert torch.equal(H[:, :h], y1a) and torch.equal(H[:, h:], y2a)
    # in-place inverse on the strided tensor equals the out-of-place one
    x1o, x2o = case.inverse(y1a, y2a, n_iters=2)
    R.revffn_inverse(case.ctx, case.Wd, p1, p2, p1, p2, wl.B, wl.S, d, None)
    torch.cuda.synchronize()
    assert torch.equal(H[:, :h], x1o) and torch.equal(H[:, h:], x2o)
    # backward twice: bit-identical gradients; dx may alias dy
    dx1, dx2, G1 = case.backward(x1o, x2o, y1a)
    dy1d, dy2d = case.up(case.dy1), case.up(case.dy2)
    G2 = Hn.alloc_grads(case.Wd)
    R.revffn_backward(case.ctx, case.Wd, x1o, x2o, y1a, dy1d, dy2d, dy1d, dy2d, G2, wl.B, wl.S, h)
    torch.cuda.synchronize()
    assert torch.equal(dy1d, dx1) and torch.equal(dy2d, dx2)
    for k in G1:
        if G1[k] is not None:
            assert torch.equal(G1[k], G2[k]), k
    # y1 = NULL recomputes it from x: same result when x is the exact input
    x1d, x2d = case.up(case.x1), case.up(case.x2)
    dxa, dxb, Ga = case.backward(x1d, x2d, y1a)
    dxc, dxd, Gb = case.backward(x1d, x2d, None)
    assert torch.equal(dxa, dxc) and torch.equal(dxb, dxd)


@pytest.mark.parametrize("name", ["mid_f32", "mid_bf16"])
def test_inverse_backward_equals_the_two_calls(name):
    wl = synth.WORKLOADS[name]
    case = Case(wl)
    case.ctx.set_inv_iters(2)
    y1d, y2d = case.forward()
    x1d, x2d, res_a = case.inverse(y1d, y2d, want_residual=True)
    dx1, dx2, G = case.backward(x1d, x2d, y1d)
    # fused, out of place
    r1, r2, o1, o2 = case.empty(), case.empty(), case.empty(), case.empty()
    G2 = Hn.alloc_grads(case.Wd)
    res = torch.zeros((1,), dtype=torch.float32, device="cuda")
    R.revffn_inverse_backward(case.ctx, case.Wd, y1d, y2d, r1, r2, case.up(case.dy1), case.up(case.dy2), o1, o2, G2,
                              wl.B, wl.S, wl.h, res)
    torch.cuda.synchronize()
    assert torch.equal(r1, x1d) and torch.equal(r2, x2d) and torch.equal(o1, dx1) and torch.equal(o2, dx2)
    assert float(res.item()) == res_a
    for k in G:
        if G[k] is not None:
            assert torch.equal(G[k], G2[k]), k
    # fused, fully in place (the sweep's calling pattern)
    a, b, ga, gb = y1d.clone(), y2d.clone(), case.up(case.dy1), case.up(case.dy2)
    G3 = Hn.alloc_grads(case.Wd)
    R.revffn_inverse_backward(case.ctx, case.Wd, a, b, a, b, ga, gb, ga, gb, G3, wl.B, wl.S, wl.h, None)
    torch.cuda.synchronize()
    assert torch.equal(a, x1d) and torch.equal(b, x2d) and torch.equal(ga, dx1) and torch.equal(gb, dx2)
    for k in G:
        if G[k] is not None:
            assert torch.equal(G[k], G3[k]), k


@pytest.mark.parametrize("mode", [0, 1])
def test_fp32_residual_streams(mode):
    """bf16 block with float32 residual streams (config.fp32_streams): same parity bar for every branch term and
    gradient; the coupling adds round to float32, so stream 2 is rebuilt to float32 rounding and stream 1 far below
    the bf16 storage floor; fused / stacked calls give the same bits as the separate ones."""
    wl = synth.WORKLOADS["mid_bf16"]
    tol = TOL["bf16"]
    case = Case(wl, mode=mode, fp32_streams=True)
    y1d, y2d, rep = _forward_checks(case, tol)
    assert y1d.dtype == torch.float32
    a_gpu, m_gpu = case.branches()
    y1h, y2h = Hn.download(y1d), Hn.download(y2d)
    ulp = 2.0 ** -23
    assert np.abs(y1h - (case.x1 + a_gpu)).max() <= ulp * np.abs(y1h).max()          # Eq. 1 rounds once, to float32
    assert np.abs(y2h - (case.x2 + m_gpu)).max() <= ulp * np.abs(y2h).max()          # Eq. 2
    for n in (1, 2, 0):
        _inverse_checks(case, y1d, y2d, tol, n)
    x1d, x2d = case.inverse(y1d, y2d, n_iters=3)
    e2 = np.abs(Hn.download(x2d) - case.x2).max()
    e1 = np.abs(Hn.download(x1d) - case.x1).max()
    # the same block with bf16 streams, for scale
    ref = Case(wl, mode=mode)
    r1d, r2d = ref.forward()
    q1d, q2d = ref.inverse(r1d, r2d, n_iters=3)
    b1 = np.abs(Hn.download(q1d) - case.x1).max()
    b2 = np.abs(Hn.download(q2d) - case.x2).max()
    print(f"mode {mode}: rebuilt-input error fp32 streams x1 {e1:.2e} x2 {e2:.2e}; bf16 streams x1 {b1:.2e} x2 {b2:.2e}")
    assert e2 <= 2 * ulp * np.abs(y2h).max()            # same MoE bits subtracted again: one float32 rounding each way
    assert e1 < 0.05 * b1 and e1 < 2e-3
    errs = _backward_checks(case, x1d, x2d, y1d, tol)
    # fused sweep step in place == separate calls
    case.ctx.set_inv_iters(2)
    x1d, x2d = case.inverse(y1d, y2d)
    dx1, dx2, G = case.backward(x1d, x2d, y1d)
    a, b, ga, gb = y1d.clone(), y2d.clone(), case.up(case.dy1), case.up(case.dy2)
    G2 = Hn.alloc_grads(case.Wd)
    R.revffn_inverse_backward(case.ctx, case.Wd, a, b, a, b, ga, gb, ga, gb, G2, wl.B, wl.S, wl.h, None)
    torch.cuda.synchronize()
    assert torch.equal(a, x1d) and torch.equal(b, x2d) and torch.equal(ga, dx1) and torch.equal(gb, dx2)
    for k in G:
        if G[k] is not None:
            assert torch.equal(G[k], G2[k]), k
    # three-block stack: rebuilt stack input against the true one
    L = 3
    Wds = [Hn.upload_weights(synth.make_weights(wl, block=l), wl.dtype) for l in range(L)]
    o1, o2 = case.empty_s(), case.empty_s()
    R.revffn_stack_forward(case.ctx, Wds, case.up_s(case.x1), case.up_s(case.x2), o1, o2, wl.B, wl.S, wl.h)
    g1, g2 = case.up(case.dy1), case.up(case.dy2)
    R.revffn_stack_backward(case.ctx, Wds, None, o1, o2, g1, g2, wl.B, wl.S, wl.h)
    torch.cuda.synchronize()
    d1 = np.abs(Hn.download(o1) - case.x1).max()
    d2 = np.abs(Hn.download(o2) - case.x2).max()
    print(f"mode {mode}: 3-block stack drift fp32 streams x1 {d1:.2e} x2 {d2:.2e}")
    assert d1 < 5e-3 and d2 < 5e-3


@pytest.mark.parametrize("name,mode", [("mid_f32", 0), ("mid_bf16", 1), ("mid_bf16", 0)])
def test_symmetric_comparison_block(name, mode):
    """The symmetric variant section 3.1 contrasts the layout with (queries from stream 2 too): same parity bar for
    forward, inverse and every gradient; the inverse is closed-form, so the input comes back to storage rounding
    without any iteration, whatever the iteration settings say."""
    wl = synth.WORKLOADS[name]
    tol = TOL[wl.dtype]
    case = Case(wl, mode=mode, flags=dict(symmetric=True))
    y1d, y2d, rep = _forward_checks(case, tol)
    # the attention branch must not depend on stream 1
    a0, _ = case.branches()
    case.forward(x1=case.x1[::-1].copy())
    a1, _ = case.branches()
    assert np.array_equal(a0, a1)
    case.forward()
    for n in (1, 0):
        _inverse_checks(case, y1d, y2d, tol, n)
    case.ctx.set_inverse_tolerance(1e-9, 7)                        # ignored: nothing is iterated
    x1d, x2d, res = case.inverse(y1d, y2d, want_residual=True)
    assert res == 0.0 and case.ctx.inverse_stats()[0] == 0
    case.ctx.set_inverse_tolerance(0.0, 0)
    ulp = (2.0 ** -7 if wl.dtype == "bf16" else 2.0 ** -23) * np.abs(Hn.download(y1d)).max()
    e1 = np.abs(Hn.download(x1d) - case.x1).max()
    e2 = np.abs(Hn.download(x2d) - case.x2).max()
    print(f"{name} mode {mode}: symmetric block rebuilt-input error x1 {e1:.2e} x2 {e2:.2e} (one unit of storage {ulp:.2e})")
    assert e1 <= 4 * ulp and e2 <= 4 * ulp
    errs = _backward_checks(case, x1d, x2d, y1d, tol)
    # fused sweep step, in place == the separate calls
    dx1, dx2, G = case.backward(x1d, x2d, y1d)
    a, b, ga, gb = y1d.clone(), y2d.clone(), case.up(case.dy1), case.up(case.dy2)
    G2 = Hn.alloc_grads(case.Wd)
    R.revffn_inverse_backward(case.ctx, case.Wd, a, b, a, b, ga, gb, ga, gb, G2, wl.B, wl.S, wl.h, None)
    torch.cuda.synchronize()
    assert torch.equal(a, x1d) and torch.equal(b, x2d) and torch.equal(ga, dx1) and torch.equal(gb, dx2)
    for k in G:
        if G[k] is not None:
            assert torch.equal(G[k], G2[k]), k
    assert float(G["norm_a1"].float().abs().max()) == 0.0
    # stored-activation route gives the same bits as the recomputing one at the true input
    x1t, x2t = case.up_s(case.x1), case.up_s(case.x2)
    o1, o2 = case.empty_s(), case.empty_s()
    R.revffn_forward(case.ctx, case.Wd, x1t, x2t, o1, o2, wl.B, wl.S, wl.h)
    s1, s2 = case.empty(), case.empty()
    G3 = Hn.alloc_grads(case.Wd)
    R.revffn_backward_stored(case.ctx, case.Wd, x1t, x2t, o1, case.up(case.dy1), case.up(case.dy2), s1, s2, G3,
                             wl.B, wl.S, wl.h)
    t1, t2, G4 = case.backward(x1t, x2t, o1)
    assert torch.equal(s1, t1) and torch.equal(s2, t2)
    for k in G3:
        if G3[k] is not None:
            assert torch.equal(G3[k], G4[k]), k


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["mid_bf16", "mid_fewbig_bf16", "mid_rows137_bf16"])
def test_fused_swiglu_epilogue_matches_the_separate_kernel(name, monkeypatch):
    """The gate/up GEMMs write silu(gate) * up from their epilogue (a tile holds matching gate and up columns).  Same
    bits as the GEMM followed by the SwiGLU kernel, through forward, inverse and every gradient; the expert widths of
    these workloads (192 and 320; 712; 200 and 160) leave tiles whose gate columns end inside the tile."""
    wl = synth.WORKLOADS[name]
    outs = []
    for separate in (False, True):
        if separate:
            monkeypatch.setenv("REVFFN_NO_FUSED_SWIGLU", "1")
        else:
            monkeypatch.delenv("REVFFN_NO_FUSED_SWIGLU", raising=False)
        case = Case(wl)
        y1d, y2d = case.forward()
        x1d, x2d = case.inverse(y1d, y2d, n_iters=1)
        dx1, dx2, G = case.backward(x1d, x2d, y1d)
        outs.append([y1d, y2d, x1d, x2d, dx1, dx2] + [G[k] for k in sorted(G) if G[k] is not None])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("mode", [0, 1])
def test_fp32_weight_gradients(mode):
    """config.fp32_grads: every weight gradient lands in a float32 buffer.  Same parity bar against the oracle, and
    rounding the float32 result to bf16 gives exactly the bf16-gradient run (only the final rounding differs)."""
    wl = synth.WORKLOADS["mid_bf16"]
    tol = TOL["bf16"]
    case = Case(wl, mode=mode, fp32_grads=True)
    ref = Case(wl, mode=mode)
    y1d, y2d = case.forward()
    x1d, x2d = case.inverse(y1d, y2d, n_iters=2)
    errs = _backward_checks(case, x1d, x2d, y1d, tol)
    dx1, dx2, G32 = case.backward(x1d, x2d, y1d)
    ex1, ex2, G16 = ref.backward(x1d, x2d, y1d)
    assert torch.equal(dx1, ex1) and torch.equal(dx2, ex2)
    for k in G32:
        if G32[k] is None:
            continue
        assert G32[k].dtype == torch.float32 and G16[k].dtype == (torch.float32 if k == "b_router" else torch.bfloat16)
        assert torch.equal(G32[k].to(G16[k].dtype), G16[k]), k
        assert not torch.equal(G32[k], G16[k].float()) or k == "b_router", k      # it really carries more bits
    # frozen groups and the fused call take the same buffers
    a, b, ga, gb = y1d.clone(), y2d.clone(), case.up(case.dy1), case.up(case.dy2)
    G2 = Hn.alloc_grads(case.Wd, skip=("w_gate_up", "w_router"), fp32=True)
    case.ctx.set_inv_iters(2)
    R.revffn_inverse_backward(case.ctx, case.Wd, a, b, a, b, ga, gb, ga, gb, G2, wl.B, wl.S, wl.h, None)
    torch.cuda.synchronize()
    for k in G2:
        if G2[k] is not None:
            assert torch.equal(G2[k], G32[k]), k


def _slow_contraction_case(name):
    """The synthetic weights contract by about 1e-5 per iteration; a sharper softmax (query projection x 128) and a
    larger branch (down adapter x 128) slow that to about 1e-2, so that a tolerance separates several iteration counts."""
    wl = synth.WORKLOADS[name]
    W = dict(synth.make_weights(wl))
    W["wq"] = W["wq"] * 128.0                   # (powers of two: the stored values stay exact)
    W["pdn_a"] = W["pdn_a"] * 128.0
    return Case(wl, weights=W)


def test_inverse_tolerance_stops_where_the_oracle_does():
    """Tolerance-driven inverse: the residual after each iteration and the iteration at which a given tolerance stops
    the loop are those of the oracle's fixed-point iteration (section 3.1), and the result is bit-identical to the
    fixed-count inverse with that many iterations."""
    case = _slow_contraction_case("mid_f32")
    wl, cfg, W = case.wl, case.ocfg, case.W
    y1o, y2o = O.forward(case.x1, case.x2, W, cfg, wl.B, wl.S)
    y1d, y2d = case.up(y1o), case.up(y2o)
    y1h, y2h = Hn.download(y1d), Hn.download(y2d)
    _, _, info = O.inverse(y1h, y2h, W, cfg, wl.B, wl.S, tol=0.0, max_iters=4, return_info=True)
    r = info["residuals"]
    assert len(r) == 4 and r[0] > 0.1 and r[2] > 1e-5 and all(r[i + 1] < 0.1 * r[i] for i in range(3)), r
    floor = 8 * np.abs(y1h).max() * 2.0 ** -23
    # residual sequence: cap the loop at k iterations with a tolerance it cannot reach
    for k in (1, 2, 3):
        case.ctx.set_inverse_tolerance(1e-30, k)
        case.inverse(y1d, y2d)
        calls, total, last, res = case.ctx.inverse_stats()
        assert (calls, total, last) == (1, k, k)
        assert abs(res - r[k - 1]) <= 0.02 * r[k - 1] + floor, (k, res, r)
    # stopping point: a tolerance between two residuals of the sequence
    for k in (1, 2, 3):
        tol = 2.0 if k == 1 else float(np.sqrt(r[k - 2] * r[k - 1]))
        xo, _, oi = O.inverse(y1h, y2h, W, cfg, wl.B, wl.S, tol=tol, max_iters=16, return_info=True)
        assert oi["iters"] == k
        case.ctx.set_inverse_tolerance(tol, 16)
        x1d, x2d, res = case.inverse(y1d, y2d, want_residual=True)
        calls, total, last, res_host = case.ctx.inverse_stats()
        assert last == k and res == res_host and res <= tol
        assert relerr(Hn.download(x1d), xo) < 1e-4
        case.ctx.set_inverse_tolerance(0.0, 0)                    # back to the fixed count
        f1, f2 = case.inverse(y1d, y2d, n_iters=k)
        assert case.ctx.inverse_stats() == (0, 0, 0, 0.0)
        assert torch.equal(f1, x1d) and torch.equal(f2, x2d)
    # the fused sweep step and the in-place form follow the same rule
    tol = float(np.sqrt(r[0] * r[1]))
    case.ctx.set_inverse_tolerance(0.0, 0)
    case.ctx.set_inv_iters(2)
    a, b, ga, gb = y1d.clone(), y2d.clone(), case.up(case.dy1), case.up(case.dy2)
    G1 = Hn.alloc_grads(case.Wd)
    R.revffn_inverse_backward(case.ctx, case.Wd, a, b, a, b, ga, gb, ga, gb, G1, wl.B, wl.S, wl.h, None)
    case.ctx.set_inv_iters(7)                                      # ignored while a tolerance is set
    case.ctx.set_inverse_tolerance(tol, 16)
    c, d, gc, gd = y1d.clone(), y2d.clone(), case.up(case.dy1), case.up(case.dy2)
    G2 = Hn.alloc_grads(case.Wd)
    R.revffn_inverse_backward(case.ctx, case.Wd, c, d, c, d, gc, gd, gc, gd, G2, wl.B, wl.S, wl.h, None)
    torch.cuda.synchronize()
    assert case.ctx.inverse_stats()[:3] == (1, 2, 2)
    assert torch.equal(a, c) and torch.equal(b, d) and torch.equal(ga, gc) and torch.equal(gb, gd)
    for k in G1:
        if G1[k] is not None:
            assert torch.equal(G1[k], G2[k]), k
    # argument checks
    lib = case.ctx.lib
    assert lib.revffn_set_inverse_tolerance(case.ctx.handle, -1.0, 4) == -1
    assert lib.revffn_set_inverse_tolerance(case.ctx.handle, float("nan"), 4) == -1
    assert lib.revffn_set_inverse_tolerance(case.ctx.handle, 1e-3, 0) == -1
    assert lib.revffn_set_inverse_tolerance(case.ctx.handle, 1e-3, 1025) == -1


def test_inverse_tolerance_bf16_floor_and_stack():
    """In bf16 successive iterates stop changing at the rounding of the stored iterate: a tolerance above the first
    residual takes one iteration, one between the first residual and that floor takes two, one below the floor runs
    to the cap.  The stack sweep applies the rule block by block."""
    wl = synth.WORKLOADS["mid_bf16"]
    case = Case(wl)
    y1d, y2d = case.forward()
    y1h, y2h = Hn.download(y1d), Hn.download(y2d)
    _, _, info = O.inverse(y1h, y2h, case.W, case.ocfg, wl.B, wl.S, tol=0.0, max_iters=3, return_info=True)
    r1 = info["residuals"][0]
    ulp = 2.0 ** (np.floor(np.log2(np.abs(y1h).max())) - 7)        # spacing of bf16 at the largest element
    assert r1 > 3 * ulp
    for tol, want in ((2 * r1, 1), (float(np.sqrt(r1 * 1.5 * ulp)), 2), (ulp / 64, 5)):
        case.ctx.set_inverse_tolerance(tol, 5)
        x1d, x2d = case.inverse(y1d, y2d)
        calls, total, last, res = case.ctx.inverse_stats()
        assert last == want, (tol, want, last, res)
        oi = O.inverse(y1h, y2h, case.W, case.ocfg, wl.B, wl.S, tol=tol, max_iters=5, return_info=True)[2]
        if want < 5:
            assert oi["iters"] == want
        case.ctx.set_inverse_tolerance(0.0, 0)
        f1, f2 = case.inverse(y1d, y2d, n_iters=want)
        assert torch.equal(f1, x1d) and torch.equal(f2, x2d)
    # stack: the sweep applies the rule in every block; same bits and same iteration counts as block-by-block calls
    L = 3
    Wds = [Hn.upload_weights(synth.make_weights(wl, block=l), wl.dtype) for l in range(L)]
    o1, o2 = case.empty(), case.empty()
    R.revffn_stack_forward(case.ctx, Wds, case.up(case.x1), case.up(case.x2), o1, o2, wl.B, wl.S, wl.h)
    tol = float(np.sqrt(r1 * 1.5 * ulp))
    case.ctx.set_inverse_tolerance(tol, 8)
    s1, s2, g1, g2 = o1.clone(), o2.clone(), case.up(case.dy1), case.up(case.dy2)
    R.revffn_stack_backward(case.ctx, Wds, None, s1, s2, g1, g2, wl.B, wl.S, wl.h)
    torch.cuda.synchronize()
    calls, total = case.ctx.inverse_stats()[:2]
    case.ctx.set_inverse_tolerance(tol, 8)                         # (resets the statistics)
    c1, c2, d1, d2 = o1.clone(), o2.clone(), case.up(case.dy1), case.up(case.dy2)
    iters = []
    for l in reversed(range(L)):
        R.revffn_inverse_backward(case.ctx, Wds[l], c1, c2, c1, c2, d1, d2, d1, d2, None, wl.B, wl.S, wl.h, None)
        iters.append(case.ctx.inverse_stats()[2])
    torch.cuda.synchronize()
    assert calls == L and total == sum(iters) and all(1 <= it <= 3 for it in iters), (calls, total, iters)
    assert torch.equal(c1, s1) and torch.equal(c2, s2) and torch.equal(d1, g1) and torch.equal(d2, g2)


def test_helper_streams_do_not_change_results(monkeypatch):
    """Same bits with the work spread over the helper streams and with everything on one stream."""
    wl = synth.WORKLOADS["mid_bf16"]
    outs = []
    for no_streams in (False, True):
        if no_streams:
            monkeypatch.setenv("REVFFN_NO_STREAMS", "1")
        else:
            monkeypatch.delenv("REVFFN_NO_STREAMS", raising=False)
        case = Case(wl)
        y1d, y2d = case.forward()
        x1d, x2d = case.inverse(y1d, y2d, n_iters=2)
        dx1, dx2, G = case.backward(x1d, x2d, y1d)
        outs.append([y1d, y2d, x1d, x2d, dx1, dx2] + [G[k] for k in sorted(G) if G[k] is not None])
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    # the same switch through the C-ABI on a live context, with the fused call at the paper's single iteration
    monkeypatch.delenv("REVFFN_NO_STREAMS", raising=False)
    case = Case(wl)
    y1d, y2d = case.forward()
    fused = []
    for on in (True, False, True):
        case.ctx.set_helper_streams(on)
        r1, r2, o1, o2 = case.empty(), case.empty(), case.empty(), case.empty()
        G = Hn.alloc_grads(case.Wd)
        R.revffn_inverse_backward(case.ctx, case.Wd, y1d, y2d, r1, r2, case.up(case.dy1), case.up(case.dy2), o1, o2, G,
                                  wl.B, wl.S, wl.h, None)
        torch.cuda.synchronize()
        fused.append([r1, r2, o1, o2] + [G[k] for k in sorted(G) if G[k] is not None])
    for other in fused[1:]:
        for a, b in zip(fused[0], other):
            assert torch.equal(a, b)


def test_frozen_groups_are_skipped():
    """NULL gradient fields (adapter-only stage; frozen routers) leave the others unchanged."""
    wl = synth.WORKLOADS["mid_f32"]
    case = Case(wl)
    y1d, y2d = case.forward()
    x1d, x2d = case.up(case.x1), case.up(case.x2)
    dx1, dx2, G = case.backward(x1d, x2d, y1d)
    frozen = [n for n in R.WEIGHT_FIELDS if n not in ("pup_a", "pdn_a", "pup_m", "pdn_m")]
    dx1b, dx2b, Gs = case.backward(x1d, x2d, y1d, skip=frozen)
    assert torch.equal(dx1, dx1b) and torch.equal(dx2, dx2b)
    for n in ("pup_a", "pdn_a", "pup_m", "pdn_m"):
        assert torch.equal(G[n], Gs[n])
    dy1d, dy2d = case.up(case.dy1), case.up(case.dy2)
    o1, o2 = case.empty(), case.empty()
    R.revffn_backward(case.ctx, case.Wd, x1d, x2d, y1d, dy1d, dy2d, o1, o2, None, wl.B, wl.S, wl.h)
    torch.cuda.synchronize()
    assert torch.equal(o1, dx1) and torch.equal(o2, dx2)


@pytest.mark.parametrize("name", ["tiny_shared_f32", "mid_bf16", "mid_rows137_bf16"])
def test_stored_activation_backward(name):
    """The non-reversible comparison route: gradients from the activations the forward call left in the workspace.
    Same bits as the recomputing backward at the true input, within tolerance of the oracle's stored route, and
    refused when the workspace no longer holds that forward call."""
    wl = synth.WORKLOADS[name]
    tol = TOL[wl.dtype]
    case = Case(wl)
    x1d, x2d = case.up(case.x1), case.up(case.x2)
    dy1d, dy2d = case.up(case.dy1), case.up(case.dy2)
    # reference: recomputing backward at the true input
    y1d, y2d = case.empty(), case.empty()
    R.revffn_forward(case.ctx, case.Wd, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h)
    dx1, dx2, G = case.backward(x1d, x2d, y1d)
    # stored route
    R.revffn_forward(case.ctx, case.Wd, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h)
    o1, o2 = case.empty(), case.empty()
    Gs = Hn.alloc_grads(case.Wd)
    R.revffn_backward_stored(case.ctx, case.Wd, x1d, x2d, y1d, dy1d, dy2d, o1, o2, Gs, wl.B, wl.S, wl.h)
    torch.cuda.synchronize()
    assert torch.equal(o1, dx1) and torch.equal(o2, dx2)
    for k in G:
        if G[k] is not None:
            assert torch.equal(G[k], Gs[k]), k
    # against the oracle's stored route
    _, _, go = O.grads_stored(Hn.download(x1d), Hn.download(x2d), case.dy1, case.dy2, case.W, case.ocfg, wl.B, wl.S)
    for k in ("pup_a", "pdn_m", "wq", "w_down", "w_gate_up"):
        assert relerr(Hn.download(Gs[k]), go[k]) < tol, k
    # the stored state serves one call, and only right after a matching out-of-place forward
    with pytest.raises(R.RevffnError):
        R.revffn_backward_stored(case.ctx, case.Wd, x1d, x2d, y1d, dy1d, dy2d, o1, o2, Gs, wl.B, wl.S, wl.h)
    R.revffn_forward(case.ctx, case.Wd, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h)
    R.revffn_inverse(case.ctx, case.Wd, y1d, y2d, case.empty(), case.empty(), wl.B, wl.S, wl.h, None)
    with pytest.raises(R.RevffnError):
        R.revffn_backward_stored(case.ctx, case.Wd, x1d, x2d, y1d, dy1d, dy2d, o1, o2, Gs, wl.B, wl.S, wl.h)
    R.revffn_forward(case.ctx, case.Wd, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h)
    with pytest.raises(R.RevffnError):
        R.revffn_backward_stored(case.ctx, case.Wd, x2d, x1d, y1d, dy1d, dy2d, o1, o2, Gs, wl.B, wl.S, wl.h)
    a, b = x1d.clone(), x2d.clone()
    R.revffn_forward(case.ctx, case.Wd, a, b, a, b, wl.B, wl.S, wl.h)            # in place: nothing stored
    with pytest.raises(R.RevffnError):
        R.revffn_backward_stored(case.ctx, case.Wd, a, b, a, dy1d, dy2d, o1, o2, Gs, wl.B, wl.S, wl.h)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["mid_f32", "mid_bf16"])
def test_stack_sweep_matches_blockwise_calls(name):
    import dataclasses
    wl = dataclasses.replace(synth.WORKLOADS[name], n_blocks=3)
    case = Case(wl)
    Ws = [synth.make_weights(wl, block=l) for l in range(3)]
    Wds = [Hn.upload_weights(W, wl.dtype) for W in Ws]
    case.ctx.set_inv_iters(2)
    x1d, x2d = case.up(case.x1), case.up(case.x2)
    y1d, y2d = case.empty(), case.empty()
    R.revffn_stack_forward(case.ctx, Wds, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h)
    # block by block through the single-block entry points
    a, b = x1d, x2d
    for l in range(3):
        na, nb = case.empty(), case.empty()
        R.revffn_forward(case.ctx, Wds[l], a, b, na, nb, wl.B, wl.S, wl.h)
        a, b = na, nb
    torch.cuda.synchronize()
    assert torch.equal(a, y1d) and torch.equal(b, y2d)
    Gs = [Hn.alloc_grads(Wd) for Wd in Wds]
    s1, s2 = y1d.clone(), y2d.clone()
    g1, g2 = case.up(case.dy1), case.up(case.dy2)
    R.revffn_stack_backward(case.ctx, Wds, Gs, s1, s2, g1, g2, wl.B, wl.S, wl.h)
    torch.cuda.synchronize()
    c1, c2 = y1d.clone(), y2d.clone()
    d1, d2 = case.up(case.dy1), case.up(case.dy2)
    for l in (2, 1, 0):
        r1, r2 = case.empty(), case.empty()
        R.revffn_inverse(case.ctx, Wds[l], c1, c2, r1, r2, wl.B, wl.S, wl.h, None)
        Gl = Hn.alloc_grads(Wds[l])
        n1, n2 = case.empty(), case.empty()
        R.revffn_backward(case.ctx, Wds[l], r1, r2, c1, d1, d2, n1, n2, Gl, wl.B, wl.S, wl.h)
        torch.cuda.synchronize()
        for k in Gl:
            if Gl[k] is not None:
                assert torch.equal(Gl[k], Gs[l][k]), (l, k)
        c1, c2, d1, d2 = r1, r2, n1, n2
    assert torch.equal(c1, s1) and torch.equal(c2, s2) and torch.equal(d1, g1) and torch.equal(d2, g2)
    # and the sweep as a whole against the oracle's sweep from the same stack output
    tol = TOL[wl.dtype]
    ocfg = case.ocfg
    dx1o, dx2o, go, rebuilt = O.stack_backward_sweep(Hn.download(y1d), Hn.download(y2d), case.dy1, case.dy2,
                                                     Ws, ocfg, wl.B, wl.S, n_iters=2)
    assert relerr(Hn.download(s1), rebuilt[0][0]) < tol and relerr(Hn.download(s2), rebuilt[0][1]) < tol
    # below the top block the oracle routes on its own fp64 rebuilt Y1 and the GPU on its stored one, so
    # near-tie tokens may pick other experts there; the MoE-side gradients of the bf16 sweep are therefore
    # compared block by block above (same inputs on both sides), and here only for the top block
    attn_side = ("pdn_a", "wo", "wq", "wk", "wv", "pup_a")
    for l in range(3):
        for k, ref in go[l].items():
            if wl.dtype == "f32" or l == 2 or k in attn_side:
                assert relerr(Hn.download(Gs[l][k]), ref) < 3 * tol, (l, k)


def test_smaller_call_on_larger_context_and_ragged_sizes():
    """A context sized for more tokens serves smaller (B, S); odd sizes exercise every tile tail."""
    import dataclasses
    base = synth.WORKLOADS["mid_f32"]
    for (B, S) in ((1, 1), (1, 67), (2, 33)):
        wl = dataclasses.replace(base, B=B, S=S)
        case = Case(wl, max_B=3, max_S=80)
        y1d, y2d, _ = _forward_checks(case, 1e-4)
        x1d, x2d = _inverse_checks(case, y1d, y2d, 1e-4, 1)
        _backward_checks(case, x1d, x2d, y1d, 1e-4)


@pytest.mark.parametrize("mode", [0, 1])
def test_degenerate_routing_and_limits_bf16(mode):
    """The routing shapes at the edges, on the bf16 path: experts without any row, one expert that takes every
    token, top_k = n_experts (no selection), and the largest expert count and top_k the library accepts."""
    import dataclasses
    base = synth.WORKLOADS["mid_bf16"]
    tol = TOL["bf16"]

    def run(wl, W=None, n_iters=1, min_same=0.97):
        case = Case(wl, mode=mode, weights=W)
        y1d, y2d, _ = _forward_checks(case, tol, min_same)
        x1d, x2d = _inverse_checks(case, y1d, y2d, tol, n_iters)
        errs = _backward_checks(case, x1d, x2d, y1d, tol)
        return case, errs

    # (1) 3 tokens x top-3 over 12 experts: at least three experts get no row; their weight gradients are exact zeros
    wl = dataclasses.replace(base, B=1, S=3)
    case, _ = run(wl)
    counts = case.routing()[2]
    assert (counts == 0).sum() >= 3
    x1d, x2d = case.up_s(case.x1), case.up_s(case.x2)
    y1d, _ = case.forward()
    _, _, G = case.backward(x1d, x2d, y1d)
    for e in np.nonzero(counts == 0)[0]:
        assert float(G["w_gate_up"][e].float().abs().max()) == 0.0 and float(G["w_down"][e].float().abs().max()) == 0.0
    # (2) a router bias that sends every token to expert 5 first: one expert holds T rows, several 256-row tiles
    wl = dataclasses.replace(base, B=3, S=200)
    W = synth.make_weights(wl)
    b = np.zeros(wl.n_experts)
    b[5] = 1.5                      # ten times the spread of the logits at these weights
    W["b_router"] = b
    case, _ = run(wl, W)
    assert case.routing()[2][5] == wl.T
    # (3) top_k = n_experts: every expert for every token
    wl = dataclasses.replace(base, n_experts=4, top_k=4, B=2, S=70)
    case, _ = run(wl)
    assert np.all(case.routing()[2] == wl.T)
    # (4) the largest expert count and top_k accepted (256, 16), narrow experts, no shared expert
    wl = dataclasses.replace(base, d_model=256, n_heads=2, head_dim=128, n_experts=256, top_k=16, d_expert=64,
                             d_shared=0, B=2, S=40)
    # (16 of 256 nearly equal logits: the selection at the oracle's own Y1 and at the GPU's bf16 Y1 differs for more
    # tokens than elsewhere; at one and the same Y1 it is still bit-exact outside ties)
    run(wl, min_same=0.6)


def test_calls_can_be_captured_into_a_hip_graph():
    """A step (forward + fused inverse/backward, helper streams included) captured once into a HIP graph and
    replayed gives the bits of the eager calls, on every replay, with eager work and synchronisations between the
    replays: the calls only enqueue kernels and event dependencies (no allocation, no memset node, no host wait)."""
    wl = synth.WORKLOADS["mid_bf16"]
    case = Case(wl)
    x1d, x2d, dy1d, dy2d = case.up(case.x1), case.up(case.x2), case.up(case.dy1), case.up(case.dy2)
    y1d, y2d, r1d, r2d, dx1d, dx2d = (case.empty() for _ in range(6))
    G = Hn.alloc_grads(case.Wd)

    def step(stream=None):
        R.revffn_forward(case.ctx, case.Wd, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h, stream)
        R.revffn_inverse_backward(case.ctx, case.Wd, y1d, y2d, r1d, r2d, dy1d, dy2d, dx1d, dx2d, G, wl.B, wl.S, wl.h,
                                  None, stream)

    outs = lambda: [t.clone() for t in (y1d, y2d, r1d, r2d, dx1d, dx2d)] + [G[k].clone() for k in sorted(G) if G[k] is not None]
    step()
    torch.cuda.synchronize()
    want = outs()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(side)                                  # every kernel variant has run once before the capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (y1d, y2d, r1d, r2d, dx1d, dx2d):
            t.fill_(float("nan"))
        for k in G:
            if G[k] is not None:
                G[k].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = outs()
        assert all(torch.equal(a, b) for a, b in zip(got, want)), rep
        # eager work on the same context between replays
        case.ctx.set_inv_iters(2)
        case.inverse(y1d, y2d)
        case.ctx.set_inv_iters(1)
        torch.cuda.synchronize()


def test_non_finite_token_does_not_disturb_other_tokens():
    """One token whose stream-1 row holds a NaN: its own outputs are not numbers, but it selects top_k distinct valid
    experts (a logit that is not a number ranks as minus infinity, ties to the lower index: experts 0..k-1), and
    every other token's indices, weights and MoE output are bit-identical to the clean run; counts, offsets and the
    row map are the stable grouping of those indices."""
    wl = synth.WORKLOADS["mid_bf16"]
    case = Case(wl)
    y1a, y2a = case.forward()
    idx0, wts0, counts0, offsets0, row_map0 = case.routing()
    t_bad = 7
    x1 = case.x1.copy()
    x1[t_bad, 3] = np.nan
    y1b, y2b = case.forward(x1=x1)
    idx1, wts1, counts1, offsets1, row_map1 = case.routing()
    keep = np.arange(wl.T) != t_bad
    assert torch.isnan(y1b[t_bad].float()).any()
    assert idx1[t_bad].tolist() == list(range(wl.top_k))
    assert np.array_equal(idx1[keep], idx0[keep]) and np.array_equal(wts1[keep], wts0[keep])
    c2, o2, r2 = O.permutation(idx1, wl.n_experts)
    assert np.array_equal(counts1, c2) and np.array_equal(offsets1, o2) and np.array_equal(row_map1, r2)
    assert counts1.sum() == wl.T * wl.top_k
    keep_t = torch.from_numpy(keep).cuda()
    assert torch.equal(y1b[keep_t], y1a[keep_t]) and torch.equal(y2b[keep_t], y2a[keep_t])
    # the oracle's rule on the same stored stream gives the same selection for the poisoned token
    _, cm = O.moe_half_forward(Hn.download(y1b), case.W, case.ocfg)
    assert cm["idx"][t_bad].tolist() == idx1[t_bad].tolist()


@pytest.mark.parametrize("name,bp", [("mid_f32", 16), ("mid_bf16", 128)])
def test_inverse_tolerance_per_position_block(name, bp):
    """The stopping rule applied per (sequence, range of positions), decided on the device: every block's rebuilt rows
    are bit for bit those of the fixed-count inverse run as many times as that block ran; the per-block counts are the
    oracle's wherever the residuals are clear of the tolerance; stream 2 and the residual follow; the call is
    asynchronous, so a captured graph of it replays to the same bits."""
    case = _slow_contraction_case(name)
    wl, cfg, W = case.wl, case.ocfg, case.W
    y1o, y2o = O.forward(case.x1, case.x2, W, cfg, wl.B, wl.S)
    y1d, y2d = case.up(y1o), case.up(y2o)
    y1h, y2h = Hn.download(y1d), Hn.download(y2d)
    _, _, whole = O.inverse(y1h, y2h, W, cfg, wl.B, wl.S, tol=0.0, max_iters=4, return_info=True)
    r = whole["residuals"]
    tol = float(np.sqrt(r[1] * r[2])) if name == "mid_f32" else float(np.sqrt(r[0] * r[1]))
    cap = 6
    xo, x2o, oi = O.inverse(y1h, y2h, W, cfg, wl.B, wl.S, tol=tol, max_iters=cap, return_info=True, block_positions=bp)
    case.ctx.set_inverse_tolerance(tol, cap, block_positions=bp)
    x1d, x2d, res = case.inverse(y1d, y2d, want_residual=True)
    its, rs = case.ctx.inverse_blocks()
    nj = -(-wl.S // bp)
    assert len(its) == wl.B * nj == len(oi["block_iters"])
    calls, total, last, res_host = case.ctx.inverse_stats()
    assert (calls, total, last) == (1, int(its.max()), int(its.max())) and res == res_host == float(rs.max())
    print(f"{name}: block iterations gpu {its.tolist()} oracle {oi['block_iters']}")
    # counts: the oracle's, except where an oracle residual sits within rounding of the tolerance
    floor = 8 * np.abs(y1h).max() * (2.0 ** -23 if wl.dtype == "f32" else 2.0 ** -8)
    for q, (a, b) in enumerate(zip(its.tolist(), oi["block_iters"])):
        if abs(oi["block_residuals"][q] - tol) > 0.05 * tol + floor and b < cap:
            assert a == b or (wl.dtype == "bf16" and abs(a - b) <= 1), (q, a, b)
    assert relerr(Hn.download(x1d), xo) < TOL[wl.dtype] and relerr(Hn.download(x2d), x2o) < TOL[wl.dtype]
    # bits: each block equals the fixed-count run with its own count
    case.ctx.set_inverse_tolerance(0.0, 0)
    fixed = {}
    for n in sorted(set(its.tolist())):
        f1, f2 = case.inverse(y1d, y2d, n_iters=n)
        fixed[n] = f1.clone()
        assert torch.equal(f2, x2d)
    for q, n in enumerate(its.tolist()):
        b, j = divmod(q, nj)
        lo, hi = b * wl.S + j * bp, b * wl.S + min(wl.S, (j + 1) * bp)
        assert torch.equal(x1d[lo:hi], fixed[n][lo:hi]), (q, n)
    # captured graph of the tolerance-driven sweep step: replays give the eager bits, with eager work in between
    case.ctx.set_inverse_tolerance(tol, cap, block_positions=bp)
    dy1d, dy2d = case.up(case.dy1), case.up(case.dy2)
    r1d, r2d, dx1d, dx2d = (case.empty() for _ in range(4))
    resd = torch.zeros((1,), dtype=torch.float32, device="cuda")
    G = Hn.alloc_grads(case.Wd)

    def step(stream=None):
        R.revffn_inverse_backward(case.ctx, case.Wd, y1d, y2d, r1d, r2d, dy1d, dy2d, dx1d, dx2d, G, wl.B, wl.S, wl.h,
                                  resd, stream)

    outs = lambda: [t.clone() for t in (r1d, r2d, dx1d, dx2d, resd)] + [G[k].clone() for k in sorted(G) if G[k] is not None]
    step()
    torch.cuda.synchronize()
    want = outs()
    assert torch.equal(r1d, x1d) and torch.equal(r2d, x2d) and float(resd.item()) == res
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (r1d, r2d, dx1d, dx2d):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(outs(), want)), rep
        case.forward()                                   # eager work on the same context between replays
        torch.cuda.synchronize()
    assert case.ctx.inverse_stats()[0] == 1 + 1 + 3      # the eager step, the warm-up on the side stream, three replays


# ---- pre-merged adapters (section 3.2) -------------------------------------------------------------------------
STORED_MERGED = ("wq", "wk", "wv", "wo", "w_gate_up", "w_down", "ws_gate_up", "ws_down")


def _oracle_merged(case):
    """The oracle's products, with the tensors that the library stores in the compute dtype rounded to it by the
    oracle side itself (the router rows stay unrounded: the library keeps them in float32)."""
    M = O.merge_adapters(case.W)
    Mr = dict(M)
    if case.dt == "bf16":
        for n in STORED_MERGED:
            if M.get(n) is not None:
                Mr[n] = synth.round_bf16(M[n])
    return M, Mr


@pytest.mark.parametrize("name", ["tiny_shared_f32", "mid_f32", "mid_bf16", "mid_fewbig_bf16", "mid_rows137_bf16"])
def test_merged_adapters_parity(name):
    wl = synth.WORKLOADS[name]
    tol = TOL[wl.dtype]
    case = Case(wl)
    M, Mr = _oracle_merged(case)
    Md = Hn.alloc_merged(wl)
    R.revffn_merge_adapters(case.ctx, case.Wd, Md)
    torch.cuda.synchronize()
    # the products themselves: rounding to storage (half a unit of bfloat16 is up to 2^-8 of the largest element)
    # plus the accumulation order
    wtol = 4.5e-3 if wl.dtype == "bf16" else 1e-5
    for n in STORED_MERGED:
        if M.get(n) is None:
            assert Md[n] is None
            continue
        g = Hn.download(Md[n])
        assert g.shape == M[n].shape, n
        assert relerr(g, M[n]) < wtol, n
    # forward from the merged set against the oracle evaluating its own merged set
    x1d, x2d = case.up_s(case.x1), case.up_s(case.x2)
    y1d, y2d = case.empty_s(), case.empty_s()
    R.revffn_forward_merged(case.ctx, case.Wd, Md, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h)
    torch.cuda.synchronize()
    y1g, y2g = Hn.download(y1d), Hn.download(y2d)
    a_gpu, m_gpu = case.branches()
    A_ref, _ = O.attn_half_forward(case.x1, case.x2, Mr, case.ocfg, wl.B, wl.S, keep_probs=False)
    assert relerr(a_gpu, A_ref) < tol, "attention branch"
    assert relerr(y1g, case.x1 + A_ref) < tol
    rep = {}
    cm, safe, idx_gpu = check_routing(case, y1g, rep)
    M_ref, _ = O.moe_half_forward(y1g, Mr, case.ocfg, forced_idx=idx_gpu)
    assert relerr(m_gpu, M_ref) < tol, "MoE branch"
    assert relerr(y2g, case.x2 + M_ref) < tol
    # and against the unmerged definition (the merged products carry one more rounding)
    A_def, _ = O.attn_half_forward(case.x1, case.x2, case.W, case.ocfg, wl.B, wl.S, keep_probs=False)
    M_def, _ = O.moe_half_forward(y1g, case.W, case.ocfg, forced_idx=idx_gpu)
    assert relerr(a_gpu, A_def) < 2 * tol and relerr(m_gpu, M_def) < 2 * tol
    # inverse from the merged set
    for n in (1, 2, 0):
        case.ctx.set_inv_iters(n)
        r1d, r2d = case.empty_s(), case.empty_s()
        res = torch.zeros((1,), dtype=torch.float32, device="cuda")
        R.revffn_inverse_merged(case.ctx, case.Wd, Md, y1d, y2d, r1d, r2d, wl.B, wl.S, wl.h, res)
        torch.cuda.synchronize()
        a_inv, m_inv = case.branches()
        _, _, idx_inv = check_routing(case, y1g)
        x1o, x2o, info = O.inverse(y1g, y2g, Mr, case.ocfg, wl.B, wl.S, n_iters=n, return_info=True, forced_idx=idx_inv)
        assert relerr(m_inv, y2g - x2o) < tol, "MoE branch in the inverse"
        assert relerr(Hn.download(r2d), x2o) < tol and relerr(Hn.download(r1d), x1o) < tol
        if n > 0:
            assert relerr(a_inv, y1g - x1o) < tol, "attention branch in the inverse"
            r = float(res.item())
            assert abs(r - info["residual"]) <= max(tol * info["residual"], 2 * np.abs(y1g).max() * (2.0 ** -8 if case.dt == "bf16" else 2.0 ** -22))
        else:
            assert torch.equal(r1d, y1d)
        # in place on the two halves of one [T, d] tensor
        H = torch.cat([y1d, y2d], dim=1).contiguous()
        p1, p2 = H.data_ptr(), H.data_ptr() + wl.h * H.element_size()
        R.revffn_inverse_merged(case.ctx, case.Wd, Md, p1, p2, p1, p2, wl.B, wl.S, wl.d_model, None)
        torch.cuda.synchronize()
        assert torch.equal(H[:, :wl.h], r1d) and torch.equal(H[:, wl.h:], r2d)
    print(name, "merged", rep)


def test_merged_adapters_argument_errors():
    wl = synth.WORKLOADS["tiny_shared_f32"]
    case = Case(wl)
    Md = Hn.alloc_merged(wl)
    bad = dict(Md)
    bad["w_down"] = None
    with pytest.raises(RuntimeError):
        R.revffn_merge_adapters(case.ctx, case.Wd, bad)
    sym = Case(wl, flags=dict(symmetric=True))
    with pytest.raises(RuntimeError):
        R.revffn_merge_adapters(sym.ctx, sym.Wd, Md)
