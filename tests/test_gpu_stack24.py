"""The 24-block reversible stack at the Qwen1.5-MoE-A2.7B layer shape (batch 1 x seq 1024, bf16, distinct weights
per block): forward keeping only the last state, then the backward sweep that rebuilds every block's input from its
output (section 3.1).  Against the fp64 oracle:

 * per layer, the drift of the rebuilt input from the oracle's exact forward state H_l, for 1 (the paper's count)
   and 3 fixed-point iterations, and from the GPU's own forward state (which separates reconstruction drift from
   forward rounding);
 * block-level parity chained through the sweep: at sampled layers the oracle runs inverse + backward from the very
   (Y, dY) the GPU sweep holds there, and the rebuilt input, both input gradients and every weight gradient are
   compared at the 2e-2 bar;
 * peak device memory: weights + gradients + one block's workspace (activations do not grow with depth);
 * revffn_stack_backward gives the same bits as the block-by-block sweep.
"""
import threading
import time

import numpy as np
import pytest
import torch

import synth
from oracle import revffn_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2512_20920_amd as R
    from paper_2512_20920_amd import harness as Hn
    from helpers import relerr, TOL, delta_err, oracle_cfg, safe_tokens


def _host_weights(Wd):
    """One block's weights back from the device as float64 (bf16 values are exact in float64)."""
    return {k: (None if v is None else Hn.download(v)) for k, v in Wd.items()}


def test_qwen_stack24_sweep_against_oracle(capsys):
    wl = synth.WORKLOADS["qwen_stack24_b1s1024"]
    L, B, S, h, T = wl.n_blocks, wl.B, wl.S, wl.h, wl.T
    cfg = oracle_cfg(wl)
    tol = TOL["bf16"]
    x1, x2, dy1, dy2 = synth.make_inputs(wl)

    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)

    # ---- weights block by block: generated on the host (next block in a helper thread), uploaded, pushed through
    # the oracle's forward, and dropped on the host.  The oracle keeps every state H_l.
    t0 = time.time()
    torch.cuda.reset_peak_memory_stats()
    Wds, states = [], [(x1, x2)]
    nxt = {}

    def gen(l):
        nxt[l] = synth.make_weights(wl, block=l, f64=False)

    th = threading.Thread(target=gen, args=(0,))
    th.start()
    a, b = x1, x2
    for l in range(L):
        th.join()
        W32 = nxt.pop(l)
        if l + 1 < L:
            th = threading.Thread(target=gen, args=(l + 1,))
            th.start()
        Wds.append(Hn.upload_weights(W32, wl.dtype))
        a, b = O.forward(a, b, O.as_f64(W32), cfg, B, S)
        states.append((a, b))
        del W32
        if l % 4 == 3:
            say(f"STACK24 oracle forward through block {l} ({time.time() - t0:.0f} s)")
    Gs = [Hn.alloc_grads(Wd) for Wd in Wds]
    ctx = R.Context(Hn.make_config(wl), B, S)
    up = lambda v: Hn.upload(v, wl.dtype)
    new = lambda: torch.empty((T, h), dtype=torch.bfloat16, device="cuda")

    # ---- GPU forward: the stack call, and block by block to keep the GPU's own states for the drift split
    x1d, x2d = up(x1), up(x2)
    y1d, y2d = new(), new()
    R.revffn_stack_forward(ctx, Wds, x1d, x2d, y1d, y2d, B, S, h)
    own = [(x1d.clone(), x2d.clone())]
    p1, p2 = x1d.clone(), x2d.clone()
    for l in range(L):
        R.revffn_forward(ctx, Wds[l], p1, p2, p1, p2, B, S, h)
        own.append((p1.clone(), p2.clone()))
    torch.cuda.synchronize()
    assert torch.equal(p1, y1d) and torch.equal(p2, y2d)
    # forward rounding accumulated over 24 blocks, measured on the update H_24 - H_0
    e1 = relerr(Hn.download(y1d) - x1, states[L][0] - x1)
    e2 = relerr(Hn.download(y2d) - x2, states[L][1] - x2)
    say(f"STACK24 forward: relative error of H_24 - H_0 against the oracle: stream 1 {e1:.2e}, stream 2 {e2:.2e}")
    assert e1 < 5 * tol and e2 < 5 * tol

    # ---- the sweep, block by block (the calls revffn_stack_backward makes), for 1 and 3 iterations
    sampled = (L - 1, 2 * L // 3, L // 3, 0)
    final = {}
    for n in (1, 3):
        ctx.set_inv_iters(n)
        s1, s2, g1, g2 = y1d.clone(), y2d.clone(), up(dy1), up(dy2)
        drift_o, drift_g = [None] * L, [None] * L
        for l in range(L - 1, -1, -1):
            check = n == 3 and l in sampled
            if check:
                yh = (Hn.download(s1), Hn.download(s2))
                dyh = (Hn.download(g1), Hn.download(g2))
            R.revffn_inverse_backward(ctx, Wds[l], s1, s2, s1, s2, g1, g2, g1, g2, Gs[l], B, S, h, None)
            r1, r2 = Hn.download(s1), Hn.download(s2)
            drift_o[l] = (float(np.abs(r1 - states[l][0]).max()), float(np.abs(r2 - states[l][1]).max()))
            drift_g[l] = (float((s1.float() - own[l][0].float()).abs().max()),
                          float((s2.float() - own[l][1].float()).abs().max()))
            if check:
                # block-level parity from the very (Y, dY) the sweep holds at this layer
                W = _host_weights(Wds[l])
                idx = torch.empty((T, wl.top_k), dtype=torch.int32, device="cuda")
                R.revffn_get_routing(ctx, idx)
                torch.cuda.synchronize()
                idx = idx.cpu().numpy()
                _, cm = O.moe_half_forward(yh[0], W, cfg)
                safe = safe_tokens(cm, cfg)
                assert np.array_equal(idx[safe], cm["idx"][safe])
                xo1, xo2 = O.inverse(yh[0], yh[1], W, cfg, B, S, n_iters=n, forced_idx=idx)
                # the rebuilt input is stored as Y - (small branch term): resolvable to the rounding of the stored value
                for nme, gpu, ref, base in (("x1", r1, xo1, yh[0]), ("x2", r2, xo2, yh[1])):
                    e, bnd = delta_err(gpu, ref, base, "bf16")
                    assert e <= bnd, (l, nme, e, bnd)
                do1, do2, go = O.backward(r1, r2, yh[0], dyh[0], dyh[1], W, cfg, B, S, forced_idx=idx)
                errs = {k: relerr(Hn.download(Gs[l][k]), ref) for k, ref in go.items()}
                for nme, gd, ref, base in (("dx1", g1, do1, dyh[0]), ("dx2", g2, do2, dyh[1])):
                    e, bnd = delta_err(Hn.download(gd), ref, base, "bf16")
                    errs[nme] = e / bnd * tol
                worst = max(errs, key=errs.get)
                say(f"STACK24 n_inv_iters={n} block {l}: chained block parity, worst {worst} {errs[worst]:.2e} "
                    f"(ties {int((~safe).sum())}, flips {int((idx != cm['idx']).any(-1).sum())})")
                assert errs[worst] < tol, (l, errs)
                del W
        torch.cuda.synchronize()
        final[n] = (s1, s2, g1, g2)
        for l in range(L - 1, -1, -1):
            say(f"STACK24 n_inv_iters={n} layer {l:2d}: max|X^-H(oracle)| x1 {drift_o[l][0]:.3e} x2 {drift_o[l][1]:.3e}   "
                f"max|X^-H(gpu forward)| x1 {drift_g[l][0]:.3e} x2 {drift_g[l][1]:.3e}")
        # bounds: the values are of size ~4 (bf16 spacing 2^-6 there); the drift stays below a few tens of units in the
        # last place over 24 blocks, and three iterations must not be worse than one
        worst1 = max(d[0] for d in drift_o)
        worst2 = max(d[1] for d in drift_o)
        assert np.isfinite(worst1) and worst2 < 0.6, (n, worst1, worst2)
        assert worst1 < (1.0 if n == 1 else 0.6), (n, worst1)
        final[n] += (drift_o,)
    assert final[3][4][0][0] <= final[1][4][0][0] + 0.05          # stack input, stream 1: 3 iterations vs 1

    # ---- the stack call gives the same bits as the block-by-block sweep (3 iterations are still set)
    s1, s2, g1, g2 = y1d.clone(), y2d.clone(), up(dy1), up(dy2)
    R.revffn_stack_backward(ctx, Wds, Gs, s1, s2, g1, g2, B, S, h)
    torch.cuda.synchronize()
    f = final[3]
    assert torch.equal(s1, f[0]) and torch.equal(s2, f[1]) and torch.equal(g1, f[2]) and torch.equal(g2, f[3])

    # ---- peak device memory: weights + gradients + one workspace + a handful of [T, h] tensors
    wbytes = sum(t.numel() * t.element_size() for w in Wds for t in w.values() if t is not None)
    gbytes = sum(t.numel() * t.element_size() for g in Gs for t in g.values() if t is not None)
    ws = int(ctx.workspace_bytes(B, S))
    peak = int(torch.cuda.max_memory_allocated()) + ws
    states_bytes = (2 * (L + 1) + 16) * T * h * 2            # this test's own copies of the GPU forward states
    # (the upload helper holds one float32 copy of the tensor it is converting: the largest weight tensor once)
    states_bytes += 4 * max(t.numel() for t in Wds[0].values() if t is not None)
    say(f"STACK24 peak device bytes {peak} = weights {wbytes} + gradients {gbytes} + workspace {ws} + test copies; "
        f"total {time.time() - t0:.0f} s")
    assert peak <= wbytes + gbytes + ws + states_bytes + (256 << 20)
    assert ws < 0.5e9                                        # one block's activations, whatever the depth
