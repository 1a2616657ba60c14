"""Shared pieces of the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

import synth
from oracle import revffn_oracle as O
import paper_2512_20920_amd as R
from paper_2512_20920_amd import harness as Hn


def oracle_cfg(wl, **kw):
    c = O.Config(wl.d_model, wl.n_heads, wl.head_dim, wl.n_experts, wl.top_k, wl.d_expert, wl.d_shared)
    return O.replace(c, **kw)


def relerr(gpu, ref):
    """max |gpu - ref| / max |ref|  (the tolerance measure of the parity bar)."""
    ref = np.asarray(ref, dtype=np.float64)
    gpu = np.asarray(gpu, dtype=np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), "non-finite GPU output"
    den = np.abs(ref).max()
    if den == 0:
        return float(np.abs(gpu).max())
    return float(np.abs(gpu - ref).max() / den)


TOL = {"f32": 1e-4, "bf16": 2e-2}
# relative spacing of the storage dtype: a stored value x carries a rounding error up to UNIT*|x|/2
UNIT = {"f32": 2.0 ** -23, "bf16": 2.0 ** -8}


def delta_err(gpu, ref, base, dt):
    """Error of the update (gpu - base) against (ref - base), as a multiple of what is resolvable:
    tol * max|ref - base| plus the rounding of storing `gpu` itself.  Returns (error, bound at tol)."""
    gpu, ref, base = (np.asarray(a, dtype=np.float64) for a in (gpu, ref, base))
    assert np.all(np.isfinite(gpu)), "non-finite GPU output"
    err = float(np.abs(gpu - ref).max())
    bound = TOL[dt] * float(np.abs(ref - base).max()) + UNIT[dt] * float(np.abs(ref).max())
    return err, bound


class Case:
    """One workload on the GPU: uploaded inputs/weights plus a context."""

    def __init__(self, wl, flags=None, mode=0, max_B=None, max_S=None, weights=None, inputs=None, fp32_streams=False,
                 fp32_grads=False):
        self.wl = wl
        self.flags = dict(flags or {})
        self.ocfg = oracle_cfg(wl, **self.flags)
        self.W = weights if weights is not None else synth.make_weights(wl)
        self.x1, self.x2, self.dy1, self.dy2 = inputs if inputs is not None else synth.make_inputs(wl)
        self.cfg = Hn.make_config(wl, fp32_streams=fp32_streams, fp32_grads=fp32_grads, **self.flags)
        self.fp32_grads = fp32_grads
        self.ctx = R.Context(self.cfg, max_B or wl.B, max_S or wl.S)
        self.ctx.set_kernel_mode(mode)
        self.ctx.enable_taps(True)
        self.Wd = Hn.upload_weights(self.W, wl.dtype)
        self.dt = wl.dtype
        self.sdt = "f32" if fp32_streams else wl.dtype      # element type of the residual streams x1, x2, y1, y2
        self.B, self.S, self.T, self.h = wl.B, wl.S, wl.T, wl.h

    def up(self, x):
        return Hn.upload(x, self.dt)

    def empty(self):
        return torch.empty((self.T, self.h), dtype=Hn.torch_dtype(self.dt), device="cuda")

    def up_s(self, x):
        return Hn.upload(x, self.sdt)

    def empty_s(self):
        return torch.empty((self.T, self.h), dtype=Hn.torch_dtype(self.sdt), device="cuda")

    def forward(self, x1=None, x2=None):
        x1d = self.up_s(self.x1 if x1 is None else x1)
        x2d = self.up_s(self.x2 if x2 is None else x2)
        y1d, y2d = self.empty_s(), self.empty_s()
        R.revffn_forward(self.ctx, self.Wd, x1d, x2d, y1d, y2d, self.B, self.S, self.h)
        torch.cuda.synchronize()
        return y1d, y2d

    def branches(self):
        a = torch.empty((self.T, self.h), dtype=torch.float32, device="cuda")
        m = torch.empty((self.T, self.h), dtype=torch.float32, device="cuda")
        R.revffn_get_branch(self.ctx, 0, a)
        R.revffn_get_branch(self.ctx, 1, m)
        torch.cuda.synchronize()
        return Hn.download(a), Hn.download(m)

    def routing(self):
        T, k, E = self.T, self.wl.top_k, self.wl.n_experts
        idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
        wts = torch.empty((T, k), dtype=torch.float32, device="cuda")
        counts = torch.empty((E,), dtype=torch.int32, device="cuda")
        offsets = torch.empty((E + 1,), dtype=torch.int32, device="cuda")
        row_map = torch.empty((T * k,), dtype=torch.int32, device="cuda")
        R.revffn_get_routing(self.ctx, idx, wts, counts, offsets, row_map)
        torch.cuda.synchronize()
        return (idx.cpu().numpy(), wts.cpu().numpy().astype(np.float64), counts.cpu().numpy(),
                offsets.cpu().numpy(), row_map.cpu().numpy())

    def inverse(self, y1d, y2d, n_iters=None, want_residual=False):
        if n_iters is not None:
            self.ctx.set_inv_iters(n_iters)
        x1d, x2d = self.empty_s(), self.empty_s()
        res = torch.zeros((1,), dtype=torch.float32, device="cuda") if want_residual else None
        R.revffn_inverse(self.ctx, self.Wd, y1d, y2d, x1d, x2d, self.B, self.S, self.h, res)
        torch.cuda.synchronize()
        return (x1d, x2d, float(res.item())) if want_residual else (x1d, x2d)

    def backward(self, x1d, x2d, y1d, dy1=None, dy2=None, skip=()):
        dy1d = self.up(self.dy1 if dy1 is None else dy1)
        dy2d = self.up(self.dy2 if dy2 is None else dy2)
        dx1d, dx2d = self.empty(), self.empty()
        G = Hn.alloc_grads(self.Wd, skip=skip, fp32=self.fp32_grads)
        R.revffn_backward(self.ctx, self.Wd, x1d, x2d, y1d, dy1d, dy2d, dx1d, dx2d, G, self.B, self.S, self.h)
        torch.cuda.synchronize()
        return dx1d, dx2d, G


def safe_tokens(cm, cfg):
    """Tokens whose selection and slot order are decided by clear margins in the oracle's fp64 logits: the top-k
    margin and every gap between selected logits exceed 1e-3.  The rest are near-ties."""
    margin = O.topk_margin(cm["z"], cfg.top_k)
    zsel = np.take_along_axis(cm["z"], cm["idx"].astype(np.int64), axis=-1)
    gaps = np.min(-np.diff(zsel, axis=-1), axis=-1) if cfg.top_k > 1 else np.full(len(margin), np.inf)
    return (margin > 1e-3) & (gaps > 1e-3)


def check_routing(case, y1_host, report=None):
    """Routing of the most recent call on case.ctx against the oracle router evaluated at the
    same stream-1 values y1_host.  Bit-exact wherever the oracle's top-k logit margin exceeds
    1e-3 (no flip is tolerated there); the rest are counted (ties).  Returns the oracle's MoE
    cache, the mask of clear tokens and the GPU's own indices, with which a caller evaluates the
    oracle (forced_idx) so that every token is compared whatever a near-tie did."""
    cfg, W = case.ocfg, case.W
    _, cm = O.moe_half_forward(y1_host, W, cfg)
    safe = safe_tokens(cm, cfg)
    idx, wts, counts, offsets, row_map = case.routing()
    assert np.array_equal(idx[safe], cm["idx"][safe]), "routing index mismatch on a token with margin > 1e-3"
    n_unsafe = int((~safe).sum())
    flips = int((idx != cm["idx"]).any(axis=-1).sum())
    if flips == 0:
        assert np.array_equal(counts, cm["counts"]) and np.array_equal(offsets, cm["offsets"])
        assert np.array_equal(row_map, cm["row_map"])
    # on a near-tie the GPU may pick the other expert of the tie, or order two slots the other way, never anything
    # else: its choice is a set of k distinct experts whose logits are within 2e-3 of the oracle's choice, slot by slot
    assert idx.min() >= 0 and idx.max() < cfg.n_experts
    assert all(len(set(r)) == cfg.top_k for r in idx[~safe].tolist())
    zg = np.take_along_axis(cm["z"], idx.astype(np.int64), axis=-1)
    zo = np.take_along_axis(cm["z"], cm["idx"].astype(np.int64), axis=-1)
    assert np.abs(zg - zo).max() <= 2e-3, "a near-tie was resolved to an expert that is not part of the tie"
    # whatever the ties did, the permutation must be the stable grouping of the GPU's own indices
    c2, o2, r2 = O.permutation(idx, cfg.n_experts)
    assert np.array_equal(counts, c2) and np.array_equal(offsets, o2) and np.array_equal(row_map, r2)
    assert relerr(wts[safe], cm["w"][safe]) < 1e-4
    # the weights of all tokens, near-ties included, against this softmax taken at the GPU's indices
    psel = np.take_along_axis(cm["p"], idx.astype(np.int64), axis=-1)
    assert relerr(wts, psel / psel.sum(-1, keepdims=True) if cfg.norm_topk_prob else psel) < 1e-4
    print(f"ROUTING {case.wl.name}: tokens {len(safe)} ties {n_unsafe} flips {flips}")
    if report is not None:
        report["ties"] = n_unsafe
        report["flips"] = flips
    return cm, safe, idx
