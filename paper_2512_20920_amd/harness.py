"""Device-memory helpers around the binding: upload seeded host arrays, allocate gradient
buffers, download results.  No arithmetic of the method lives here."""
import numpy as np
import torch

from .binding import Config, WEIGHT_FIELDS

F32_ONLY = ("b_router",)


def torch_dtype(dtype):
    return torch.bfloat16 if dtype in ("bf16", 1) else torch.float32


def make_config(wl, causal=True, use_rope=True, norm_topk_prob=False, n_inv_iters=1,
                rope_theta=1.0e6, rms_eps=1.0e-6, dtype=None, fp32_streams=False, symmetric=False, fp32_grads=False):
    """Config for a synth.Workload-like object (needs d_model, n_heads, ... and dtype)."""
    dt = wl.dtype if dtype is None else dtype
    return Config(d_model=wl.d_model, n_heads=wl.n_heads, head_dim=wl.head_dim, n_experts=wl.n_experts,
                  top_k=wl.top_k, d_expert=wl.d_expert, d_shared=wl.d_shared,
                  dtype=1 if dt == "bf16" else 0, causal=int(causal), use_rope=int(use_rope),
                  norm_topk_prob=int(norm_topk_prob), n_inv_iters=n_inv_iters,
                  rope_theta=rope_theta, rms_eps=rms_eps, fp32_streams=int(bool(fp32_streams)), symmetric=int(bool(symmetric)), fp32_grads=int(bool(fp32_grads)))


def upload(x, dtype, device="cuda"):
    """float64 host array (already holding storage-rounded values) -> device tensor."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device).to(torch_dtype(dtype)).contiguous()


def upload_weights(W, dtype, device="cuda"):
    out = {}
    for n in WEIGHT_FIELDS:
        v = W.get(n)
        if v is None:
            out[n] = None
        else:
            out[n] = upload(v, "f32" if n in F32_ONLY else dtype, device)
    return out


def alloc_grads(Wdev, skip=(), fp32=False):
    """A gradient buffer per present weight (filled with NaN so an unwritten one is noticed); float32 buffers with
    fp32=True (config.fp32_grads)."""
    out = {}
    for n in WEIGHT_FIELDS:
        v = Wdev.get(n)
        if v is None or n in skip:
            out[n] = None
        else:
            out[n] = torch.full_like(v, float("nan"), dtype=torch.float32 if fp32 else v.dtype)
    return out


def download(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def alloc_merged(wl, device="cuda"):
    """Device buffers for the pre-merged adapter weights of one block (binding.Merged fields)."""
    d, h, E, I, Is = wl.d_model, wl.d_model // 2, wl.n_experts, wl.d_expert, wl.d_shared
    dt = torch_dtype(wl.dtype)
    new = lambda *shape, t=dt: torch.full(shape, float("nan"), dtype=t, device=device)
    return {"wq": new(d, h), "wk": new(d, h), "wv": new(d, h), "wo": new(h, d), "w_gate_up": new(E, 2 * I, h),
            "w_down": new(E, h, I), "ws_gate_up": new(2 * Is, h) if Is else None, "ws_down": new(h, Is) if Is else None,
            "w_router": new(E + (1 if Is else 0), h, t=torch.float32)}
