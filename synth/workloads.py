"""Workload table and seeded tensor generators (no method arithmetic here)."""
from dataclasses import dataclass, field
import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    d_model: int
    n_heads: int
    head_dim: int
    n_experts: int
    top_k: int
    d_expert: int
    d_shared: int
    B: int
    S: int
    dtype: str            # "f32" or "bf16" (storage; accumulation is always fp32 on the GPU)
    n_blocks: int = 1
    zipf: bool = False    # add the Zipf(1.2) router bias
    gain_jitter: float = 0.0   # std of the N(0, .) perturbation of the RMSNorm gains around 1
    seed: int = 0

    @property
    def T(self):
        return self.B * self.S

    @property
    def h(self):
        return self.d_model // 2


_QWEN = dict(d_model=2048, n_heads=16, head_dim=128, n_experts=60, top_k=4,
             d_expert=1408, d_shared=5632)

WORKLOADS = {
    # tiny fp32 block: the case the oracle finishes in seconds
    "tiny_f32": Workload("tiny_f32", 64, 4, 16, 8, 2, 128, 0, 2, 32, "f32", gain_jitter=0.02),
    # the same tiny geometry with a shared expert, used by CPU-side oracle pins
    "tiny_shared_f32": Workload("tiny_shared_f32", 64, 4, 16, 8, 2, 128, 96, 2, 32, "f32", gain_jitter=0.02),
    # headline: one block at the Qwen1.5-MoE-A2.7B shape, batch 4 x seq 512
    "qwen_b4s512": Workload("qwen_b4s512", B=4, S=512, dtype="bf16", **_QWEN),
    # load imbalance: Zipf router bias, batch 2 x seq 2048
    "qwen_zipf_b2s2048": Workload("qwen_zipf_b2s2048", B=2, S=2048, dtype="bf16", zipf=True, **_QWEN),
    # 24-block stack, batch 1 x seq 1024
    "qwen_stack24_b1s1024": Workload("qwen_stack24_b1s1024", B=1, S=1024, dtype="bf16", n_blocks=24, **_QWEN),
    # long context, batch 1 x seq 8192
    "qwen_b1s8192": Workload("qwen_b1s8192", B=1, S=8192, dtype="bf16", **_QWEN),
    # a second MoE geometry for the grouped GEMMs: few large experts (8 experts, top-2, width 14336, d 4096, no shared
    # expert), 512 rows per expert at batch 2 x seq 1024 -- the compute-bound end, where the Qwen shape is the
    # weight-streaming end
    "e8k2_d4096_b2s1024": Workload("e8k2_d4096_b2s1024", 4096, 32, 128, 8, 2, 14336, 0, 2, 1024, "bf16"),
    # reduced-size bf16 cases for element-by-element parity (several tiles + ragged tails)
    "mid_bf16": Workload("mid_bf16", 512, 4, 128, 12, 3, 192, 320, 2, 200, "bf16", gain_jitter=0.02),
    "mid_f32": Workload("mid_f32", 128, 4, 32, 6, 2, 96, 160, 3, 50, "f32", gain_jitter=0.02),
    # few large experts, no shared expert, reduced: rows per expert span several 128- and 256-row tiles
    "mid_fewbig_bf16": Workload("mid_fewbig_bf16", 512, 4, 128, 3, 2, 712, 0, 3, 232, "bf16", gain_jitter=0.02),
    # 137 rows per expert on average, the Qwen shape's figure at 2048 tokens: the routed forward GEMMs take the tiles
    # that are 160 rows high; expert width 200 leaves a gate column tile that ends inside the tile
    "mid_rows137_bf16": Workload("mid_rows137_bf16", 512, 4, 128, 6, 2, 200, 160, 2, 206, "bf16", gain_jitter=0.02),
}

WEIGHT_FIELDS = (
    "norm_a1", "norm_a2", "norm_m", "pup_a", "pdn_a", "pup_m", "pdn_m",
    "wq", "wk", "wv", "wo", "bq", "bk", "bv", "w_router", "b_router",
    "w_gate_up", "w_down", "ws_gate_up", "ws_down", "ws_gate",
)

# Scale of the Zipf router bias b_e = ZIPF_ALPHA * (-1.2 * ln rank_e), chosen so the
# hottest expert gets about 8x the mean load on the zipf workload.  The value is
# written by tests/golden/calibrate_zipf.py (which calls only the oracle).
ZIPF_ALPHA = 0.2691


def weight_shapes(wl):
    d, h, E, I, Is = wl.d_model, wl.h, wl.n_experts, wl.d_expert, wl.d_shared
    shapes = {
        "norm_a1": (h,), "norm_a2": (h,), "norm_m": (h,),
        "pup_a": (d, h), "pdn_a": (h, d), "pup_m": (d, h), "pdn_m": (h, d),
        "wq": (d, d), "wk": (d, d), "wv": (d, d), "wo": (d, d),
        "bq": (d,), "bk": (d,), "bv": (d,),
        "w_router": (E, d), "b_router": (E,),
        "w_gate_up": (E, 2 * I, d), "w_down": (E, d, I),
    }
    if Is:
        shapes.update({"ws_gate_up": (2 * Is, d), "ws_down": (d, Is), "ws_gate": (d,)})
    return shapes


def bf16_bits(x):
    """float array -> uint16 bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))     # finite inputs: no wrap-around
    return (u >> np.uint32(16)).astype(np.uint16)


def bits_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def round_bf16(x):
    """float array -> float64 array holding exactly the bf16-rounded values."""
    return bits_to_f64(bf16_bits(x))


def _store(x, dtype, f64=True):
    """Round float32 values to the storage dtype.  Returns an array holding exactly the stored
    values: float64 if f64 else float32 (both represent bf16 and fp32 values exactly)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        if x.size > (1 << 20):
            # same round-to-nearest-even as bf16_bits, done by torch's multi-threaded cast
            import torch
            x = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
        else:
            x = (bf16_bits(x).astype(np.uint32) << 16).view(np.float32)
    return x.astype(np.float64) if f64 else x


def zipf_router_bias(wl, seed, alpha=None):
    """b_e = alpha * (-1.2 * ln rank_e), ranks 1..E assigned by a seeded permutation."""
    a = ZIPF_ALPHA if alpha is None else alpha
    rng = np.random.default_rng(seed + 77)
    rank = rng.permutation(wl.n_experts) + 1
    return a * (-1.2 * np.log(rank.astype(np.float64)))


def make_weights(wl, block=0, alpha=None, f64=True):
    """One block's weights as float64 (or, with f64=False, float32) arrays holding
    storage-rounded values.  b_router is fp32 at the boundary in both dtypes.
    Block l of a stack uses seed + 1000*(l+1)."""
    rng = np.random.default_rng(wl.seed + 1000 * (block + 1))
    W = {}
    for name, shp in weight_shapes(wl).items():
        if name.startswith("norm_"):
            v = 1.0 + wl.gain_jitter * rng.standard_normal(shp)
        elif name == "b_router":
            if not wl.zipf:
                continue
            W[name] = np.asarray(zipf_router_bias(wl, wl.seed, alpha), dtype=np.float32).astype(np.float64)
            continue
        else:
            v = rng.standard_normal(shp, dtype=np.float32)
            v *= np.float32(0.02)
        W[name] = _store(v, wl.dtype, f64)
    for name in WEIGHT_FIELDS:
        W.setdefault(name, None)
    return W


def make_inputs(wl):
    """X1, X2 and upstream gradients dY1, dY2, each [T, h], float64 holding
    storage-rounded values; drawn in that order from default_rng(seed)."""
    rng = np.random.default_rng(wl.seed)
    out = []
    for _ in range(4):
        out.append(_store(rng.standard_normal((wl.T, wl.h), dtype=np.float32), wl.dtype))
    return tuple(out)
