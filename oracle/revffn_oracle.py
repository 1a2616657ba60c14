"""Plain fp64 CPU oracle of the RevFFN reversible block.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may import
this module; the product library never does, and this module imports nothing
from the product.  It is deliberately slow and literal: one numpy statement per
line of the method, no blocking, no fusion, no reordering.

What it computes (paper section 3.1, Eq. 1-2, the inverse display below them, and
the adapter display of section 3.2):

    Y1 = X1 + Attn(Norm X1, Norm X2, Norm X2)          Eq. 1
    Y2 = X2 + MLP(Norm Y1)                              Eq. 2
    Attn(a, b, b) = P_dn( Attn_pt(P_up a, P_up b, P_up b) )     section 3.2
    MLP(c)        = P_dn( MLP_pt(P_up c) )                      section 3.2
    X2^ = Y2 - MLP(Norm Y1)                            inverse, first line
    X1^ = Y1 - Attn(Norm X1^, Norm X2^, Norm X2^)      inverse, second line,
          solved by fixed-point iteration started at X1^ = Y1

The symmetric comparison block of section 3.1 (the coupling the asymmetric layout is
contrasted with; Config.symmetric) takes the queries from stream 2 as well,

    Y1 = X1 + Attn(Norm X2, Norm X2, Norm X2),   Y2 = X2 + MLP(Norm Y1),

so its inverse has no implicit term: X2^ = Y2 - MLP(Norm Y1), X1^ = Y1 - Attn(Norm X2^, ...).

Attn_pt is multi-head softmax attention with q/k/v biases and rotary position
encoding (half-split pairing); MLP_pt is a sparse mixture of SwiGLU experts with
softmax-then-top-k routing plus an optional sigmoid-gated shared SwiGLU expert.
Those two follow the public Qwen2-MoE layer conventions, which the paper names
as its base model (section 3, first paragraph) but does not restate; Norm is
RMSNorm with a learnable gain for the same reason.  These readings are NOT fixed
by the paper ("parity unpinned by the paper"); every one is a Config flag.

The backward pass is ordinary reverse-mode differentiation of Eq. 1-2 evaluated
at a supplied block input (section 3.1: activations are recomputed from the
rebuilt input instead of being cached); it is not differentiated through the
fixed-point loop.

All arrays are float64 numpy.  Token-major layout: a stream is [T, h] with
T = B*S tokens (token t = b*S + s) and h = d_model/2.  Linear weights are
[out, in], applied as x @ W.T.
"""
from dataclasses import dataclass, replace
import numpy as np


@dataclass
class Config:
    d_model: int
    n_heads: int
    head_dim: int
    n_experts: int
    top_k: int
    d_expert: int
    d_shared: int = 0
    causal: bool = True
    use_rope: bool = True
    norm_topk_prob: bool = False
    n_inv_iters: int = 1          # the paper's value (section 3.1, last paragraph)
    symmetric: bool = False       # queries from stream 2 too (the symmetric variant section 3.1 compares against)
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6

    @property
    def h(self):
        return self.d_model // 2


PARAM_NAMES = (
    "norm_a1", "norm_a2", "norm_m", "pup_a", "pdn_a", "pup_m", "pdn_m",
    "wq", "wk", "wv", "wo", "bq", "bk", "bv", "w_router", "b_router",
    "w_gate_up", "w_down", "ws_gate_up", "ws_down", "ws_gate",
)


def as_f64(W):
    """Weights dict with every array promoted to float64 (no copy where it already is)."""
    return {k: (None if v is None else np.asarray(v, dtype=np.float64)) for k, v in W.items()}


# --------------------------------------------------------------------------
# element functions
# --------------------------------------------------------------------------
def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def silu(x):
    return x * sigmoid(x)


def silu_grad(x):
    s = sigmoid(x)
    return s * (1.0 + x * (1.0 - s))


def rmsnorm(x, g, eps):
    """Norm of Eq. 1-2, read as RMSNorm: x / sqrt(mean_j x_j^2 + eps) * g, per token."""
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x * r * g


def rmsnorm_bwd(dy, x, g, eps):
    n = x.shape[-1]
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    gdy = g * dy
    dx = r * gdy - x * (r ** 3) * np.sum(x * gdy, axis=-1, keepdims=True) / n
    dg = np.sum(x * r * dy, axis=0)
    return dx, dg


def rope(v, theta, sign=1.0):
    """Rotary encoding of v[B, S, H, dh], half-split pairing: element i is paired
    with element i + dh/2 and the pair is rotated by angle s * theta^(-2i/dh) at
    sequence position s.  sign=-1 rotates back (the transpose, used in backward)."""
    B, S, H, dh = v.shape
    half = dh // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = np.arange(S, dtype=np.float64)[:, None] * inv_freq[None, :]   # [S, half]
    c = np.cos(ang)[None, :, None, :]
    s = sign * np.sin(ang)[None, :, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


# --------------------------------------------------------------------------
# attention half:  A = P_dn_a( Attn_pt(P_up_a Norm X1, P_up_a Norm X2, P_up_a Norm X2) )
# --------------------------------------------------------------------------
def attention_core(Q, K, V, causal, keep_probs=True):
    """softmax(Q K^T / sqrt(dh) + mask) V for Q, K, V of shape [B, S, H, dh].
    Returns O [B, S, H, dh] and the probabilities P [B, H, S, S] (None unless keep_probs)."""
    B, S, H, dh = Q.shape
    O = np.zeros_like(Q)
    P = np.zeros((B, H, S, S)) if keep_probs else None
    for b in range(B):
        for hh in range(H):
            sc = Q[b, :, hh, :] @ K[b, :, hh, :].T / np.sqrt(dh)
            if causal:
                sc = np.where(np.tril(np.ones((S, S), dtype=bool)), sc, -np.inf)
            sc = sc - sc.max(axis=-1, keepdims=True)
            e = np.exp(sc)
            p = e / e.sum(axis=-1, keepdims=True)
            if keep_probs:
                P[b, hh] = p
            O[b, :, hh, :] = p @ V[b, :, hh, :]
    return O, P


def attention_core_backward(dO, Q, K, V, P):
    """Reverse-mode through attention_core given its probabilities P: returns dQ, dK, dV."""
    B, S, H, dh = Q.shape
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for b in range(B):
        for hh in range(H):
            p = P[b, hh]
            do = dO[b, :, hh, :]
            dV[b, :, hh, :] = p.T @ do
            dp = do @ V[b, :, hh, :].T
            ds = p * (dp - np.sum(dp * p, axis=-1, keepdims=True))
            dQ[b, :, hh, :] = ds @ K[b, :, hh, :] / np.sqrt(dh)
            dK[b, :, hh, :] = ds.T @ Q[b, :, hh, :] / np.sqrt(dh)
    return dQ, dK, dV


def attention_core_backward_streaming(dO, Q, K, V, causal):
    """The same gradients as attention_core_backward without a stored probability tensor: the
    probabilities of one (batch, head) pair are evaluated again from Q and K (the statements of
    attention_core), used, and dropped, so the memory in flight is one S x S matrix."""
    B, S, H, dh = Q.shape
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for b in range(B):
        for hh in range(H):
            sc = Q[b, :, hh, :] @ K[b, :, hh, :].T / np.sqrt(dh)
            if causal:
                sc = np.where(np.tril(np.ones((S, S), dtype=bool)), sc, -np.inf)
            sc = sc - sc.max(axis=-1, keepdims=True)
            e = np.exp(sc)
            p = e / e.sum(axis=-1, keepdims=True)
            do = dO[b, :, hh, :]
            dV[b, :, hh, :] = p.T @ do
            dp = do @ V[b, :, hh, :].T
            ds = p * (dp - np.sum(dp * p, axis=-1, keepdims=True))
            dQ[b, :, hh, :] = ds @ K[b, :, hh, :] / np.sqrt(dh)
            dK[b, :, hh, :] = ds.T @ Q[b, :, hh, :] / np.sqrt(dh)
    return dQ, dK, dV


def attn_half_forward(x1, x2, W, cfg, B, S, keep_probs=True):
    W = as_f64(W)
    T = B * S
    H, dh, d = cfg.n_heads, cfg.head_dim, cfg.d_model
    n1 = rmsnorm(x1, W["norm_a1"], cfg.rms_eps)
    n2 = rmsnorm(x2, W["norm_a2"], cfg.rms_eps)
    U1 = n1 @ W["pup_a"].T                      # the same P_up serves both streams
    U2 = n2 @ W["pup_a"].T
    if cfg.symmetric:                           # self-attention on stream 2: x1 plays no part in the branch
        n1, U1 = None, U2
    Ql = U1 @ W["wq"].T
    Kl = U2 @ W["wk"].T
    Vl = U2 @ W["wv"].T
    if W.get("bq") is not None:
        Ql = Ql + W["bq"]
    if W.get("bk") is not None:
        Kl = Kl + W["bk"]
    if W.get("bv") is not None:
        Vl = Vl + W["bv"]
    Q = Ql.reshape(B, S, H, dh)
    K = Kl.reshape(B, S, H, dh)
    V = Vl.reshape(B, S, H, dh)
    if cfg.use_rope:
        Q = rope(Q, cfg.rope_theta)
        K = rope(K, cfg.rope_theta)
    O4, P = attention_core(Q, K, V, cfg.causal, keep_probs)
    O = O4.reshape(T, d)
    AO = O @ W["wo"].T
    A = AO @ W["pdn_a"].T
    cache = dict(x1=x1, x2=x2, n1=n1, n2=n2, U1=U1, U2=U2, Q=Q, K=K, V=V,
                 P=P, O=O, AO=AO)
    return A, cache


def attn_half_backward(dA, c, W, cfg, B, S):
    """Reverse-mode through attn_half_forward.  Returns dx1, dx2, grads."""
    W = as_f64(W)
    T = B * S
    H, dh, d = cfg.n_heads, cfg.head_dim, cfg.d_model
    g = {}
    g["pdn_a"] = dA.T @ c["AO"]
    dAO = dA @ W["pdn_a"]
    g["wo"] = dAO.T @ c["O"]
    dO = (dAO @ W["wo"]).reshape(B, S, H, dh)
    if c["P"] is None:                          # forward ran with keep_probs=False (long sequences)
        dQ, dK, dV = attention_core_backward_streaming(dO, c["Q"], c["K"], c["V"], cfg.causal)
    else:
        dQ, dK, dV = attention_core_backward(dO, c["Q"], c["K"], c["V"], c["P"])
    if cfg.use_rope:
        dQ = rope(dQ, cfg.rope_theta, sign=-1.0)
        dK = rope(dK, cfg.rope_theta, sign=-1.0)
    dQl, dKl, dVl = dQ.reshape(T, d), dK.reshape(T, d), dV.reshape(T, d)
    g["wq"] = dQl.T @ c["U1"]
    g["wk"] = dKl.T @ c["U2"]
    g["wv"] = dVl.T @ c["U2"]
    g["bq"] = dQl.sum(axis=0)
    g["bk"] = dKl.sum(axis=0)
    g["bv"] = dVl.sum(axis=0)
    dU1 = dQl @ W["wq"]
    dU2 = dKl @ W["wk"] + dVl @ W["wv"]
    if cfg.symmetric:                           # the query path ends in stream 2 as well
        dU2 = dU2 + dU1
        g["pup_a"] = dU2.T @ c["n2"]
        dx2, g["norm_a2"] = rmsnorm_bwd(dU2 @ W["pup_a"], c["x2"], W["norm_a2"], cfg.rms_eps)
        g["norm_a1"] = np.zeros_like(W["norm_a1"])
        return np.zeros_like(c["x2"]), dx2, g
    g["pup_a"] = dU1.T @ c["n1"] + dU2.T @ c["n2"]
    dn1 = dU1 @ W["pup_a"]
    dn2 = dU2 @ W["pup_a"]
    dx1, g["norm_a1"] = rmsnorm_bwd(dn1, c["x1"], W["norm_a1"], cfg.rms_eps)
    dx2, g["norm_a2"] = rmsnorm_bwd(dn2, c["x2"], W["norm_a2"], cfg.rms_eps)
    return dx1, dx2, g


# --------------------------------------------------------------------------
# routing: integer, deterministic
# --------------------------------------------------------------------------
def route(z, cfg, forced_idx=None):
    """Softmax over all experts, then the top_k largest logits per token.
    Slots are ordered by descending logit; equal logits go to the lower expert
    index.  A logit that is not a number ranks as minus infinity in the selection
    (so a token with a non-finite input still selects top_k distinct, valid experts;
    its weights are not numbers).  Routing weight = softmax probability (renormalised
    over the selected set only if norm_topk_prob).  forced_idx [T,k]: take this
    selection instead of ranking the logits (used to evaluate the block under a
    selection that differs from this one's on a near-tie); the weights are still
    this softmax's.  Returns idx [T,k] int32, w [T,k], p [T,E]."""
    zs = z - z.max(axis=-1, keepdims=True)
    e = np.exp(zs)
    p = e / e.sum(axis=-1, keepdims=True)
    if forced_idx is not None:
        idx = np.asarray(forced_idx).astype(np.int32)
        assert idx.shape == (z.shape[0], cfg.top_k)
    else:
        zr = np.where(np.isnan(z), -np.inf, z)
        order = np.argsort(-zr, axis=-1, kind="stable")
        idx = order[:, :cfg.top_k].astype(np.int32)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=-1)
    if cfg.norm_topk_prob:
        w = w / w.sum(axis=-1, keepdims=True)
    return idx, w, p


def topk_margin(z, k):
    """z_(k) - z_(k+1) per token: how far the selection is from flipping."""
    if k >= z.shape[-1]:
        return np.full(z.shape[0], np.inf)
    zs = -np.sort(-z, axis=-1)
    return zs[:, k - 1] - zs[:, k]


def permutation(idx, n_experts):
    """Group the T*k (token, slot) pairs by expert, keeping (token, slot) order
    inside each expert.  counts[e] rows per expert, offsets = exclusive prefix sum
    (length E+1), row_map[pos] = t*k + slot for permuted position pos."""
    flat = idx.reshape(-1)
    counts = np.bincount(flat, minlength=n_experts).astype(np.int32)
    offsets = np.zeros(n_experts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    row_map = np.argsort(flat, kind="stable").astype(np.int32)
    return counts, offsets, row_map


# --------------------------------------------------------------------------
# MoE half:  M = P_dn_m( MLP_pt(P_up_m Norm Y1) )
# --------------------------------------------------------------------------
def moe_half_forward(y1, W, cfg, forced_idx=None):
    W = as_f64(W)
    T = y1.shape[0]
    E, k, I, d = cfg.n_experts, cfg.top_k, cfg.d_expert, cfg.d_model
    n3 = rmsnorm(y1, W["norm_m"], cfg.rms_eps)
    Um = n3 @ W["pup_m"].T
    z = Um @ W["w_router"].T
    if W.get("b_router") is not None:
        z = z + W["b_router"]
    idx, w, p = route(z, cfg, forced_idx)
    counts, offsets, row_map = permutation(idx, E)
    d = W["w_down"].shape[1]                    # width of the pre-trained space (h when the adapters are merged in)
    R = np.zeros((T, d))
    per_expert = []
    for e in range(E):
        rows = row_map[offsets[e]:offsets[e + 1]]
        tl, sl = rows // k, rows % k
        x = Um[tl]
        Wg, Wu = W["w_gate_up"][e, :I], W["w_gate_up"][e, I:]
        G = x @ Wg.T
        U = x @ Wu.T
        Hh = silu(G) * U
        Yp = Hh @ W["w_down"][e].T
        np.add.at(R, tl, w[tl, sl][:, None] * Yp)
        per_expert.append(dict(tl=tl, sl=sl, G=G, U=U, Hh=Hh, Yp=Yp))
    c = dict(y1=y1, n3=n3, Um=Um, z=z, p=p, idx=idx, w=w, counts=counts,
             offsets=offsets, row_map=row_map, per_expert=per_expert, R=R)
    Sh = np.zeros((T, d))
    if cfg.d_shared:
        Is = cfg.d_shared
        Gs = Um @ W["ws_gate_up"][:Is].T
        Us = Um @ W["ws_gate_up"][Is:].T
        Hs = silu(Gs) * Us
        Ys = Hs @ W["ws_down"].T
        gam = sigmoid(Um @ W["ws_gate"])
        Sh = gam[:, None] * Ys
        c.update(Gs=Gs, Us=Us, Hs=Hs, Ys=Ys, gam=gam)
    RS = R + Sh
    M = RS @ W["pdn_m"].T
    c.update(RS=RS, Sh=Sh)
    return M, c


def merge_adapters(W):
    """Section 3.2 wraps each pre-trained module as P_dn(module(P_up .)).  With static weights the products can be
    formed first: every matrix that reads the up-projected input is multiplied by P_up from the right, every matrix
    whose output is down-projected by P_dn from the left.  Returned in the layout of W with identity adapters, so the
    same functions evaluate it; in exact arithmetic nothing changes (associativity)."""
    W = as_f64(W)
    h = W["pup_a"].shape[1]
    M = dict(W)
    M["pup_a"] = np.eye(h)
    M["pdn_a"] = np.eye(h)
    M["pup_m"] = np.eye(h)
    M["pdn_m"] = np.eye(h)
    for n in ("wq", "wk", "wv"):
        M[n] = W[n] @ W["pup_a"]                                    # [d,d][d,h]
    M["wo"] = W["pdn_a"] @ W["wo"]                                  # [h,d][d,d]
    M["w_router"] = W["w_router"] @ W["pup_m"]                      # [E,d][d,h]
    M["w_gate_up"] = W["w_gate_up"] @ W["pup_m"]                    # [E,2I,d][d,h]
    M["w_down"] = np.einsum("hd,edi->ehi", W["pdn_m"], W["w_down"])
    if W.get("ws_gate_up") is not None:
        M["ws_gate_up"] = W["ws_gate_up"] @ W["pup_m"]
        M["ws_down"] = W["pdn_m"] @ W["ws_down"]
        M["ws_gate"] = W["pup_m"].T @ W["ws_gate"]                  # gamma = sigmoid(Um . ws_gate) = sigmoid(n3 . (P_up^T ws_gate))
    return M


def moe_half_backward(dM, c, W, cfg):
    """Reverse-mode through moe_half_forward.  The top-k selection itself has zero
    gradient; the routing probabilities do carry gradient to every logit."""
    W = as_f64(W)
    T = dM.shape[0]
    E, k, I, d = cfg.n_experts, cfg.top_k, cfg.d_expert, cfg.d_model
    Um = c["Um"]
    g = {}
    g["pdn_m"] = dM.T @ c["RS"]
    dRS = dM @ W["pdn_m"]
    dUm = np.zeros_like(Um)
    if cfg.d_shared:
        Is = cfg.d_shared
        gam = c["gam"]
        dgam = np.sum(dRS * c["Ys"], axis=-1)
        dYs = gam[:, None] * dRS
        dlg = dgam * gam * (1.0 - gam)
        g["ws_down"] = dYs.T @ c["Hs"]
        dHs = dYs @ W["ws_down"]
        dGs = dHs * c["Us"] * silu_grad(c["Gs"])
        dUs = dHs * silu(c["Gs"])
        g["ws_gate_up"] = np.concatenate([dGs.T @ Um, dUs.T @ Um], axis=0)
        dUm += dGs @ W["ws_gate_up"][:Is] + dUs @ W["ws_gate_up"][Is:]
        g["ws_gate"] = dlg @ Um
        dUm += dlg[:, None] * W["ws_gate"][None, :]
    dw = np.zeros((T, k))
    g["w_gate_up"] = np.zeros_like(W["w_gate_up"])
    g["w_down"] = np.zeros_like(W["w_down"])
    for e in range(E):
        pe = c["per_expert"][e]
        tl, sl = pe["tl"], pe["sl"]
        if tl.size == 0:
            continue
        x = Um[tl]
        dR_e = dRS[tl]
        dw[tl, sl] = np.sum(dR_e * pe["Yp"], axis=-1)
        dYp = c["w"][tl, sl][:, None] * dR_e
        g["w_down"][e] = dYp.T @ pe["Hh"]
        dHh = dYp @ W["w_down"][e]
        dG = dHh * pe["U"] * silu_grad(pe["G"])
        dU = dHh * silu(pe["G"])
        g["w_gate_up"][e, :I] = dG.T @ x
        g["w_gate_up"][e, I:] = dU.T @ x
        np.add.at(dUm, tl, dG @ W["w_gate_up"][e, :I] + dU @ W["w_gate_up"][e, I:])
    p, idx = c["p"], c["idx"].astype(np.int64)
    if cfg.norm_topk_prob:
        psel = np.take_along_axis(p, idx, axis=-1)
        ssum = psel.sum(axis=-1, keepdims=True)
        dpsel = (dw - np.sum(dw * c["w"], axis=-1, keepdims=True)) / ssum
    else:
        dpsel = dw
    dp = np.zeros_like(p)
    np.put_along_axis(dp, idx, dpsel, axis=-1)
    dz = p * (dp - np.sum(dp * p, axis=-1, keepdims=True))
    g["w_router"] = dz.T @ Um
    g["b_router"] = dz.sum(axis=0)
    dUm += dz @ W["w_router"]
    g["pup_m"] = dUm.T @ c["n3"]
    dn3 = dUm @ W["pup_m"]
    dy1, g["norm_m"] = rmsnorm_bwd(dn3, c["y1"], W["norm_m"], cfg.rms_eps)
    return dy1, g


# --------------------------------------------------------------------------
# block: forward (Eq. 1-2), inverse, backward
# --------------------------------------------------------------------------
def forward(x1, x2, W, cfg, B, S, return_cache=False, forced_idx=None):
    A, ca = attn_half_forward(x1, x2, W, cfg, B, S, keep_probs=return_cache)
    y1 = x1 + A                                  # Eq. 1
    M, cm = moe_half_forward(y1, W, cfg, forced_idx)
    y2 = x2 + M                                  # Eq. 2
    if return_cache:
        return y1, y2, dict(attn=ca, moe=cm, A=A, M=M)
    return y1, y2


def inverse(y1, y2, W, cfg, B, S, n_iters=None, converge=False, return_info=False, tol=None, max_iters=64,
            forced_idx=None, block_positions=0):
    """Rebuild the block input from its output.  Stream 2 is exact.  Stream 1 is
    the fixed-point iteration x <- Y1 - Attn(Norm x, Norm X2^, Norm X2^) started
    from x = Y1, run n_iters times (default cfg.n_inv_iters), or, if converge, until
    successive iterates differ by less than 1e-14 * max|Y1| (at most 64 times), or, if
    tol is given, until max|x_n - x_(n-1)| <= tol (at most max_iters times).
    With tol and block_positions > 0 the rule is applied to each run of block_positions positions
    of each sequence on its own (a query row's iterate depends on that row alone, since keys and
    values come from X2^): a block that has met the tolerance keeps its iterate while the others go
    on; info then also holds block_iters and block_residuals in (sequence, range) order, and
    residual / iters are the largest over the blocks."""
    M, cm = moe_half_forward(y1, W, cfg)
    x2 = y2 - M
    if cfg.symmetric:                            # closed form: the branch depends on X2^ alone
        A, _ = attn_half_forward(y1, x2, W, cfg, B, S, keep_probs=False)
        x = y1 - A
        return (x, x2, dict(residual=0.0, iters=0, moe=cm, residuals=[])) if return_info else (x, x2)
    if tol is not None and block_positions > 0:
        nj = -(-S // block_positions)
        rows = [np.arange(b * S + j * block_positions, b * S + min(S, (j + 1) * block_positions))
                for b in range(B) for j in range(nj)]
        x = y1.copy()
        active = [True] * len(rows)
        b_it, b_res = [0] * len(rows), [0.0] * len(rows)
        for it in range(1, max_iters + 1):
            A, _ = attn_half_forward(x, x2, W, cfg, B, S, keep_probs=False)
            xn = y1 - A
            for q, r in enumerate(rows):
                if not active[q]:
                    continue
                b_res[q] = float(np.max(np.abs(xn[r] - x[r])))
                b_it[q] = it
                x[r] = xn[r]
                if b_res[q] <= tol:
                    active[q] = False
            if not any(active):
                break
        if return_info:
            return x, x2, dict(residual=max(b_res), iters=max(b_it), moe=cm, residuals=[],
                               block_iters=b_it, block_residuals=b_res)
        return x, x2
    x = y1.copy()
    n = cfg.n_inv_iters if n_iters is None else n_iters
    res, it = np.inf, 0
    limit = max_iters if tol is not None else (64 if converge else n)
    history = []
    while it < limit:
        A, _ = attn_half_forward(x, x2, W, cfg, B, S, keep_probs=False)
        xn = y1 - A
        res = float(np.max(np.abs(xn - x)))
        history.append(res)
        x = xn
        it += 1
        if tol is not None:
            if res <= tol:
                break
        elif converge and res < 1e-14 * float(np.max(np.abs(y1))):
            break
    if return_info:
        return x, x2, dict(residual=res, iters=it, moe=cm, residuals=history)
    return x, x2


def backward(x1, x2, y1, dy1, dy2, W, cfg, B, S, forced_idx=None, keep_probs=True):
    """Gradients of the block at input (x1, x2) for upstream (dy1, dy2).
    The attention half is recomputed at (x1, x2); the MoE half is recomputed at
    y1 (the exact block output the sweep holds) or at x1 + A(x1, x2) if y1 is None.
    keep_probs=False: the attention probabilities are not stored but evaluated again
    head by head in the backward pass (same statements; for long sequences).
    Returns dx1, dx2, grads (dict keyed like the weights)."""
    A, ca = attn_half_forward(x1, x2, W, cfg, B, S, keep_probs=keep_probs)
    if y1 is None:
        y1 = x1 + A
    _, cm = moe_half_forward(y1, W, cfg, forced_idx)
    dy1_moe, gm = moe_half_backward(dy2, cm, W, cfg)      # Y2 = X2 + M(Y1)
    g1 = dy1 + dy1_moe                                     # total gradient at Y1
    dx1_att, dx2_att, ga = attn_half_backward(g1, ca, W, cfg, B, S)  # Y1 = X1 + A(X1, X2)
    dx1 = g1 + dx1_att
    dx2 = dy2 + dx2_att
    grads = {}
    grads.update(ga)
    grads.update(gm)
    for name in ("bq", "bk", "bv", "b_router"):
        if W.get(name) is None:
            grads.pop(name, None)
    return dx1, dx2, grads


def grads_stored(x1, x2, dy1, dy2, W, cfg, B, S):
    """Ordinary stored-activation route: forward on the true input, backprop there."""
    y1, _ = forward(x1, x2, W, cfg, B, S)
    return backward(x1, x2, y1, dy1, dy2, W, cfg, B, S)


def grads_reconstructed(y1, y2, dy1, dy2, W, cfg, B, S, n_iters=None, converge=False):
    """Reversible route: rebuild the input from the output, then backprop at the
    rebuilt input with the MoE half evaluated at the exact y1."""
    x1h, x2h = inverse(y1, y2, W, cfg, B, S, n_iters=n_iters, converge=converge)
    dx1, dx2, grads = backward(x1h, x2h, y1, dy1, dy2, W, cfg, B, S)
    return x1h, x2h, dx1, dx2, grads


# --------------------------------------------------------------------------
# stack of blocks (section 3.1: only the last hidden state is kept; the backward
# sweep walks down, rebuilding each block's input from its output)
# --------------------------------------------------------------------------
def stack_forward(x1, x2, Ws, cfg, B, S, keep_all=False):
    states = [(x1, x2)] if keep_all else None
    for W in Ws:
        x1, x2 = forward(x1, x2, W, cfg, B, S)        # no stream swap between layers
        if keep_all:
            states.append((x1, x2))
    return (x1, x2, states) if keep_all else (x1, x2)


def stack_backward_sweep(y1, y2, dy1, dy2, Ws, cfg, B, S, n_iters=None):
    """Returns dx1, dx2 at the stack input, per-layer grads (list, layer order) and
    the rebuilt per-layer inputs (list, layer order)."""
    grads, rebuilt = [None] * len(Ws), [None] * len(Ws)
    for l in range(len(Ws) - 1, -1, -1):
        x1h, x2h, dy1, dy2, g = grads_reconstructed(y1, y2, dy1, dy2, Ws[l], cfg, B, S, n_iters=n_iters)
        grads[l], rebuilt[l] = g, (x1h, x2h)
        y1, y2 = x1h, x2h
    return dy1, dy2, grads, rebuilt
