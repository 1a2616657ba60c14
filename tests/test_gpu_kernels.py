"""Kernel-level GPU parity: the bf16 MFMA GEMM in its three operand layouts and the flash
attention kernels, each against the fp64 oracle on the same bf16-rounded inputs, at sizes
that span several tiles and end in ragged tails."""
import numpy as np
import pytest
import torch

import synth
from oracle import revffn_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2512_20920_amd as R
    from paper_2512_20920_amd import harness as Hn
    from helpers import relerr


def _bf(rng, shape, scale=1.0):
    return synth.round_bf16(scale * rng.standard_normal(shape).astype(np.float32))


@pytest.mark.parametrize("layout", ["nt", "nn", "tn"])
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (200, 328, 136), (1, 64, 520), (300, 8, 72), (257, 129 * 8, 24),
                                   # 64 tiles or more: the XCD-aware tile placement, with ragged last tiles and
                                   # rectangles that do not divide the tile grid evenly
                                   (1100, 1304, 72), (2056, 520, 40), (392, 4104, 24)])
def test_mfma_gemm_layouts(layout, M, N, K):
    if layout == "tn":
        M = (M + 7) // 8 * 8
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    A, Bm = _bf(rng, (M, K)), _bf(rng, (K, N))
    ref = A @ Bm
    a_trans, b_trans = layout == "tn", layout in ("nn", "tn")
    a_host = A.T.copy() if a_trans else A
    b_host = Bm if b_trans else Bm.T.copy()
    ad, bd = Hn.upload(a_host, "bf16"), Hn.upload(b_host, "bf16")
    for out_f32 in (False, True):
        cd = torch.full((M, N), float("nan"), dtype=torch.float32 if out_f32 else torch.bfloat16, device="cuda")
        R.revffn_op_gemm(1, 2, ad, bd, cd, M, N, K, a_host.shape[1], b_host.shape[1], N, a_trans, b_trans, out_f32)
        torch.cuda.synchronize()
        assert relerr(Hn.download(cd), ref) < (1e-5 if out_f32 else 6e-3), (layout, out_f32)
    # the generic kernel computes the same thing
    cd = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    R.revffn_op_gemm(1, 1, ad, bd, cd, M, N, K, a_host.shape[1], b_host.shape[1], N, a_trans, b_trans, False)
    torch.cuda.synchronize()
    assert relerr(Hn.download(cd), ref) < 6e-3


@pytest.mark.parametrize("tile", [1, 2, 3, 4])
@pytest.mark.parametrize("layout", ["nt", "nn", "tn"])
def test_mfma_gemm_every_tile_shape(layout, tile):
    """Every tile shape of the MFMA kernel (forced per launch) on shapes with ragged last tiles in m, n and k,
    including problems smaller than one tile."""
    for (M, N, K) in [(264, 328, 136), (520, 264, 200), (40, 72, 24)]:
        rng = np.random.default_rng(M + 3 * N + 5 * K + tile)
        A, Bm = _bf(rng, (M, K)), _bf(rng, (K, N))
        ref = A @ Bm
        a_trans, b_trans = layout == "tn", layout in ("nn", "tn")
        a_host = A.T.copy() if a_trans else A
        b_host = Bm if b_trans else Bm.T.copy()
        ad, bd = Hn.upload(a_host, "bf16"), Hn.upload(b_host, "bf16")
        for out_f32 in (False, True):
            cd = torch.full((M, N), float("nan"), dtype=torch.float32 if out_f32 else torch.bfloat16, device="cuda")
            R.revffn_op_gemm(1, 2 + 256 * tile, ad, bd, cd, M, N, K, a_host.shape[1], b_host.shape[1], N, a_trans,
                             b_trans, out_f32)
            torch.cuda.synchronize()
            assert relerr(Hn.download(cd), ref) < (1e-5 if out_f32 else 6e-3), (layout, tile, M, N, K, out_f32)


def _attention_case(B, S, H, dh, causal, mode, dtype):
    rng = np.random.default_rng(S * 31 + H + (7 if causal else 0))
    rnd = (lambda s, sc=1.0: _bf(rng, s, sc)) if dtype == 1 else \
          (lambda s, sc=1.0: (sc * rng.standard_normal(s)).astype(np.float32).astype(np.float64))
    d = H * dh
    q, k, v, do = rnd((B * S, d), 1.5), rnd((B * S, d), 1.5), rnd((B * S, d)), rnd((B * S, d))
    r4 = lambda a: a.reshape(B, S, H, dh)
    if S > 2048:          # long sequences: one S x S matrix in flight instead of a stored probability tensor
        o_ref, _ = O.attention_core(r4(q), r4(k), r4(v), causal, keep_probs=False)
        dq_ref, dk_ref, dv_ref = O.attention_core_backward_streaming(r4(do), r4(q), r4(k), r4(v), causal)
    else:
        o_ref, P = O.attention_core(r4(q), r4(k), r4(v), causal)
        dq_ref, dk_ref, dv_ref = O.attention_core_backward(r4(do), r4(q), r4(k), r4(v), P)
    sname = "bf16" if dtype == 1 else "f32"
    qd, kd, vd, dod = (Hn.upload(a, sname) for a in (q, k, v, do))
    od = torch.full_like(qd, float("nan"))
    lse = torch.full((B, H, S), float("nan"), dtype=torch.float32, device="cuda")
    R.revffn_op_attention_fwd(dtype, mode, qd, kd, vd, od, lse, B, S, H, dh, causal)
    torch.cuda.synchronize()
    tol = 2e-2 if dtype == 1 else 1e-4
    assert relerr(Hn.download(od), o_ref.reshape(B * S, d)) < tol
    sc = np.einsum("bshd,bthd->bhst", r4(q), r4(k)) / np.sqrt(dh)
    if causal:
        sc = np.where(np.tril(np.ones((S, S), dtype=bool)), sc, -np.inf)
    lse_ref = np.log(np.exp(sc - sc.max(-1, keepdims=True)).sum(-1)) + sc.max(-1)
    assert np.abs(Hn.download(lse) - lse_ref).max() < (2e-2 if dtype == 1 else 1e-4)
    dvec = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    dqd, dkd, dvd = (torch.full_like(qd, float("nan")) for _ in range(3))
    R.revffn_op_attention_bwd(dtype, mode, qd, kd, vd, od, dod, lse, dvec, dqd, dkd, dvd, B, S, H, dh, causal)
    torch.cuda.synchronize()
    assert relerr(Hn.download(dvd), dv_ref.reshape(B * S, d)) < tol
    assert relerr(Hn.download(dqd), dq_ref.reshape(B * S, d)) < tol
    assert relerr(Hn.download(dkd), dk_ref.reshape(B * S, d)) < tol


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("B,S,H", [(1, 128, 1), (2, 200, 3), (1, 64, 2), (1, 1, 1), (1, 451, 2)])
def test_flash_attention(B, S, H, causal):
    _attention_case(B, S, H, 128, causal, 2, 1)


@pytest.mark.parametrize("causal", [True, False])
def test_flash_attention_long_sequence(causal):
    """One head at the long-context sequence length (S = 8192): forward, dQ, dK and dV element by element."""
    _attention_case(1, 8192, 1, 128, causal, 2, 1)


def test_flash_attention_ragged_long_sequence():
    _attention_case(1, 2500, 2, 128, True, 2, 1)


@pytest.mark.parametrize("dtype,dh", [(0, 16), (1, 32), (0, 80)])
def test_generic_attention(dtype, dh):
    _attention_case(2, 70, 3, dh, True, 1, dtype)
    _attention_case(1, 33, 2, dh, False, 1, dtype)
