"""The entry point that allocates nothing: revffn_op_attention_bwd_noalloc (scratch in a device array built into the
library) against revffn_op_attention_bwd (scratch passed by the caller), through the C ABI, on two calls in a row,
the second with a smaller input.  Same kernels, so the results must be the same bits; the allocating entry point is
itself checked against the fp64 oracle here (and at more shapes in test_gpu_kernels.py)."""
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


def _run(B, S, H, dh, causal, seed):
    rng = np.random.default_rng(seed)
    d = H * dh
    bf = lambda sc=1.0: synth.round_bf16((sc * rng.standard_normal((B * S, d))).astype(np.float32))
    q, k, v, do = bf(1.5), bf(1.5), bf(), bf()
    qd, kd, vd, dod = (Hn.upload(a, "bf16") for a in (q, k, v, do))
    od = torch.empty_like(qd)
    lse = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    R.revffn_op_attention_fwd(1, 0, qd, kd, vd, od, lse, B, S, H, dh, causal)
    # reference: the existing entry point, scratch from the caller
    dvec = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    ref = [torch.full_like(qd, float("nan")) for _ in range(3)]
    R.revffn_op_attention_bwd(1, 0, qd, kd, vd, od, dod, lse, dvec, *ref, B, S, H, dh, causal)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    out = [torch.full_like(qd, float("nan")) for _ in range(3)]
    after_alloc = torch.cuda.memory_allocated()
    R.revffn_op_attention_bwd_noalloc(1, 0, qd, kd, vd, od, dod, lse, *out, B, S, H, dh, causal)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == after_alloc and after_alloc > before
    for a, b in zip(out, ref):
        assert torch.equal(a, b)
    # and the reference itself against the oracle, at the bf16 bar
    r4 = lambda a: a.reshape(B, S, H, dh)
    _, P = O.attention_core(r4(q), r4(k), r4(v), causal)
    for g, r in zip(out, O.attention_core_backward(r4(do), r4(q), r4(k), r4(v), P)):
        assert relerr(Hn.download(g), r.reshape(B * S, d)) < 2e-2


def test_no_alloc_attention_backward_two_calls_second_smaller():
    _run(2, 300, 3, 128, True, 1)       # matrix-core kernels, ragged tiles
    _run(1, 77, 2, 128, True, 2)        # smaller: the scratch still holds the first call's values beyond these rows
    _run(2, 50, 3, 32, False, 3)        # head width without matrix-core kernels: the generic route uses the scratch too


def test_no_alloc_rejects_sizes_beyond_the_scratch():
    t = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(R.RevffnError, match="-2"):
        R.revffn_op_attention_bwd_noalloc(1, 0, t, t, t, t, t, f, t, t, t, 64, 8192, 16, 128, True)
