"""The entry point that allocates nothing (atp_attention_static) against atp_attention.

Two calls in a row through the raw C ABI, the second with a smaller input: the built-in scratch buffer
keeps the first call's contents, so the second call shows that stale data is never read."""
import ctypes as C

import numpy as np
import pytest
import torch

from util import to_dev

pytestmark = pytest.mark.gpu


def test_attention_static_matches_attention_on_two_calls_in_a_row():
    import paper_2403_02352_amd as atp
    lib = atp.lib
    rng = np.random.default_rng(2403)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptr = lambda t: C.c_void_p(t.data_ptr())
    # (batch, L, r, heads, d_h): ragged r and L in both; the second is smaller in every dimension
    for case, dtype in (((2, 300, 200, 4, 64), "bf16"), ((1, 130, 70, 2, 64), "bf16"),
                        ((2, 96, 50, 2, 32), "f32"), ((1, 40, 20, 2, 32), "f32")):
        batch, L, r, heads, dh = case
        dq = heads * dh
        print(f"attention_static {case} {dtype}", flush=True)
        Q = to_dev(rng.standard_normal((batch, L, dq)), dtype)
        K = to_dev(rng.standard_normal((batch, r, dq)), dtype)
        V = to_dev(rng.standard_normal((batch, r, dq)), dtype)
        ref = atp.attention(Q, K, V, heads)
        out = torch.full_like(Q, float("nan"))
        t = atp.ATP_BF16 if dtype == "bf16" else atp.ATP_F32
        st = lib.atp_attention_static(ptr(Q), ptr(K), ptr(V), ptr(out), batch, L, r, dq, heads, C.c_float(0.0), t, stream)
        assert st == 0, lib.atp_status_string(st)
        torch.cuda.synchronize()
        assert torch.isfinite(out.float()).all()
        # same kernels, same launch shapes, same inputs: the results are the same bits
        assert torch.equal(out, ref)


def test_attention_static_rejects_inputs_beyond_the_limit():
    import paper_2403_02352_amd as atp
    lib = atp.lib
    # 8·4096·1024·2 bytes = 64 MiB > 32 MiB: refused on the host before any pointer is touched
    one = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    p = C.c_void_p(one.data_ptr())
    st = lib.atp_attention_static(p, p, p, p, 8, 4096, 1024, 4096, 32, C.c_float(0.0), atp.ATP_BF16, None)
    assert st == 6 and b"scratch" in lib.atp_status_string(st)
    assert atp.attention_workspace(8, 4096, 1024, 4096, 32, torch.bfloat16) > atp.STATIC_SCRATCH_BYTES
    # the largest benchmark shape fits exactly
    assert atp.attention_workspace(4, 4096, 1024, 4096, 32, torch.bfloat16) == atp.STATIC_SCRATCH_BYTES
