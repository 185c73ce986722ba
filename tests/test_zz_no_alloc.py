"""The entry point that allocates nothing (ntp_attn_proj_shard_fwd_static): split-K partial sums in the library's
static device array.  Two calls in a row through the C ABI, the second on a smaller input, each compared bit for
bit with ntp_attn_proj_shard_fwd on a handle whose workspace has the same size, and with the oracle.
On a real MI355X."""
import sys

import numpy as np
import pytest

from paper_2504_06095_amd import binding as K
from tests.helpers import TOL, AttnCase, dev_bf16_to_f64, rel_err, to_dev_bf16

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def _run(case, fn, handle):
    import torch
    M, H, wq, wo = case.M, case.H, case.w_qkv, case.w_o
    X, Cc, Wqkv, Wo = (to_dev_bf16(b) for b in (case.X_bits, case.C_bits, case.Wqkv_bits, case.Wo_bits))
    QKV = torch.full((M, wq), float("nan"), dtype=torch.bfloat16, device="cuda")
    Z = torch.full((M, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    fn(M, H, wq, wo, X, Wqkv, QKV, Cc, Wo, Z, handle=handle)
    torch.cuda.synchronize()
    return QKV, Z


def test_static_scratch_entry_point_matches_the_workspace_one_twice():
    import torch
    import paper_2504_06095_amd as N
    static_h, ref_h = N.ntp_create(), N.ntp_create()
    N.ntp_set_workspace(torch.full((K.NTP_STATIC_SCRATCH_BYTES // 4,), float("nan"), dtype=torch.float32, device="cuda"),
                        handle=ref_h)
    # first call: 3 heads of a 64-head model at TP 30 (4096 tokens, hidden 8192): X W_qkv is cut into K chunks;
    # second call: a smaller input (fewer tokens, narrower, other ranks' widths), cut again
    cases = [AttnCase(4096, 8192, 64, 8, 128, 30, 0, tag="static.a"), AttnCase(2200, 4104, 32, 4, 64, 11, 1, tag="static.b")]
    for i, case in enumerate(cases):
        c = K.ntp_gemm_choice(0, case.M, case.w_qkv, case.H, handle=ref_h)
        _say(f"static scratch call {i}: M={case.M} H={case.H} w_qkv={case.w_qkv} w_o={case.w_o}, K chunks {c['k_splits']}")
        assert c["k_splits"] > 1, "the case is meant to use the scratch array"
        got_q, got_z = _run(case, N.ntp_attn_proj_shard_fwd_static, static_h)
        ref_q, ref_z = _run(case, N.ntp_attn_proj_shard_fwd, ref_h)
        assert torch.equal(got_q.view(torch.int16), ref_q.view(torch.int16))
        assert torch.equal(got_z.view(torch.int16), ref_z.view(torch.int16))
        want = case.oracle()
        assert rel_err(dev_bf16_to_f64(got_q), want["QKV"]) <= TOL
        assert rel_err(dev_bf16_to_f64(got_z), want["Z"]) <= TOL
    # a shape that could use more room than the array has is refused, and nothing is written
    probe = N.ntp_create()
    assert K.lib().ntp_set_workspace(probe.ptr, 0x10000000, 1 << 40) == 0  # (an address for the host-only choice call)
    c = K.ntp_gemm_choice(0, 8192, 512, 16384, handle=probe)
    assert c["k_splits"] * 8192 * 512 * 4 > K.NTP_STATIC_SCRATCH_BYTES
    N.ntp_destroy(probe)
    X = torch.zeros(8192, 16384, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros(512, 16384, dtype=torch.bfloat16, device="cuda")
    QKV = torch.full((8192, 512), 3.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(N.NtpError) as e:
        N.ntp_attn_proj_shard_fwd_static(8192, 16384, 512, 256, X, W, QKV, None, None, None, handle=static_h)
    assert e.value.status == K.NTP_ERR_SCRATCH_TOO_SMALL
    torch.cuda.synchronize()
    assert bool((QKV == 3.0).all())
    N.ntp_destroy(static_h)
    N.ntp_destroy(ref_h)
