"""Weight gradients written straight into the destination layout (the gradient GEMM's epilogue does the
reshard): bit-identical to the unfused backward followed by ntp_reshard_grad, and within the GEMM tolerance
of the oracle's reshard of the oracle's gradients.  On a real MI355X."""
import sys

import numpy as np
import pytest

from paper_2504_06095_amd import binding as K

from oracle import ntp_oracle as O
from tests import helpers as Hh

pytestmark = pytest.mark.gpu
SENTINEL = -12345.0


def _say(msg):
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def _dst_shards(torch, widths, H, pad=0):
    """Destination shards [w x H] (leading dimension H + pad), filled with a sentinel."""
    out = []
    for w in widths:
        buf = torch.full((max(w, 1), H + pad), SENTINEL, dtype=torch.float32, device="cuda")
        out.append(buf[:w, :H])
    return out


def _mlp_case(M, H, n, a, b, rank, seed, pad, accumulate):
    import torch
    import paper_2504_06095_amd as N
    c = Hh.MlpCase(M, H, n, a, rank, seed=seed, tag="fused")
    n_r = c.n_r
    X, At, B, dZ = (Hh.to_dev_bf16(x) for x in (c.X_bits, c.At_bits, c.B_bits, c.dZ_bits))
    ld = max(Hh.round_up(n_r, 8), 8)
    mk = lambda r, cc: torch.full((r, cc), float("nan"), dtype=torch.bfloat16, device="cuda")
    P, Y, dP = mk(M, ld)[:, :n_r], mk(M, ld)[:, :n_r], mk(M, ld)[:, :n_r]
    Z, dX = mk(M, H), mk(M, H)
    N.ntp_mlp_shard_fwd(X, At, B, P, Y, Z, n_r)
    spec = N.tensor_spec(n, H, 0, 1, 4)
    widths = [O.shard_plan(n, b, d)[1] for d in range(b)]
    # unfused: gradients of this rank, then the reshard with only this rank present
    dA = torch.full((n_r, H), float("nan"), dtype=torch.float32, device="cuda")
    dB = torch.full((n_r, H), float("nan"), dtype=torch.float32, device="cuda")
    ref = {}
    for name, g in (("dA", dA), ("dB", dB)):
        ref[name] = _dst_shards(torch, widths, H, pad)
    reps = 2 if accumulate else 1
    for i in range(reps):
        N.ntp_mlp_shard_bwd(dZ, X, At, B, P, Y, dP, dX, dA, dB, n_r, 0, i > 0)
    src = [None] * a
    for name, g in (("dA", dA), ("dB", dB)):
        src[rank] = g
        N.ntp_reshard_grad(spec, a, b, src, ref[name])
    # fused
    got = {name: _dst_shards(torch, widths, H, pad) for name in ("dA", "dB")}
    segs = {name: N.ntp_reshard_row_segments(spec, a, rank, b, got[name]) for name in ("dA", "dB")}
    dX2 = mk(M, H)
    for i in range(reps):
        N.ntp_mlp_shard_bwd_resharded(dZ, X, At, B, P, Y, dP, dX2, segs["dA"], segs["dB"], n_r, 0, i > 0)
    torch.cuda.synchronize()
    for name in ("dA", "dB"):
        for d in range(b):
            assert torch.equal(got[name][d], ref[name][d]), (name, d)
    assert torch.equal(dX2.view(torch.int16), dX.view(torch.int16))
    # against the oracle: this rank's gradient rows, cut where the TP = b layout cuts them
    w = c.oracle()
    for name, key in (("dA", "dA_t"), ("dB", "dB")):
        full = w[key] * reps
        for d in range(b):
            o_d, w_d = O.shard_plan(n, b, d)
            lo, hi = max(o_d, c.off), min(o_d + w_d, c.off + n_r)
            g = got[name][d].cpu().numpy().astype(np.float64)
            if lo < hi:
                assert Hh.rel_err(g[lo - o_d: hi - o_d], full[lo - c.off: hi - c.off]) <= Hh.TOL, (name, d)
            untouched = np.ones(w_d, dtype=bool)
            untouched[max(lo - o_d, 0): max(hi - o_d, 0)] = False
            assert (g[untouched] == SENTINEL).all(), (name, d)


@pytest.mark.parametrize("M,H,n,a,b,rank,pad,accumulate", [
    (512, 1024, 4096, 7, 8, 0, 0, False),   # config 1
    (512, 1024, 4096, 7, 8, 3, 4, False),   # a middle rank: two destinations, padded rows
    (512, 1024, 4096, 7, 8, 6, 0, True),    # last rank, accumulated twice
    (300, 512, 1000, 8, 7, 5, 0, False),    # full -> reduced, ragged tokens
    (256, 512, 1003, 3, 8, 1, 0, False),    # one source shard over four destinations
])
def test_mlp_bwd_resharded_matches_unfused(M, H, n, a, b, rank, pad, accumulate):
    _say(f"mlp bwd resharded M={M} H={H} n={n} {a}->{b} rank {rank} pad {pad} acc {accumulate}")
    _mlp_case(M, H, n, a, b, rank, 4, pad, accumulate)


@pytest.mark.parametrize("tile", ["auto", "256x256", "224x256", "256x192", "128x256", "128x128", "generic"])
def test_mlp_bwd_resharded_every_kernel_family(opts, tile):
    # large enough for the ring kernel's weight-gradient variants; the tile shape is forced in turn
    _say(f"mlp bwd resharded, gradient GEMM tile {tile}")
    if tile != "auto":
        opts(K.NTP_OPT_GEMM_TILE, tile)
    _mlp_case(1024, 2048, 8192, 7, 8, 2, 5, 0, tile == "256x256")


@pytest.mark.parametrize("splits,accumulate", [(2, False), (3, True)])
def test_mlp_bwd_resharded_with_split_k(opts, splits, accumulate):
    """The gradient GEMMs cut along the token axis: the kernel that adds the partial sums stores them through the
    same row segments (two destination shards per gradient here), overwriting or accumulating."""
    import torch
    import paper_2504_06095_amd as N
    _say(f"mlp bwd resharded with split-K, {splits} chunks, accumulate {accumulate}")
    N.ntp_set_workspace(torch.full((32 << 20,), float("nan"), dtype=torch.float32, device="cuda"))
    N.ntp_kernel_timing_enable(1)
    N.ntp_kernel_timing_read()
    try:
        opts(K.NTP_OPT_GEMM_SPLIT, splits)
        _mlp_case(1100, 1096, 8197, 7, 8, 3, 6, 4, accumulate)
        names = [r["name"] for r in N.ntp_kernel_timing_read() if r["name"].startswith("gemm_tn")]
        assert names and all(n.endswith(f"k{splits}") for n in names), names
    finally:
        N.ntp_kernel_timing_enable(0)
        N.ntp_kernel_timing_read()
        N.ntp_set_workspace(None)


def test_attn_bwd_resharded_refuses_replicated_kv_heads():
    """16 query heads, 4 KV heads over 5 ranks: rank 2 holds heads 7-9, i.e. KV heads 1 and 2, which ranks 1 and 3
    hold too.  Its dW rows of those heads are partial sums; the fused store would drop the other holders' shares."""
    import paper_2504_06095_amd as N
    K = N.binding
    spec_q = N.tensor_spec((16 + 8) * 32, 512, 0, 32, 4, K.NTP_KIND_QKV_GQA, 16, 4)
    dst = [(0x10000000 + 0x1000000 * r, 512) for r in range(7)]
    with pytest.raises(N.NtpError) as e:
        N.ntp_reshard_row_segments(spec_q, 5, 2, 7, dst)
    assert e.value.status == K.NTP_ERR_UNSUPPORTED
    assert len(N.ntp_reshard_row_segments(spec_q, 5, 0, 7, dst)) > 0  # rank 0 holds KV head 0 alone


# (source ranks whose KV heads no other source rank holds)
@pytest.mark.parametrize("a,b,rank", [(5, 7, 0), (4, 7, 2), (4, 4, 1), (2, 7, 1), (1, 5, 0)])
def test_attn_bwd_resharded_matches_unfused(a, b, rank):
    import torch
    import paper_2504_06095_amd as N
    _say(f"attn bwd resharded {a}->{b} rank {rank}")
    M, H, n_q, n_kv, d = 320, 512, 16, 4, 32
    c = Hh.AttnCase(M, H, n_q, n_kv, d, a, rank, seed=6, tag="fusedattn")
    wq, wo = c.w_qkv, c.w_o
    X, Cc, dZ, dQKV, Wqkv, Wo = (Hh.to_dev_bf16(x) for x in (c.X_bits, c.C_bits, c.dZ_bits, c.dQKV_bits, c.Wqkv_bits,
                                                             c.Wo_bits))
    mk = lambda r, cc: torch.full((r, cc), float("nan"), dtype=torch.bfloat16, device="cuda")
    K = N.binding
    spec_q = N.tensor_spec((n_q + 2 * n_kv) * d, H, 0, d, 4, K.NTP_KIND_QKV_GQA, n_q, n_kv)
    spec_o = N.tensor_spec(n_q * d, H, 0, d, 4)
    wq_dst = [N.ntp_attn_shard_plan(n_q, n_kv, d, b, r)["w_qkv"] for r in range(b)]
    wo_dst = [N.ntp_attn_shard_plan(n_q, n_kv, d, b, r)["w_o"] for r in range(b)]
    # unfused
    dC, dX = mk(M, wo), mk(M, H)
    dWqkv = torch.full((wq, H), float("nan"), dtype=torch.float32, device="cuda")
    dWo = torch.full((wo, H), float("nan"), dtype=torch.float32, device="cuda")
    N.ntp_attn_proj_shard_bwd(M, H, wq, wo, dZ, dQKV, X, Cc, Wqkv, Wo, dC, dX, dWqkv, dWo, False)
    ref_q, ref_o = _dst_shards(torch, wq_dst, H), _dst_shards(torch, wo_dst, H)
    src = [None] * a
    src[rank] = dWqkv
    N.ntp_reshard_grad(spec_q, a, b, src, ref_q)
    src[rank] = dWo
    N.ntp_reshard_grad(spec_o, a, b, src, ref_o)
    # fused
    got_q, got_o = _dst_shards(torch, wq_dst, H), _dst_shards(torch, wo_dst, H)
    sq = N.ntp_reshard_row_segments(spec_q, a, rank, b, got_q)
    so = N.ntp_reshard_row_segments(spec_o, a, rank, b, got_o)
    dC2, dX2 = mk(M, wo), mk(M, H)
    N.ntp_attn_proj_shard_bwd_resharded(M, H, wq, wo, dZ, dQKV, X, Cc, Wqkv, Wo, dC2, dX2, sq, so, False)
    torch.cuda.synchronize()
    for r in range(b):
        assert torch.equal(got_q[r], ref_q[r]), ("dWqkv", r)
        assert torch.equal(got_o[r], ref_o[r]), ("dWo", r)
    assert torch.equal(dC2.view(torch.int16), dC.view(torch.int16)) and torch.equal(dX2.view(torch.int16), dX.view(torch.int16))
    # against the oracle on the rows this rank feeds: the destination copy of every unit it is the source of
    w = c.oracle()
    n_units = n_q + 2 * n_kv
    for r in range(b):
        g = got_q[r].cpu().numpy().astype(np.float64)
        for j in range(wq_dst[r] // d):
            sr, sl = O.reshard_source_of(O.QKV_GQA, n_units, a, b, r, j, n_q, n_kv)
            blk = g[j * d: (j + 1) * d]
            if sr == rank:
                assert Hh.rel_err(blk, w["dWqkv"][sl * d: (sl + 1) * d]) <= Hh.TOL, (r, j)
            else:
                assert (blk == SENTINEL).all(), (r, j)


def test_resharded_rejects_bad_segments():
    import torch
    import paper_2504_06095_amd as N
    _say("resharded: error paths")
    M, H, n_r = 64, 256, 40
    bf = dict(dtype=torch.bfloat16, device="cuda")
    dZ, X = torch.zeros(M, H, **bf), torch.zeros(M, H, **bf)
    At, B = torch.zeros(n_r, H, **bf), torch.zeros(n_r, H, **bf)
    P, Y, dP = torch.zeros(M, n_r, **bf), torch.zeros(M, n_r, **bf), torch.zeros(M, n_r, **bf)
    dX = torch.zeros(M, H, **bf)
    buf = torch.zeros(2 * n_r, H, dtype=torch.float32, device="cuda")
    other = torch.zeros(n_r, H, dtype=torch.float32, device="cuda")
    K = N.binding
    good = N.row_segments([(0, n_r, other, H)])

    def call(a_segs, b_segs=good):
        N.ntp_mlp_shard_bwd_resharded(dZ, X, At, B, P, Y, dP, dX, a_segs, b_segs, n_r)

    with pytest.raises(N.NtpError) as e:  # rows past the end of the gradient
        call(N.row_segments([(0, n_r + 1, buf, H)]))
    assert e.value.status == K.NTP_ERR_INVALID_ARG
    with pytest.raises(N.NtpError) as e:  # two segments that overlap in memory
        call(N.row_segments([(0, 20, buf, H), (20, 20, buf[10:], H)]))
    assert e.value.status == K.NTP_ERR_INVALID_ARG
    with pytest.raises(N.NtpError) as e:  # destination rows shorter than the gradient's
        call(N.row_segments([(0, n_r, buf, H - 4)]))
    assert e.value.status == K.NTP_ERR_INVALID_ARG
    with pytest.raises(N.NtpError) as e:  # misaligned destination
        call(N.row_segments([(0, n_r, buf.data_ptr() + 4, H)]))
    assert e.value.status == K.NTP_ERR_ALIGNMENT
    with pytest.raises(N.NtpError) as e:  # more segments than one launch takes
        call(N.row_segments([(i, 1, buf[i: i + 1], H) for i in range(17)]))
    assert e.value.status == K.NTP_ERR_UNSUPPORTED
    # a row listed nowhere is simply not stored
    buf.fill_(SENTINEL)
    call(N.row_segments([(0, 10, buf, H), (30, 10, buf[30:], H)]))
    torch.cuda.synchronize()
    assert (buf[10:30] == SENTINEL).all() and (buf[:10] == 0).all() and (buf[30:40] == 0).all()
