"""Parity of the attention core (Eq. 5) on a rank's local heads against the oracle, on a real MI355X:
forward output and log-sum-exp, uneven head counts, grouped KV heads, ragged sequence lengths, causal and
unmasked."""
import sys

import numpy as np
import pytest

from paper_2504_06095_amd import binding as K

from oracle import ntp_oracle as O
from paper_2504_06095_amd import inputs as I
from tests import helpers as Hh

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def _case(n_q, n_kv, tp, rank, d, n_seq, S, causal, seed=0, pad=0, std=1.0):
    import torch
    import paper_2504_06095_amd as N
    plan = N.ntp_attn_shard_plan(n_q, n_kv, d, tp, rank)
    oplan = O.attn_shard_plan(n_q, n_kv, tp, rank)
    group = n_q // n_kv
    M = n_seq * S
    wq, wo = plan["w_qkv"], plan["w_o"]
    bits, vals = I.normal_bf16(seed, f"core.QKV.{n_q}.{n_kv}.{tp}.{rank}.{d}.{M}", (M, wq), std)
    QKV = Hh.to_dev_bf16(bits, wq + pad)
    C = torch.full((M, wo + pad), float("nan"), dtype=torch.bfloat16, device="cuda")[:, :wo]
    LSE = torch.full((plan["q_cnt"], M), float("nan"), dtype=torch.float32, device="cuda")
    shape = N.attn_core_shape(n_seq, S, plan, group, causal)
    N.ntp_attn_core_shard_fwd(shape, QKV, C, LSE)
    torch.cuda.synchronize()
    if wo == 0:
        return 0.0  # a rank without heads: the call is a no-op
    x = vals.astype(np.float64)
    want = O.attn_core_shard_fwd(x, oplan, group, d, n_seq, causal)
    got = Hh.dev_bf16_to_f64(C)
    assert np.isfinite(got).all()
    assert Hh.rel_err(got, want) <= Hh.TOL, Hh.rel_err(got, want)
    qc, kc = oplan["q_cnt"], oplan["kv_cnt"]
    lse = LSE.cpu().numpy().astype(np.float64)
    for s in range(n_seq):
        rows = slice(s * S, (s + 1) * S)
        for j in range(qc):
            g = (oplan["q_off"] + j) // group - oplan["kv_off"]
            w = O.attention_lse(x[rows, j * d:(j + 1) * d], x[rows, (qc + g) * d:(qc + g + 1) * d], causal)
            assert np.abs(lse[j, rows] - w).max() <= 2e-2 * max(1.0, np.abs(w).max()), (s, j)
    return Hh.rel_err(got, want)


CASES = [
    # n_q, n_kv, tp, rank, d, n_seq, S
    (8, 2, 3, 0, 128, 2, 200),    # 3 local heads over 1-2 KV heads, ragged length, two sequences
    (8, 2, 3, 2, 128, 1, 129),    # 2 local heads; one row past a 128-row tile
    (64, 8, 30, 3, 128, 1, 512),  # config-3 head plan (3 heads), several key tiles
    (64, 8, 30, 29, 128, 1, 384), # a rank with 2 heads
    (6, 6, 4, 1, 128, 3, 64),     # no grouping, exactly one key tile
    (4, 4, 2, 0, 64, 2, 100),     # head dimension 64
    (4, 1, 4, 3, 128, 1, 1),      # a single token
    (4, 2, 8, 6, 128, 1, 50),     # more ranks than heads: this rank has none
]


@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("n_q,n_kv,tp,rank,d,n_seq,S", CASES)
def test_attn_core_fwd_matches_oracle(n_q, n_kv, tp, rank, d, n_seq, S, causal):
    _say(f"attn core fwd n_q={n_q} n_kv={n_kv} tp={tp} rank={rank} d={d} n_seq={n_seq} S={S} causal={causal}")
    _case(n_q, n_kv, tp, rank, d, n_seq, S, causal)


@pytest.mark.parametrize("copy", [1, 2], ids=["registers", "dma"])
@pytest.mark.parametrize("n_q,n_kv,n_seq,S,causal,pad", [(24, 24, 4, 512, False, 0), (32, 32, 8, 512, True, 0), (32, 4, 7, 449, True, 8),
                                                         (32, 4, 6, 449, False, 8), (48, 48, 3, 1100, True, 0)])
def test_attn_core_fwd_many_workgroups(opts, n_q, n_kv, n_seq, S, causal, pad, copy):
    """Enough (sequence, head, tile) workgroups for the variants with 32 query rows per wavefront (tiles copied through
    registers, or by DMA): whole tiles, ragged lengths with an odd number of 128-row tiles, grouped KV heads, padded rows."""
    import paper_2504_06095_amd as N
    _say(f"attn core fwd, many workgroups: heads {n_q}/{n_kv} n_seq {n_seq} S {S} causal {causal} pad {pad} copy {copy}")
    opts(K.NTP_OPT_ATTN_COPY, copy)
    plan = N.ntp_attn_shard_plan(n_q, n_kv, 128, 1, 0)
    assert N.ntp_attn_core_choice(N.attn_core_shape(n_seq, S, plan, n_q // n_kv, causal))["fwd_rows_per_wavefront"] == 32
    _case(n_q, n_kv, 1, 0, 128, n_seq, S, causal, seed=2, pad=pad)


def _bwd_case(n_q, n_kv, tp, rank, d, n_seq, S, causal, seed=1, pad=0):
    import torch
    import paper_2504_06095_amd as N
    plan = N.ntp_attn_shard_plan(n_q, n_kv, d, tp, rank)
    oplan = O.attn_shard_plan(n_q, n_kv, tp, rank)
    group = n_q // n_kv
    M = n_seq * S
    wq, wo = plan["w_qkv"], plan["w_o"]
    qc, kc = plan["q_cnt"], plan["kv_cnt"]
    bits, vals = I.normal_bf16(seed, f"coreb.QKV.{n_q}.{n_kv}.{tp}.{rank}.{d}.{M}", (M, wq), 1.0)
    gbits, gvals = I.normal_bf16(seed, f"coreb.dC.{n_q}.{n_kv}.{tp}.{rank}.{d}.{M}", (M, wo), 1.0)
    QKV, dC = Hh.to_dev_bf16(bits, wq + pad), Hh.to_dev_bf16(gbits, wo + pad)
    nanbf = lambda r, c: torch.full((r, c + pad), float("nan"), dtype=torch.bfloat16, device="cuda")[:, :c]
    C, dQKV = nanbf(M, wo), nanbf(M, wq)
    LSE = torch.full((qc, M), float("nan"), dtype=torch.float32, device="cuda")
    Delta = torch.full((qc, M), float("nan"), dtype=torch.float32, device="cuda")
    shape = N.attn_core_shape(n_seq, S, plan, group, causal)
    N.ntp_attn_core_shard_fwd(shape, QKV, C, LSE)
    N.ntp_attn_core_shard_bwd(shape, QKV, C, dC, LSE, Delta, dQKV)
    torch.cuda.synchronize()
    x, gC = vals.astype(np.float64), gvals.astype(np.float64)
    want = O.attn_core_shard_bwd(x, gC, oplan, group, d, n_seq, causal)
    got = Hh.dev_bf16_to_f64(dQKV)
    assert np.isfinite(got).all()
    for name, lo, hi in (("dQ", 0, qc * d), ("dK", qc * d, (qc + kc) * d), ("dV", (qc + kc) * d, (qc + 2 * kc) * d)):
        assert Hh.rel_err(got[:, lo:hi], want[:, lo:hi]) <= Hh.TOL, (name, Hh.rel_err(got[:, lo:hi], want[:, lo:hi]))
    # the scratch holds rowsum(dC .* C) per head and token
    Cw = O.attn_core_shard_fwd(x, oplan, group, d, n_seq, causal)
    dl = Delta.cpu().numpy().astype(np.float64)
    for j in range(qc):
        w = (gC[:, j * d:(j + 1) * d] * Cw[:, j * d:(j + 1) * d]).sum(1)
        assert np.abs(dl[j] - w).max() <= 2e-2 * max(1.0, np.abs(w).max()), j


@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("n_q,n_kv,tp,rank,d,n_seq,S", CASES[:7])
def test_attn_core_bwd_matches_oracle(n_q, n_kv, tp, rank, d, n_seq, S, causal):
    _say(f"attn core bwd n_q={n_q} n_kv={n_kv} tp={tp} rank={rank} d={d} n_seq={n_seq} S={S} causal={causal}")
    _bwd_case(n_q, n_kv, tp, rank, d, n_seq, S, causal)


@pytest.fixture
def workspace():
    """A registered workspace full of NaN (partial sums must all be written before they are read), timing on."""
    import torch
    import paper_2504_06095_amd as N
    ws = torch.full((32 << 20,), float("nan"), dtype=torch.float32, device="cuda")  # 128 MiB
    N.ntp_set_workspace(ws)
    N.ntp_kernel_timing_enable(1)
    N.ntp_kernel_timing_read()
    yield ws
    N.ntp_kernel_timing_enable(0)
    N.ntp_kernel_timing_read()
    N.ntp_set_workspace(None)


def _core_names():
    import paper_2504_06095_amd as N
    return [r["name"] for r in N.ntp_kernel_timing_read() if r["name"].startswith("attn_core")]


@pytest.mark.parametrize("parts", [2, 5, 16])
@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("n_q,n_kv,tp,rank,d,n_seq,S", [CASES[0], CASES[2], CASES[3], CASES[5], CASES[6]])
def test_attn_core_bwd_cut_walks(workspace, opts, n_q, n_kv, tp, rank, d, n_seq, S, causal, parts):
    """Each workgroup's walk cut into 2, 5 and 16 parts (more parts than tiles leaves some empty), fp32 partial
    sums added by the second kernel."""
    _say(f"attn core bwd cut into {parts}: n_q={n_q} n_kv={n_kv} tp={tp} rank={rank} d={d} n_seq={n_seq} S={S} causal={causal}")
    opts(K.NTP_OPT_ATTN_PARTS, parts)
    _bwd_case(n_q, n_kv, tp, rank, d, n_seq, S, causal)
    names = _core_names()
    if d == 128:  # both kernels in one launch
        assert "attn_core_bwd_both_cut" in names, names
    else:
        assert "attn_core_bwd_dq_cut" in names and "attn_core_bwd_dkv_cut" in names, names


@pytest.mark.parametrize("parts", [2, 5, 16])
@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("n_q,n_kv,tp,rank,d,n_seq,S", [CASES[0], CASES[1], CASES[2], CASES[5], CASES[6]])
def test_attn_core_fwd_cut_walks(workspace, opts, n_q, n_kv, tp, rank, d, n_seq, S, causal, parts):
    """The forward walk over the key tiles cut into pieces that are merged by their running maxima and sums."""
    _say(f"attn core fwd cut into {parts}: n_q={n_q} n_kv={n_kv} tp={tp} rank={rank} d={d} n_seq={n_seq} S={S} causal={causal}")
    opts(K.NTP_OPT_ATTN_PARTS, parts)
    _case(n_q, n_kv, tp, rank, d, n_seq, S, causal)
    assert _core_names() == ["attn_core_fwd_causal_cut" if causal else "attn_core_fwd_cut"]


@pytest.mark.parametrize("parts", [1, 3])
@pytest.mark.parametrize("n_q,n_kv,tp,rank,d,n_seq,S", [(8, 2, 3, 0, 128, 2, 440), (6, 6, 4, 1, 128, 1, 1100), (4, 4, 2, 0, 64, 3, 1)])
def test_attn_core_causal_pairs_odd_tile_counts(workspace, opts, n_q, n_kv, tp, rank, d, n_seq, S, parts):
    """Under the causal mask a workgroup takes a pair of tiles, one from each end of the sequence: 7 and 18 tiles (an odd
    count leaves the middle tile alone), a single tile, several sequences, whole walks and walks cut in three."""
    _say(f"attn core causal pairs: n_q={n_q} n_kv={n_kv} d={d} n_seq={n_seq} S={S} parts={parts}")
    opts(K.NTP_OPT_ATTN_PARTS, parts)
    _bwd_case(n_q, n_kv, tp, rank, d, n_seq, S, True, seed=11)


@pytest.mark.parametrize("copy", [1, 2], ids=["registers", "dma"])
@pytest.mark.parametrize("parts", [1, 3])
@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("n_q,n_kv,tp,rank,d,n_seq,S,pad", [(8, 2, 3, 0, 128, 2, 200, 0), (6, 6, 4, 1, 128, 1, 1100, 8),
                                                          (64, 8, 30, 3, 128, 2, 449, 0), (4, 1, 4, 3, 128, 1, 1, 0),
                                                          (6, 6, 4, 1, 128, 3, 64, 0), (8, 2, 3, 2, 128, 1, 129, 0)])
def test_attn_core_fwd_both_copy_forms(workspace, opts, n_q, n_kv, tp, rank, d, n_seq, S, pad, causal, parts, copy):
    """The kernels bring key / value tiles to LDS through registers or by DMA (the default at head dimension
    128 with 16 query rows per wavefront): both forms on ragged lengths, 1, 2, 3, 4, 8 and 18 key tiles, grouped KV
    heads, rows with padding between them, whole and cut walks."""
    _say(f"attn core fwd copy form {copy}: n_q={n_q} n_kv={n_kv} d={d} n_seq={n_seq} S={S} pad={pad} causal={causal} parts={parts}")
    opts(K.NTP_OPT_ATTN_PARTS, parts)
    opts(K.NTP_OPT_ATTN_COPY, copy)
    _case(n_q, n_kv, tp, rank, d, n_seq, S, causal, seed=17, pad=pad)


@pytest.mark.parametrize("copy", [1, 2], ids=["registers", "dma"])
@pytest.mark.parametrize("parts", [1, 3])
@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("n_q,n_kv,tp,rank,d,n_seq,S,pad", [(8, 2, 3, 0, 128, 2, 200, 0), (6, 6, 4, 1, 128, 1, 1100, 8),
                                                          (64, 8, 30, 3, 128, 2, 449, 0)])
def test_attn_core_bwd_both_copy_forms(workspace, opts, n_q, n_kv, tp, rank, d, n_seq, S, pad, causal, parts, copy):
    """The same two copy forms in the backward kernels, all three gradients against the oracle."""
    _say(f"attn core bwd copy form {copy}: n_q={n_q} n_kv={n_kv} d={d} n_seq={n_seq} S={S} pad={pad} causal={causal} parts={parts}")
    opts(K.NTP_OPT_ATTN_PARTS, parts)
    opts(K.NTP_OPT_ATTN_COPY, copy)
    _bwd_case(n_q, n_kv, tp, rank, d, n_seq, S, causal, seed=19, pad=pad)


@pytest.mark.parametrize("launches", [1, 2], ids=["two_launches", "one_launch"])
@pytest.mark.parametrize("parts", [1, 4])
@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("n_q,n_kv,tp,rank,d,n_seq,S,pad", [(8, 2, 3, 0, 128, 2, 200, 0), (6, 6, 4, 1, 128, 1, 1100, 8),
                                                          (64, 8, 30, 3, 128, 2, 449, 0), (4, 1, 4, 3, 128, 1, 1, 0)])
def test_attn_core_bwd_one_or_two_launches(workspace, opts, n_q, n_kv, tp, rank, d, n_seq, S, pad, causal, parts, launches):
    """The dQ and the dK/dV kernel as two launches or as one launch whose workgroups are of both kinds (after a kernel
    that stores the rows' delta values): grouped and ungrouped KV heads, ragged lengths, whole and cut walks (both
    kernels' parts side by side in the workspace)."""
    _say(f"attn core bwd, launches option {launches}: n_q={n_q} n_kv={n_kv} d={d} n_seq={n_seq} S={S} pad={pad} causal={causal} parts={parts}")
    opts(K.NTP_OPT_ATTN_PARTS, parts)
    opts(K.NTP_OPT_ATTN_BWD_LAUNCHES, launches)
    _bwd_case(n_q, n_kv, tp, rank, d, n_seq, S, causal, seed=23, pad=pad)
    names = [n for n in _core_names() if "bwd" in n]
    cut = "_cut" if parts > 1 else ""
    assert names == (["attn_core_bwd_both" + cut] if launches == 2 else ["attn_core_bwd_dq" + cut, "attn_core_bwd_dkv" + cut]), names


def test_attn_core_bwd_one_launch_needs_room_for_both_kernels_parts(opts):
    """With a workspace that holds either kernel's parts but not both, the cut kernels go out as two launches."""
    import torch
    import paper_2504_06095_amd as N
    _say("attn core bwd: workspace too small for one launch")
    # 3 heads on 1 KV head, 449 x 2 tokens: 16 tiles; 4 parts: dQ 16 x 3 x 4 x 32 KiB = 6 MiB, dK/dV 16 x 4 x 64 KiB = 4 MiB
    ws = torch.full(((7 << 20) // 4,), float("nan"), dtype=torch.float32, device="cuda")
    N.ntp_set_workspace(ws)
    N.ntp_kernel_timing_enable(1)
    N.ntp_kernel_timing_read()
    try:
        opts(K.NTP_OPT_ATTN_PARTS, 4)
        _bwd_case(64, 8, 30, 3, 128, 2, 449, True, seed=29)
        names = [n for n in _core_names() if "bwd" in n]
        assert names == ["attn_core_bwd_dq_cut", "attn_core_bwd_dkv_cut"], names
    finally:
        N.ntp_kernel_timing_enable(0)
        N.ntp_kernel_timing_read()
        N.ntp_set_workspace(None)


@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
def test_attn_core_at_the_step_shape(workspace, causal):
    """14 heads x 128, one sequence of 2048 tokens (the benchmark step's rank), the launcher's own choices with a
    workspace registered: forward, log-sum-exp and all three gradients against the oracle."""
    _say(f"attn core at the step's shape, causal={causal}")
    _bwd_case(96, 96, 7, 0, 128, 1, 2048, causal, seed=13)


@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
def test_attn_core_long_sequence_sampled_rows(workspace, causal):
    """14 heads x 128, one sequence of 8192 tokens (128 key tiles per walk; the forward kernel with 32 query rows per
    wavefront, the backward kernels with their longest walks of the benchmark): the oracle computes sampled query rows
    one by one (Eq. 5 is separable over query rows: row t needs the keys and values it sees and nothing else), output,
    log-sum-exp and dQ; the rows include the first and last of the sequence and both sides of tile borders.  One
    head is also computed in full for dQ, dK and dV."""
    import torch
    import paper_2504_06095_amd as N
    _say(f"attn core, 8192 tokens, sampled rows, causal={causal}")
    n_q, tp, d, S = 96, 7, 128, 8192
    plan = N.ntp_attn_shard_plan(n_q, n_q, d, tp, 0)
    qc = plan["q_cnt"]
    wq, wo = plan["w_qkv"], plan["w_o"]
    bits, vals = I.normal_bf16(31, f"core.long.QKV.{causal}", (S, wq), 1.0)
    gbits, gvals = I.normal_bf16(31, f"core.long.dC.{causal}", (S, wo), 1.0)
    QKV, dC = Hh.to_dev_bf16(bits, wq), Hh.to_dev_bf16(gbits, wo)
    nan = lambda r, c: torch.full((r, c), float("nan"), dtype=torch.bfloat16, device="cuda")
    C, dQKV = nan(S, wo), nan(S, wq)
    LSE = torch.full((qc, S), float("nan"), dtype=torch.float32, device="cuda")
    Delta = torch.full((qc, S), float("nan"), dtype=torch.float32, device="cuda")
    shape = N.attn_core_shape(1, S, plan, 1, causal)
    assert N.ntp_attn_core_choice(shape)["fwd_rows_per_wavefront"] == 32
    N.ntp_attn_core_shard_fwd(shape, QKV, C, LSE)
    N.ntp_attn_core_shard_bwd(shape, QKV, C, dC, LSE, Delta, dQKV)
    torch.cuda.synchronize()
    got_c, got_dq = Hh.dev_bf16_to_f64(C), Hh.dev_bf16_to_f64(dQKV)[:, :qc * d]
    assert np.isfinite(got_c).all() and np.isfinite(Hh.dev_bf16_to_f64(dQKV)).all()
    lse = LSE.cpu().numpy().astype(np.float64)
    rows = sorted({0, 1, 15, 16, 63, 64, 65, 127, 128, 129, 4095, 4096, 4097, 8127, 8128, 8190, 8191} |
                  {int(r) for r in np.random.default_rng(5).integers(0, S, 16)})
    x, g = vals.astype(np.float64), gvals.astype(np.float64)
    worst_c = worst_dq = 0.0
    for j in range(qc):
        Kh, Vh = x[:, (qc + j) * d:(qc + j + 1) * d], x[:, (2 * qc + j) * d:(2 * qc + j + 1) * d]
        want_c, want_dq, want_l = [], [], []
        for t in rows:
            n = t + 1 if causal else S
            q = x[t:t + 1, j * d:(j + 1) * d]
            want_c.append(O.attention_core(q, Kh[:n], Vh[:n])[0])
            want_l.append(O.attention_lse(q, Kh[:n])[0])
            want_dq.append(O.attention_core_bwd(q, Kh[:n], Vh[:n], g[t:t + 1, j * d:(j + 1) * d])[0][0])
        want_c, want_dq, want_l = np.array(want_c), np.array(want_dq), np.array(want_l)
        worst_c = max(worst_c, Hh.rel_err(got_c[rows, j * d:(j + 1) * d], want_c))
        worst_dq = max(worst_dq, Hh.rel_err(got_dq[rows, j * d:(j + 1) * d], want_dq))
        assert np.abs(lse[j, rows] - want_l).max() <= 2e-2 * max(1.0, np.abs(want_l).max()), j
    assert worst_c <= Hh.TOL and worst_dq <= Hh.TOL, (worst_c, worst_dq)
    # one head in full (its 8192 x 8192 scores fit the host): dQ, dK and dV of every token
    j = 5
    cols = lambda base: slice((base + j) * d, (base + j + 1) * d)
    dq, dk, dv = O.attention_core_bwd(x[:, cols(0)], x[:, cols(qc)], x[:, cols(2 * qc)], g[:, cols(0)], causal)
    got = Hh.dev_bf16_to_f64(dQKV)
    for name, base, want in (("dQ", 0, dq), ("dK", qc, dk), ("dV", 2 * qc, dv)):
        assert Hh.rel_err(got[:, cols(base)], want) <= Hh.TOL, (name, Hh.rel_err(got[:, cols(base)], want))


def test_attn_core_fwd_cut_peaked_scores(workspace, opts):
    """Large scores: the pieces' maxima differ by hundreds, so most pieces merge with weight zero."""
    _say("attn core fwd cut: peaked scores")
    opts(K.NTP_OPT_ATTN_PARTS, 7)
    _case(8, 2, 3, 1, 128, 1, 700, False, seed=4, std=6.0)
    _case(8, 2, 3, 1, 128, 1, 700, True, seed=4, std=6.0)


def test_attn_core_bwd_cut_chosen_for_few_heads(workspace):
    """No override: 3 heads of a 4096-token causal sequence are 192 (dQ) and 64 (dK, dV) workgroups with walks of
    up to 64 and 192 tiles, so both are cut; without a workspace neither is."""
    import paper_2504_06095_amd as N
    _say("attn core bwd: cut chosen at the config-3 shape")
    _bwd_case(64, 8, 30, 0, 128, 1, 4096, True, seed=5)
    names = _core_names()
    assert names == ["attn_core_fwd_causal_cut", "attn_core_bwd_both_cut"], names
    N.ntp_set_workspace(None)
    _bwd_case(64, 8, 30, 0, 128, 1, 1024, True, seed=5)
    names = _core_names()
    assert names == ["attn_core_fwd_causal", "attn_core_bwd_both"], names


def test_attn_core_bwd_padded_rows():
    _say("attn core bwd: padded leading dimensions")
    _bwd_case(8, 2, 3, 1, 128, 1, 300, True, seed=3, pad=8)


def test_attn_core_fwd_padded_rows_and_peaked_scores():
    _say("attn core fwd: padded leading dimensions, large scores")
    _case(8, 2, 3, 1, 128, 1, 300, True, seed=3, pad=8)
    # scores with a standard deviation of ~30: the softmax is nearly one-hot, the running maximum moves a lot
    _case(8, 2, 3, 1, 128, 1, 300, False, seed=4, std=5.0)


def test_attention_layer_end_to_end_sums_to_the_unsharded_layer():
    """Projection, core, projection on every rank of an uneven head split (3, 3, 2 heads): the partial
    outputs sum to the unsharded attention layer (Eq. 4-6)."""
    import torch
    import paper_2504_06095_amd as N
    _say("attention layer end to end, all ranks of TP 3 with 8 heads")
    n_q, n_kv, d, tp, H, S = 8, 2, 64, 3, 256, 160
    group = n_q // n_kv
    Xb, X = I.normal_bf16(9, "layer.X", (S, H), 1.0)
    ws = {}
    for name, shape in (("Wq", (H, n_q * d)), ("Wk", (H, n_kv * d)), ("Wv", (H, n_kv * d)), ("Wo", (n_q * d, H))):
        ws[name] = I.normal_bf16(9, "layer." + name, shape, 0.05)
    f = lambda k: ws[k][1].astype(np.float64)
    want = O.attn_unsharded_fwd(X.astype(np.float64), f("Wq"), f("Wk"), f("Wv"), f("Wo"), n_q, n_kv, d)
    Xd = Hh.to_dev_bf16(Xb)
    total = np.zeros((S, H))
    for r in range(tp):
        plan = N.ntp_attn_shard_plan(n_q, n_kv, d, tp, r)
        _, Wqkv_i, Wo_i = O.attn_shard_weights(ws["Wq"][0], ws["Wk"][0], ws["Wv"][0], ws["Wo"][0], n_q, n_kv, d, tp, r)
        wq, wo = plan["w_qkv"], plan["w_o"]
        Wqkv = Hh.to_dev_bf16(np.ascontiguousarray(Wqkv_i.T))  # stored [w_qkv x H]
        Wo = Hh.to_dev_bf16(np.ascontiguousarray(Wo_i))
        mk = lambda rr, cc: torch.full((rr, cc), float("nan"), dtype=torch.bfloat16, device="cuda")
        QKV, Cc, Z = mk(S, wq), mk(S, wo), mk(S, H)
        N.ntp_attn_proj_shard_fwd(S, H, wq, wo, Xd, Wqkv, QKV, None, None, None)
        N.ntp_attn_core_shard_fwd(N.attn_core_shape(1, S, plan, group, False), QKV, Cc, None)
        N.ntp_attn_proj_shard_fwd(S, H, wq, wo, None, None, None, Cc, Wo, Z)
        torch.cuda.synchronize()
        total += Hh.dev_bf16_to_f64(Z)
    assert Hh.rel_err(total, want) <= Hh.TOL, Hh.rel_err(total, want)


def test_attn_core_rejects_bad_arguments():
    import torch
    import paper_2504_06095_amd as N
    _say("attn core: error paths")
    K = N.binding
    plan = dict(q_cnt=2, kv_cnt=1, q_off=0, kv_off=0, head_dim=128)
    QKV = torch.zeros(64, 4 * 128, dtype=torch.bfloat16, device="cuda")
    Cc = torch.zeros(64, 2 * 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(N.NtpError) as e:  # head dimension not built
        N.ntp_attn_core_shard_fwd(N.attn_core_shape(1, 64, dict(plan, head_dim=96), 2), QKV, Cc)
    assert e.value.status == K.NTP_ERR_UNSUPPORTED
    with pytest.raises(N.NtpError) as e:  # a query head whose KV head is not local
        N.ntp_attn_core_shard_fwd(N.attn_core_shape(1, 64, dict(plan, q_off=2), 2), QKV, Cc)
    assert e.value.status == K.NTP_ERR_INVALID_ARG
    with pytest.raises(N.NtpError) as e:  # QKV narrower than the heads need
        N.ntp_attn_core_shard_fwd(N.attn_core_shape(1, 64, plan, 2), torch.zeros(64, 384, dtype=torch.bfloat16, device="cuda"), Cc)
    assert e.value.status == K.NTP_ERR_INVALID_ARG
    # one sequence's rows of QKV spanning 2 GiB or more (2^21 rows of 512 values): refused before anything is launched
    import ctypes as C
    big = N.attn_core_shape(1, 1 << 21, plan, 2)
    st = K.lib().ntp_attn_core_shard_fwd(N.default_handle().ptr, C.byref(big), QKV.data_ptr(), 512, Cc.data_ptr(), 256, None, None)
    assert st == K.NTP_ERR_UNSUPPORTED
