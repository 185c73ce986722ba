"""The shard calls inside a captured HIP graph: they allocate nothing and never synchronise, so a training
loop can capture a layer's calls once and replay them.  Every replay is compared bit for bit with the same
calls made eagerly on the same inputs, with eager work and synchronisations between the replays.
On a real MI355X."""
import sys

import pytest

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def _bf(torch, r, c, seed, scale=1.0):
    g = torch.Generator(device="cuda").manual_seed(seed)
    return (torch.randn(r, c, device="cuda", generator=g) * scale).to(torch.bfloat16)


def _layer(torch, N, M, H, n_r, plan, n_seq, with_workspace):
    """Buffers and a function that runs MLP shard fwd+bwd and the attention core fwd+bwd on them."""
    ld = (n_r + 7) // 8 * 8
    e = lambda r, c, dt=torch.bfloat16: torch.zeros(r, c, dtype=dt, device="cuda")
    b = dict(X=_bf(torch, M, H, 1), At=_bf(torch, n_r, H, 2, 0.03), B=_bf(torch, n_r, H, 3, 0.03), dZ=_bf(torch, M, H, 4),
             P=e(M, ld), Y=e(M, ld), dP=e(M, ld), Z=e(M, H), dX=e(M, H), dA=e(n_r, H, torch.float32), dB=e(n_r, H, torch.float32))
    wq, wo, q = plan["w_qkv"], plan["w_o"], plan["q_cnt"]
    b.update(QKV=_bf(torch, M, wq, 5), dC=_bf(torch, M, wo, 6), C=e(M, wo), dQKV=e(M, wq),
             LSE=e(q, M, torch.float32), Delta=e(q, M, torch.float32))
    shape = N.attn_core_shape(n_seq, M // n_seq, plan, 8, True)

    def run():
        N.ntp_mlp_shard_fwd(b["X"], b["At"], b["B"], b["P"][:, :n_r], b["Y"][:, :n_r], b["Z"], n_r, 0)
        N.ntp_mlp_shard_bwd(b["dZ"], b["X"], b["At"], b["B"], b["P"][:, :n_r], b["Y"][:, :n_r], b["dP"][:, :n_r], b["dX"],
                            b["dA"], b["dB"], n_r, 0, False)
        N.ntp_attn_core_shard_fwd(shape, b["QKV"], b["C"], b["LSE"])
        N.ntp_attn_core_shard_bwd(shape, b["QKV"], b["C"], b["dC"], b["LSE"], b["Delta"], b["dQKV"])
    return b, run


OUTPUTS = ("P", "Y", "Z", "dP", "dX", "dA", "dB", "C", "LSE", "dQKV")


@pytest.mark.parametrize("with_workspace", [False, True], ids=["plain", "split-K and cut walks"])
def test_layer_calls_replay_in_a_graph(with_workspace):
    import torch
    import paper_2504_06095_amd as N
    _say(f"graph capture of MLP shard + attention core, workspace {with_workspace}")
    M, H, n_r = 2048, 2048, 586                      # skinny: fc1 and dY are split when a workspace is there
    plan = N.ntp_attn_shard_plan(64, 8, 128, 30, 0)  # 3 heads: the core's walks are cut when a workspace is there
    if with_workspace:
        N.ntp_set_workspace(torch.empty(64 << 20, dtype=torch.float32, device="cuda"))
    try:
        b, run = _layer(torch, N, M, H, n_r, plan, 1, with_workspace)
        if with_workspace:
            N.ntp_kernel_timing_enable(1)
            N.ntp_kernel_timing_read()
            run()
            names = [r["name"] for r in N.ntp_kernel_timing_read()]
            N.ntp_kernel_timing_enable(0)
            assert any(n.startswith("gemm_") and "k" in n.split("_")[-1] for n in names), names
            assert "attn_core_bwd_both_cut" in names, names
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            run()  # warm-up on the capture stream
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                run()
        torch.cuda.synchronize()
        for rep in range(3):
            # new inputs in the captured buffers, eager reference first
            b["X"].copy_(_bf(torch, M, H, 10 + rep))
            b["dZ"].copy_(_bf(torch, M, H, 20 + rep))
            b["QKV"].copy_(_bf(torch, M, plan["w_qkv"], 30 + rep))
            run()
            torch.cuda.synchronize()
            want = {k: b[k].clone() for k in OUTPUTS}
            for k in OUTPUTS:
                b[k].fill_(7.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for k in OUTPUTS:
                same = torch.equal(b[k].view(torch.int16 if b[k].dtype == torch.bfloat16 else torch.int32),
                                   want[k].view(torch.int16 if want[k].dtype == torch.bfloat16 else torch.int32))
                assert same, f"replay {rep}: {k} differs from the eager result"
    finally:
        N.ntp_set_workspace(None)


def test_prepared_reshard_plan_replays_in_a_graph():
    """A reshard between the comp and sync layouts of the rank assignment (Alg. 1), prepared so that its run
    allocates nothing, captured and replayed with new gradients each time."""
    import numpy as np
    import torch
    import paper_2504_06095_amd as N
    _say("graph capture of a prepared reshard plan")
    k, t, tr, rows = 4096, 8, 7, 512
    comp, sync = N.ntp_comp_sync_plan(k, t, tr)
    comp, sync = np.asarray(comp), np.asarray(sync)
    plan = N.ntp_reshard_plan_create(N.tensor_spec(rows, k, 1, 1, 4), t, comp, tr, sync)
    try:
        src = [torch.zeros(rows, int((comp == r).sum()), dtype=torch.float32, device="cuda") for r in range(t)]
        dst = [torch.zeros(rows, int((sync == r).sum()), dtype=torch.float32, device="cuda") for r in range(tr)]
        plan.ntp_reshard_plan_prepare()
        side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                plan.ntp_reshard_plan_run(src, dst)
        torch.cuda.synchronize()
        for rep in range(3):
            G = torch.randn(rows, k, device="cuda", generator=torch.Generator(device="cuda").manual_seed(rep))
            for r in range(t):
                src[r].copy_(G[:, torch.from_numpy(np.nonzero(comp == r)[0]).cuda()])
            for d in dst:
                d.fill_(-1.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for r in range(tr):
                want = G[:, torch.from_numpy(np.nonzero(sync == r)[0]).cuda()]
                assert torch.equal(dst[r], want), f"replay {rep}: destination shard {r}"
    finally:
        plan.destroy()
